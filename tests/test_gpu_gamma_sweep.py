"""Memory decay sweep (Sec. III (iii)) on the 4-bit format of Sec. IV-C ([sign mantissa exponent] =
[1 2 1], i.e. E1M2; the best decay there is 0.9): for gamma in {0, 0.1, 0.5, 0.9, 1} a chain of
iterations is compared with the oracle bit for bit, and the diagnostic of Sec. IV-B (L1 norm of the
memory relative to the L1 norm of the gradient) and the rate are read from the device and compared
with the oracle's.

The two-rounding form x = fl32(g + fl32(gamma * m)) matters for every gamma that is not 0 or 1.
"""
import numpy as np
import pytest

import oracle
import co3_inputs as inp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

GAMMAS = (0.0, 0.1, 0.5, 0.9, 1.0)


@pytest.fixture(scope="module")
def co3():
    import paper_2203_09044_amd as pkg
    return pkg


def device_l1(co3, x2d, n):
    """sum |x| per row through the library's moment kernel (gamma = 0 drops the second operand)."""
    U = x2d.shape[0]
    sums = torch.zeros((U, 1, 2), dtype=torch.float64, device="cuda")
    co3.binding.moments(x2d, x2d, n, 0.0, sums)
    return sums[:, 0, 0].cpu().numpy()


@pytest.mark.parametrize("bias", ["absmax", "moments"])
def test_gamma_sweep_chain(co3, bias):
    fmt = co3.Fmt(1, 2)
    f = oracle.Fmt(1, 2)
    U, n, T, C = 2, 60_000 + 13, 6, 256
    ratios = {}
    rates = {}
    for gamma in GAMMAS:
        pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, gamma=gamma, bias=bias, grid_anchor=1)
        g = pipe.new_gradient_buffer()
        errs = [np.zeros(n, np.float32) for _ in range(U)]
        for t in range(1, T + 1):
            gh = [inp.gennorm(inp.rng_for(55, u, t), n, (0.8, 1.3)[u], 1e-3) for u in range(U)]
            g[:, :n] = torch.from_numpy(np.stack(gh)).cuda()
            if bias == "moments":
                scale_o = np.stack([oracle.bias_scales(gh[u], errs[u], gamma) for u in range(U)])
                pipe.fit_bias(g)
                got = pipe.scale.cpu().numpy()
                assert np.all(np.abs(got.view(np.int32).astype(np.int64) - scale_o.view(np.int32).astype(np.int64)) <= 2)
                pipe.scale.copy_(torch.from_numpy(scale_o).cuda())
            pipe.convert(g)
            pipe.build()
            pipe.encode()
            pipe.aggregate()
            assert pipe.poll() == 0
            syms, anchors = [], []
            for u in range(U):
                if bias == "moments":
                    A = np.array([1], np.int32)
                    sym, e_new = oracle.convert_ef(gh[u], errs[u], A, gamma, f, scale=scale_o[u])
                else:
                    A = oracle.anchor(gh[u], f)
                    sym, e_new = oracle.convert_ef(gh[u], errs[u], A, gamma, f)
                assert np.array_equal(pipe.sym[u, :n].cpu().numpy(), sym), (gamma, t, u)
                assert np.array_equal(pipe.err[u, :n].cpu().numpy().view(np.uint32), e_new.view(np.uint32)), (gamma, t, u)
                cnt = oracle.histogram(sym, f)
                l = oracle.huffman_lengths(cnt)
                _, _, total = oracle.encode(sym, l, oracle.canonical_codes(l), C)
                assert int(pipe.total_bits[u].item()) == total
                errs[u] = e_new
                syms.append(sym)
                anchors.append(A)
            want = oracle.aggregate(np.stack(syms), np.stack(anchors), f,
                                    scale=scale_o if bias == "moments" else None)
            assert np.array_equal(pipe.avg[:n].cpu().numpy().view(np.uint32), want.view(np.uint32))
        # diagnostic after the last iteration: ||m||_1 / ||g||_1 per user, device vs oracle
        l1_m = device_l1(co3, pipe.err, n)
        l1_g = device_l1(co3, g, n)
        for u in range(U):
            om = oracle.moments(errs[u], errs[u], 0.0)[0, 0]
            og = oracle.moments(gh[u], gh[u], 0.0)[0, 0]
            assert l1_m[u] == pytest.approx(om, rel=1e-12)
            assert l1_g[u] == pytest.approx(og, rel=1e-12)
        ratios[gamma] = float(np.mean(l1_m / l1_g))
        rates[gamma] = float(pipe.total_bits.sum().item()) / (U * n)
    # carried memory grows with the decay coefficient (the trend the paper's diagnostic shows)
    r = [ratios[gm] for gm in GAMMAS]
    assert all(b >= a * 0.999 for a, b in zip(r, r[1:])), r
    print(f"\n[gamma sweep, bias={bias}] " +
          "  ".join(f"gamma={gm}: |m|1/|g|1={ratios[gm]:.4f} rate={rates[gm]:.3f} b/elem" for gm in GAMMAS))
