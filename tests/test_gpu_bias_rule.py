"""HIP path vs CPU oracle for the paper's bias rule (Sec. III (i), Eq. (exp bias); Sec. IV-B,
Eq. (approximate)), through the C ABI (GPU only).

Bars.  Moment sums: fp64 sums whose order of additions differs from the oracle's sequential order:
1e-12 relative.  Fit and multiplier: the device evaluates log-gamma with its own math library: shape and
scale within 1e-9 relative, the fp32 multiplier within 2 units in the last place.  Conversion, memory,
histogram, streams and the average with GIVEN multipliers: bit for bit (the multipliers handed to both
sides are the oracle's).
"""
import numpy as np
import pytest

import oracle
import co3_inputs as inp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def co3():
    import paper_2203_09044_amd as pkg
    return pkg


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def u64(t):
    return t.cpu().numpy().view(np.uint64)


def ulp_distance(a, b):
    a = np.asarray(a, np.float32).view(np.int32).astype(np.int64)
    b = np.asarray(b, np.float32).view(np.int32).astype(np.int64)
    return np.abs(a - b)


CASES = [
    # U, n, sizes, gamma
    (1, 1, None, 1.0),
    (1, 100, None, 1.0),
    (3, 4096, None, 0.9),
    (2, 16385, None, 1.0),
    (4, 70001, None, 0.0),
    (2, 50000, [10, 0, 4086, 1, 33000, 12903], 1.0),
    (1, 300000, [64, 64, 147456, 128, 128, 152160], 0.9),
]


def draw(U, n, seed):
    g = np.stack([inp.gennorm(inp.rng_for(77, seed, u), n, (0.6, 1.0, 1.4)[u % 3], 10.0 ** -(1 + u % 4)) for u in range(U)])
    e = np.stack([inp.gennorm(inp.rng_for(78, seed, u), n, 1.0, 10.0 ** -(2 + u % 4)) for u in range(U)])
    return g.astype(np.float32), e.astype(np.float32)


@pytest.mark.parametrize("U,n,sizes,gamma", CASES)
def test_moments_and_fit(co3, U, n, sizes, gamma):
    B = co3.binding
    seg = None if sizes is None else inp.seg_offsets(sizes)
    nseg = 1 if seg is None else len(seg) - 1
    stride = (n + 15) // 16 * 16
    gh, eh = draw(U, n, n)
    g = torch.zeros((U, stride), dtype=torch.float32, device="cuda")
    e = torch.zeros_like(g)
    g[:, :n] = torch.from_numpy(gh).cuda()
    e[:, :n] = torch.from_numpy(eh).cuda()
    seg_t = None if seg is None else torch.as_tensor(seg, dtype=torch.int64).cuda()
    sums = torch.full((U, nseg, 2), -1.0, dtype=torch.float64, device="cuda")
    B.moments(g, e, n, gamma, sums, seg_off=seg_t)
    want = np.stack([oracle.moments(gh[u], eh[u], gamma, seg) for u in range(U)])
    got = sums.cpu().numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=0.0)
    assert np.array_equal(got == 0.0, want == 0.0)

    # the fit and the multiplier from the ORACLE's sums (uploaded), so that only the fit is compared
    sums_o = torch.from_numpy(want).cuda()
    scale = torch.zeros((U, nseg), dtype=torch.float32, device="cuda")
    fit = torch.zeros((U, nseg, 2), dtype=torch.float64, device="cuda")
    B.bias_scale(sums_o, n, U, scale, fit=fit, seg_off=seg_t)
    so = [0, n] if seg is None else seg
    for u in range(U):
        for s in range(nseg):
            b, a = oracle.gennorm_fit(want[u, s, 0], want[u, s, 1], so[s + 1] - so[s])
            fb, fa = fit[u, s].cpu().numpy()
            assert fb == pytest.approx(b, rel=1e-9)
            assert fa == pytest.approx(a, rel=1e-9, abs=0.0)
            c = oracle.bias_scale(b, a)
            assert ulp_distance(scale[u, s].item(), c) <= 2, (scale[u, s].item(), c)


def test_fit_edge_cases(co3):
    """Zero tensor, constant magnitude (ratio 1, above the uniform limit), a single spike (ratio ~ 0),
    exact Gaussian / Laplace population moments, huge and tiny scales."""
    B = co3.binding
    n = 1000
    rows = [(0.0, 0.0), (1000.0, 1000.0), (1.0, 1.0),
            (n * np.sqrt(2 / np.pi), n * 1.0), (n * 1.0, n * 2.0),
            (n * 1e-30, n * 2e-60), (n * 1e30, n * 2e60)]
    sums = torch.tensor(rows, dtype=torch.float64, device="cuda").reshape(len(rows), 1, 2)
    scale = torch.zeros((len(rows), 1), dtype=torch.float32, device="cuda")
    fit = torch.zeros((len(rows), 1, 2), dtype=torch.float64, device="cuda")
    B.bias_scale(sums, n, len(rows), scale, fit=fit)
    for r, (s1, s2) in enumerate(rows):
        b, a = oracle.gennorm_fit(s1, s2, n)
        assert fit[r, 0, 0].item() == pytest.approx(b, rel=1e-9)
        assert fit[r, 0, 1].item() == pytest.approx(a, rel=1e-9, abs=0.0)
        assert ulp_distance(scale[r, 0].item(), oracle.bias_scale(b, a)) <= 2
    assert scale[0, 0].item() == 1.0
    assert fit[1, 0, 0].item() == 50.0 and fit[2, 0, 0].item() < 0.1
    assert fit[3, 0, 0].item() == pytest.approx(2.0, rel=1e-9) and fit[4, 0, 0].item() == pytest.approx(1.0, rel=1e-9)
    assert scale[5, 0].item() == 2.0 ** 96 or scale[5, 0].item() == pytest.approx(0.65 / 1e-30, rel=1e-6)


FORMATS = [(1, 2, 1), (2, 1, 2), (3, 0, 4), (3, 1, 4), (4, 3, 8), (5, 2, 16)]


@pytest.mark.parametrize("E,M,A0", FORMATS)
@pytest.mark.parametrize("U,n,sizes,gamma", CASES[2:])
def test_scaled_path_bit_exact(co3, E, M, A0, U, n, sizes, gamma):
    """Whole iteration with the multipliers of the oracle's bias rule handed to both sides."""
    fmt = co3.Fmt(E, M)
    f = oracle.Fmt(E, M)
    seg = None if sizes is None else inp.seg_offsets(sizes)
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=128, seg_off=seg, gamma=gamma, bias="moments", grid_anchor=A0)
    gh, eh = draw(U, n, 1000 + n + E)
    g = pipe.new_gradient_buffer()
    g[:, :n] = torch.from_numpy(gh).cuda()
    pipe.err[:, :n] = torch.from_numpy(eh).cuda()
    scale_o = np.stack([oracle.bias_scales(gh[u], eh[u], gamma, seg) for u in range(U)])
    # the device's own multipliers agree to rounding; then the oracle's are installed for the bit-exact part
    pipe.fit_bias(g)
    assert np.all(ulp_distance(pipe.scale.cpu().numpy(), scale_o) <= 2)
    pipe.scale.copy_(torch.from_numpy(scale_o).cuda())
    pipe.convert(g)
    pipe.build()
    pipe.encode()
    pipe.aggregate()
    pipe.decode()
    assert pipe.poll() == 0
    A = np.full(pipe.nseg, A0, np.int32)
    syms = []
    for u in range(U):
        sym, e_new = oracle.convert_ef(gh[u], eh[u], A, gamma, f, seg, scale=scale_o[u])
        syms.append(sym)
        assert np.array_equal(pipe.sym[u, :n].cpu().numpy(), sym), "symbols"
        assert np.array_equal(u32(pipe.err[u, :n]), e_new.view(np.uint32)), "memory"
        cnt = oracle.histogram(sym, f)
        assert np.array_equal(u32(pipe.counts[u]), cnt), "histogram"
        l = oracle.huffman_lengths(cnt)
        words, off, total = oracle.encode(sym, l, oracle.canonical_codes(l), 128)
        assert int(pipe.total_bits[u].item()) == total
        nw = (total + 63) // 64
        assert np.array_equal(u64(pipe.words[u, :nw]), words[:nw]), "stream"
        assert np.array_equal(pipe.sym_dec[u, :n].cpu().numpy(), sym), "round trip"
    want = oracle.aggregate(np.stack(syms), np.tile(A, (U, 1)), f, seg, scale=scale_o)
    assert np.array_equal(u32(pipe.avg[:n]), want.view(np.uint32)), "average"


def test_scaled_adversarial_values(co3):
    """Multipliers at the limits and values whose product overflows, underflows or lands on midpoints."""
    fmt = co3.Fmt(1, 2)
    f = oracle.Fmt(1, 2)
    vals = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-38, 3.4e38, -3.4e38, np.inf, -np.inf, 0.25, 0.75, 1.25, 1.75, 2.25,
                     2.75, 3.25, 3.5, 3.75, 4.0, 1e-3, -1e-3, 0.4999999, 0.5000001], np.float32)
    for c in (2.0 ** -96, 1e-10, 0.3, 1.0, 3.0, 650.0, 1e10, 2.0 ** 96):
        gh = np.concatenate([vals, (vals / np.float32(c)).astype(np.float32)])
        gh = gh[np.isfinite(gh) | np.isinf(gh)]
        n = gh.size
        pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=64, bias="moments", grid_anchor=1)
        g = pipe.new_gradient_buffer()
        g[0, :n] = torch.from_numpy(gh).cuda()
        pipe.scale.fill_(float(np.float32(c)))
        pipe.convert(g)
        assert pipe.poll() == 0
        sc = np.array([c], np.float32)
        sym, e_new = oracle.convert_ef(gh, np.zeros(n, np.float32), np.array([1], np.int32), 1.0, f, scale=sc)
        assert np.array_equal(pipe.sym[0, :n].cpu().numpy(), sym), c
        got, want = u32(pipe.err[0, :n]), e_new.view(np.uint32)
        nan = np.isnan(e_new)
        assert np.array_equal(got[~nan], want[~nan]), c
        assert np.all(np.isnan(pipe.err[0, :n].cpu().numpy()[nan]))


def test_rule_lowers_l2_error_on_device(co3):
    """The purpose of the bias (Sec. III (i)): on the 4-bit format the rule's squared error is well below
    the max-anchor's, measured from the device's own memory vectors after one iteration."""
    fmt = co3.Fmt(1, 2)
    n = 1 << 20
    x = inp.device_gennorm(n, 1.0, 1e-3, 4242)
    out = {}
    for bias in ("absmax", "moments"):
        pipe = co3.Co3Pipeline(1, n, fmt, bias=bias, grid_anchor=1)
        g = pipe.new_gradient_buffer()
        g[0, :n] = x
        pipe.step(g)
        assert pipe.poll() == 0
        out[bias] = float((pipe.err[0, :n].double() ** 2).sum().item())
        # the server's average of one user is that user's reconstruction: g - m'
        recon = (g[0, :n] - pipe.err[0, :n])
        assert torch.allclose(pipe.avg[:n], recon, rtol=1e-6, atol=1e-12)
    assert out["moments"] < 0.5 * out["absmax"]


def test_host_rejected_arguments(co3):
    B = co3.binding
    g = torch.zeros((1, 64), dtype=torch.float32, device="cuda")
    sums = torch.zeros((1, 1, 2), dtype=torch.float64, device="cuda")
    scale = torch.zeros((1, 1), dtype=torch.float32, device="cuda")
    with pytest.raises(co3.Co3Error):
        B.moments(g, g, -1, 1.0, sums)
    with pytest.raises(co3.Co3Error):
        B._chk(B._lib.co3_bias_scale(None, 64, 1, None, 1, B._dp(scale), None, B._stream()), "co3_bias_scale")
    with pytest.raises(co3.Co3Error):
        B._chk(B._lib.co3_bias_scale(B._dp(sums), 64, 1, None, 2, B._dp(scale), None, B._stream()), "co3_bias_scale")
