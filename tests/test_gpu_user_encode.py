"""co3_user_encode (the user's steps of an iteration in one call; where the batch fits, a resident grid
that reads every gradient once) against the CPU oracle, through the C ABI: anchors, symbols, memory,
counts, code lengths, streams, chunk offsets and the average, bit for bit."""
import numpy as np
import pytest

import oracle
import co3_inputs as inp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import oracle_user_side, check_user_side, ofmt, host_u32, host_u64   # noqa: E402


@pytest.fixture(scope="module")
def co3():
    import paper_2203_09044_amd as pkg
    return pkg


def run_one_call(co3, U, n, fmt, C, betas, alpha=1e-3, T=2, gamma=1.0, sizes=None, seed=0, keep_symbols=True,
                 adversarial=None):
    seg_off = None if sizes is None else inp.seg_offsets(sizes)
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, seg_off=seg_off, gamma=gamma, one_call=True,
                           keep_symbols=keep_symbols)
    errs = [np.zeros(n, np.float32) for _ in range(U)]
    g = pipe.new_gradient_buffer()
    for t in range(1, T + 1):
        g_host = []
        for u in range(U):
            r = inp.rng_for(98, seed, u, t)
            x = inp.gennorm(r, n, betas[u % len(betas)], alpha * (1.0 + 3.0 * ((u + t) % 3)))
            if adversarial is not None:
                x = adversarial(x, u, t)
            g_host.append(x)
        if n:
            g[:, :n] = torch.from_numpy(np.stack(g_host)).cuda()
        pipe.step(g)
        assert pipe.poll() == 0
        refs = []
        for u in range(U):
            ref = oracle_user_side(g_host[u], errs[u], fmt, seg_off, gamma, C)
            if keep_symbols:
                check_user_side(pipe, u, ref, n)
            else:
                assert np.array_equal(pipe.anchor[u].cpu().numpy(), ref["A"]), "anchor"
                assert np.array_equal(host_u32(pipe.err[u, :n]), ref["err"].view(np.uint32)), "error vector"
                assert np.array_equal(host_u32(pipe.counts[u]), ref["cnt"]), "histogram"
                assert np.array_equal(pipe.codes[u, :fmt.K].cpu().numpy(), ref["len"]), "code lengths"
                assert int(pipe.total_bits[u].item()) == ref["total"], "total bits"
                assert np.array_equal(host_u64(pipe.chunk_bitoff[u]), ref["off"]), "chunk offsets"
                nw = (ref["total"] + 63) // 64
                assert np.array_equal(host_u64(pipe.words[u, :nw]), ref["words"][:nw]), "stream words"
            errs[u] = ref["err"]
            refs.append(ref)
        want = oracle.aggregate(np.stack([r["sym"] for r in refs]) if n else np.zeros((U, 0), np.uint8),
                                np.stack([r["A"] for r in refs]), ofmt(fmt), seg_off)
        got = pipe.avg[:n].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), "average"
    return pipe


@pytest.mark.parametrize("E,M", [(3, 0), (3, 1), (2, 0), (4, 3), (5, 2), (1, 2)])
def test_one_call_formats(co3, E, M):
    # more than one run of 256 per wavefront on 256 compute units, ragged end, users of different shape and scale
    run_one_call(co3, 3, 256 * 2048 * 2 + 1237, co3.Fmt(E, M), 256, betas=[0.6, 1.0, 1.4], T=3)


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 255, 256, 257, 2047, 2048, 2049, 65_536, 65_541, 524_288, 524_289,
                               1_048_576 + 2048 + 7])
@pytest.mark.parametrize("keep", [True, False])
def test_one_call_sizes(co3, n, keep):
    run_one_call(co3, 2, n, co3.Fmt(3, 1), 64, betas=[1.0, 0.7], T=2, keep_symbols=keep)


def test_one_call_single_user_and_many_users(co3):
    run_one_call(co3, 1, 700_001, co3.Fmt(3, 0), 256, betas=[1.0], T=3)
    run_one_call(co3, 16, 70_001, co3.Fmt(3, 0), 128, betas=[0.5, 1.5], T=2)


def test_one_call_gamma_and_adversarial_values(co3):
    def adv(x, u, t):
        x = x.copy()
        # the largest magnitude sits in different workgroups' ranges, at both ends, and changes binade per user
        x[0 if (u + t) % 2 else -1] = np.float32(3.9 * 2.0 ** (u - t))
        x[len(x) // 2] = np.float32(-1e-30)        # far below every level
        x[len(x) // 3] = np.float32(0.0)
        return x
    run_one_call(co3, 4, 300_007, co3.Fmt(3, 1), 256, betas=[0.8], T=4, gamma=0.9, adversarial=adv)
    run_one_call(co3, 2, 300_007, co3.Fmt(1, 2), 256, betas=[1.2], T=3, gamma=0.0, adversarial=adv)


def test_one_call_zero_gradients_and_subnormal_maxima(co3):
    def zeros(x, u, t):
        return np.zeros_like(x) if u == 0 else (x * np.float32(1e-38)).astype(np.float32)
    run_one_call(co3, 2, 100_000, co3.Fmt(3, 1), 256, betas=[1.0], T=2, adversarial=zeros)


def test_one_call_with_tensors(co3):
    """Several tensors per user, one anchor each: up to six users the resident grid (maxima per tensor through
    atomics, runs with a tensor boundary converted with an anchor per element), more users the separate kernels."""
    sizes = [10, 1, 4097, 64, 3, 20_000, 7, 128, 0, 5, 12_345]
    run_one_call(co3, 2, sum(sizes), co3.Fmt(4, 3), 256, betas=[0.8], T=2, sizes=sizes)
    run_one_call(co3, 2, sum(sizes), co3.Fmt(4, 3), 256, betas=[0.8], T=2, sizes=sizes, keep_symbols=False)
    run_one_call(co3, 6, sum(sizes), co3.Fmt(4, 3), 256, betas=[0.8], T=2, sizes=sizes)
    run_one_call(co3, 9, sum(sizes), co3.Fmt(4, 3), 256, betas=[0.8], T=2, sizes=sizes)


def tensor_sizes(total, seed):
    """Tensors of a network-like mix: a few large ones, runs of small ones (64 ... 512), single elements and empty ones."""
    rng = inp.rng_for(97, seed)
    sizes = []
    while sum(sizes) < total:
        kind = rng.integers(0, 10)
        if kind < 3:
            sizes.append(int(rng.integers(total // 40, total // 8)))
        elif kind < 8:
            sizes.extend([int(rng.choice([64, 128, 256, 512]))] * 2)
        elif kind == 8:
            sizes.extend([1, 0, int(rng.integers(2, 300))])
        else:
            sizes.append(int(rng.integers(1000, 50_000)))
    sizes[-1] -= sum(sizes) - total
    if sizes[-1] < 0:
        sizes = sizes[:-1] + [0]
        while sum(sizes) > total:
            sizes.pop(0)
        sizes.append(total - sum(sizes))
    return sizes


@pytest.mark.parametrize("total,U,E,M,keep", [(1_200_003, 3, 3, 1, True), (2_600_017, 2, 2, 0, False), (6_000_001, 1, 4, 3, False),
                                              (14_000_021, 2, 3, 0, False)])
def test_tensors_in_every_form_of_the_resident_grid(co3, total, U, E, M, keep):
    """Sizes that select, on 256 compute units, 4, 12, 22 and 32 runs per lane of the form with one anchor per tensor;
    tensor boundaries inside runs, runs that hold several small tensors, empty and one-element tensors."""
    sizes = tensor_sizes(total, total % 97)
    assert sum(sizes) == total and min(sizes) >= 0
    run_one_call(co3, U, total, co3.Fmt(E, M), 256, betas=[0.7, 1.2, 1.0], T=2, sizes=sizes, keep_symbols=keep)


def test_one_call_deterministic(co3):
    a = run_one_call(co3, 3, 400_003, co3.Fmt(3, 0), 256, betas=[0.5, 1.0, 1.5], T=2)
    b = run_one_call(co3, 3, 400_003, co3.Fmt(3, 0), 256, betas=[0.5, 1.0, 1.5], T=2)
    assert torch.equal(a.words, b.words) and torch.equal(a.err, b.err) and torch.equal(a.avg, b.avg)


@pytest.mark.parametrize("kind,n,sizes", [("one tensor", 300_000, None), ("tensors", 300_000, [100_000, 7, 150_000, 0, 49_993]),
                                          ("long vector", 17_000_003, None)])
def test_a_wait_that_runs_out_is_reported_and_the_kernel_ends(co3, kind, n, sizes):
    """No poll allowed: every exchange of the resident grid runs out at once (in each of its forms: one anchor per
    user, one per tensor, part of the gradient in LDS).  The call must come back with CO3_ETIMEOUT in the status
    word, having written nothing out of bounds (canaries), and the next call works."""
    B = co3.binding
    fmt = co3.Fmt(3, 0)
    U = 2
    assert sizes is None or sum(sizes) == n
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=256, one_call=True, seg_off=None if sizes is None else inp.seg_offsets(sizes))
    g = pipe.new_gradient_buffer()
    for u in range(U):
        g[u, :n] = inp.device_gennorm(n, 1.0, 1e-3, 40 + u)
    pad = pipe.err[:, n:].clone()
    try:
        B.set_exchange_spin_limit(0)
        pipe.user_encode(g)
        assert pipe.poll() == B.ETIMEOUT
    finally:
        B.set_exchange_spin_limit(-1)
    assert torch.equal(pipe.err[:, n:], pad)
    pipe.status.zero_()
    pipe.err.zero_()
    pipe.step(g)
    assert pipe.poll() == 0


@pytest.mark.parametrize("n", [1, 255, 256, 1023, 5631, 5632, 5633, 256 * 2048 * 3 + 17])
def test_ragged_ends_of_the_resident_grid(co3, n):
    """Sizes around the boundaries of the resident grid's parts (whole parts in the grid, the ragged end in
    the kernel that finishes the users, parts with no element at all)."""
    run_one_call(co3, 4, n, co3.Fmt(3, 1), 64, betas=[0.7, 1.2], T=2, seed=n)
    run_one_call(co3, 4, n, co3.Fmt(3, 0), 64, betas=[0.7, 1.2], T=2, seed=n + 1, keep_symbols=False)


@pytest.mark.parametrize("n,E,M,keep", [(12_000_037, 3, 0, False), (16_777_216 + 333, 4, 3, True), (17_000_003, 2, 0, False),
                                        (20_900_001, 3, 1, True), (24_000_005, 3, 0, False), (25_165_824, 4, 3, False)])
def test_vectors_beyond_the_registers_of_the_device(co3, n, E, M, keep):
    """On 256 compute units these sizes select the forms of the resident grid with 32 runs of 256 elements per
    lane in registers, and with 34 in registers plus 6 or 14 in LDS (the last size fills that form exactly)."""
    run_one_call(co3, 2, n, co3.Fmt(E, M), 256, betas=[0.8, 1.3], T=2, keep_symbols=keep)


def test_ten_chained_iterations_at_a_size_that_fills_the_device(co3):
    run_one_call(co3, 6, 256 * 2048 * 8 + 999, co3.Fmt(3, 0), 256, betas=[0.5, 1.5, 1.0], T=10, keep_symbols=False)
    run_one_call(co3, 2, 256 * 2048 * 12 + 1, co3.Fmt(4, 3), 256, betas=[0.8], T=2)


def test_the_two_halves_of_the_aggregate(co3):
    """co3_ps_decode_users for groups of users followed by co3_ps_average = co3_ps_aggregate, bit for bit."""
    B = co3.binding
    fmt = co3.Fmt(3, 1)
    U, n, C = 7, 200_003, 256
    pipe = run_one_call(co3, U, n, fmt, C, betas=[0.6, 1.0, 1.5], T=1)
    want = pipe.avg.clone()
    for cuts in ([0, 3, 7], [0, 1, 2, 7], [0, 7]):
        ws = torch.zeros((B.ps_aggregate_workspace_bytes(n, U, C),), dtype=torch.uint8, device="cuda")
        for a, b in reversed(list(zip(cuts[:-1], cuts[1:]))):         # any order of the groups
            B.ps_decode_users(pipe.words[a:b], pipe.chunk_bitoff[a:b], C, pipe.codes[a:b], fmt, n, b - a, a, U, ws, pipe.status)
        out = torch.full_like(pipe.avg, float("nan"))
        B.ps_average(ws, C, fmt, n, U, pipe.anchor, out)
        assert pipe.poll() == 0
        assert torch.equal(out[:n].view(torch.int32), want[:n].view(torch.int32)), cuts
    L = B._lib
    assert L.co3_ps_decode_users(None, 2, None, 256, None, fmt.c(), 10, 1, 0, 1, None, 0, None, None) == B.EINVAL
    assert L.co3_ps_average(None, 0, 256, fmt.c(), 10, 1, None, None, 1, None, None) == B.EINVAL


def test_average_continued_over_groups_of_users(co3):
    """co3_ps_aggregate_partial: sums over groups of users chained through acc_in, one division at the end =
    co3_ps_aggregate over all users = the oracle's average, bit for bit; acc_in may be the output array; an
    undivided partial sum is the plain fp32 sum of the group's values."""
    B = co3.binding
    fmt = co3.Fmt(3, 1)
    U, n, C = 7, 200_003, 256
    pipe = run_one_call(co3, U, n, fmt, C, betas=[0.6, 1.0, 1.5], T=1)
    want = pipe.avg.clone()
    for cuts in ([0, 3, 7], [0, 1, 2, 7], [0, 7], [0, 2, 4, 6, 7]):
        acc = torch.zeros_like(pipe.avg)
        out = torch.full_like(pipe.avg, float("nan"))
        for j, (a, b) in enumerate(zip(cuts[:-1], cuts[1:])):
            last = b == U
            ws = torch.zeros((B.ps_aggregate_workspace_bytes(n, b - a, C),), dtype=torch.uint8, device="cuda")
            B.ps_aggregate_partial(pipe.words[a:b], pipe.chunk_bitoff[a:b], C, pipe.codes[a:b], fmt, n, b - a,
                                   pipe.anchor[a:b], None if j == 0 else acc, U if last else 0, out if last else acc,
                                   ws, pipe.status)
        assert pipe.poll() == 0
        assert torch.equal(out[:n].view(torch.int32), want[:n].view(torch.int32)), cuts
    # an undivided sum of users 2..4 against the oracle's values added in order
    f = ofmt(fmt)
    ws = torch.zeros((B.ps_aggregate_workspace_bytes(n, 3, C),), dtype=torch.uint8, device="cuda")
    part = torch.zeros_like(pipe.avg)
    B.ps_aggregate_partial(pipe.words[2:5], pipe.chunk_bitoff[2:5], C, pipe.codes[2:5], fmt, n, 3, pipe.anchor[2:5], None, 0,
                           part, ws, pipe.status)
    s = np.zeros(n, np.float32)
    for u in range(2, 5):
        s = s + oracle.aggregate(pipe.sym[u:u + 1, :n].cpu().numpy(), pipe.anchor[u:u + 1].cpu().numpy(), f)
    assert np.array_equal(part[:n].cpu().numpy().view(np.uint32), s.view(np.uint32))
    assert B._lib.co3_ps_aggregate_partial(None, 2, None, 256, None, fmt.c(), 10, 1, None, None, 1, None, -1, None, None, 0,
                                           None, None) == B.EINVAL


@pytest.mark.parametrize("E,M", [(3, 0), (2, 0), (1, 2)])
@pytest.mark.parametrize("n", [1, 3, 5, 255, 1023, 1025, 5631, 5633, 65_541, 256 * 2048 + 4097])
def test_symbols_kept_inside_the_call_take_four_bits(co3, E, M, n):
    """Alphabets of at most 16 symbols with no symbol array asked for: between conversion and compression
    the symbols are held two per byte.  Everything that leaves the call must be what the oracle says."""
    run_one_call(co3, 3, n, co3.Fmt(E, M), 64, betas=[0.6, 1.0, 1.6], T=2, keep_symbols=False, seed=n)


def test_symbols_kept_inside_the_call_with_tensors(co3):
    """The same on the path of the separate kernels (several tensors per user: anchors per tensor, tiles that
    straddle tensors, one-element and empty tensors, a ragged end)."""
    for sizes in ([70_000, 13, 300_001, 1, 0, 50_000], [3, 3, 3, 2], [1024, 1, 1023, 2048 + 7]):
        run_one_call(co3, 2, sum(sizes), co3.Fmt(3, 0), 256, betas=[0.8, 1.3], T=2, sizes=sizes, keep_symbols=False)
        run_one_call(co3, 3, sum(sizes), co3.Fmt(1, 2), 64, betas=[1.0], T=2, sizes=sizes, keep_symbols=False, gamma=0.9)
