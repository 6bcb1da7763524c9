"""Parity at the full sizes of the five benchmark workloads, in the launch configurations that
bench.py times (chunk 256, fused histogram, tiled averaging workspace; one call per iteration for the
user side where the benchmark uses it).

Every element of every client goes through the oracle (threads over clients; the oracle itself stays
single-threaded per call): C1 for its 5 iterations, C2, C3, C4 and all 12 points of C5 for iterations
1-2 of all clients, and one client of each of C2, C3, C4 and C5 point 7 over the workload's full
number of chained iterations.  On top, properties that hold at any size are checked on every client:
decode(encode(s)) = s, coded length = sum of count * length, chunk offsets consistent with the stream
length, histogram total = n.
Inputs are drawn on the device with the seeded sampler and copied back, so both sides consume
the same bytes.
"""
from concurrent.futures import ThreadPoolExecutor

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


def oracle_client(args):
    g, err, E, M, seg_off, C, weights = args
    f = oracle.Fmt(E, M)
    A = oracle.anchor(g, f, seg_off)
    sym, e_new = oracle.convert_ef(g, err, A, 1.0, f, seg_off)
    cnt = oracle.histogram(sym, f)
    l = oracle.huffman_lengths(cnt if weights is None else weights)
    words, off, total = oracle.encode(sym, l, oracle.canonical_codes(l), C)
    return dict(A=A, sym=sym, err=e_new, cnt=cnt, len=l, words=words, off=off, total=total)


def compare_client(pipe, u, ref, n):
    assert np.array_equal(pipe.anchor[u].cpu().numpy(), ref["A"]), "anchor"
    assert np.array_equal(pipe.sym[u, :n].cpu().numpy(), ref["sym"]), "symbols"
    assert np.array_equal(u32(pipe.err[u, :n]), ref["err"].view(np.uint32)), "error vector"
    assert np.array_equal(u32(pipe.counts[u]), ref["cnt"]), "histogram"
    assert np.array_equal(pipe.codes[u, :pipe.fmt.K].cpu().numpy(), ref["len"]), "code lengths"
    assert int(pipe.total_bits[u].item()) == ref["total"], "total bits"
    assert np.array_equal(u64(pipe.chunk_bitoff[u]), ref["off"]), "chunk offsets"
    nw = (ref["total"] + 63) // 64
    assert np.array_equal(u64(pipe.words[u, :nw]), ref["words"][:nw]), "stream words"


def properties_all_clients(pipe, n):
    """Size-independent checks on every client, from GPU results only."""
    pipe.decode()
    assert pipe.poll() == 0
    assert torch.equal(pipe.sym_dec[:, :n], pipe.sym[:, :n]), "decode(encode(s)) = s"
    cnt = pipe.counts.cpu().numpy().view(np.uint32).astype(np.int64)
    lens = pipe.codes[:, :pipe.fmt.K].cpu().numpy().astype(np.int64)
    assert np.all(cnt.sum(axis=1) == n)
    tot = pipe.total_bits.cpu().numpy().astype(np.int64)
    assert np.array_equal(tot, (cnt * lens).sum(axis=1)), "coded length = sum count * length"
    off = pipe.chunk_bitoff.cpu().numpy().astype(np.int64)
    assert np.all(off[:, 0] == 0) and np.array_equal(off[:, -1], tot) and np.all(np.diff(off, axis=1) > 0)
    for u in range(pipe.U):          # Kraft equality of every client's code
        l = lens[u][lens[u] > 0]
        if l.size >= 2:
            assert abs(float(np.sum(np.exp2(-l.astype(np.float64)))) - 1.0) < 1e-12


def fill_from_device(pipe, g, draw):
    host = []
    for u in range(pipe.U):
        x = draw(u)
        g[u, :pipe.n] = x
        host.append(x.cpu().numpy())
    return host


def test_c1_full(co3):
    """C1: 65,536 elements, E3M1, 5 error-feedback iterations, every element."""
    w = inp.c1()
    fmt = co3.Fmt(w.E, w.M)
    pipe = co3.Co3Pipeline(1, w.n, fmt, chunk_syms=256)
    g = pipe.new_gradient_buffer()
    err = np.zeros(w.n, np.float32)
    for t in range(1, w.T + 1):
        gh = inp.host_gradient(w, 0, t)
        g[0, :w.n] = torch.from_numpy(gh).cuda()
        pipe.step(g)
        assert pipe.poll() == 0
        ref = oracle_client((gh, err, w.E, w.M, None, 256, None))
        compare_client(pipe, 0, ref, w.n)
        want = oracle.aggregate(ref["sym"][None, :], ref["A"][None, :], oracle.Fmt(w.E, w.M))
        assert np.array_equal(u32(pipe.avg[:w.n]), want.view(np.uint32))
        err = ref["err"]
    properties_all_clients(pipe, w.n)


def test_c2_full(co3):
    """C2: 62 tensors, 11,173,962 elements, E4M3, per-tensor anchors; 3 chained iterations checked on
    every element (the workload's 100 iterations repeat the same code path)."""
    w = inp.c2()
    fmt = co3.Fmt(w.E, w.M)
    pipe = co3.Co3Pipeline(1, w.n, fmt, chunk_syms=256, seg_off=w.seg_off)
    g = pipe.new_gradient_buffer()
    err = np.zeros(w.n, np.float32)
    scales = inp.c2_tensor_scales()
    for t in range(1, 4):
        parts = [inp.device_gennorm(s, 0.8, float(a), 2000 + 100 * t + k) for k, (s, a) in enumerate(zip(w.sizes, scales))]
        x = torch.cat(parts)
        g[0, :w.n] = x
        gh = x.cpu().numpy()
        pipe.step(g)
        assert pipe.poll() == 0
        ref = oracle_client((gh, err, w.E, w.M, w.seg_off, 256, None))
        compare_client(pipe, 0, ref, w.n)
        want = oracle.aggregate(ref["sym"][None, :], ref["A"][None, :], oracle.Fmt(w.E, w.M), w.seg_off)
        assert np.array_equal(u32(pipe.avg[:w.n]), want.view(np.uint32))
        err = ref["err"]
    properties_all_clients(pipe, w.n)


@pytest.mark.parametrize("one_call", [True, False])
def test_c3_full(co3, one_call):
    """C3 (the benchmark workload): 10 clients x 11,173,962, E3M0; 2 chained iterations, every element of
    every client, and the average; through co3_user_encode (the benchmark's configuration) and through the
    separate calls."""
    w = inp.c3()
    fmt = co3.Fmt(w.E, w.M)
    betas = inp.c3_client_betas(w.U)
    pipe = co3.Co3Pipeline(w.U, w.n, fmt, chunk_syms=256, one_call=one_call)
    g = pipe.new_gradient_buffer()
    errs = [np.zeros(w.n, np.float32) for _ in range(w.U)]
    with ThreadPoolExecutor(max_workers=10) as pool:
        for t in range(1, 3):
            host = fill_from_device(pipe, g, lambda u: inp.device_gennorm(w.n, float(betas[u]), 1e-3, 3000 + 10 * t + u))
            pipe.step(g)
            assert pipe.poll() == 0
            refs = list(pool.map(oracle_client, [(host[u], errs[u], w.E, w.M, None, 256, None) for u in range(w.U)]))
            for u in range(w.U):
                compare_client(pipe, u, refs[u], w.n)
                errs[u] = refs[u]["err"]
            want = oracle.aggregate(np.stack([r["sym"] for r in refs]), np.stack([r["A"] for r in refs]),
                                    oracle.Fmt(w.E, w.M))
            assert np.array_equal(u32(pipe.avg[:w.n]), want.view(np.uint32)), "average"
    properties_all_clients(pipe, w.n)


def test_c3_single_pass_full(co3):
    """The C3 shape with tables fixed before the iteration (designed from a GenNorm model, one per client) and
    conversion + compression in one pass: 2 chained iterations, memory, stream words, chunk offsets and
    the average of every client against the oracle's convert_ef followed by encode, bit for bit."""
    w = inp.c3()
    fmt = co3.Fmt(w.E, w.M)
    f = oracle.Fmt(w.E, w.M)
    betas = inp.c3_client_betas(w.U)
    pipe = co3.Co3Pipeline(w.U, w.n, fmt, chunk_syms=256, statistics=False, single_pass=True, cap_words=w.n // 4)
    g = pipe.new_gradient_buffer()
    weights = np.stack([oracle.model_weights(-7, f, float(betas[u]), 1e-3) for u in range(w.U)])
    pipe.build(torch.from_numpy(weights.view(np.int32)).cuda())
    errs = [np.zeros(w.n, np.float32) for _ in range(w.U)]
    with ThreadPoolExecutor(max_workers=10) as pool:
        for t in range(1, 3):
            host = fill_from_device(pipe, g, lambda u: inp.device_gennorm(w.n, float(betas[u]), 1e-3, 3700 + 10 * t + u))
            pipe.step(g, rebuild=False)
            assert pipe.poll() == 0
            refs = list(pool.map(oracle_client, [(host[u], errs[u], w.E, w.M, None, 256, weights[u]) for u in range(w.U)]))
            for u in range(w.U):
                ref = refs[u]
                assert np.array_equal(pipe.anchor[u].cpu().numpy(), ref["A"]), "anchor"
                assert np.array_equal(u32(pipe.err[u, :w.n]), ref["err"].view(np.uint32)), "error vector"
                assert int(pipe.total_bits[u].item()) == ref["total"], "total bits"
                assert np.array_equal(u64(pipe.chunk_bitoff[u]), ref["off"]), "chunk offsets"
                nw = (ref["total"] + 63) // 64
                assert np.array_equal(u64(pipe.words[u, :nw]), ref["words"][:nw]), "stream words"
                errs[u] = ref["err"]
            want = oracle.aggregate(np.stack([r["sym"] for r in refs]), np.stack([r["A"] for r in refs]), f)
            assert np.array_equal(u32(pipe.avg[:w.n]), want.view(np.uint32)), "average"


def test_c3_bias_rule_full(co3):
    """The C3 shape (10 clients x 11,173,962) on the paper's 4-bit format E1M2 with the bias rule: moment
    sums and multipliers against the oracle (1e-12 relative / 2 units in the last place), then one whole
    iteration with the oracle's multipliers installed on both sides, every element of every client bit for
    bit, and the average."""
    w = inp.c3()
    fmt = co3.Fmt(1, 2)
    f = oracle.Fmt(1, 2)
    betas = inp.c3_client_betas(w.U)
    pipe = co3.Co3Pipeline(w.U, w.n, fmt, chunk_syms=256, bias="moments")
    g = pipe.new_gradient_buffer()
    host = fill_from_device(pipe, g, lambda u: inp.device_gennorm(w.n, float(betas[u]), 1e-3, 3500 + u))
    errs = [inp.gennorm(inp.rng_for(35, u), w.n, 1.0, 1e-4) for u in range(w.U)]
    for u in range(w.U):
        pipe.err[u, :w.n] = torch.from_numpy(errs[u]).cuda()
    pipe.fit_bias(g)
    with ThreadPoolExecutor(max_workers=10) as pool:
        sums_o = np.stack(list(pool.map(lambda u: oracle.moments(host[u], errs[u], 1.0), range(w.U))))
        assert np.allclose(pipe.sums.cpu().numpy(), sums_o, rtol=1e-12, atol=0.0)
        scale_o = np.zeros((w.U, 1), np.float32)
        for u in range(w.U):
            b, a = oracle.gennorm_fit(sums_o[u, 0, 0], sums_o[u, 0, 1], w.n)
            scale_o[u, 0] = oracle.bias_scale(b, a)
            assert abs(b - betas[u]) < 0.35          # the memory term is Laplace: the mixture's shape moves a little
        got = pipe.scale.cpu().numpy()
        assert np.all(np.abs(got.view(np.int32).astype(np.int64) - scale_o.view(np.int32).astype(np.int64)) <= 2)
        pipe.scale.copy_(torch.from_numpy(scale_o).cuda())
        pipe.convert(g)
        pipe.build()
        pipe.encode()
        pipe.aggregate()
        assert pipe.poll() == 0
        A = np.array([1], np.int32)

        def client(u):
            sym, e_new = oracle.convert_ef(host[u], errs[u], A, 1.0, f, scale=scale_o[u])
            cnt = oracle.histogram(sym, f)
            l = oracle.huffman_lengths(cnt)
            words, off, total = oracle.encode(sym, l, oracle.canonical_codes(l), 256)
            return dict(A=A, sym=sym, err=e_new, cnt=cnt, len=l, words=words, off=off, total=total)

        refs = list(pool.map(client, range(w.U)))
    for u in range(w.U):
        compare_client(pipe, u, refs[u], w.n)
    want = oracle.aggregate(np.stack([r["sym"] for r in refs]), np.tile(A, (w.U, 1)), f, scale=scale_o)
    assert np.array_equal(u32(pipe.avg[:w.n]), want.view(np.uint32)), "average"
    properties_all_clients(pipe, w.n)


def test_c3_paper_scheme_single_pass_full(co3):
    """The scheme as Sec. III states it, at the C3 shape: the 4-bit format E1M2, the bias rule's multiplier
    on a fixed grid, one code designed from the GenNorm model and shared by all users, and the user side in
    one pass (co3_convert_encode_layers).  One iteration from a non-zero memory, the oracle's multipliers
    on both sides; memory, stream words, chunk offsets of every user and the average, bit for bit."""
    w = inp.c3()
    fmt = co3.Fmt(1, 2)
    f = oracle.Fmt(1, 2)
    betas = inp.c3_client_betas(w.U)
    pipe = co3.Co3Pipeline(w.U, w.n, fmt, chunk_syms=256, bias="moments", codes="layer", statistics=False,
                           single_pass=True, cap_words=w.n // 4)
    g = pipe.new_gradient_buffer()
    host = fill_from_device(pipe, g, lambda u: inp.device_gennorm(w.n, float(betas[u]), 1e-3, 3900 + u))
    errs = [inp.gennorm(inp.rng_for(39, u), w.n, 1.0, 1e-4) for u in range(w.U)]
    for u in range(w.U):
        pipe.err[u, :w.n] = torch.from_numpy(errs[u]).cuda()
    A = np.array([1], np.int32)
    assert np.all(pipe.anchor.cpu().numpy() == 1)
    with ThreadPoolExecutor(max_workers=10) as pool:
        scale_o = np.stack(list(pool.map(lambda u: oracle.bias_scales(host[u], errs[u], 1.0), range(w.U))))
        pipe.scale.copy_(torch.from_numpy(scale_o).cuda())
        weights = oracle.model_weights(1, f, 1.0, 1e-3 * float(scale_o.mean()))[None, :]
        pipe.build(torch.from_numpy(weights.view(np.int32)).cuda())
        lens = oracle.huffman_lengths(weights[0])[None, :]
        cods = oracle.canonical_codes(lens[0])[None, :]
        assert np.array_equal(pipe.codes[:, :fmt.K].cpu().numpy(), lens)
        pipe.convert_encode(g)
        pipe.aggregate()
        assert pipe.poll() == 0

        def client(u):
            sym, e_new = oracle.convert_ef(host[u], errs[u], A, 1.0, f, scale=scale_o[u])
            words, off, total = oracle.encode_layers(sym, lens, cods, [0, w.n], 256)
            return sym, e_new, words, off, total

        refs = list(pool.map(client, range(w.U)))
    for u, (sym, e_new, words, off, total) in enumerate(refs):
        assert np.array_equal(u32(pipe.err[u, :w.n]), e_new.view(np.uint32)), "error vector"
        assert int(pipe.total_bits[u].item()) == total, "total bits"
        assert np.array_equal(u64(pipe.chunk_bitoff[u]), off), "chunk offsets"
        nw = (total + 63) // 64
        assert np.array_equal(u64(pipe.words[u, :nw]), words[:nw]), "stream words"
    want = oracle.aggregate(np.stack([r[0] for r in refs]), np.tile(A, (w.U, 1)), f, scale=scale_o)
    assert np.array_equal(u32(pipe.avg[:w.n]), want.view(np.uint32)), "average"


def test_c4_full(co3):
    """C4: 100M elements, E5M2, with outliers; empirical table and the fixed GenNorm-model table, one
    iteration each on every element."""
    w = inp.c4()
    fmt = co3.Fmt(w.E, w.M)
    f = oracle.Fmt(w.E, w.M)
    n = w.n
    x = inp.device_gennorm_outliers(n, 1.0, 1e-4, 1e-4, 100.0, 4001)
    gh = x.cpu().numpy()
    for table in ("empirical", "model"):
        pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=256, cap_words=None if table == "empirical" else n // 4)
        g = pipe.new_gradient_buffer()
        g[0, :n] = x
        del_g = g
        weights = None
        if table == "model":
            pipe.convert(g)
            A = int(pipe.anchor[0, 0].item())
            wdev = co3.binding.model_weights(A, fmt, 1.0, 1e-4)
            weights = oracle.model_weights(A, f, 1.0, 1e-4)
            assert np.array_equal(wdev.numpy().view(np.uint32), weights)
            pipe.build(wdev.cuda().reshape(1, -1))
            pipe.encode()
            pipe.aggregate()
        else:
            pipe.step(g)
        assert pipe.poll() == 0
        ref = oracle_client((gh, np.zeros(n, np.float32), w.E, w.M, None, 256, weights))
        compare_client(pipe, 0, ref, n)
        want = oracle.aggregate(ref["sym"][None, :], ref["A"][None, :], f)
        assert np.array_equal(u32(pipe.avg[:n]), want.view(np.uint32))
        pipe.decode()
        assert pipe.poll() == 0
        assert torch.equal(pipe.sym_dec[0, :n], pipe.sym[0, :n])
        del pipe, g, del_g
        torch.cuda.empty_cache()


def oracle_average(pool, refs, f, n, parts=16):
    """The oracle's average of all users, element ranges spread over the pool (each call stays single-threaded)."""
    syms = [r["sym"] for r in refs]
    A = np.stack([r["A"] for r in refs])
    cuts = np.linspace(0, n, parts + 1).astype(np.int64)

    def piece(k):
        a, b = int(cuts[k]), int(cuts[k + 1])
        return oracle.aggregate(np.stack([s[a:b] for s in syms]), A, f)

    return np.concatenate(list(pool.map(piece, range(parts))))


@pytest.mark.parametrize("point", range(12))
def test_c5_points(co3, point):
    """C5: 16 clients x 25M, all 12 points of the sweep (E2M0 / E3M1 / E4M3 / E5M2 x beta 0.5 / 1 / 2): every
    element of every client and the average through the oracle for iterations 1 and 2 (chained through the
    memory), in the one-call launch configuration that the benchmark times."""
    w = inp.c5(point)
    beta = inp.C5_BETAS[point % 3]
    fmt = co3.Fmt(w.E, w.M)
    f = oracle.Fmt(w.E, w.M)
    pipe = co3.Co3Pipeline(w.U, w.n, fmt, chunk_syms=256, one_call=True)
    g = pipe.new_gradient_buffer()
    errs = [np.zeros(w.n, np.float32) for _ in range(w.U)]
    with ThreadPoolExecutor(max_workers=16) as pool:
        for t in (1, 2):
            host = fill_from_device(pipe, g, lambda u: inp.device_gennorm(w.n, beta, 1e-3, 50000 + 1000 * point + 20 * t + u))
            pipe.step(g)
            assert pipe.poll() == 0
            refs = list(pool.map(oracle_client, [(host[u], errs[u], w.E, w.M, None, 256, None) for u in range(w.U)]))
            for u in range(w.U):
                compare_client(pipe, u, refs[u], w.n)
                errs[u] = refs[u]["err"]
            want = oracle_average(pool, refs, f, w.n)
            assert np.array_equal(u32(pipe.avg[:w.n]), want.view(np.uint32)), "average"
            del refs, want, host
    properties_all_clients(pipe, w.n)


# ---- one client of every workload over the workload's full number of iterations ------------------------
# The memory chains the iterations, so the oracle's conversion of iteration t + 1 waits for that of
# iteration t; its statistics, code and compression of iteration t run beside it in a worker thread.
def run_chain(co3, pipe, w, T, draw, client=0, seg_off=None):
    n = w.n
    f = oracle.Fmt(w.E, w.M)
    g = pipe.new_gradient_buffer()
    err = np.zeros(n, np.float32)

    def finish(t, snap, A, sym):
        cnt = oracle.histogram(sym, f)
        l = oracle.huffman_lengths(cnt)
        words, off, total = oracle.encode(sym, l, oracle.canonical_codes(l), 256)
        assert np.array_equal(snap["cnt"], cnt), (t, "histogram")
        assert np.array_equal(snap["len"], l), (t, "code lengths")
        assert snap["total"] == total, (t, "total bits")
        assert np.array_equal(snap["off"], off), (t, "chunk offsets")
        nw = (total + 63) // 64
        assert np.array_equal(snap["words"][:nw], words[:nw]), (t, "stream words")
        return total

    with ThreadPoolExecutor(max_workers=2) as pool:
        pending = []
        for t in range(1, T + 1):
            gh = draw(pipe, g, t)
            pipe.step(g)
            assert pipe.poll() == 0
            u = client
            snap = dict(cnt=u32(pipe.counts[u]), len=pipe.codes[u, :pipe.fmt.K].cpu().numpy(),
                        total=int(pipe.total_bits[u].item()), off=u64(pipe.chunk_bitoff[u]),
                        words=u64(pipe.words[u, :(int(pipe.total_bits[u].item()) + 63) // 64]))
            A = oracle.anchor(gh, f, seg_off)
            sym, err = oracle.convert_ef(gh, err, A, 1.0, f, seg_off)
            assert np.array_equal(pipe.anchor[u].cpu().numpy(), A), (t, "anchor")
            assert np.array_equal(pipe.sym[u, :n].cpu().numpy(), sym), (t, "symbols")
            assert np.array_equal(u32(pipe.err[u, :n]), err.view(np.uint32)), (t, "error vector")
            if pipe.U == 1:
                want = oracle.aggregate(sym[None, :], A[None, :], f, seg_off)
                assert np.array_equal(u32(pipe.avg[:n]), want.view(np.uint32)), (t, "average")
            pending.append(pool.submit(finish, t, snap, A, sym))
            while len(pending) > 2:
                pending.pop(0).result()
        for fut in pending:
            fut.result()


def test_c2_all_100_iterations(co3):
    """C2 over its 100 chained iterations: every output of every iteration against the oracle."""
    w = inp.c2()
    pipe = co3.Co3Pipeline(1, w.n, co3.Fmt(w.E, w.M), chunk_syms=256, seg_off=w.seg_off)
    scales = inp.c2_tensor_scales()

    def draw(pipe, g, t):
        x = torch.cat([inp.device_gennorm(s, 0.8, float(a), 20000 + 100 * t + k) for k, (s, a) in enumerate(zip(w.sizes, scales))])
        g[0, :w.n] = x
        return x.cpu().numpy()

    run_chain(co3, pipe, w, w.T, draw, seg_off=w.seg_off)


def test_c3_client_0_all_50_iterations(co3):
    """C3 over its 50 chained iterations (all 10 clients run on the device, one call per iteration as in the
    benchmark): every output of client 0 against the oracle at every iteration."""
    w = inp.c3()
    betas = inp.c3_client_betas(w.U)
    pipe = co3.Co3Pipeline(w.U, w.n, co3.Fmt(w.E, w.M), chunk_syms=256, one_call=True)

    def draw(pipe, g, t):
        for u in range(w.U):
            g[u, :w.n] = inp.device_gennorm(w.n, float(betas[u]), 1e-3, 30000 + 100 * t + u)
        return g[0, :w.n].cpu().numpy()

    run_chain(co3, pipe, w, w.T, draw)


def test_c4_all_20_iterations(co3):
    """C4 (100M elements with outliers, empirical table) over its 20 chained iterations."""
    w = inp.c4()
    pipe = co3.Co3Pipeline(1, w.n, co3.Fmt(w.E, w.M), chunk_syms=256, one_call=True)

    def draw(pipe, g, t):
        x = inp.device_gennorm_outliers(w.n, 1.0, 1e-4, 1e-4, 100.0, 40000 + 10 * t)
        g[0, :w.n] = x
        return x.cpu().numpy()

    run_chain(co3, pipe, w, w.T, draw)


def test_c5_point_7_client_0_all_10_iterations(co3):
    """One point of the C5 sweep (E4M3, beta = 1) over its 10 chained iterations, client 0 through the oracle."""
    w = inp.c5(7)
    pipe = co3.Co3Pipeline(w.U, w.n, co3.Fmt(w.E, w.M), chunk_syms=256, one_call=True)

    def draw(pipe, g, t):
        for u in range(w.U):
            g[u, :w.n] = inp.device_gennorm(w.n, 1.0, 1e-3, 57000 + 100 * t + u)
        return g[0, :w.n].cpu().numpy()

    run_chain(co3, pipe, w, w.T, draw)


def test_beyond_2_to_the_31_elements(co3):
    """One client with 2^31 + 2^20 + 13 elements (the interface admits n < 2^32): every index computation must
    be 64-bit.  Inputs are drawn on the device in pieces; the anchor is checked against torch's own maximum;
    windows at the start, across element 2^31 and at the ragged end go through the oracle element by element
    (symbols, memory, average); all elements through the size-independent properties."""
    n = (1 << 31) + (1 << 20) + 13
    fmt = co3.Fmt(3, 0)
    f = oracle.Fmt(3, 0)
    pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=256)
    g = pipe.new_gradient_buffer()
    piece = 1 << 28
    for k, a in enumerate(range(0, n, piece)):
        b = min(n, a + piece)
        g[0, a:b] = inp.device_gennorm(b - a, 1.0, 1e-3, 8100 + k)
    pipe.step(g)
    assert pipe.poll() == 0
    amax = float(g[0, :n].abs().max().item())
    A = int(np.floor(np.log2(amax)))
    assert int(pipe.anchor[0, 0].item()) == A
    windows = [(0, 70_000), ((1 << 31) - 50_001, (1 << 31) + 50_003), (n - 66_001, n)]
    for a, b in windows:
        gh = g[0, a:b].cpu().numpy()
        sym, e_new = oracle.convert_ef(gh, np.zeros(b - a, np.float32), np.array([A], np.int32), 1.0, f)
        assert np.array_equal(pipe.sym[0, a:b].cpu().numpy(), sym), (a, b)
        assert np.array_equal(u32(pipe.err[0, a:b]), e_new.view(np.uint32)), (a, b)
        want = oracle.aggregate(sym[None, :], np.array([[A]], np.int32), f)
        assert np.array_equal(u32(pipe.avg[a:b]), want.view(np.uint32)), (a, b)
    # stream of the first window against the oracle's encoder (the code comes from the device histogram,
    # itself checked against the symbols by the properties below)
    cnt = u32(pipe.counts[0])
    lens = oracle.huffman_lengths(cnt)
    assert np.array_equal(pipe.codes[0, :fmt.K].cpu().numpy(), lens)
    m = 65_536
    words, off, total = oracle.encode(pipe.sym[0, :m].cpu().numpy(), lens, oracle.canonical_codes(lens), 256)
    assert np.array_equal(u64(pipe.chunk_bitoff[0, :m // 256 + 1]), off)
    assert np.array_equal(u64(pipe.words[0, :total // 64]), words[:total // 64])
    hist = torch.bincount(pipe.sym[0, :n].to(torch.int32), minlength=fmt.K).cpu().numpy()
    assert np.array_equal(hist, cnt.astype(np.int64))
    properties_all_clients(pipe, n)


def test_single_pass_beyond_2_to_the_31_elements(co3):
    """The one-pass user side at 2^31 + 2^20 + 13 elements (64-bit indices everywhere): with the code that
    the two-pass path built from the same gradients, memory, stream words, chunk offsets and total must
    equal the two-pass results over the whole length (those are checked against the oracle in the test
    above); windows of the memory across element 2^31 and at the ragged end, and the stream of the first
    65,536 symbols, go through the oracle directly."""
    n = (1 << 31) + (1 << 20) + 13
    fmt = co3.Fmt(3, 0)
    f = oracle.Fmt(3, 0)
    two = co3.Co3Pipeline(1, n, fmt, chunk_syms=256)
    g = two.new_gradient_buffer()
    piece = 1 << 28
    for k, a in enumerate(range(0, n, piece)):
        b = min(n, a + piece)
        g[0, a:b] = inp.device_gennorm(b - a, 1.0, 1e-3, 8300 + k)
    two.convert(g)
    two.build()
    two.encode()
    assert two.poll() == 0
    one = co3.Co3Pipeline(1, n, fmt, chunk_syms=256, statistics=False, single_pass=True)
    one.codes.copy_(two.codes)
    one.convert_encode(g)
    assert one.poll() == 0
    assert torch.equal(one.anchor, two.anchor)
    assert torch.equal(one.total_bits, two.total_bits)
    assert torch.equal(one.chunk_bitoff, two.chunk_bitoff), "chunk offsets"
    nw = (int(two.total_bits[0].item()) + 63) // 64
    assert torch.equal(one.words[0, :nw], two.words[0, :nw]), "stream words"
    assert torch.equal(one.err.view(torch.int32), two.err.view(torch.int32)), "memory"
    A = one.anchor[0].cpu().numpy()
    for a, b in [((1 << 31) - 50_001, (1 << 31) + 50_003), (n - 66_001, n)]:
        sym, e_new = oracle.convert_ef(g[0, a:b].cpu().numpy(), np.zeros(b - a, np.float32), A, 1.0, f)
        assert np.array_equal(u32(one.err[0, a:b]), e_new.view(np.uint32)), (a, b)
    lens = one.codes[0, :fmt.K].cpu().numpy()
    m = 65_536
    sym, _ = oracle.convert_ef(g[0, :m].cpu().numpy(), np.zeros(m, np.float32), A, 1.0, f)
    words, off, total = oracle.encode(sym, lens, oracle.canonical_codes(lens), 256)
    assert np.array_equal(u64(one.chunk_bitoff[0, :m // 256 + 1]), off)
    assert np.array_equal(u64(one.words[0, :total // 64]), words[:total // 64])
