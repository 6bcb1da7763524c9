"""HIP path vs CPU oracle, element by element, through the C ABI (GPU only).

Bars: symbols, error vectors, histograms, code lengths, streams, chunk offsets and decoded
symbols are compared bit for bit.  The average is produced in the same user order as the
oracle, so it is compared bit for bit as well (the stated tolerance would be 1e-6 relative).
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


def ofmt(fmt):
    return oracle.Fmt(fmt.E, fmt.M)


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)


def host_u64(t):
    return t.cpu().numpy().view(np.uint64)


def oracle_user_side(g, err, fmt, seg_off, gamma, C, weights=None):
    """Oracle run of one user: returns dict of every intermediate."""
    f = ofmt(fmt)
    A = oracle.anchor(g, f, seg_off)
    sym, e_new = oracle.convert_ef(g, err, A, gamma, f, seg_off)
    cnt = oracle.histogram(sym, f)
    l = oracle.huffman_lengths(cnt if weights is None else weights)
    codes = oracle.canonical_codes(l)
    words, off, total = oracle.encode(sym, l, codes, C)
    return dict(A=A, sym=sym, err=e_new, cnt=cnt, len=l, codes=codes, words=words, off=off, total=total)


def check_user_side(pipe, u, ref, n):
    assert np.array_equal(pipe.anchor[u].cpu().numpy(), ref["A"]), "anchor"
    assert np.array_equal(pipe.sym[u, :n].cpu().numpy(), ref["sym"]), "symbols"
    assert np.array_equal(host_u32(pipe.err[u, :n]), ref["err"].view(np.uint32)), "error vector"
    assert np.array_equal(host_u32(pipe.counts[u]), ref["cnt"]), "histogram"
    K = pipe.fmt.K
    assert np.array_equal(pipe.codes[u, :K].cpu().numpy(), ref["len"]), "code lengths"
    assert int(pipe.total_bits[u].item()) == ref["total"], "total bits"
    assert np.array_equal(host_u64(pipe.chunk_bitoff[u]), ref["off"]), "chunk offsets"
    nw = (ref["total"] + 63) // 64
    assert np.array_equal(host_u64(pipe.words[u, :nw]), ref["words"][:nw]), "stream words"


def run_case(co3, U, n, fmt, C, betas, alpha=1e-3, T=2, gamma=1.0, sizes=None, seed=0):
    seg_off = None if sizes is None else inp.seg_offsets(sizes)
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, seg_off=seg_off, gamma=gamma)
    errs = [np.zeros(n, np.float32) for _ in range(U)]
    g = pipe.new_gradient_buffer()
    for t in range(1, T + 1):
        g_host = []
        for u in range(U):
            r = inp.rng_for(99, seed, u, t)
            g_host.append(inp.gennorm(r, n, betas[u % len(betas)], alpha))
        if n:
            g[:, :n] = torch.from_numpy(np.stack(g_host)).cuda()
        pipe.step(g)
        assert pipe.poll() == 0
        pipe.decode()
        assert pipe.poll() == 0
        refs = []
        for u in range(U):
            ref = oracle_user_side(g_host[u], errs[u], fmt, seg_off, gamma, C)
            check_user_side(pipe, u, ref, n)
            assert np.array_equal(pipe.sym_dec[u, :n].cpu().numpy(), ref["sym"]), "decode(encode(s)) = s"
            errs[u] = ref["err"]
            refs.append(ref)
        want = oracle.aggregate(np.stack([r["sym"] for r in refs]) if n else np.zeros((U, 0), np.uint8),
                                np.stack([r["A"] for r in refs]), ofmt(fmt), seg_off)
        got = pipe.avg[:n].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), "average"
    return pipe


# ---------------------------------------------------------------- whole path, many shapes
@pytest.mark.parametrize("E,M", [(3, 1), (3, 0), (2, 0), (4, 3), (5, 2), (1, 2), (1, 0), (1, 6)])
def test_whole_path_formats(co3, E, M):
    fmt = co3.Fmt(E, M)
    # several encoder blocks (2048 symbols) and a ragged tail, two users with different shapes
    run_case(co3, 2, 2048 * 5 + 1237, fmt, 256, betas=[0.7, 1.4], T=3)


@pytest.mark.parametrize("n", [0, 1, 3, 4, 63, 64, 65, 255, 256, 257, 2047, 2048, 2049, 4096 + 8, 10_000, 65_536 + 5])
def test_whole_path_sizes(co3, n):
    run_case(co3, 1, n, co3.Fmt(3, 1), 64, betas=[1.0], T=2)
    run_case(co3, 3, n, co3.Fmt(3, 0), 128, betas=[0.5, 1.0, 1.5], T=2)


@pytest.mark.parametrize("C", [64, 128, 256, 512, 1024, 2048, 4096])
def test_whole_path_chunk_sizes(co3, C):
    run_case(co3, 2, 3 * 4096 + 100, co3.Fmt(4, 3), C, betas=[0.8], T=2)


def test_whole_path_gamma_decay(co3):
    run_case(co3, 2, 30_000, co3.Fmt(1, 2), 256, betas=[1.0], T=4, gamma=0.9)
    run_case(co3, 1, 30_000, co3.Fmt(3, 1), 256, betas=[1.0], T=3, gamma=0.0)


def test_whole_path_segments(co3):
    """Per-tensor anchors: tiny tensors beside large ones, boundaries not aligned to anything."""
    sizes = [10, 1, 4097, 64, 3, 20_000, 7, 128, 0, 5, 12_345]
    n = sum(sizes)
    seg_off = inp.seg_offsets(sizes)
    fmt = co3.Fmt(4, 3)
    U, C = 2, 256
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, seg_off=seg_off)
    g = pipe.new_gradient_buffer()
    errs = [np.zeros(n, np.float32) for _ in range(U)]
    scales = 10.0 ** inp.rng_for(98).uniform(-5, -2, len(sizes))
    for t in range(1, 4):
        g_host = []
        for u in range(U):
            r = inp.rng_for(98, 1, u, t)
            g_host.append(np.concatenate([inp.gennorm(r, s, 0.8, a) for s, a in zip(sizes, scales)]))
        g[:, :n] = torch.from_numpy(np.stack(g_host)).cuda()
        pipe.step(g)
        pipe.decode()
        assert pipe.poll() == 0
        refs = []
        for u in range(U):
            ref = oracle_user_side(g_host[u], errs[u], fmt, seg_off, 1.0, C)
            check_user_side(pipe, u, ref, n)
            assert np.array_equal(pipe.sym_dec[u, :n].cpu().numpy(), ref["sym"])
            errs[u] = ref["err"]
            refs.append(ref)
        want = oracle.aggregate(np.stack([r["sym"] for r in refs]), np.stack([r["A"] for r in refs]), ofmt(fmt),
                                seg_off)
        assert np.array_equal(host_u32(pipe.avg[:n]), want.view(np.uint32))


# ------------------------------------------------------------- conversion: adversarial values
@pytest.mark.parametrize("E,M", [(3, 1), (4, 3), (5, 2), (2, 0), (1, 6)])
def test_convert_adversarial_values(co3, E, M):
    fmt = co3.Fmt(E, M)
    f = ofmt(fmt)
    rng = np.random.default_rng(5)
    for A in (f.F - 126, -60, -9, 0, 30, 127):
        lv = np.array([oracle.level(c >> M, c & ((1 << M) - 1), A, f) for c in range(fmt.K // 2)])
        mids = 0.5 * (lv[:-1] + lv[1:])
        base = np.concatenate([lv, mids]).astype(np.float32)
        pts = np.concatenate([base, np.nextafter(base, np.float32(np.inf)), np.nextafter(base, np.float32(0)),
                              base * np.float32(1.5), [np.float32(lv[-1] * 2), np.float32(lv[-1] * 1e6)],
                              np.array([0.0, 1e-45, 1e-40, 1.1754944e-38, 3e38, np.inf], dtype=np.float32),
                              (rng.standard_normal(3000) * lv[-1] * 0.3).astype(np.float32),
                              np.exp2(rng.uniform(-149, 127.9, 3000)).astype(np.float32)])
        x = np.concatenate([pts, -pts]).astype(np.float32)
        x = x[~np.isnan(x)]
        n = x.size
        pipe = co3.Co3Pipeline(1, n, fmt)
        g = pipe.new_gradient_buffer()
        g[0, :n] = torch.from_numpy(x).cuda()
        pipe.anchor[0, 0] = A
        # carried error: zero, then a second pass with the produced error and a decay
        e_prev = np.zeros(n, np.float32)
        for gamma in (1.0, 0.9):
            pipe.gamma = gamma
            co3.binding.convert_ef(g, pipe.err, pipe.sym, n, pipe.anchor, co3.binding.ANCHOR_GIVEN, gamma, fmt,
                                   counts=pipe.counts)
            sym, e_new = oracle.convert_ef(x, e_prev, np.array([A], np.int32), gamma, f)
            finite = np.isfinite(e_new)
            assert np.array_equal(pipe.sym[0, :n].cpu().numpy(), sym)
            got_e = pipe.err[0, :n].cpu().numpy()
            assert np.array_equal(got_e.view(np.uint32)[finite], e_new.view(np.uint32)[finite])
            assert np.array_equal(host_u32(pipe.counts[0]), oracle.histogram(sym, f))
            # keep the carried error finite for the second pass on both sides
            e_prev = np.where(finite, e_new, 0).astype(np.float32)
            pipe.err[0, :n] = torch.from_numpy(e_prev).cuda()


def test_anchor_from_absmax_edges(co3):
    fmt = co3.Fmt(3, 1)
    f = ofmt(fmt)
    cases = [np.zeros(100, np.float32), np.array([1e-40, -3e-41, 0], np.float32), np.array([2.0 ** -124], np.float32),
             np.array([3e38, -1.0], np.float32), np.array([-0.75, 0.5], np.float32), np.array([1.0], np.float32),
             np.array([np.nextafter(np.float32(2), np.float32(0))], np.float32)]
    for x in cases:
        n = x.size
        pipe = co3.Co3Pipeline(1, n, fmt)
        g = pipe.new_gradient_buffer()
        g[0, :n] = torch.from_numpy(x).cuda()
        pipe.convert(g)
        assert int(pipe.anchor[0, 0].item()) == int(oracle.anchor(x, f)[0]), x


# ------------------------------------------------------------------ histogram (stand-alone)
@pytest.mark.parametrize("K_fmt", [(1, 0), (3, 0), (3, 1), (4, 3)])
def test_histogram_standalone(co3, K_fmt):
    fmt = co3.Fmt(*K_fmt)
    rng = np.random.default_rng(3)
    for n in (0, 1, 15, 16, 17, 4095, 100_003):
        U = 2
        stride = (max(n, 1) + 15) // 16 * 16
        # heavily skewed symbols: one symbol holds most of the mass
        s = np.where(rng.random((U, stride)) < 0.9, 0, rng.integers(0, fmt.K, (U, stride))).astype(np.uint8)
        sym = torch.from_numpy(s).cuda()
        counts = torch.full((U, fmt.K), -1, dtype=torch.int32, device="cuda")
        co3.binding.histogram(sym, n, fmt, counts)
        for u in range(U):
            assert np.array_equal(host_u32(counts[u]), np.bincount(s[u, :n], minlength=fmt.K))


# --------------------------------------------------------------------- Huffman construction
def test_build_code_adversarial_weights(co3):
    rng = np.random.default_rng(4)
    fib = [1, 1]
    while len(fib) < 46:
        fib.append(fib[-1] + fib[-2])
    rows = []
    for K in (256,):
        rows.append(np.array(fib + [0] * (K - len(fib)), dtype=np.uint64))                 # deepest tree (45 bits)
        rows.append(np.full(K, 2 ** 32 - 1, dtype=np.uint64))                              # merged weights > 2^32
        rows.append(np.full(K, 1, dtype=np.uint64))                                        # all ties
        rows.append(np.zeros(K, dtype=np.uint64))                                          # nothing active
        one = np.zeros(K, dtype=np.uint64); one[77] = 5; rows.append(one)                  # a single symbol
        two = np.zeros(K, dtype=np.uint64); two[3] = 9; two[200] = 9; rows.append(two)
        rows.append(rng.integers(1, 4, K).astype(np.uint64))                               # many ties
        rows.append((rng.pareto(0.5, K) * 10).astype(np.uint64).clip(0, 2 ** 32 - 1))      # heavy tail, zeros
        rows.append(np.array([2 ** (i % 31) for i in range(K)], dtype=np.uint64))
        rows.append(np.arange(K, dtype=np.uint64)[::-1].copy())
    w = np.stack(rows).astype(np.uint32)
    U = w.shape[0]
    fmt = co3.Fmt(4, 3)
    weights = torch.from_numpy(w.view(np.int32)).cuda()
    codes = torch.zeros((U, co3.binding.CODE_BYTES), dtype=torch.uint8, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    co3.binding.build_code(weights, U, fmt, codes, status)
    assert co3.binding.poll_status(status) == 0
    for u in range(U):
        want = oracle.huffman_lengths(w[u])
        assert np.array_equal(codes[u, :256].cpu().numpy(), want), u
    # smaller alphabets use only the first K weights of each row
    for E, M in ((3, 0), (2, 0), (3, 1)):
        f2 = co3.Fmt(E, M)
        w2 = np.ascontiguousarray(w[:, :f2.K])
        co3.binding.build_code(torch.from_numpy(w2.view(np.int32)).cuda(), U, f2, codes, status)
        assert co3.binding.poll_status(status) == 0
        for u in range(U):
            assert np.array_equal(codes[u, :f2.K].cpu().numpy(), oracle.huffman_lengths(w2[u])), (E, M, u)


# ------------------------------------------------- streams with long codewords (table miss path)
@pytest.mark.parametrize("C", [64, 256])
def test_long_codewords_roundtrip(co3, C):
    """Symbols drawn so that the empirical code has lengths far beyond the decoder table prefix."""
    fmt = co3.Fmt(4, 3)
    f = ofmt(fmt)
    n = 300_007
    rng = np.random.default_rng(6)
    # geometric law over 40 symbols (probability halves each step) -> lengths 1, 2, ..., ~20+
    p = 0.5 ** np.arange(1, 41)
    p[-1] += 1 - p.sum()
    order = rng.permutation(256)[:40]
    s = order[rng.choice(40, size=n, p=p)].astype(np.uint8)
    pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=C)
    pipe.sym[0, :n] = torch.from_numpy(s).cuda()
    co3.binding.histogram(pipe.sym, n, fmt, pipe.counts)
    pipe.build()
    pipe.encode()
    pipe.decode()
    assert pipe.poll() == 0
    cnt = oracle.histogram(s, f)
    l = oracle.huffman_lengths(cnt)
    assert int(l.max()) > 14
    words, off, total = oracle.encode(s, l, oracle.canonical_codes(l), C)
    assert np.array_equal(pipe.codes[0, :256].cpu().numpy(), l)
    assert int(pipe.total_bits[0].item()) == total
    assert np.array_equal(host_u64(pipe.chunk_bitoff[0]), off)
    assert np.array_equal(host_u64(pipe.words[0, :(total + 63) // 64]), words[:(total + 63) // 64])
    assert np.array_equal(pipe.sym_dec[0, :n].cpu().numpy(), s)


def test_very_long_codewords_model_style_table(co3):
    """Codes up to 45 bits (Fibonacci weights given as a table, not measured from the data):
    runs of long codewords cross several 64-bit words and overflow the staging average."""
    fmt = co3.Fmt(4, 3)
    fib = [1, 1]
    while len(fib) < 46:
        fib.append(fib[-1] + fib[-2])
    w = np.zeros(256, np.uint32)
    w[:46] = fib
    l = oracle.huffman_lengths(w)
    assert int(l.max()) == 45
    rng = np.random.default_rng(8)
    n = 3 * 2048 + 77
    # mostly the rarest symbols (longest codes): about 40 bits per symbol
    s = rng.integers(0, 8, n).astype(np.uint8)
    s[rng.integers(0, n, 200)] = 45
    C = 64
    cap = (int(l[s].astype(np.int64).sum()) + 63) // 64 + 2
    pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=C, cap_words=cap)
    pipe.sym[0, :n] = torch.from_numpy(s).cuda()
    pipe.build(torch.from_numpy(w.view(np.int32)).cuda().reshape(1, 256))
    pipe.encode()
    pipe.decode()
    assert pipe.poll() == 0
    words, off, total = oracle.encode(s, l, oracle.canonical_codes(l), C)
    assert int(pipe.total_bits[0].item()) == total
    assert np.array_equal(host_u64(pipe.chunk_bitoff[0]), off)
    assert np.array_equal(host_u64(pipe.words[0, :(total + 63) // 64]), words[:(total + 63) // 64])
    assert np.array_equal(pipe.sym_dec[0, :n].cpu().numpy(), s)


# ------------------------------ alphabets of at most 16 symbols: two symbols per lookup, packed workspace
@pytest.mark.parametrize("E,M,C", [(3, 0, 64), (3, 0, 512), (3, 0, 4096), (2, 0, 64), (1, 2, 1024), (2, 1, 128), (1, 0, 64)])
def test_small_alphabet_chunk_sizes(co3, E, M, C):
    # several tiles of 64 chunks where the chunk is small, a ragged last chunk and a ragged last run
    run_case(co3, 3, 70 * C + 45 if C <= 512 else 5 * C + 45, co3.Fmt(E, M), C, betas=[0.5, 1.0, 2.0], T=2)


@pytest.mark.parametrize("C", [64, 256])
def test_small_alphabet_long_codewords(co3, C):
    """K = 16 with a table of Fibonacci weights (codewords of 1..14 bits) and data in which the rare
    symbols are frequent: pairs that do not fit the table prefix, codewords longer than it, and runs
    that fall back to the careful decoder, in the plain and in the averaging path."""
    fmt = co3.Fmt(3, 0)
    f = ofmt(fmt)
    fib = [1, 1]
    while len(fib) < 15:
        fib.append(fib[-1] + fib[-2])
    w = np.zeros((1, 16), np.uint32)
    order = np.random.default_rng(3).permutation(16)[:15]
    w[0, order] = fib
    l = oracle.huffman_lengths(w[0])
    assert int(l.max()) == 14
    U, n = 2, 40 * 64 * C // 16 + 21
    rng = np.random.default_rng(12)
    syms = []
    for u in range(U):
        # user 0: all active symbols equally likely (about 8 bits per symbol); user 1: the table's own law
        p = np.full(15, 1 / 15) if u == 0 else np.asarray(fib, float) / sum(fib)
        syms.append(order[rng.choice(15, size=n, p=p)].astype(np.uint8))
    cap = 2 * ((max(int(l[s].astype(np.int64).sum()) for s in syms) + 127) // 128) + 2
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, cap_words=cap)
    pipe.sym[:, :n] = torch.from_numpy(np.stack(syms)).cuda()
    pipe.build(torch.from_numpy(np.repeat(w, U, 0).view(np.int32)).cuda())
    pipe.anchor[:, 0] = torch.tensor([-3, 2], dtype=torch.int32)
    pipe.encode()
    pipe.decode()
    pipe.aggregate()
    assert pipe.poll() == 0
    for u in range(U):
        words, off, total = oracle.encode(syms[u], l, oracle.canonical_codes(l), C)
        assert int(pipe.total_bits[u].item()) == total
        assert np.array_equal(host_u64(pipe.chunk_bitoff[u]), off)
        assert np.array_equal(host_u64(pipe.words[u, :(total + 63) // 64]), words[:(total + 63) // 64])
        assert np.array_equal(pipe.sym_dec[u, :n].cpu().numpy(), syms[u])
    want = oracle.aggregate(np.stack(syms), np.array([[-3], [2]], np.int32), f)
    assert np.array_equal(pipe.avg[:n].cpu().numpy().view(np.uint32), want.view(np.uint32))
    # a flipped stream bit: the decoders run to the end and report the stream unless it still parses
    pipe.words[0, 5] ^= 1 << 17
    pipe.status.zero_()
    pipe.aggregate()
    pipe.decode()
    rc = pipe.poll()
    assert rc in (0, co3.binding.EBADSTREAM)


# ----------------------------------------------------------------------------- error paths
def test_device_reported_errors(co3):
    fmt = co3.Fmt(3, 0)
    n, C = 10_000, 256
    rng = np.random.default_rng(9)
    s = rng.integers(0, 8, n).astype(np.uint8)
    # capacity: a 3-bit flat code over 8 symbols needs 30000 bits; give 100 words
    pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=C, cap_words=100)
    pipe.sym[0, :n] = torch.from_numpy(s).cuda()
    co3.binding.histogram(pipe.sym, n, fmt, pipe.counts)
    pipe.build()
    # the word buffer continues past the stated capacity: nothing may land there
    big = torch.full((1, 1000), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")
    rc = co3.binding._lib.co3_encode(pipe.sym.data_ptr(), n, 1, pipe.stride, fmt.c(), pipe.codes.data_ptr(),
                                     big.data_ptr(), 100, C, pipe.chunk_bitoff.data_ptr(),
                                     pipe.total_bits.data_ptr(), pipe.enc_ws.data_ptr(), pipe.enc_ws.numel() * 8,
                                     pipe.status.data_ptr(), None)
    assert rc == 0
    assert pipe.poll() == co3.binding.ECAP
    assert bool((big[0, 100:] == 0x5A5A5A5A5A5A5A5A).all())
    assert int(pipe.total_bits[0].item()) == 3 * n    # the needed length is still reported
    # symbol without a code: table built from weights that miss symbol 7
    pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=C)
    pipe.sym[0, :n] = torch.from_numpy(s).cuda()
    w = np.ones((1, 16), np.int32)
    w[0, 7] = 0
    pipe.build(torch.from_numpy(w).cuda())
    pipe.encode()
    assert pipe.poll() == co3.binding.ENOCODE
    # corrupt index: decoder reports it and stays in bounds
    pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=C)
    pipe.sym[0, :n] = torch.from_numpy(s).cuda()
    co3.binding.histogram(pipe.sym, n, fmt, pipe.counts)
    pipe.build()
    pipe.encode()
    assert pipe.poll() == 0
    pipe.chunk_bitoff[0, 3] += 1
    pipe.decode()
    assert pipe.poll() == co3.binding.EBADSTREAM
    pipe.status.zero_()
    pipe.chunk_bitoff[0, 3] = 1 << 50                 # far outside the buffer
    pipe.decode()
    assert pipe.poll() == co3.binding.EBADSTREAM


def test_host_rejected_arguments(co3):
    B = co3.binding
    fmt = co3.Fmt(3, 1)
    pipe = co3.Co3Pipeline(2, 1000, fmt)
    g = pipe.new_gradient_buffer()
    with pytest.raises(co3.Co3Error) as ei:
        B.convert_ef(g, pipe.err, pipe.sym, 1000, pipe.anchor, B.ANCHOR_GIVEN, 1.0, co3.Fmt(5, 3))   # 9 bits
    assert ei.value.code == B.EINVAL
    with pytest.raises(co3.Co3Error):
        B.convert_ef(g, pipe.err, pipe.sym, -1, pipe.anchor, B.ANCHOR_GIVEN, 1.0, fmt)
    with pytest.raises(co3.Co3Error):
        B.convert_ef(g, pipe.err, pipe.sym, 1000, pipe.anchor, 7, 1.0, fmt)
    with pytest.raises(co3.Co3Error):   # chunk size not a power of two
        B.encode(pipe.sym, 1000, fmt, pipe.codes, pipe.words, 100, pipe.chunk_bitoff, pipe.total_bits, pipe.enc_ws,
                 pipe.status)
    with pytest.raises(co3.Co3Error):   # workspace too small
        B.encode(pipe.sym, 1000, fmt, pipe.codes, pipe.words, 256, pipe.chunk_bitoff, pipe.total_bits,
                 torch.zeros(1, dtype=torch.int64, device="cuda"), pipe.status)
    with pytest.raises(co3.Co3Error):   # misaligned gradient pointer
        B.convert_ef(g.view(-1)[1:1001], pipe.err.view(-1)[1:1001], pipe.sym.view(-1)[:1000], 1000,
                     pipe.anchor[:1], B.ANCHOR_GIVEN, 1.0, fmt)
    assert B.strerror(B.ECAP) and B.strerror(-99)


# --------------------------------------------------------------- determinism and canaries
def test_deterministic_and_no_stray_writes(co3):
    fmt = co3.Fmt(3, 0)
    U, n, C = 3, 50_000 + 13, 256
    outs = []
    for rep in range(2):
        pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C)
        # poison everything the kernels are supposed to overwrite or leave alone
        pipe.words.fill_(0x5A5A5A5A5A5A5A5A)
        pipe.sym.fill_(0xEE)
        pipe.avg.fill_(123.0)
        pipe.counts.fill_(-7)
        g = pipe.new_gradient_buffer()
        g.fill_(float("nan"))
        for u in range(U):
            g[u, :n] = torch.from_numpy(inp.gennorm(inp.rng_for(97, 0, u, 1), n, 0.5 + 0.5 * u, 1e-3)).cuda()
        pipe.step(g)
        assert pipe.poll() == 0
        # padding between n and stride is never touched
        assert bool((pipe.sym[:, n:] == 0xEE).all())
        assert bool((pipe.avg[n:] == 123.0).all())
        assert bool((pipe.err[:, n:] == 0).all())
        for u in range(U):
            nw = (int(pipe.total_bits[u].item()) + 63) // 64
            assert bool((pipe.words[u, nw:] == 0x5A5A5A5A5A5A5A5A).all())
        outs.append((pipe.words.clone(), pipe.chunk_bitoff.clone(), pipe.avg.clone(), pipe.err.clone()))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)


# ------------------------------------------------------------------ model table (host call)
def test_model_weights_match_oracle(co3):
    for (E, M), beta, alpha, A in [((5, 2), 1.0, 1e-4, -7), ((5, 2), 1.0, 1e-4, -6), ((3, 1), 1.0, 1e-3, -7),
                                   ((4, 3), 0.8, 1e-3, -5), ((2, 0), 0.5, 1e-3, -3), ((3, 0), 1.5, 1e-3, -8),
                                   ((4, 3), 2.0, 1e-3, -8)]:
        fmt = co3.Fmt(E, M)
        got = co3.binding.model_weights(A, fmt, beta, alpha).numpy().view(np.uint32)
        want = oracle.model_weights(A, ofmt(fmt), beta, alpha)
        assert np.array_equal(got, want), (E, M, beta, A)


def test_model_table_encodes_data(co3):
    """C4-style: a fixed table from the GenNorm model codes data drawn from that model."""
    fmt = co3.Fmt(5, 2)
    f = ofmt(fmt)
    n, C = 200_000, 256
    x = inp.gennorm_outliers(inp.rng_for(4, 0, 0, 1), n, 1.0, 1e-4, 1e-4, 100.0)
    pipe = co3.Co3Pipeline(1, n, fmt, chunk_syms=C, cap_words=n)       # model tables have no length bound
    g = pipe.new_gradient_buffer()
    g[0, :n] = torch.from_numpy(x).cuda()
    pipe.convert(g)
    A = int(pipe.anchor[0, 0].item())
    assert A == int(oracle.anchor(x, f)[0])
    w = co3.binding.model_weights(A, fmt, 1.0, 1e-4)
    pipe.build(w.cuda().reshape(1, -1))
    pipe.encode()
    pipe.aggregate()
    pipe.decode()
    assert pipe.poll() == 0
    ref = oracle_user_side(x, np.zeros(n, np.float32), fmt, None, 1.0, C, weights=oracle.model_weights(A, f, 1.0, 1e-4))
    assert np.array_equal(pipe.codes[0, :256].cpu().numpy(), ref["len"])
    assert int(pipe.total_bits[0].item()) == ref["total"]
    nw = (ref["total"] + 63) // 64
    assert np.array_equal(host_u64(pipe.words[0, :nw]), ref["words"][:nw])
    assert np.array_equal(pipe.sym_dec[0, :n].cpu().numpy(), ref["sym"])
