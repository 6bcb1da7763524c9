"""HIP path vs CPU oracle for one code per tensor shared by all users (Sec. III (ii) as the paper states
it), through the C ABI (GPU only).  Everything is integer / byte work: bit for bit."""
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


SHAPES = {
    "odd": [10, 0, 4086, 1, 33000, 12903],
    "resnet_head": [1728, 64, 64, 36864, 64, 64, 73728, 128, 128, 5120, 10],
    "single": [70001],
    "tiny_many": [5] * 300 + [2000] + [1] * 70 + [9000],
    "two_big": [300000, 300001],
    "aligned": [4096, 8192, 1024, 1024],
}


def run_layers(co3, U, sizes, E, M, C, table, seed=0):
    B = co3.binding
    fmt = co3.Fmt(E, M)
    f = oracle.Fmt(E, M)
    seg = inp.seg_offsets(sizes)
    nseg = len(sizes)
    n = int(seg[-1])
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, seg_off=seg)
    g = pipe.new_gradient_buffer()
    scales = 10.0 ** inp.rng_for(88, seed).uniform(-4, -2, nseg)
    gh = [np.concatenate([inp.gennorm(inp.rng_for(88, seed, u, k), m, 0.9, a) for k, (m, a) in enumerate(zip(sizes, scales))]
                         ).astype(np.float32) for u in range(U)]
    g[:, :n] = torch.from_numpy(np.stack(gh)).cuda()
    pipe.convert(g)                                   # per-tensor anchors, symbols (parity covered elsewhere)
    A = np.stack([oracle.anchor(gh[u], f, seg) for u in range(U)])
    syms = [oracle.convert_ef(gh[u], np.zeros(n, np.float32), A[u], 1.0, f, seg)[0] for u in range(U)]
    for u in range(U):
        assert np.array_equal(pipe.sym[u, :n].cpu().numpy(), syms[u])

    # per-tensor histograms
    cnt = torch.full((U, nseg, fmt.K), 7, dtype=torch.int32, device="cuda")
    B.histogram_layers(pipe.sym, n, fmt, pipe.seg_off, cnt)
    cnt_o = np.stack([oracle.histogram_layers(syms[u], f, seg) for u in range(U)])
    assert np.array_equal(u32(cnt), cnt_o), "per-tensor histogram"

    # one code per tensor: pooled counts of all users, or the GenNorm model of the tensor
    if table == "pooled":
        w = cnt_o.astype(np.int64).sum(axis=0).astype(np.uint32)
    else:
        # the anchor of user 0 designs the table; symbols other users emit always have a codeword because
        # every emit-able symbol gets weight >= 1
        w = np.stack([oracle.model_weights(int(A[0, k]), f, 0.9, float(scales[k])) for k in range(nseg)])
    wd = torch.from_numpy(w.view(np.int32)).cuda()
    codes = torch.zeros((nseg, B.CODE_BYTES), dtype=torch.uint8, device="cuda")
    B.build_code(wd, nseg, fmt, codes, pipe.status)
    lens = np.stack([oracle.huffman_lengths(w[k]) for k in range(nseg)])
    cods = np.stack([oracle.canonical_codes(lens[k]) for k in range(nseg)])
    assert np.array_equal(codes[:, :fmt.K].cpu().numpy(), lens), "code lengths per tensor"

    cap = max(2, ((int(lens.max(initial=1)) * n + 63) // 64 + 1) // 2 * 2)
    words = torch.zeros((U, cap), dtype=torch.int64, device="cuda")
    B.encode_layers(pipe.sym, n, fmt, codes, pipe.seg_off, words, C, pipe.chunk_bitoff, pipe.total_bits, pipe.enc_ws,
                    pipe.status)
    assert pipe.poll() == 0
    for u in range(U):
        wo, off, total = oracle.encode_layers(syms[u], lens, cods, seg, C)
        assert int(pipe.total_bits[u].item()) == total, "total bits"
        assert np.array_equal(u64(pipe.chunk_bitoff[u]), off), "chunk offsets"
        nw = (total + 63) // 64
        assert np.array_equal(u64(words[u, :nw]), wo[:nw]), "stream words"

    B.decode_layers(words, pipe.chunk_bitoff, C, codes, pipe.seg_off, fmt, n, pipe.sym_dec, pipe.status)
    assert pipe.poll() == 0
    assert torch.equal(pipe.sym_dec[:, :n], pipe.sym[:, :n]), "decode(encode(s)) = s"

    B.ps_aggregate_layers(words, pipe.chunk_bitoff, C, codes, pipe.seg_off, fmt, n, U, pipe.anchor, pipe.avg,
                          pipe.agg_ws, pipe.status, seg_off=pipe.seg_off)
    assert pipe.poll() == 0
    want = oracle.aggregate(np.stack(syms), A, f, seg)
    assert np.array_equal(u32(pipe.avg[:n]), want.view(np.uint32)), "average"
    return pipe, words, codes


@pytest.mark.parametrize("shape", list(SHAPES))
def test_layer_codes_shapes(co3, shape):
    run_layers(co3, 2, SHAPES[shape], 3, 1, 256, "pooled", seed=len(shape))


@pytest.mark.parametrize("E,M", [(3, 0), (4, 3), (5, 2), (1, 2)])
def test_layer_codes_formats(co3, E, M):
    run_layers(co3, 3, SHAPES["resnet_head"], E, M, 256, "pooled", seed=E * 8 + M)


@pytest.mark.parametrize("C", [64, 1024, 4096])
def test_layer_codes_chunk_sizes(co3, C):
    run_layers(co3, 2, SHAPES["odd"], 4, 3, C, "pooled", seed=C)


def test_layer_codes_from_model(co3):
    """Tables designed from the GenNorm law of each tensor (no statistics of the data): long codewords for
    the rare symbols, every emit-able symbol has one."""
    run_layers(co3, 2, SHAPES["resnet_head"], 4, 3, 256, "model", seed=5)
    run_layers(co3, 2, SHAPES["two_big"], 3, 1, 256, "model", seed=6)


def test_code_groups_differ_from_anchor_tensors(co3):
    """Anchors per tensor, codes per group of tensors (each small tensor grouped with the large one before
    it), pooled over 3 users, through the pipeline class; two chained iterations."""
    sizes = [1728, 64, 64, 36864, 64, 64, 73728, 128, 128, 5120, 10]
    groups = [1728 + 64 + 64, 36864 + 64 + 64, 73728 + 128 + 128, 5120 + 10]
    seg, cseg = inp.seg_offsets(sizes), inp.seg_offsets(groups)
    n, U, C = int(seg[-1]), 3, 256
    fmt, f = co3.Fmt(4, 3), oracle.Fmt(4, 3)
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, seg_off=seg, codes="layer", code_seg_off=cseg)
    g = pipe.new_gradient_buffer()
    errs = [np.zeros(n, np.float32) for _ in range(U)]
    for t in range(2):
        gh = [np.concatenate([inp.gennorm(inp.rng_for(89, t, u, k), m, 0.9, 10.0 ** -(2 + k % 3))
                              for k, m in enumerate(sizes)]).astype(np.float32) for u in range(U)]
        g[:, :n] = torch.from_numpy(np.stack(gh)).cuda()
        pipe.step(g)
        pipe.decode()
        assert pipe.poll() == 0
        A = np.stack([oracle.anchor(gh[u], f, seg) for u in range(U)])
        syms = []
        for u in range(U):
            sym, errs[u] = oracle.convert_ef(gh[u], errs[u], A[u], 1.0, f, seg)
            syms.append(sym)
        w = np.stack([oracle.histogram_layers(s_, f, cseg) for s_ in syms]).astype(np.int64).sum(axis=0).astype(np.uint32)
        assert np.array_equal(u32(pipe.layer_counts), w), "pooled counts per code group"
        lens = np.stack([oracle.huffman_lengths(w[k]) for k in range(len(groups))])
        cods = np.stack([oracle.canonical_codes(lens[k]) for k in range(len(groups))])
        for u in range(U):
            wo, off, total = oracle.encode_layers(syms[u], lens, cods, cseg, C)
            assert int(pipe.total_bits[u].item()) == total
            assert np.array_equal(u64(pipe.chunk_bitoff[u]), off)
            assert np.array_equal(u64(pipe.words[u, :(total + 63) // 64]), wo[:(total + 63) // 64])
            assert np.array_equal(pipe.sym_dec[u, :n].cpu().numpy(), syms[u])
            assert np.array_equal(u32(pipe.err[u, :n]), errs[u].view(np.uint32))
        want = oracle.aggregate(np.stack(syms), A, f, seg)
        assert np.array_equal(u32(pipe.avg[:n]), want.view(np.uint32))


def test_layer_codes_errors(co3):
    B = co3.binding
    pipe, words, codes = run_layers(co3, 1, [3000, 3000], 3, 1, 256, "pooled", seed=9)
    fmt, n = pipe.fmt, pipe.n
    # a symbol of tensor 1 loses its codeword: reported from the device, as for per-user codes
    cnt = oracle.histogram_layers(pipe.sym[0, :n].cpu().numpy(), oracle.Fmt(3, 1), [0, 3000, 6000]).astype(np.uint32)
    cnt[1, int(pipe.sym[0, 4000].item())] = 0
    B.build_code(torch.from_numpy(cnt.view(np.int32)).cuda(), 2, fmt, codes, pipe.status)
    B.encode_layers(pipe.sym, n, fmt, codes, pipe.seg_off, words, 256, pipe.chunk_bitoff, pipe.total_bits, pipe.enc_ws,
                    pipe.status)
    assert pipe.poll() == B.ENOCODE
    pipe.status.zero_()
    # host-rejected: tensor boundaries are required
    with pytest.raises(co3.Co3Error):
        B._chk(B._lib.co3_encode_layers(B._dp(pipe.sym), n, 1, pipe.stride, fmt.c(), B._dp(codes), None, 2,
                                        B._dp(words), words.shape[-1], 256, B._dp(pipe.chunk_bitoff),
                                        B._dp(pipe.total_bits), B._dp(pipe.enc_ws), pipe.enc_ws.numel() * 8,
                                        B._dp(pipe.status), B._stream()), "co3_encode_layers")
    with pytest.raises(co3.Co3Error):
        B._chk(B._lib.co3_decode_layers(B._dp(words), words.shape[-1], B._dp(pipe.chunk_bitoff), 256, B._dp(codes),
                                        None, 2, fmt.c(), n, 1, B._dp(pipe.sym_dec), pipe.stride, B._dp(pipe.status),
                                        B._stream()), "co3_decode_layers")
