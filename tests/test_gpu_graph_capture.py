"""The whole iteration captured in a HIP graph (the library allocates nothing, records no memset and keeps
no state between calls while launch timing is off): every replay, with eager work and synchronisations
in between and fresh inputs written into the captured buffers, must equal the eager result bit for bit."""
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


@pytest.mark.parametrize("mode", ["user", "layer", "moments"])
def test_graph_replays_equal_eager(co3, mode):
    sizes = [5000, 64, 64, 40000, 3]
    seg = inp.seg_offsets(sizes)
    n, U = int(seg[-1]), 3
    fmt = co3.Fmt(3, 1)
    kw = dict(chunk_syms=256, seg_off=seg)
    if mode == "layer":
        kw.update(codes="layer", code_seg_off=inp.seg_offsets(inp.group_small_tensors(sizes, 1000)))
    if mode == "moments":
        kw.update(bias="moments")
    eager = co3.Co3Pipeline(U, n, fmt, **kw)
    graphed = co3.Co3Pipeline(U, n, fmt, **kw)
    g_e = eager.new_gradient_buffer()
    g_g = graphed.new_gradient_buffer()

    def draw(t):
        x = np.stack([inp.gennorm(inp.rng_for(71, t, u), n, 1.0, 1e-3) for u in range(U)]).astype(np.float32)
        return torch.from_numpy(x).cuda()

    # warm-up on a side stream, then capture one iteration
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        g_g[:, :n] = draw(0)
        graphed.step(g_g)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    graphed.err.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graphed.step(g_g)
    torch.cuda.synchronize()
    graphed.err.zero_()                      # the capture does not run the kernels; start both from m = 0

    for t in range(1, 5):
        x = draw(t)
        g_e[:, :n] = x
        g_g[:, :n] = x
        eager.step(g_e)
        graph.replay()
        torch.cuda.synchronize()
        junk = torch.rand(1 << 20, device="cuda").sum().item()      # eager work between replays
        assert junk > 0
        assert eager.poll() == 0 and graphed.poll() == 0
        for name in ("sym", "err", "anchor", "total_bits", "chunk_bitoff", "avg"):
            a, b = getattr(eager, name), getattr(graphed, name)
            assert torch.equal(a.view(torch.uint8) if a.dtype == torch.float32 else a,
                               b.view(torch.uint8) if b.dtype == torch.float32 else b), (mode, t, name)
        for u in range(U):                   # words past a user's own stream are left untouched by the encoder
            nw = int((eager.total_bits[u].item() + 63) // 64)
            assert torch.equal(eager.words[u, :nw], graphed.words[u, :nw]), (mode, t, u, "words")
    # and the eager side is the oracle's (last iteration, user 0, plain mode only)
    if mode == "user":
        f = oracle.Fmt(3, 1)
        assert np.array_equal(graphed.anchor[0].cpu().numpy(), oracle.anchor(x[0].cpu().numpy(), f, seg))


@pytest.mark.parametrize("mode", ["user", "layer-moments"])
def test_graph_replays_of_the_one_pass_user_side(co3, mode):
    """Fixed tables, conversion and compression in one pass: the captured iteration against the eager one."""
    sizes = [5000, 64, 64, 40000, 3]
    seg = inp.seg_offsets(sizes)
    n, U = int(seg[-1]), 3
    fmt = co3.Fmt(3, 1)
    kw = dict(chunk_syms=256, seg_off=seg, statistics=False, single_pass=True, cap_words=n)
    if mode == "layer-moments":
        kw.update(codes="layer", code_seg_off=inp.seg_offsets(inp.group_small_tensors(sizes, 1000)), bias="moments")
    eager = co3.Co3Pipeline(U, n, fmt, **kw)
    graphed = co3.Co3Pipeline(U, n, fmt, **kw)
    rows = eager.codes.shape[0]
    weights = np.random.default_rng(5).integers(1, 500, (rows, fmt.K)).astype(np.uint32) ** 2
    weights[:, fmt.K // 2] = 0
    for p in (eager, graphed):
        p.build(torch.from_numpy(weights.view(np.int32)).cuda())
    g_e = eager.new_gradient_buffer()
    g_g = graphed.new_gradient_buffer()

    def draw(t):
        x = np.stack([inp.gennorm(inp.rng_for(72, t, u), n, 1.0, 1e-3) for u in range(U)]).astype(np.float32)
        return torch.from_numpy(x).cuda()

    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        g_g[:, :n] = draw(0)
        graphed.step(g_g, rebuild=False)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    graphed.err.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graphed.step(g_g, rebuild=False)
    torch.cuda.synchronize()
    graphed.err.zero_()

    for t in range(1, 5):
        x = draw(t)
        g_e[:, :n] = x
        g_g[:, :n] = x
        eager.step(g_e, rebuild=False)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.rand(1 << 20, device="cuda").sum().item() > 0      # eager work between replays
        assert eager.poll() == 0 and graphed.poll() == 0
        for name in ("err", "anchor", "total_bits", "chunk_bitoff", "avg"):
            a, b = getattr(eager, name), getattr(graphed, name)
            assert torch.equal(a.view(torch.uint8) if a.dtype == torch.float32 else a,
                               b.view(torch.uint8) if b.dtype == torch.float32 else b), (mode, t, name)
        for u in range(U):
            nw = int((eager.total_bits[u].item() + 63) // 64)
            assert torch.equal(eager.words[u, :nw], graphed.words[u, :nw]), (mode, t, u, "words")
