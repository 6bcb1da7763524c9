"""Two workloads driven from two HIP streams at the same time (default priority): the library keeps no
state between calls, so interleaved launches on different streams give each workload the result it
gets alone."""
import numpy as np
import pytest

import co3_inputs as inp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def co3():
    import paper_2203_09044_amd as pkg
    return pkg


def test_two_streams_interleaved(co3):
    cfgs = [(2, 300_000 + 7, co3.Fmt(3, 0), 0.7), (3, 150_000 + 3, co3.Fmt(4, 3), 1.3)]
    alone, both = [], []
    data = []
    for U, n, fmt, beta in cfgs:
        x = torch.from_numpy(np.stack([inp.gennorm(inp.rng_for(61, U, u), n, beta, 1e-3) for u in range(U)])).cuda()
        data.append(x)
        p = co3.Co3Pipeline(U, n, fmt)
        g = p.new_gradient_buffer()
        g[:, :n] = x
        for _ in range(3):
            p.step(g)
        torch.cuda.synchronize()
        assert p.poll() == 0
        alone.append(p)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    gs = []
    for (U, n, fmt, _), x in zip(cfgs, data):
        p = co3.Co3Pipeline(U, n, fmt)
        g = p.new_gradient_buffer()
        g[:, :n] = x
        both.append(p)
        gs.append(g)
    torch.cuda.synchronize()
    for _ in range(3):                       # launches of the two workloads alternate
        for p, g, s in zip(both, gs, streams):
            with torch.cuda.stream(s):
                p.step(g)
    for s in streams:
        s.synchronize()
    for a, b, (U, n, fmt, _) in zip(alone, both, cfgs):
        assert b.poll() == 0
        assert torch.equal(a.sym, b.sym) and torch.equal(a.err.view(torch.int32), b.err.view(torch.int32))
        assert torch.equal(a.total_bits, b.total_bits) and torch.equal(a.chunk_bitoff, b.chunk_bitoff)
        assert torch.equal(a.avg.view(torch.int32), b.avg.view(torch.int32))
        for u in range(U):
            nw = int((a.total_bits[u].item() + 63) // 64)
            assert torch.equal(a.words[u, :nw], b.words[u, :nw])
