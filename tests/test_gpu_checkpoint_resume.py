"""Checkpoint and resume: the only state that Algorithm 1 carries from one iteration to the next on the
user side is the memory m (and, where the codes lag one iteration behind, the codes).  T iterations in one
go must give the same streams, averages and memories as T/2 iterations, a save of that state through a
file, a fresh pipeline that loads it, and the remaining T/2 iterations."""
import io

import numpy as np
import pytest

import co3_inputs as inp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def co3():
    import paper_2203_09044_amd as pkg
    return pkg


def gradients(U, n, t, g):
    for u in range(U):
        g[u, :n] = torch.from_numpy(inp.gennorm(inp.rng_for(90, 0, u, t), n, 0.7 + 0.3 * u, 1e-3 * (1.0 + 0.2 * t))).cuda()


def snapshot(pipe):
    nw = [(int(b) + 63) // 64 for b in pipe.total_bits.cpu().tolist()]
    return dict(words=[pipe.words[u, :nw[u]].clone() for u in range(pipe.U)], total=pipe.total_bits.clone(),
                off=pipe.chunk_bitoff.clone(), avg=pipe.avg.clone(), err=pipe.err.clone(), anchor=pipe.anchor.clone())


def same(a, b):
    return (all(torch.equal(x, y) for x, y in zip(a["words"], b["words"])) and torch.equal(a["total"], b["total"])
            and torch.equal(a["off"], b["off"]) and torch.equal(a["avg"].view(torch.int32), b["avg"].view(torch.int32))
            and torch.equal(a["err"].view(torch.int32), b["err"].view(torch.int32)) and torch.equal(a["anchor"], b["anchor"]))


@pytest.mark.parametrize("mode", ["separate", "one_call", "lagged"])
@pytest.mark.parametrize("gamma", [1.0, 0.9])
def test_resume_from_saved_memory_gives_identical_streams(co3, mode, gamma):
    U, n, T = 3, 300_007, 6
    fmt = co3.Fmt(3, 1)
    kw = dict(chunk_syms=256, gamma=gamma, one_call=mode == "one_call", single_pass=mode == "lagged",
              lagged_codes=mode == "lagged")

    whole = co3.Co3Pipeline(U, n, fmt, **kw)
    g = whole.new_gradient_buffer()
    ref = []
    for t in range(1, T + 1):
        gradients(U, n, t, g)
        whole.step(g)
        ref.append(snapshot(whole))
    assert whole.poll() == 0

    first = co3.Co3Pipeline(U, n, fmt, **kw)
    for t in range(1, T // 2 + 1):
        gradients(U, n, t, g)
        first.step(g)
        assert same(snapshot(first), ref[t - 1])
    f = io.BytesIO()
    torch.save({"err": first.err.cpu(), "codes": first.codes.cpu(), "have_codes": first.have_codes}, f)
    del first

    f.seek(0)
    state = torch.load(f, weights_only=True)
    second = co3.Co3Pipeline(U, n, fmt, **kw)
    second.err.copy_(state["err"])
    if mode == "lagged":
        second.codes.copy_(state["codes"])
        second.have_codes = bool(state["have_codes"])
    for t in range(T // 2 + 1, T + 1):
        gradients(U, n, t, g)
        second.step(g)
        assert same(snapshot(second), ref[t - 1]), t
    assert second.poll() == 0
    # the memory matters: without it the continuation differs
    third = co3.Co3Pipeline(U, n, fmt, **kw)
    gradients(U, n, T // 2 + 1, g)
    third.step(g)
    assert not torch.equal(third.err.view(torch.int32), ref[T // 2]["err"].view(torch.int32))
