"""co3_convert_encode (fixed codes: conversion and compression in one pass) against the oracle's
convert_ef followed by encode, bit for bit, through the C ABI."""
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


def u64(t):
    return t.cpu().numpy().view(np.uint64)


def run(co3, U, n, E, M, C, betas, sizes=None, T=2, gamma=1.0, weights=None, seed=0):
    fmt, f = co3.Fmt(E, M), oracle.Fmt(E, M)
    seg_off = None if sizes is None else inp.seg_offsets(sizes)
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C, seg_off=seg_off, gamma=gamma, statistics=False, single_pass=True,
                           cap_words=2 * ((n * 57 + 127) // 128 + 1))        # a fixed table has no length bound
    # fixed tables: every emit-able symbol has a codeword (weight >= 1), skewed so that lengths differ
    if weights is None:
        rng = np.random.default_rng(seed + 5)
        weights = rng.integers(1, 1000, (U, fmt.K)).astype(np.uint32) ** 2
        weights[:, 1 << (E + M)] = 0                               # the negative zero is never emitted
    pipe.build(torch.from_numpy(weights.view(np.int32)).cuda())
    lens = [oracle.huffman_lengths(weights[u]) for u in range(U)]
    errs = [np.zeros(n, np.float32) for _ in range(U)]
    g = pipe.new_gradient_buffer()
    for t in range(1, T + 1):
        gh = [inp.gennorm(inp.rng_for(98, seed, u, t), n, betas[u % len(betas)], 1e-3) for u in range(U)]
        if n:
            g[:, :n] = torch.from_numpy(np.stack(gh)).cuda()
        pipe.step(g, rebuild=False)
        assert pipe.poll() == 0
        syms, anchors = [], []
        for u in range(U):
            A = oracle.anchor(gh[u], f, seg_off)
            s, errs[u] = oracle.convert_ef(gh[u], errs[u], A, gamma, f, seg_off)
            words, off, total = oracle.encode(s, lens[u], oracle.canonical_codes(lens[u]), C)
            assert np.array_equal(pipe.anchor[u].cpu().numpy(), A), "anchor"
            assert np.array_equal(pipe.err[u, :n].cpu().numpy().view(np.uint32), errs[u].view(np.uint32)), "memory"
            assert int(pipe.total_bits[u].item()) == total, "total bits"
            assert np.array_equal(u64(pipe.chunk_bitoff[u]), off), "chunk offsets"
            nw = (total + 63) // 64
            assert np.array_equal(u64(pipe.words[u, :nw]), words[:nw]), "stream words"
            syms.append(s)
            anchors.append(A)
        want = oracle.aggregate(np.stack(syms) if n else np.zeros((U, 0), np.uint8), np.stack(anchors), f, seg_off)
        assert np.array_equal(pipe.avg[:n].cpu().numpy().view(np.uint32), want.view(np.uint32)), "average"
    return pipe


@pytest.mark.parametrize("E,M", [(3, 0), (3, 1), (4, 3), (5, 2), (1, 2), (2, 0)])
def test_formats(co3, E, M):
    run(co3, 2, 5 * 2048 + 1237, E, M, 256, betas=[0.7, 1.4], T=3)


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 255, 256, 257, 1023, 1024, 1025, 2047, 4095, 4096, 4096 + 8, 65_535, 65_536,
                               65_536 + 5, 2 * 65_536 + 1024, 300_001])
def test_sizes(co3, n):
    run(co3, 3, n, 3, 1, 64, betas=[0.5, 1.0, 1.5])


@pytest.mark.parametrize("C", [64, 128, 256, 512, 1024, 4096])
def test_chunk_sizes(co3, C):
    run(co3, 2, 3 * 4096 + 100, 4, 3, C, betas=[0.8])


def test_tensors_and_decay(co3):
    sizes = (1000, 3, 64, 5000, 129, 70_000, 1, 256, 4000)
    run(co3, 2, sum(sizes), 4, 3, 256, betas=[0.8, 1.2], sizes=sizes, T=3, gamma=0.9)


def test_long_codewords(co3):
    """Fibonacci weights: codewords up to 45 bits, so a lane's four codewords often exceed 64 bits (staged one by
    one) and a unit's bits fill several hundred words of its slot."""
    fib = [1, 1]
    while len(fib) < 46:
        fib.append(fib[-1] + fib[-2])
    w = np.ones((1, 256), np.uint32)
    w[0, 128] = 0
    w[0, :46] = fib
    w[0, 46:128] = fib[-1]
    run(co3, 1, 3 * 2048 + 77, 4, 3, 64, betas=[1.0], weights=w)


def test_symbol_without_code_is_reported(co3):
    fmt = co3.Fmt(3, 0)
    n = 10_000
    pipe = co3.Co3Pipeline(1, n, fmt, statistics=False, single_pass=True)
    w = np.ones((1, 16), np.int32)
    w[0, 0] = 0                       # the zero level has no codeword
    pipe.build(torch.from_numpy(w).cuda())
    g = pipe.new_gradient_buffer()
    g[0, :n] = torch.from_numpy(inp.gennorm(inp.rng_for(98, 1, 0, 1), n, 1.0, 1e-3)).cuda()
    pipe.convert_encode(g)
    assert pipe.poll() == co3.binding.ENOCODE


def test_capacity_is_respected(co3):
    fmt = co3.Fmt(3, 0)
    n = 20_000
    pipe = co3.Co3Pipeline(1, n, fmt, statistics=False, single_pass=True, cap_words=100)
    pipe.build(torch.ones((1, 16), dtype=torch.int32, device="cuda"))         # flat 4-bit code: 80,000 bits
    pipe.words.fill_(0x5A5A5A5A5A5A5A5A)
    g = pipe.new_gradient_buffer()
    g[0, :n] = torch.from_numpy(inp.gennorm(inp.rng_for(98, 2, 0, 1), n, 1.0, 1e-3)).cuda()
    pipe.convert_encode(g)
    assert pipe.poll() == co3.binding.ECAP
    assert int(pipe.total_bits[0].item()) == 4 * n          # the needed length is still reported
