"""Pins for the oracle's per-layer codes (Sec. III (ii): a different code per layer, shared by all users):
the stream is the bit-level concatenation of the per-tensor plain streams (the plain encoder is pinned in
test_oracle_pins.py), built here from bit strings without the oracle's packing code."""
import numpy as np
import pytest

import oracle
import co3_inputs as inp


def bits_of(words, total):
    return "".join(format(int(w), "064b") for w in words)[:total]


def make(nsizes, K, seed):
    rng = inp.rng_for(66, seed)
    sizes = list(nsizes)
    seg = inp.seg_offsets(sizes)
    n = int(seg[-1])
    f = oracle.Fmt(3, 1) if K == 32 else oracle.Fmt(2, 0)
    syms, lens, codes = [], [], []
    for s, m in enumerate(sizes):
        p = rng.dirichlet(np.full(K, 0.3 + 0.4 * (s % 3)))
        w = np.maximum(1, np.rint(p * 1e6)).astype(np.uint32)
        if s % 4 == 3:
            w[rng.integers(0, K, K // 2)] = 0            # some tensors leave symbols without a code
        l = oracle.huffman_lengths(w)
        c = oracle.canonical_codes(l)
        active = np.flatnonzero(l)
        syms.append(rng.choice(active, size=m, p=w[active] / w[active].sum()).astype(np.uint8))
        lens.append(l)
        codes.append(c)
    return f, seg, n, np.concatenate(syms) if n else np.zeros(0, np.uint8), np.stack(lens), np.stack(codes)


@pytest.mark.parametrize("sizes", [[1000], [10, 0, 700, 1, 333, 64, 5000], [1, 1, 1, 1], [257, 255, 256]])
@pytest.mark.parametrize("C", [1, 64, 256])
def test_stream_is_concatenation_of_tensor_streams(sizes, C):
    f, seg, n, sym, lens, codes = make(sizes, 32, len(sizes) * 7 + C)
    words, off, total = oracle.encode_layers(sym, lens, codes, seg, C)
    want = ""
    for s in range(len(sizes)):
        part = sym[seg[s]:seg[s + 1]]
        if part.size:
            w, _, t = oracle.encode(part, lens[s], codes[s], 64)
            want += bits_of(w, t)
    assert bits_of(words, total) == want
    assert total == len(want)
    assert all(int(b) == 0 for b in "".join(format(int(w), "064b") for w in words)[total:])
    # chunk offsets: prefix sums of the per-symbol lengths under each symbol's own tensor code
    per = np.concatenate([lens[s][sym[seg[s]:seg[s + 1]]] for s in range(len(sizes))]).astype(np.int64)
    cum = np.concatenate([[0], np.cumsum(per)])
    nchunks = (n + C - 1) // C
    assert np.array_equal(off.astype(np.int64), np.array([cum[min(c * C, n)] for c in range(nchunks + 1)]))
    # coded length from the per-tensor histograms
    cnt = oracle.histogram_layers(sym, f, seg)
    assert total == int((cnt.astype(np.int64) * lens.astype(np.int64)).sum())
    assert np.array_equal(cnt, np.stack([np.bincount(sym[seg[s]:seg[s + 1]], minlength=f.K) for s in range(len(sizes))]))
    # round trip
    assert np.array_equal(oracle.decode_layers(words, total, lens, codes, seg, n), sym)


def test_single_tensor_reduces_to_plain_functions():
    f, seg, n, sym, lens, codes = make([5000], 32, 3)
    w1, o1, t1 = oracle.encode_layers(sym, lens, codes, seg, 128)
    w0, o0, t0 = oracle.encode(sym, lens[0], codes[0], 128)
    assert t1 == t0 and np.array_equal(o1, o0) and np.array_equal(w1[:(t0 + 63) // 64], w0[:(t0 + 63) // 64])
    assert np.array_equal(oracle.decode_layers(w1, t1, lens, codes, seg, n), oracle.decode(w0, t0, lens[0], codes[0], n))


def test_error_paths():
    f, seg, n, sym, lens, codes = make([100, 100], 8, 4)
    bad = lens.copy()
    bad[1, sym[150]] = 0
    with pytest.raises(oracle.OracleError) as e:
        oracle.encode_layers(sym, bad, codes, seg, 64)
    assert e.value.code == oracle.ENOCODE
    with pytest.raises(oracle.OracleError) as e:
        oracle.encode_layers(sym, lens, codes, seg, 64, cap_words=1)
    assert e.value.code == oracle.ECAP
    words, off, total = oracle.encode_layers(sym, lens, codes, seg, 64)
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode_layers(words, total - 1, lens, codes, seg, n)
    assert e.value.code == oracle.EBADSTREAM
    # decoding with the tensors' codes swapped does not give the symbols back
    try:
        out = oracle.decode_layers(words, total, lens[::-1].copy(), codes[::-1].copy(), seg, n)
        assert not np.array_equal(out, sym)
    except oracle.OracleError as e2:
        assert e2.code == oracle.EBADSTREAM
