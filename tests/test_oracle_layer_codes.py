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
    # a byte that is not a symbol of the format is rejected by both histogram functions alike
    f3 = oracle.Fmt(2, 0)
    good = np.array([0, 1, 7, 3, 2, 7], np.uint8)
    assert np.array_equal(oracle.histogram_layers(good, f3, [0, 2, 6]).sum(axis=0), oracle.histogram(good, f3))
    for fn in (lambda x: oracle.histogram(x, f3), lambda x: oracle.histogram_layers(x, f3, [0, 2, 6])):
        with pytest.raises(oracle.OracleError) as e:
            fn(np.array([0, 1, 8, 3, 2, 7], np.uint8))
        assert e.value.code == oracle.EINVAL
    # decoding with the tensors' codes swapped does not give the symbols back
    try:
        out = oracle.decode_layers(words, total, lens[::-1].copy(), codes[::-1].copy(), seg, n)
        assert not np.array_equal(out, sym)
    except oracle.OracleError as e2:
        assert e2.code == oracle.EBADSTREAM


# ---- model tables of shared per-layer codes: which tensor designs a group's table, and the pooled law ----
def test_design_tables_pick_the_largest_tensor_that_starts_in_the_group():
    """Hand-built layout: expected design tensors written out by hand.  Every tensor gets a law of its own
    (all users alike), so the table of a group tells which tensor designed it."""
    f = oracle.Fmt(3, 1)
    sizes = [5, 100, 100, 7, 300, 2, 0, 40]
    seg = inp.seg_offsets(sizes)                      # 0 5 105 205 212 512 514 514 554
    code_seg = [0, 205, 212, 514, 554, 554]           # groups: {0,1,2} {3} {4,5,6} {7} {} (empty range at the end)
    want_tensor = [1, 3, 4, 7]                        # first of the two equal tensors 1 and 2; 6 is empty
    U, nseg = 3, len(sizes)
    fit = np.zeros((U, nseg, 2))
    fit[:, :, 0] = 0.5 + 0.1 * np.arange(nseg)        # shape per tensor
    fit[:, :, 1] = 1e-3 * (1 + np.arange(nseg))       # scale per tensor
    scale = np.ones((U, nseg), np.float32)
    got = oracle.design_layer_tables(fit, scale, seg, code_seg[:5], -3, f)
    for k, s in enumerate(want_tensor):
        assert np.array_equal(got[k], oracle.model_weights(-3, f, 0.5 + 0.1 * s, 1e-3 * (1 + s))), k
    # a group in which no tensor starts takes the tensor that holds its first element
    got = oracle.design_layer_tables(fit, scale, seg, [0, 250, 400, 554], -3, f)
    assert np.array_equal(got[1], oracle.model_weights(-3, f, 0.5 + 0.1 * 4, 1e-3 * 5))   # element 250 lies in tensor 4


def test_design_tables_pool_the_users_by_the_mean_of_the_fitted_parameters():
    """One tensor, one group: the law is (mean shape, mean of scale x multiplier), checked against exact
    rational arithmetic; identical users reduce to a single user; the limits on the shape hold."""
    from fractions import Fraction
    f = oracle.Fmt(1, 2)
    rng = inp.rng_for(67, 1)
    U = 5
    fit = np.zeros((U, 1, 2))
    fit[:, 0, 0] = rng.uniform(0.6, 1.8, U)
    fit[:, 0, 1] = rng.uniform(1e-4, 1e-2, U)
    scale = rng.uniform(50, 500, (U, 1)).astype(np.float32)
    beta = float(sum(Fraction(float(b)) for b in fit[:, 0, 0]) / U)
    alpha = float(sum(Fraction(float(a)) * Fraction(float(c)) for a, c in zip(fit[:, 0, 1], scale[:, 0])) / U)
    got = oracle.design_layer_tables(fit, scale, [0, 1000], [0, 1000], 1, f)[0]
    want = oracle.model_weights(1, f, beta, alpha)
    # the double-precision sums are within a few units in the last place of the exact means: the weights
    # (32-bit roundings of probabilities) can differ by one unit at most
    assert np.max(np.abs(got.astype(np.int64) - want.astype(np.int64))) <= 1
    # a multiplier moves the scale, not the shape: twice the multiplier = twice the scale of the law
    twice = oracle.design_layer_tables(fit, 2 * scale, [0, 1000], [0, 1000], 1, f)[0]
    assert np.max(np.abs(twice.astype(np.int64) - oracle.model_weights(1, f, beta, 2 * alpha).astype(np.int64))) <= 1
    same = np.repeat(fit[:1], 4, axis=0), np.repeat(scale[:1], 4, axis=0)
    one = oracle.design_layer_tables(fit[:1], scale[:1], [0, 1000], [0, 1000], 1, f)[0]
    assert np.array_equal(oracle.design_layer_tables(same[0], same[1], [0, 1000], [0, 1000], 1, f)[0], one)
    assert np.array_equal(one, oracle.model_weights(1, f, float(fit[0, 0, 0]), float(fit[0, 0, 1]) * float(scale[0, 0])))
    lo, hi = fit.copy(), fit.copy()
    lo[:, 0, 0], hi[:, 0, 0] = 0.01, 40.0
    ones = np.ones((U, 1), np.float32)
    a = float(np.sum([Fraction(float(x)) for x in fit[:, 0, 1]]) / U)
    assert np.max(np.abs(oracle.design_layer_tables(lo, ones, [0, 9], [0, 9], 1, f)[0].astype(np.int64) -
                         oracle.model_weights(1, f, 0.2, a).astype(np.int64))) <= 1
    assert np.max(np.abs(oracle.design_layer_tables(hi, ones, [0, 9], [0, 9], 1, f)[0].astype(np.int64) -
                         oracle.model_weights(1, f, 4.0, a).astype(np.int64))) <= 1
