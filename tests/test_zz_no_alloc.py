"""co3_encode_static (the encoder for callers that cannot allocate: its tile and group sizes live in a
fixed array inside the library) against co3_encode, through the C ABI: every stream word, every chunk
offset and the stream lengths, on two calls in a row, the second with a smaller input (the array keeps
the first call's contents).  Collected last: the file name sorts after every other test file."""
import numpy as np
import pytest

import co3_inputs as inp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _u64(t):
    return t.cpu().numpy().view(np.uint64)


def _encode_both(co3, U, n, fmt, C, seed):
    """Symbols and codes from the library's own user side, then both encoders on the same inputs."""
    B = co3.binding
    pipe = co3.Co3Pipeline(U, n, fmt, chunk_syms=C)
    g = pipe.new_gradient_buffer()
    host = np.stack([inp.gennorm(inp.rng_for(77, seed, u, 1), n, 0.6 + 0.3 * u, 1e-3) for u in range(U)])
    g[:, :n] = torch.from_numpy(host).cuda()
    pipe.convert(g)
    pipe.build()
    pipe.encode()                       # co3_encode, caller's workspace
    assert pipe.poll() == 0
    nw = [int((int(t) + 63) // 64) for t in pipe.total_bits.cpu().numpy()]
    want = dict(words=[_u64(pipe.words[u, :nw[u]]).copy() for u in range(U)], off=_u64(pipe.chunk_bitoff).copy(),
                total=_u64(pipe.total_bits).copy())
    # fresh outputs with a recognisable filling
    words = torch.full_like(pipe.words, -1)
    off = torch.full_like(pipe.chunk_bitoff, -1)
    total = torch.full_like(pipe.total_bits, -1)
    B.encode_static(pipe.sym, n, fmt, pipe.codes, words, C, off, total, pipe.status)
    assert pipe.poll() == 0
    assert np.array_equal(_u64(total), want["total"]), "stream lengths"
    assert np.array_equal(_u64(off), want["off"]), "chunk offsets"
    for u in range(U):
        assert np.array_equal(_u64(words[u, :nw[u]]), want["words"][u]), f"stream words of user {u}"
        assert bool((words[u, nw[u]:] == -1).all()), "nothing is written past the stream"
    return pipe


def test_encode_static_matches_encode_twice_in_a_row():
    import paper_2203_09044_amd as co3
    fmt = co3.Fmt(3, 1)
    # several groups of 16 tiles and a ragged tail; then a smaller batch with another format and chunk size
    _encode_both(co3, 3, 16 * 1024 * 5 + 1237, fmt, 256, seed=1)
    _encode_both(co3, 2, 1024 * 3 + 17, co3.Fmt(4, 3), 128, seed=2)
    _encode_both(co3, 1, 5, fmt, 64, seed=3)


def test_encode_static_rejects_batches_beyond_the_fixed_workspace():
    import paper_2203_09044_amd as co3
    B = co3.binding
    fmt = co3.Fmt(2, 0)
    U, n = 64, 10_000_000                   # 64 x 9766 tiles x 8 B > 4 MiB
    assert B.encode_workspace_bytes(n, U) > B.ENCODE_STATIC_WS_BYTES
    one = torch.zeros(16, dtype=torch.uint8, device="cuda")
    w = torch.zeros(2, dtype=torch.int64, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc = B._lib.co3_encode_static(B._dp(one), n, U, n + 16 - n % 16, fmt.c(), B._dp(one), B._dp(w), 2, 256, B._dp(w),
                                  B._dp(w), B._dp(st), B._stream())
    assert rc == B.EINVAL
