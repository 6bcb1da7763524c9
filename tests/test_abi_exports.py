"""The C-ABI library loads and exports every function declared in include/co3.h (CPU only:
no GPU work is issued; the host-only helpers are exercised)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "co3.h")
LIB = os.path.join(ROOT, "paper_2203_09044_amd", "libco3.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(co3_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as ge
        ge.build()
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"co3_convert_ef", "co3_histogram", "co3_build_code", "co3_encode", "co3_decode",
            "co3_ps_aggregate"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_covers_header():
    from paper_2203_09044_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()
    for name in binding.EXPORTS:
        assert hasattr(binding, name[len("co3_"):]), name


def test_host_helpers_without_gpu():
    from paper_2203_09044_amd import binding as B
    fmt = B.Fmt(3, 1)
    assert B.strerror(0) == "ok" and B.strerror(B.ECAP) and B.strerror(-1234)
    assert B.encode_workspace_bytes(0, 1) == 16
    assert B.encode_workspace_bytes(1024, 3) == 48
    assert B.encode_workspace_bytes(1025, 3) == 72
    assert B.ps_aggregate_workspace_bytes(32, 4, 256) == 4 * 64 * 256      # one tile of 64 chunks per user
    assert B.ps_aggregate_workspace_bytes(64 * 256 + 1, 1, 256) == 2 * 64 * 256
    assert B.cap_words_empirical(64, fmt) == 6          # 5 bits * 64 = 320 bits = 5 words, even -> 6
    assert B.cap_words_empirical(0, fmt) == 0
    assert B.CODE_BYTES == 12288


def test_host_argument_checks_launch_nothing():
    """Invalid arguments are rejected on the host before any HIP call (safe without a GPU)."""
    from paper_2203_09044_amd import binding as B
    L = B._lib
    f = B.Fmt(6, 3).c()       # 10 bits: invalid
    assert L.co3_convert_ef(None, None, None, 10, 1, 16, None, 1, None, 0, 1.0, f, None, None) == B.EINVAL
    assert L.co3_histogram(None, 10, 1, 16, B.Fmt(3, 1).c(), None, None) == B.EINVAL
    assert L.co3_build_code(None, 1, B.Fmt(3, 1).c(), None, None, None) == B.EINVAL
    assert L.co3_encode(None, 10, 1, 16, B.Fmt(3, 1).c(), None, None, 1, 100, None, None, None, 0, None, None) == B.EINVAL
    assert L.co3_decode(None, 1, None, 256, None, B.Fmt(3, 1).c(), 10, 1, None, 16, None, None) == B.EINVAL
    assert L.co3_ps_aggregate(None, 1, None, 256, None, B.Fmt(3, 1).c(), 10, 1, None, None, 1, None, None, 0, None,
                              None) == B.EINVAL
    assert L.co3_poll_status(None, None) == B.EINVAL
    ok = B.Fmt(3, 1).c()
    assert L.co3_moments(None, None, 10, 1, 16, None, 1, 1.0, None, None) == B.EINVAL
    assert L.co3_bias_scale(None, 10, 1, None, 1, None, None, None) == B.EINVAL
    assert L.co3_convert_ef_scaled(None, None, None, 10, 1, 16, None, 1, None, None, 1.0, ok, None, None) == B.EINVAL
    assert L.co3_ps_aggregate_scaled(None, 2, None, 256, None, ok, 10, 1, None, None, None, 1, None, None, 0, None,
                                     None) == B.EINVAL
    assert L.co3_histogram_layers(None, 10, 1, 16, None, 1, ok, 0, None, None) == B.EINVAL
    assert L.co3_encode_layers(None, 10, 1, 16, ok, None, None, 1, None, 2, 256, None, None, None, 0, None,
                               None) == B.EINVAL
    assert L.co3_decode_layers(None, 2, None, 256, None, None, 1, ok, 10, 1, None, 16, None, None) == B.EINVAL
    assert L.co3_ps_aggregate_layers(None, 2, None, 256, None, None, 1, ok, 10, 1, None, None, None, 1, None, None, 0,
                                     None, None) == B.EINVAL
    assert L.co3_convert_encode(None, None, 10, 1, 16, None, 1, None, 0, 1.0, ok, None, None, None, 2, 256, None, None, None,
                                0, None, None) == B.EINVAL
    assert L.co3_convert_encode_layers(None, None, 10, 1, 16, None, 1, None, 0, None, 1.0, ok, None, None, 1, None, None, 2,
                                       256, None, None, None, 0, None, None) == B.EINVAL
    assert B.convert_encode_workspace_bytes(0, 1, 256) > 0 and B.convert_encode_workspace_bytes(10, 1, 100) == 0
    # sizes at and beyond the interface's limit (n < 2^32), with plausible non-null pointers: rejected before
    # anything is launched
    import ctypes as C
    fake = C.c_void_p(1 << 20)
    big = 1 << 32
    assert L.co3_histogram(fake, big, 1, big, ok, fake, None) == B.EINVAL
    assert L.co3_convert_ef(fake, fake, fake, big, 1, big, None, 1, fake, 0, 1.0, ok, None, None) == B.EINVAL
    assert L.co3_moments(fake, fake, big, 1, big, None, 1, 1.0, fake, None) == B.EINVAL
    assert L.co3_decode(fake, 2, fake, 256, fake, ok, big, 1, fake, big, None, None) == B.EINVAL
    # users of a batch must be 16-element aligned rows at least n long
    assert L.co3_histogram(fake, 100, 2, 100, ok, fake, None) == B.EINVAL
    assert L.co3_histogram(fake, 100, 2, 96, ok, fake, None) == B.EINVAL


def test_model_weights_host_matches_oracle_model():
    """The library's own GenNorm-CDF arithmetic against the oracle's scipy-based table."""
    import oracle
    from paper_2203_09044_amd import binding as B
    for (E, M), beta, alpha, A in [((5, 2), 1.0, 1e-4, -7), ((3, 1), 1.0, 1e-3, -7), ((4, 3), 0.8, 1e-3, -5),
                                   ((2, 0), 0.5, 1e-3, -3), ((3, 0), 1.5, 1e-3, -8), ((4, 3), 2.0, 1e-3, -8),
                                   ((5, 2), 0.5, 1e-3, 2)]:
        got = B.model_weights(A, B.Fmt(E, M), beta, alpha).numpy().view(np.uint32)
        want = oracle.model_weights(A, oracle.Fmt(E, M), beta, alpha)
        assert np.array_equal(got, want), (E, M, beta, A)
        assert got[(1 << (E + M))] == 0 and got.min(initial=1, where=np.arange(got.size) != (1 << (E + M))) >= 1


def test_design_layer_tables_host_matches_oracle():
    """co3_design_layer_tables (which tensor designs a group's shared table, the law pooled over the users,
    its limits) against the oracle's statement of the same rule, bit for bit on the weights."""
    import oracle
    import co3_inputs as inp
    from paper_2203_09044_amd import binding as B
    import torch
    rng = inp.rng_for(68, 2)
    for case, (sizes, gmin, U, (E, M), A) in enumerate([([5, 100, 100, 7, 300, 2, 0, 40], 50, 3, (3, 1), -3),
                                                        (inp.resnet18_cifar_tensor_sizes(), 16384, 10, (1, 2), 1),
                                                        ([1000], 1, 1, (4, 3), 8), ([3, 3, 3], 100, 4, (2, 0), 0)]):
        seg = inp.seg_offsets(sizes)
        cso = inp.seg_offsets(inp.group_small_tensors(sizes, gmin))
        nseg = len(sizes)
        fit = np.zeros((U, nseg, 2))
        fit[:, :, 0] = rng.uniform(0.1, 5.0, (U, nseg))              # beyond the limits on both sides
        fit[:, :, 1] = 10.0 ** rng.uniform(-6, -1, (U, nseg))
        scale = (10.0 ** rng.uniform(0, 4, (U, nseg))).astype(np.float32)
        got = B.design_layer_tables(torch.from_numpy(fit), torch.from_numpy(scale), seg, cso, A, B.Fmt(E, M))
        want = oracle.design_layer_tables(fit, scale, seg, cso, A, oracle.Fmt(E, M))
        assert np.array_equal(got.numpy().view(np.uint32), want), case
    # boundaries of the groups that are not tensor boundaries
    sizes = [5, 100, 100, 7, 300]
    seg = inp.seg_offsets(sizes)
    fit = np.zeros((2, 5, 2))
    fit[:, :, 0] = rng.uniform(0.5, 1.5, (2, 5))
    fit[:, :, 1] = 1e-3
    scale = np.ones((2, 5), np.float32)
    cso = [0, 250, 400, 512]
    got = B.design_layer_tables(torch.from_numpy(fit), torch.from_numpy(scale), seg, cso, -2, B.Fmt(3, 1))
    assert np.array_equal(got.numpy().view(np.uint32), oracle.design_layer_tables(fit, scale, seg, cso, -2, oracle.Fmt(3, 1)))
    L = B._lib
    assert L.co3_design_layer_tables(None, None, 1, 1, None, None, 1, 0, B.Fmt(3, 1).c(), None) == B.EINVAL
