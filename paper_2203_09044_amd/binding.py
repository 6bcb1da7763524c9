"""ctypes binding of libco3: argument marshalling only.

Every function has the name and meaning of the C entry point in ``include/co3.h``.
Tensors are torch CUDA tensors (PyTorch is used for device memory and streams only);
all arithmetic of the codec runs in the HIP kernels of the library.  There is no
fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libco3.so")

OK, EINVAL, ECAP, ENOCODE, EBADSTREAM, EHIP, ETIMEOUT = 0, -1, -2, -3, -4, -5, -6
ANCHOR_GIVEN, ANCHOR_FROM_ABSMAX_G = 0, 1
CODE_BYTES = 12288
PACK_SYMS = 1024

EXPORTS = (
    "co3_strerror", "co3_encode_workspace_bytes", "co3_ps_aggregate_workspace_bytes", "co3_cap_words_empirical",
    "co3_poll_status", "co3_convert_ef", "co3_histogram", "co3_build_code", "co3_encode", "co3_decode",
    "co3_ps_aggregate", "co3_model_weights", "co3_timing_enable", "co3_timing_read", "co3_timing_reset",
    "co3_kernel_name", "co3_moments", "co3_bias_scale", "co3_convert_ef_scaled", "co3_ps_aggregate_scaled",
    "co3_histogram_layers", "co3_encode_layers", "co3_decode_layers", "co3_ps_aggregate_layers",
    "co3_convert_encode_workspace_bytes", "co3_convert_encode", "co3_convert_encode_layers", "co3_encode_static",
    "co3_user_encode_workspace_bytes", "co3_user_encode", "co3_set_exchange_spin_limit", "co3_design_layer_tables",
    "co3_ps_aggregate_partial", "co3_ps_decode_users", "co3_ps_average",
)
KERNEL_COUNT = 13


class _Fmt(C.Structure):
    _fields_ = [("exp_bits", C.c_int32), ("mant_bits", C.c_int32)]


@dataclass(frozen=True)
class Fmt:
    """1 sign bit, E exponent bits, M mantissa bits."""
    E: int
    M: int

    @property
    def K(self) -> int:
        return 1 << (1 + self.E + self.M)

    @property
    def bits(self) -> int:
        return 1 + self.E + self.M

    def c(self) -> _Fmt:
        return _Fmt(self.E, self.M)


class Co3Error(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {strerror(code)} ({code})")
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(LIB_PATH)
    p, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.co3_strerror.restype = C.c_char_p
    L.co3_strerror.argtypes = [i32]
    L.co3_encode_workspace_bytes.restype = sz
    L.co3_encode_workspace_bytes.argtypes = [i64, i32]
    L.co3_ps_aggregate_workspace_bytes.restype = sz
    L.co3_ps_aggregate_workspace_bytes.argtypes = [i64, i32, i32]
    L.co3_cap_words_empirical.restype = i64
    L.co3_cap_words_empirical.argtypes = [i64, _Fmt]
    L.co3_poll_status.restype = i32
    L.co3_poll_status.argtypes = [p, p]
    L.co3_convert_ef.restype = i32
    L.co3_convert_ef.argtypes = [p, p, p, i64, i32, i64, p, i32, p, i32, C.c_float, _Fmt, p, p]
    L.co3_convert_ef_scaled.restype = i32
    L.co3_convert_ef_scaled.argtypes = [p, p, p, i64, i32, i64, p, i32, p, p, C.c_float, _Fmt, p, p]
    L.co3_moments.restype = i32
    L.co3_moments.argtypes = [p, p, i64, i32, i64, p, i32, C.c_float, p, p]
    L.co3_bias_scale.restype = i32
    L.co3_bias_scale.argtypes = [p, i64, i32, p, i32, p, p, p]
    L.co3_ps_aggregate_scaled.restype = i32
    L.co3_ps_aggregate_scaled.argtypes = [p, i64, p, i32, p, _Fmt, i64, i32, p, p, p, i32, p, p, sz, p, p]
    L.co3_histogram.restype = i32
    L.co3_histogram.argtypes = [p, i64, i32, i64, _Fmt, p, p]
    L.co3_build_code.restype = i32
    L.co3_build_code.argtypes = [p, i32, _Fmt, p, p, p]
    L.co3_encode.restype = i32
    L.co3_encode.argtypes = [p, i64, i32, i64, _Fmt, p, p, i64, i32, p, p, p, sz, p, p]
    L.co3_encode_static.restype = i32
    L.co3_encode_static.argtypes = [p, i64, i32, i64, _Fmt, p, p, i64, i32, p, p, p, p]
    L.co3_design_layer_tables.restype = i32
    L.co3_design_layer_tables.argtypes = [p, p, i32, i32, p, p, i32, i32, _Fmt, p]
    L.co3_user_encode_workspace_bytes.restype = sz
    L.co3_user_encode_workspace_bytes.argtypes = [i64, i32, i64, i32, i32]
    L.co3_user_encode.restype = i32
    L.co3_user_encode.argtypes = [p, p, i64, i32, i64, p, i32, p, C.c_float, _Fmt, p, p, p, i64, i32, p, p, p, p, sz, p, p]
    L.co3_ps_decode_users.restype = i32
    L.co3_ps_decode_users.argtypes = [p, i64, p, i32, p, _Fmt, i64, i32, i32, i32, p, sz, p, p]
    L.co3_ps_average.restype = i32
    L.co3_ps_average.argtypes = [p, sz, i32, _Fmt, i64, i32, p, p, i32, p, p]
    L.co3_ps_aggregate_partial.restype = i32
    L.co3_ps_aggregate_partial.argtypes = [p, i64, p, i32, p, _Fmt, i64, i32, p, p, i32, p, i32, p, p, sz, p, p]
    L.co3_set_exchange_spin_limit.restype = None
    L.co3_set_exchange_spin_limit.argtypes = [C.c_int64]
    L.co3_decode.restype = i32
    L.co3_decode.argtypes = [p, i64, p, i32, p, _Fmt, i64, i32, p, i64, p, p]
    L.co3_ps_aggregate.restype = i32
    L.co3_ps_aggregate.argtypes = [p, i64, p, i32, p, _Fmt, i64, i32, p, p, i32, p, p, sz, p, p]
    L.co3_histogram_layers.restype = i32
    L.co3_histogram_layers.argtypes = [p, i64, i32, i64, p, i32, _Fmt, i32, p, p]
    L.co3_encode_layers.restype = i32
    L.co3_encode_layers.argtypes = [p, i64, i32, i64, _Fmt, p, p, i32, p, i64, i32, p, p, p, sz, p, p]
    L.co3_decode_layers.restype = i32
    L.co3_decode_layers.argtypes = [p, i64, p, i32, p, p, i32, _Fmt, i64, i32, p, i64, p, p]
    L.co3_ps_aggregate_layers.restype = i32
    L.co3_ps_aggregate_layers.argtypes = [p, i64, p, i32, p, p, i32, _Fmt, i64, i32, p, p, p, i32, p, p, sz, p, p]
    L.co3_convert_encode_workspace_bytes.restype = sz
    L.co3_convert_encode_workspace_bytes.argtypes = [i64, i32, i32]
    L.co3_convert_encode.restype = i32
    L.co3_convert_encode.argtypes = [p, p, i64, i32, i64, p, i32, p, i32, C.c_float, _Fmt, p, p, p, i64, i32, p, p, p, sz, p, p]
    L.co3_convert_encode_layers.restype = i32
    L.co3_convert_encode_layers.argtypes = [p, p, i64, i32, i64, p, i32, p, i32, p, C.c_float, _Fmt, p, p, i32, p, p, i64, i32,
                                            p, p, p, sz, p, p]
    L.co3_model_weights.restype = i32
    L.co3_model_weights.argtypes = [i32, _Fmt, C.c_double, C.c_double, p]
    L.co3_timing_enable.restype = i32
    L.co3_timing_enable.argtypes = [C.c_uint32]
    L.co3_timing_read.restype = i32
    L.co3_timing_read.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.co3_timing_reset.restype = i32
    L.co3_timing_reset.argtypes = []
    L.co3_kernel_name.restype = C.c_char_p
    L.co3_kernel_name.argtypes = [i32]
    return L


_lib = _load()


def _dp(t, dtype=None):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _chk(rc: int, where: str):
    if rc != OK:
        raise Co3Error(rc, where)


def _batch(t):
    """(U, n_or_stride) of a [U][stride] tensor (1-D tensors are one user)."""
    if t.dim() == 1:
        return 1, t.shape[0]
    if t.dim() != 2:
        raise ValueError("expected a 1-D or 2-D tensor")
    return t.shape[0], t.shape[1]


def strerror(code: int) -> str:
    return _lib.co3_strerror(code).decode()


def encode_workspace_bytes(n: int, U: int) -> int:
    return _lib.co3_encode_workspace_bytes(n, U)


def ps_aggregate_workspace_bytes(n: int, U: int, chunk_syms: int) -> int:
    return _lib.co3_ps_aggregate_workspace_bytes(n, U, chunk_syms)


def convert_encode_workspace_bytes(n: int, U: int, chunk_syms: int) -> int:
    return _lib.co3_convert_encode_workspace_bytes(n, U, chunk_syms)


def cap_words_empirical(n: int, fmt: Fmt) -> int:
    return _lib.co3_cap_words_empirical(n, fmt.c())


def poll_status(status, stream=None) -> int:
    return _lib.co3_poll_status(_dp(status, torch.int32), _stream(stream))


def convert_ef(g, err, sym, n, anchor, anchor_mode, gamma, fmt: Fmt, seg_off=None, counts=None, stream=None):
    U, stride = _batch(g)
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_convert_ef(_dp(g, torch.float32), _dp(err, torch.float32), _dp(sym, torch.uint8), n, U, stride,
                             _dp(seg_off, torch.int64), nseg, _dp(anchor, torch.int32), anchor_mode,
                             C.c_float(gamma), fmt.c(), _dp(counts, torch.int32), _stream(stream))
    _chk(rc, "co3_convert_ef")


def convert_encode(g, err, n, anchor, anchor_mode, gamma, fmt: Fmt, codes, words, chunk_syms, chunk_bitoff, total_bits,
                   workspace, status, seg_off=None, counts=None, stream=None):
    """counts: None, or [U][K] int32 out: 1 + occurrences of every symbol (weights of the next iteration's codes)."""
    U, stride = _batch(g)
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_convert_encode(_dp(g, torch.float32), _dp(err, torch.float32), n, U, stride,
                                 _dp(seg_off, torch.int64), nseg, _dp(anchor, torch.int32), anchor_mode,
                                 C.c_float(gamma), fmt.c(), _dp(codes, torch.uint8), _dp(counts, torch.int32),
                                 _dp(words, torch.int64),
                                 words.shape[-1], chunk_syms, _dp(chunk_bitoff, torch.int64), _dp(total_bits, torch.int64),
                                 _dp(workspace), workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                                 _stream(stream))
    _chk(rc, "co3_convert_encode")


def convert_encode_layers(g, err, n, anchor, anchor_mode, gamma, fmt: Fmt, codes, code_seg_off, words, chunk_syms,
                          chunk_bitoff, total_bits, workspace, status, seg_off=None, scale=None, counts=None, stream=None):
    """code_seg_off: boundaries of the codes; seg_off: boundaries of the anchors; scale: None or [U][nseg];
    counts: None or [ncodes][K] int32 out (1 + occurrences, users added up)."""
    U, stride = _batch(g)
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_convert_encode_layers(_dp(g, torch.float32), _dp(err, torch.float32), n, U, stride,
                                        _dp(seg_off, torch.int64), nseg, _dp(anchor, torch.int32), anchor_mode,
                                        _dp(scale, torch.float32), C.c_float(gamma), fmt.c(), _dp(codes, torch.uint8),
                                        _dp(code_seg_off, torch.int64), code_seg_off.numel() - 1,
                                        _dp(counts, torch.int32), _dp(words, torch.int64), words.shape[-1], chunk_syms,
                                        _dp(chunk_bitoff, torch.int64), _dp(total_bits, torch.int64), _dp(workspace),
                                        workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                                        _stream(stream))
    _chk(rc, "co3_convert_encode_layers")


def convert_ef_scaled(g, err, sym, n, anchor, scale, gamma, fmt: Fmt, seg_off=None, counts=None, stream=None):
    U, stride = _batch(g)
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_convert_ef_scaled(_dp(g, torch.float32), _dp(err, torch.float32), _dp(sym, torch.uint8), n, U,
                                    stride, _dp(seg_off, torch.int64), nseg, _dp(anchor, torch.int32),
                                    _dp(scale, torch.float32), C.c_float(gamma), fmt.c(), _dp(counts, torch.int32),
                                    _stream(stream))
    _chk(rc, "co3_convert_ef_scaled")


def moments(g, err, n, gamma, sums, seg_off=None, stream=None):
    U, stride = _batch(g)
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_moments(_dp(g, torch.float32), _dp(err, torch.float32), n, U, stride, _dp(seg_off, torch.int64),
                          nseg, C.c_float(gamma), _dp(sums, torch.float64), _stream(stream))
    _chk(rc, "co3_moments")


def bias_scale(sums, n, U, scale, fit=None, seg_off=None, stream=None):
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_bias_scale(_dp(sums, torch.float64), n, U, _dp(seg_off, torch.int64), nseg,
                             _dp(scale, torch.float32), _dp(fit, torch.float64), _stream(stream))
    _chk(rc, "co3_bias_scale")


def histogram(sym, n, fmt: Fmt, counts, stream=None):
    U, stride = _batch(sym)
    _chk(_lib.co3_histogram(_dp(sym, torch.uint8), n, U, stride, fmt.c(), _dp(counts, torch.int32), _stream(stream)),
         "co3_histogram")


def build_code(weights, U, fmt: Fmt, codes, status, stream=None):
    _chk(_lib.co3_build_code(_dp(weights, torch.int32), U, fmt.c(), _dp(codes, torch.uint8),
                             _dp(status, torch.int32), _stream(stream)), "co3_build_code")


def encode(sym, n, fmt: Fmt, codes, words, chunk_syms, chunk_bitoff, total_bits, workspace, status, stream=None):
    U, stride = _batch(sym)
    cap_words = words.shape[-1]
    rc = _lib.co3_encode(_dp(sym, torch.uint8), n, U, stride, fmt.c(), _dp(codes, torch.uint8),
                         _dp(words, torch.int64), cap_words, chunk_syms, _dp(chunk_bitoff, torch.int64),
                         _dp(total_bits, torch.int64), _dp(workspace), workspace.numel() * workspace.element_size(),
                         _dp(status, torch.int32), _stream(stream))
    _chk(rc, "co3_encode")


ENCODE_STATIC_WS_BYTES = 4 << 20


def user_encode_workspace_bytes(n: int, U: int, stride: int, nseg: int, caller_has_sym: bool) -> int:
    return _lib.co3_user_encode_workspace_bytes(n, U, stride, nseg, int(bool(caller_has_sym)))


def user_encode(g, err, n, anchor, gamma, fmt: Fmt, counts, codes, words, chunk_syms, chunk_bitoff, total_bits, workspace,
                status, sym=None, seg_off=None, stream=None):
    """The user's steps of one iteration in one call (co3_convert_ef with the anchor from max|g| and counts,
    co3_build_code, co3_encode); sym: None, or the [U][stride] uint8 array that receives the symbols."""
    U, stride = _batch(g)
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_user_encode(_dp(g, torch.float32), _dp(err, torch.float32), n, U, stride, _dp(seg_off, torch.int64),
                              nseg, _dp(anchor, torch.int32), C.c_float(gamma), fmt.c(), _dp(counts, torch.int32),
                              _dp(codes, torch.uint8), _dp(words, torch.int64), words.shape[-1], chunk_syms,
                              _dp(chunk_bitoff, torch.int64), _dp(total_bits, torch.int64), _dp(sym, torch.uint8),
                              _dp(workspace), workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                              _stream(stream))
    _chk(rc, "co3_user_encode")


def set_exchange_spin_limit(polls: int):
    _lib.co3_set_exchange_spin_limit(polls)


def encode_static(sym, n, fmt: Fmt, codes, words, chunk_syms, chunk_bitoff, total_bits, status, stream=None):
    """co3_encode with the library's own fixed workspace (no workspace argument, nothing allocated)."""
    U, stride = _batch(sym)
    rc = _lib.co3_encode_static(_dp(sym, torch.uint8), n, U, stride, fmt.c(), _dp(codes, torch.uint8),
                                _dp(words, torch.int64), words.shape[-1], chunk_syms, _dp(chunk_bitoff, torch.int64),
                                _dp(total_bits, torch.int64), _dp(status, torch.int32), _stream(stream))
    _chk(rc, "co3_encode_static")


def decode(words, chunk_bitoff, chunk_syms, codes, fmt: Fmt, n, sym_out, status, stream=None):
    U, stride = _batch(sym_out)
    rc = _lib.co3_decode(_dp(words, torch.int64), words.shape[-1], _dp(chunk_bitoff, torch.int64), chunk_syms,
                         _dp(codes, torch.uint8), fmt.c(), n, U, _dp(sym_out, torch.uint8), stride,
                         _dp(status, torch.int32), _stream(stream))
    _chk(rc, "co3_decode")


def ps_aggregate(words, chunk_bitoff, chunk_syms, codes, fmt: Fmt, n, U, anchor, avg_out, workspace, status,
                 seg_off=None, stream=None):
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_ps_aggregate(_dp(words, torch.int64), words.shape[-1], _dp(chunk_bitoff, torch.int64), chunk_syms,
                               _dp(codes, torch.uint8), fmt.c(), n, U, _dp(anchor, torch.int32),
                               _dp(seg_off, torch.int64), nseg, _dp(avg_out, torch.float32), _dp(workspace),
                               workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                               _stream(stream))
    _chk(rc, "co3_ps_aggregate")


def ps_aggregate_partial(words, chunk_bitoff, chunk_syms, codes, fmt: Fmt, n, U, anchor, acc_in, divide_by, out, workspace,
                         status, seg_off=None, stream=None):
    """co3_ps_aggregate over a group of users that continues the sum ``acc_in`` (None: zeros) and divides by
    ``divide_by`` (0: the sum is left undivided)."""
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_ps_aggregate_partial(_dp(words, torch.int64), words.shape[-1], _dp(chunk_bitoff, torch.int64),
                                       chunk_syms, _dp(codes, torch.uint8), fmt.c(), n, U, _dp(anchor, torch.int32),
                                       _dp(seg_off, torch.int64), nseg, _dp(acc_in, torch.float32), divide_by,
                                       _dp(out, torch.float32), _dp(workspace),
                                       workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                                       _stream(stream))
    _chk(rc, "co3_ps_aggregate_partial")


def ps_decode_users(words, chunk_bitoff, chunk_syms, codes, fmt: Fmt, n, U, first_user, U_total, workspace, status, stream=None):
    """Decompresses U users (tensors sliced to them) into their places of the averaging workspace of U_total users."""
    rc = _lib.co3_ps_decode_users(_dp(words, torch.int64), words.shape[-1], _dp(chunk_bitoff, torch.int64), chunk_syms,
                                  _dp(codes, torch.uint8), fmt.c(), n, U, first_user, U_total, _dp(workspace),
                                  workspace.numel() * workspace.element_size(), _dp(status, torch.int32), _stream(stream))
    _chk(rc, "co3_ps_decode_users")


def ps_average(workspace, chunk_syms, fmt: Fmt, n, U, anchor, avg_out, seg_off=None, stream=None):
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_ps_average(_dp(workspace), workspace.numel() * workspace.element_size(), chunk_syms, fmt.c(), n, U,
                             _dp(anchor, torch.int32), _dp(seg_off, torch.int64), nseg, _dp(avg_out, torch.float32),
                             _stream(stream))
    _chk(rc, "co3_ps_average")


def model_weights(A: int, fmt: Fmt, beta: float, alpha: float):
    """Host computation; returns a CPU int32 tensor holding the K uint32 weights bit-for-bit."""
    import numpy as np
    w = np.zeros(fmt.K, dtype=np.uint32)
    _chk(_lib.co3_model_weights(A, fmt.c(), beta, alpha, w.ctypes.data_as(C.c_void_p)), "co3_model_weights")
    return torch.from_numpy(w.view(np.int32).copy())


def design_layer_tables(fit, scale, seg_off, code_seg_off, A: int, fmt: Fmt):
    """Host computation on host copies of fit [U][nseg][2] f64 and scale [U][nseg] f32; returns a CPU int32
    tensor [ncodes][K] holding the uint32 weights bit for bit."""
    import numpy as np
    fit = np.ascontiguousarray(fit.detach().cpu().numpy(), dtype=np.float64)
    sc = np.ascontiguousarray(scale.detach().cpu().numpy(), dtype=np.float32)
    so = np.ascontiguousarray(np.asarray(seg_off, dtype=np.int64))
    cso = np.ascontiguousarray(np.asarray(code_seg_off, dtype=np.int64))
    U, nseg = sc.shape
    ncodes = cso.size - 1
    w = np.zeros((ncodes, fmt.K), dtype=np.uint32)
    vp = lambda a: a.ctypes.data_as(C.c_void_p)
    _chk(_lib.co3_design_layer_tables(vp(fit), vp(sc), U, nseg, vp(so), vp(cso), ncodes, A, fmt.c(), vp(w)),
         "co3_design_layer_tables")
    return torch.from_numpy(w.view(np.int32).copy())


def timing_enable(kernel_mask: int):
    _chk(_lib.co3_timing_enable(kernel_mask), "co3_timing_enable")


def timing_read(kernel: int):
    """(total milliseconds, launches) of one kernel id since the last reset."""
    ms, cnt = C.c_double(0), C.c_int64(0)
    _chk(_lib.co3_timing_read(kernel, C.byref(ms), C.byref(cnt)), "co3_timing_read")
    return ms.value, cnt.value


def timing_reset():
    _chk(_lib.co3_timing_reset(), "co3_timing_reset")


def kernel_name(kernel: int) -> str:
    return _lib.co3_kernel_name(kernel).decode()


def ps_aggregate_scaled(words, chunk_bitoff, chunk_syms, codes, fmt: Fmt, n, U, anchor, scale, avg_out, workspace,
                        status, seg_off=None, stream=None):
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_ps_aggregate_scaled(_dp(words, torch.int64), words.shape[-1], _dp(chunk_bitoff, torch.int64),
                                      chunk_syms, _dp(codes, torch.uint8), fmt.c(), n, U, _dp(anchor, torch.int32),
                                      _dp(scale, torch.float32), _dp(seg_off, torch.int64), nseg,
                                      _dp(avg_out, torch.float32), _dp(workspace),
                                      workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                                      _stream(stream))
    _chk(rc, "co3_ps_aggregate_scaled")


# ---- one code per tensor, shared by all users -------------------------------------------------
def histogram_layers(sym, n, fmt: Fmt, seg_off, counts, pool_users=False, stream=None):
    U, stride = _batch(sym)
    _chk(_lib.co3_histogram_layers(_dp(sym, torch.uint8), n, U, stride, _dp(seg_off, torch.int64),
                                   seg_off.numel() - 1, fmt.c(), int(bool(pool_users)), _dp(counts, torch.int32),
                                   _stream(stream)), "co3_histogram_layers")


def encode_layers(sym, n, fmt: Fmt, codes, seg_off, words, chunk_syms, chunk_bitoff, total_bits, workspace, status,
                  stream=None):
    U, stride = _batch(sym)
    rc = _lib.co3_encode_layers(_dp(sym, torch.uint8), n, U, stride, fmt.c(), _dp(codes, torch.uint8),
                                _dp(seg_off, torch.int64), seg_off.numel() - 1, _dp(words, torch.int64),
                                words.shape[-1], chunk_syms, _dp(chunk_bitoff, torch.int64),
                                _dp(total_bits, torch.int64), _dp(workspace),
                                workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                                _stream(stream))
    _chk(rc, "co3_encode_layers")


def decode_layers(words, chunk_bitoff, chunk_syms, codes, seg_off, fmt: Fmt, n, sym_out, status, stream=None):
    U, stride = _batch(sym_out)
    rc = _lib.co3_decode_layers(_dp(words, torch.int64), words.shape[-1], _dp(chunk_bitoff, torch.int64), chunk_syms,
                                _dp(codes, torch.uint8), _dp(seg_off, torch.int64), seg_off.numel() - 1, fmt.c(), n,
                                U, _dp(sym_out, torch.uint8), stride, _dp(status, torch.int32), _stream(stream))
    _chk(rc, "co3_decode_layers")


def ps_aggregate_layers(words, chunk_bitoff, chunk_syms, codes, code_seg_off, fmt: Fmt, n, U, anchor, avg_out,
                        workspace, status, seg_off=None, scale=None, stream=None):
    """code_seg_off: boundaries of the codes; seg_off: boundaries of the anchors (None: one anchor per user)."""
    nseg = 1 if seg_off is None else seg_off.numel() - 1
    rc = _lib.co3_ps_aggregate_layers(_dp(words, torch.int64), words.shape[-1], _dp(chunk_bitoff, torch.int64),
                                      chunk_syms, _dp(codes, torch.uint8), _dp(code_seg_off, torch.int64),
                                      code_seg_off.numel() - 1, fmt.c(), n, U, _dp(anchor, torch.int32),
                                      _dp(scale, torch.float32), _dp(seg_off, torch.int64), nseg,
                                      _dp(avg_out, torch.float32), _dp(workspace),
                                      workspace.numel() * workspace.element_size(), _dp(status, torch.int32),
                                      _stream(stream))
    _chk(rc, "co3_ps_aggregate_layers")
