"""ctypes binding of libdmath.so: same names and argument order as include/dmath.h.

Argument marshalling only.  Matrix arguments may be torch tensors (their ``data_ptr()`` is
passed) or raw integer device addresses; ``stream`` may be a ``torch.cuda.Stream``, a raw
``hipStream_t`` integer, or None for torch's current stream.  Nothing here computes; if the
native library is missing the import fails instead of falling back to anything else.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdmath.so")

OK, ERR_INVALID_ARG, ERR_NULL_PTR, ERR_UNSUPPORTED, ERR_LAUNCH, ERR_WORKSPACE = range(6)
OP_N, OP_T = 0, 1

EXPORTS = (
    "dmath_gemm", "dmath_gemm_noalloc", "dmath_conv2d_fwd", "dmath_conv2d_bwd_data", "dmath_conv2d_bwd_filter", "dmath_gemm_panels", "dmath_hgemm", "dmath_set_hgemm_path", "dmath_hgemm_workspace_bytes", "dmath_dgemm", "dmath_set_dgemm_config", "dmath_dgemm_workspace_bytes", "dmath_gemm_workspace_bytes", "dmath_set_workspace",
    "dmath_set_override", "dmath_set_clock_probe", "dmath_gemm_plan", "dmath_num_configs", "dmath_config_name", "dmath_last_error_arg",
    "dmath_status_string", "dmath_version",
)

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "%s is not built; run `python -m paper_1604_01416_amd.build` (hipcc, gfx950)" % LIB_PATH)

_lib = ctypes.CDLL(LIB_PATH)

_i64, _f32, _vp, _int = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int

_lib.dmath_gemm.restype = _int
_lib.dmath_gemm.argtypes = [_int, _int, _i64, _i64, _i64, _f32, _vp, _i64, _vp, _i64, _f32, _vp, _i64, _vp]
_lib.dmath_gemm_noalloc.restype = _int
_lib.dmath_gemm_noalloc.argtypes = list(_lib.dmath_gemm.argtypes)
_lib.dmath_conv2d_fwd.restype = _int
_lib.dmath_conv2d_fwd.argtypes = [_i64] * 11 + [_f32, _vp, _vp, _f32, _vp, _vp]
_lib.dmath_conv2d_bwd_data.restype = _int
_lib.dmath_conv2d_bwd_data.argtypes = [_i64] * 11 + [_f32, _vp, _vp, _f32, _vp, _vp]
_lib.dmath_hgemm.restype = _int
_lib.dmath_hgemm.argtypes = [_int, _int, _i64, _i64, _i64, _f32, _vp, _i64, _vp, _i64, _f32, _vp, _i64, _vp]
_lib.dmath_dgemm.restype = _int
_lib.dmath_dgemm.argtypes = [_int, _int, _i64, _i64, _i64, ctypes.c_double, _vp, _i64, _vp, _i64, ctypes.c_double, _vp,
                             _i64, _vp]
_lib.dmath_set_dgemm_config.restype = _int
_lib.dmath_set_dgemm_config.argtypes = [_int]
_lib.dmath_hgemm_workspace_bytes.restype = ctypes.c_size_t
_lib.dmath_hgemm_workspace_bytes.argtypes = [_int, _int, _i64, _i64, _i64]
_lib.dmath_dgemm_workspace_bytes.restype = ctypes.c_size_t
_lib.dmath_dgemm_workspace_bytes.argtypes = [_int, _int, _i64, _i64, _i64]
_lib.dmath_set_hgemm_path.restype = _int
_lib.dmath_set_hgemm_path.argtypes = [_int]
_lib.dmath_gemm_panels.restype = _int
_lib.dmath_gemm_panels.argtypes = [_int, _int, _i64, _i64, _i64, _i64, _f32, ctypes.POINTER(_vp), _i64,
                                   ctypes.POINTER(_vp), _i64, _f32, _vp, _i64, _vp]
_lib.dmath_conv2d_bwd_filter.restype = _int
_lib.dmath_conv2d_bwd_filter.argtypes = [_i64] * 11 + [_f32, _vp, _vp, _f32, _vp, _vp]
_lib.dmath_gemm_workspace_bytes.restype = ctypes.c_size_t
_lib.dmath_gemm_workspace_bytes.argtypes = [_int, _int, _i64, _i64, _i64]
_lib.dmath_set_workspace.restype = _int
_lib.dmath_set_workspace.argtypes = [_vp, ctypes.c_size_t]
_lib.dmath_set_override.restype = _int
_lib.dmath_set_override.argtypes = [_int, _int]
_lib.dmath_set_clock_probe.restype = _int
_lib.dmath_set_clock_probe.argtypes = [_vp]
_lib.dmath_gemm_plan.restype = _int
_lib.dmath_gemm_plan.argtypes = [_int, _int, _i64, _i64, _i64, ctypes.POINTER(_int), ctypes.POINTER(_int)]
_lib.dmath_num_configs.restype = _int
_lib.dmath_config_name.restype = ctypes.c_char_p
_lib.dmath_config_name.argtypes = [_int]
_lib.dmath_last_error_arg.restype = _int
_lib.dmath_status_string.restype = ctypes.c_char_p
_lib.dmath_status_string.argtypes = [_int]
_lib.dmath_version.restype = ctypes.c_char_p


def _addr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def dmath_gemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None):
    return _lib.dmath_gemm(transA, transB, M, N, K, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C), ldc,
                           _stream(stream))


NOALLOC_SCRATCH_BYTES = 32 << 20   # DMATH_NOALLOC_SCRATCH_BYTES of include/dmath.h


def dmath_gemm_noalloc(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None):
    return _lib.dmath_gemm_noalloc(transA, transB, M, N, K, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C), ldc,
                                   _stream(stream))


def dmath_conv2d_fwd(N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, x, w, beta, y,
                     stream=None):
    return _lib.dmath_conv2d_fwd(N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, _addr(x),
                                 _addr(w), beta, _addr(y), _stream(stream))


def dmath_conv2d_bwd_data(N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, dy, w, beta, dx,
                          stream=None):
    return _lib.dmath_conv2d_bwd_data(N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, _addr(dy),
                                      _addr(w), beta, _addr(dx), _stream(stream))


def dmath_hgemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None):
    """A, B, C: float16 device tensors (or addresses of binary16 data)."""
    return _lib.dmath_hgemm(transA, transB, M, N, K, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C), ldc,
                            _stream(stream))


def dmath_dgemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None):
    """A, B, C: float64 device tensors."""
    return _lib.dmath_dgemm(transA, transB, M, N, K, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C), ldc,
                            _stream(stream))


def dmath_set_dgemm_config(tile_config):
    return _lib.dmath_set_dgemm_config(tile_config)


def dmath_hgemm_workspace_bytes(transA, transB, M, N, K):
    return _lib.dmath_hgemm_workspace_bytes(transA, transB, M, N, K)


def dmath_dgemm_workspace_bytes(transA, transB, M, N, K):
    return _lib.dmath_dgemm_workspace_bytes(transA, transB, M, N, K)


def dmath_set_hgemm_path(path):
    return _lib.dmath_set_hgemm_path(path)


def dmath_gemm_panels(transA, transB, M, N, K, alpha, A_panels, lda, B_panels, ldb, beta, C, ldc, stream=None):
    """A_panels, B_panels: equally long sequences of device tensors / addresses (or None for a NULL table)."""
    def table(panels):
        if panels is None:
            return None, 0
        arr = (_vp * max(1, len(panels)))(*[_addr(p) for p in panels])
        return arr, len(panels)
    ta, na = table(A_panels)
    tb, nb = table(B_panels)
    if A_panels is not None and B_panels is not None and na != nb:
        raise ValueError("A_panels and B_panels differ in length")
    return _lib.dmath_gemm_panels(transA, transB, M, N, K, max(na, nb), alpha, ta, lda, tb, ldb, beta, _addr(C), ldc,
                                  _stream(stream))


def dmath_conv2d_bwd_filter(N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, x, dy, beta, dw,
                            stream=None):
    return _lib.dmath_conv2d_bwd_filter(N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, _addr(x),
                                        _addr(dy), beta, _addr(dw), _stream(stream))


def dmath_gemm_workspace_bytes(transA, transB, M, N, K):
    return int(_lib.dmath_gemm_workspace_bytes(transA, transB, M, N, K))


def dmath_set_workspace(device_ptr, nbytes):
    return _lib.dmath_set_workspace(_addr(device_ptr), nbytes)


def dmath_set_override(tile_config, split_k):
    return _lib.dmath_set_override(tile_config, split_k)


def dmath_set_clock_probe(device_ptr):
    return _lib.dmath_set_clock_probe(_addr(device_ptr))


def dmath_gemm_plan(transA, transB, M, N, K):
    """Returns (status, tile_config, split_k)."""
    cfg, split = _int(0), _int(0)
    st = _lib.dmath_gemm_plan(transA, transB, M, N, K, ctypes.byref(cfg), ctypes.byref(split))
    return st, cfg.value, split.value


def dmath_num_configs():
    return int(_lib.dmath_num_configs())


def dmath_config_name(tile_config):
    s = _lib.dmath_config_name(tile_config)
    return s.decode() if s is not None else None


def dmath_last_error_arg():
    return int(_lib.dmath_last_error_arg())


def dmath_status_string(status):
    return _lib.dmath_status_string(status).decode()


def dmath_version():
    return _lib.dmath_version().decode()


def check(status):
    """Raise if a call did not return DMATH_OK."""
    if status != OK:
        raise RuntimeError("dmath: %s (argument %d)" % (dmath_status_string(status), dmath_last_error_arg()))
