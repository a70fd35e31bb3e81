"""FP64 CPU oracle for the local GEMM / forward-convolution kernels.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``; never by the product package.
The arithmetic lives in ``dmath_oracle.c`` (plain C, FP64 sums in the order of
the definitions); this module only marshals numpy arrays into it.

Every function takes FP32 arrays (the same bytes the GPU sees) and returns
``(ref, mag)`` as FP64 arrays: the reference value and the companion sum of
absolute values used by the bound ``|gpu-ref| <= 4*K*2^-24*mag + 1e-6``.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None

_i64 = ctypes.c_int64
_dbl = ctypes.c_double
_fp = ctypes.POINTER(ctypes.c_float)
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int64)
_hp = ctypes.POINTER(ctypes.c_uint16)


def _load():
    global _lib
    if _lib is None:
        # DMATH_ORACLE_SANITIZE=1: the ASan + UBSan build (the process must preload the sanitizer runtime)
        path = _build.build(force=False, sanitize=os.environ.get("DMATH_ORACLE_SANITIZE") == "1")
        lib = ctypes.CDLL(path)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_gemm.restype = ctypes.c_int
        lib.oracle_gemm.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _dbl, _fp, _i64,
                                    _fp, _i64, _dbl, _fp, _i64, _dp, _dp]
        lib.oracle_gemm_points.restype = ctypes.c_int
        lib.oracle_gemm_points.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _dbl, _fp,
                                           _i64, _fp, _i64, _dbl, _fp, _i64, _i64, _ip, _ip, _dp, _dp]
        lib.oracle_gemm_panels.restype = ctypes.c_int
        lib.oracle_gemm_panels.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _i64, _dbl,
                                           ctypes.POINTER(_fp), _i64, ctypes.POINTER(_fp), _i64, _dbl, _fp, _i64,
                                           _i64, _ip, _ip, _dp, _dp]
        lib.oracle_half_to_double.restype = _dbl
        lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_hgemm.restype = ctypes.c_int
        lib.oracle_hgemm.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _dbl, _hp, _i64, _hp, _i64, _dbl,
                                     _hp, _i64, _i64, _ip, _ip, _dp, _dp]
        lib.oracle_dgemm.restype = ctypes.c_int
        lib.oracle_dgemm.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _dbl, _dp, _i64, _dp, _i64, _dbl,
                                     _dp, _i64, _i64, _ip, _ip, _dp, _dp]
        lib.oracle_long_double_digits.restype = ctypes.c_int
        lib.oracle_conv2d_fwd.restype = ctypes.c_int
        lib.oracle_conv2d_fwd.argtypes = [_i64] * 11 + [_dbl, _fp, _fp, _dbl, _fp, _dp, _dp]
        lib.oracle_conv2d_fwd_points.restype = ctypes.c_int
        lib.oracle_conv2d_fwd_points.argtypes = [_i64] * 11 + [_dbl, _fp, _fp, _dbl, _fp, _i64, _ip,
                                                               _dp, _dp]
        lib.oracle_conv2d_bwd_data.restype = ctypes.c_int
        lib.oracle_conv2d_bwd_data.argtypes = [_i64] * 11 + [_dbl, _fp, _fp, _dbl, _fp, _i64, _ip, _dp, _dp]
        lib.oracle_conv2d_bwd_filter.restype = ctypes.c_int
        lib.oracle_conv2d_bwd_filter.argtypes = [_i64] * 11 + [_dbl, _fp, _fp, _dbl, _fp, _i64, _ip, _dp, _dp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f32(a, name):
    if a is None:
        return None
    if not isinstance(a, np.ndarray) or a.dtype != np.float32:
        raise TypeError("%s must be a float32 numpy array" % name)
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("%s must be C-contiguous (use the ld arguments for windows)" % name)
    return a


def _ptr(a):
    return a.ctypes.data_as(_fp) if a is not None else ctypes.cast(None, _fp)


def _need(a, count, name):
    """The flat buffer must hold every element the definition may touch."""
    if a is None:
        if count > 0:
            raise ValueError("%s is required" % name)
        return
    if a.size < count:
        raise ValueError("%s holds %d elements, the call reads %d" % (name, a.size, count))


def _extent(rows, cols, ld):
    return 0 if rows == 0 or cols == 0 else (rows - 1) * ld + cols


def _check_gemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc):
    A = _f32(A, "A")
    B = _f32(B, "B")
    C0 = _f32(C0, "C0")
    if alpha != 0.0:
        _need(A, _extent(K, M, lda) if transA else _extent(M, K, lda), "A")
        _need(B, _extent(N, K, ldb) if transB else _extent(K, N, ldb), "B")
    if beta != 0.0:
        _need(C0, _extent(M, N, ldc), "C0")
    return A, B, C0


def gemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta=0.0, C0=None, ldc=None):
    """ref, mag (M x N float64) of alpha*op(A)*op(B) + beta*C0, row-major with leading dims."""
    ldc = N if ldc is None else ldc
    A, B, C0 = _check_gemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc)
    ref = np.empty((M, N), dtype=np.float64)
    mag = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_gemm(int(bool(transA)), int(bool(transB)), M, N, K, float(alpha), _ptr(A), lda,
                             _ptr(B), ldb, float(beta), _ptr(C0), ldc,
                             ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_gemm rejected its arguments")
    return ref, mag


def gemm_points(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc, pi, pj):
    """Same sums at the output positions (pi[t], pj[t]) only."""
    A, B, C0 = _check_gemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc)
    pi = np.ascontiguousarray(pi, dtype=np.int64)
    pj = np.ascontiguousarray(pj, dtype=np.int64)
    assert pi.shape == pj.shape and pi.ndim == 1
    ref = np.empty(pi.shape, dtype=np.float64)
    mag = np.empty(pi.shape, dtype=np.float64)
    rc = _load().oracle_gemm_points(int(bool(transA)), int(bool(transB)), M, N, K, float(alpha), _ptr(A),
                                    lda, _ptr(B), ldb, float(beta), _ptr(C0), ldc, pi.size,
                                    pi.ctypes.data_as(_ip), pj.ctypes.data_as(_ip),
                                    ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_gemm_points rejected its arguments")
    return ref, mag


def gemm_panels(transA, transB, M, N, K, alpha, A_panels, lda, B_panels, ldb, beta=0.0, C0=None, ldc=None, pi=None,
                pj=None):
    """ref, mag of alpha * sum_p op(A_p)*op(B_p) + beta*C0 for lists of equally shaped panels; all M x N
    elements, or only the positions (pi[t], pj[t])."""
    ldc = N if ldc is None else ldc
    assert len(A_panels) == len(B_panels)
    keep = []
    for a, b in zip(A_panels, B_panels):
        a, b, _ = _check_gemm(transA, transB, M, N, K, alpha, a, lda, b, ldb, 0.0, None, ldc)
        keep.append((a, b))
    C0 = _f32(C0, "C0")
    if beta != 0.0:
        _need(C0, _extent(M, N, ldc), "C0")
    n = len(keep)
    fpp = ctypes.POINTER(ctypes.c_float) * max(1, n)
    Ap = fpp(*[_ptr(a) for a, _ in keep])
    Bp = fpp(*[_ptr(b) for _, b in keep])
    if pi is None:
        shape, npts = (M, N), 0
        ip = jp = ctypes.cast(None, _ip)
    else:
        pi = np.ascontiguousarray(pi, dtype=np.int64)
        pj = np.ascontiguousarray(pj, dtype=np.int64)
        assert pi.shape == pj.shape and pi.ndim == 1
        shape, npts = pi.shape, pi.size
        ip, jp = pi.ctypes.data_as(_ip), pj.ctypes.data_as(_ip)
    ref = np.empty(shape, dtype=np.float64)
    mag = np.empty(shape, dtype=np.float64)
    rc = _load().oracle_gemm_panels(int(bool(transA)), int(bool(transB)), M, N, K, n, float(alpha), Ap, lda, Bp, ldb,
                                    float(beta), _ptr(C0), ldc, npts, ip, jp,
                                    ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_gemm_panels rejected its arguments")
    return ref, mag


def half_to_double(bits):
    """Value of one IEEE binary16 bit pattern (0..65535) as the oracle decodes it."""
    return _load().oracle_half_to_double(int(bits))


def _f16(a, name):
    if a is None:
        return None
    a = np.asarray(a)
    if a.dtype != np.float16 or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("%s must be a C-contiguous float16 array" % name)
    return a


def _hptr(a):
    return ctypes.cast(None, _hp) if a is None else a.ctypes.data_as(_hp)


def half_bound(K, mag, ref):
    """Acceptance bound for a result stored as IEEE half: the FP32-accumulation bound plus one rounding of the
    result to half (half an ulp: 2^-11 relative for normal numbers, 2^-25 absolute in the subnormal range)."""
    return bound(K, mag) + np.maximum(np.abs(ref) * 2.0 ** -11, 2.0 ** -25)


def hgemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta=0.0, C0=None, ldc=None, pi=None, pj=None):
    """ref, mag (float64) of alpha*op(A)*op(B) + beta*C0 for float16 arrays; all elements or the points (pi, pj)."""
    ldc = N if ldc is None else ldc
    A, B, C0 = _f16(A, "A"), _f16(B, "B"), _f16(C0, "C0")
    if alpha != 0.0:
        _need(A, _extent(K, M, lda) if transA else _extent(M, K, lda), "A")
        _need(B, _extent(N, K, ldb) if transB else _extent(K, N, ldb), "B")
    if beta != 0.0:
        _need(C0, _extent(M, N, ldc), "C0")
    if pi is None:
        shape, npts = (M, N), 0
        ip = jp = ctypes.cast(None, _ip)
    else:
        pi = np.ascontiguousarray(pi, dtype=np.int64)
        pj = np.ascontiguousarray(pj, dtype=np.int64)
        assert pi.shape == pj.shape and pi.ndim == 1
        shape, npts = pi.shape, pi.size
        ip, jp = pi.ctypes.data_as(_ip), pj.ctypes.data_as(_ip)
    ref = np.empty(shape, dtype=np.float64)
    mag = np.empty(shape, dtype=np.float64)
    rc = _load().oracle_hgemm(int(bool(transA)), int(bool(transB)), M, N, K, float(alpha), _hptr(A), lda, _hptr(B),
                              ldb, float(beta), _hptr(C0), ldc, npts, ip, jp,
                              ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_hgemm rejected its arguments")
    return ref, mag


def _f64(a, name):
    if a is None:
        return None
    a = np.asarray(a)
    if a.dtype != np.float64 or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("%s must be a C-contiguous float64 array" % name)
    return a


def _dptr(a):
    return ctypes.cast(None, _dp) if a is None else a.ctypes.data_as(_dp)


def long_double_digits():
    """Significand bits of the type the FP64 oracle accumulates in (64 on x86-64)."""
    return _load().oracle_long_double_digits()


def double_bound(K, mag):
    """Acceptance bound for FP64 results: the FP32 contract with the FP64 unit roundoff,
    4*K*2^-53*mag + 2^-49."""
    return 4.0 * K * 2.0 ** -53 * mag + 2.0 ** -49


def dgemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta=0.0, C0=None, ldc=None, pi=None, pj=None):
    """ref, mag (float64, accumulated in long double) of alpha*op(A)*op(B) + beta*C0 for float64 arrays."""
    ldc = N if ldc is None else ldc
    A, B, C0 = _f64(A, "A"), _f64(B, "B"), _f64(C0, "C0")
    if alpha != 0.0:
        _need(A, _extent(K, M, lda) if transA else _extent(M, K, lda), "A")
        _need(B, _extent(N, K, ldb) if transB else _extent(K, N, ldb), "B")
    if beta != 0.0:
        _need(C0, _extent(M, N, ldc), "C0")
    if pi is None:
        shape, npts = (M, N), 0
        ip = jp = ctypes.cast(None, _ip)
    else:
        pi = np.ascontiguousarray(pi, dtype=np.int64)
        pj = np.ascontiguousarray(pj, dtype=np.int64)
        assert pi.shape == pj.shape and pi.ndim == 1
        shape, npts = pi.shape, pi.size
        ip, jp = pi.ctypes.data_as(_ip), pj.ctypes.data_as(_ip)
    ref = np.empty(shape, dtype=np.float64)
    mag = np.empty(shape, dtype=np.float64)
    rc = _load().oracle_dgemm(int(bool(transA)), int(bool(transB)), M, N, K, float(alpha), _dptr(A), lda, _dptr(B),
                              ldb, float(beta), _dptr(C0), ldc, npts, ip, jp,
                              ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_dgemm rejected its arguments")
    return ref, mag


def conv_out_shape(H, W, R, S, pad_h, pad_w, stride_h, stride_w):
    P = (H + 2 * pad_h - R) // stride_h + 1 if H + 2 * pad_h - R >= 0 else 0
    Q = (W + 2 * pad_w - S) // stride_w + 1 if W + 2 * pad_w - S >= 0 else 0
    return P, Q


def _check_conv(x, w, y0, N, C, H, W, Kout, R, S, P, Q, alpha, beta):
    x = _f32(x, "x")
    w = _f32(w, "w")
    y0 = _f32(y0, "y0")
    if alpha != 0.0:
        _need(x, N * C * H * W, "x")
        _need(w, Kout * C * R * S, "w")
    if beta != 0.0:
        _need(y0, N * Kout * P * Q, "y0")
    return x, w, y0


def conv2d_fwd(x, w, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, y0=None):
    """ref, mag (N x Kout x P x Q float64) of the direct forward convolution of x[N,C,H,W] with w[Kout,C,R,S]."""
    N, C, H, W = x.shape
    Kout, C2, R, S = w.shape
    assert C == C2
    P, Q = conv_out_shape(H, W, R, S, pad[0], pad[1], stride[0], stride[1])
    x, w, y0 = _check_conv(x, w, y0, N, C, H, W, Kout, R, S, P, Q, alpha, beta)
    ref = np.empty((N, Kout, P, Q), dtype=np.float64)
    mag = np.empty((N, Kout, P, Q), dtype=np.float64)
    rc = _load().oracle_conv2d_fwd(N, C, H, W, Kout, R, S, pad[0], pad[1], stride[0], stride[1],
                                   float(alpha), _ptr(x), _ptr(w), float(beta), _ptr(y0),
                                   ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_conv2d_fwd rejected its arguments")
    return ref, mag


def conv2d_fwd_points(x, w, idx, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, y0=None):
    """Same sums at the flat offsets idx into the N x Kout x P x Q output."""
    N, C, H, W = x.shape
    Kout, C2, R, S = w.shape
    assert C == C2
    P, Q = conv_out_shape(H, W, R, S, pad[0], pad[1], stride[0], stride[1])
    x, w, y0 = _check_conv(x, w, y0, N, C, H, W, Kout, R, S, P, Q, alpha, beta)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    ref = np.empty(idx.shape, dtype=np.float64)
    mag = np.empty(idx.shape, dtype=np.float64)
    rc = _load().oracle_conv2d_fwd_points(N, C, H, W, Kout, R, S, pad[0], pad[1], stride[0], stride[1],
                                          float(alpha), _ptr(x), _ptr(w), float(beta), _ptr(y0),
                                          idx.size, idx.ctypes.data_as(_ip),
                                          ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_conv2d_fwd_points rejected its arguments")
    return ref, mag


def conv2d_bwd_data(dy, w, x_shape, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, dx0=None, idx=None):
    """ref, mag of the gradient of the forward convolution with respect to x (shape x_shape = N, C, H, W),
    given dy[N,Kout,P,Q] and w[Kout,C,R,S]; all elements, or the flat offsets idx only."""
    N, C, H, W = x_shape
    Kout, C2, R, S = w.shape
    assert C == C2
    P, Q = conv_out_shape(H, W, R, S, pad[0], pad[1], stride[0], stride[1])
    assert dy.shape == (N, Kout, P, Q)
    dy = _f32(dy, "dy")
    w = _f32(w, "w")
    dx0 = _f32(dx0, "dx0")
    if beta != 0.0:
        _need(dx0, N * C * H * W, "dx0")
    if idx is None:
        shape, n, ip = (N, C, H, W), 0, ctypes.cast(None, _ip)
    else:
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        shape, n, ip = idx.shape, idx.size, idx.ctypes.data_as(_ip)
    ref = np.empty(shape, dtype=np.float64)
    mag = np.empty(shape, dtype=np.float64)
    rc = _load().oracle_conv2d_bwd_data(N, C, H, W, Kout, R, S, pad[0], pad[1], stride[0], stride[1], float(alpha),
                                        _ptr(dy), _ptr(w), float(beta), _ptr(dx0), n, ip,
                                        ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_conv2d_bwd_data rejected its arguments")
    return ref, mag


def conv2d_bwd_filter(x, dy, w_shape, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, dw0=None, idx=None):
    """ref, mag of the gradient of the forward convolution with respect to w (shape w_shape = Kout, C, R, S),
    given x[N,C,H,W] and dy[N,Kout,P,Q]; all elements, or the flat offsets idx only."""
    N, C, H, W = x.shape
    Kout, C2, R, S = w_shape
    assert C == C2
    P, Q = conv_out_shape(H, W, R, S, pad[0], pad[1], stride[0], stride[1])
    assert dy.shape == (N, Kout, P, Q)
    x = _f32(x, "x")
    dy = _f32(dy, "dy")
    dw0 = _f32(dw0, "dw0")
    if beta != 0.0:
        _need(dw0, Kout * C * R * S, "dw0")
    if idx is None:
        shape, n, ip = (Kout, C, R, S), 0, ctypes.cast(None, _ip)
    else:
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        shape, n, ip = idx.shape, idx.size, idx.ctypes.data_as(_ip)
    ref = np.empty(shape, dtype=np.float64)
    mag = np.empty(shape, dtype=np.float64)
    rc = _load().oracle_conv2d_bwd_filter(N, C, H, W, Kout, R, S, pad[0], pad[1], stride[0], stride[1], float(alpha),
                                          _ptr(x), _ptr(dy), float(beta), _ptr(dw0), n, ip,
                                          ref.ctypes.data_as(_dp), mag.ctypes.data_as(_dp))
    if rc != 0:
        raise RuntimeError("oracle_conv2d_bwd_filter rejected its arguments")
    return ref, mag


def bound(K, mag):
    """Acceptance bound on |gpu - ref| per element: 4*K*2^-24*mag + 1e-6."""
    return 4.0 * K * 2.0 ** -24 * mag + 1e-6
