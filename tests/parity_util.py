"""Shared helpers of the GPU parity tests: build stored operands, run the library through its
C ABI binding, run the FP64 oracle on the same bytes, and compare under the contract bound

    |gpu - ref| <= 4 * K * 2^-24 * mag + 1e-6      (mag = |alpha| |A||B| + |beta| |C0|)
"""
import numpy as np

import oracle

GUARD = np.float32(np.nan)


def stored(op_matrix, trans, ld_extra=0, lead=0, tail=8):
    """Flat FP32 buffer holding op_matrix (N) or its transpose (T) with row padding.

    Returns (flat, offset, ld): the matrix starts at flat[offset]; padding, lead and tail are NaN.
    """
    m = np.ascontiguousarray(op_matrix.T if trans else op_matrix, dtype=np.float32)
    rows, cols = m.shape
    ld = max(1, cols + ld_extra)
    flat = np.full(lead + rows * ld + tail, GUARD, dtype=np.float32)
    view = flat[lead:lead + rows * ld].reshape(rows, ld)
    view[:, :cols] = m
    return flat, lead, ld


def check_bound(gpu, ref, mag, K, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    err = np.abs(gpu - ref)
    bnd = oracle.bound(K, mag)
    bad = ~(err <= bnd)          # also catches NaN
    if bad.any():
        idx = np.argwhere(bad)[:5]
        raise AssertionError("%s: %d of %d elements outside the bound; first at %s, err %s, bound %s, gpu %s, ref %s"
                             % (what, int(bad.sum()), bad.size, idx.tolist(),
                                err[bad][:5], bnd[bad][:5], gpu[bad][:5], ref[bad][:5]))
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(bnd > 0, err / bnd, 0.0)
    return float(ratio.max()) if ratio.size else 0.0


def run_gemm_case(dm, torch, tA, tB, M, N, K, alpha=1.0, beta=0.0, ld_extra=(0, 0, 0), lead=(0, 0, 0),
                  seed=0, ints=False, c_nan=False, exact=False):
    """One dmath_gemm call against the oracle, with a NaN guard frame around every operand.

    ints: small-integer entries (every FP32 summation order is exact) -> with exact=True the GPU
    result must equal the oracle bit for bit.  c_nan: C starts as NaN (only legal with beta == 0).
    """
    rng = np.random.default_rng(seed)
    if ints:
        A = rng.integers(-4, 5, size=(M, K)).astype(np.float32)
        B = rng.integers(-4, 5, size=(K, N)).astype(np.float32)
        C0 = rng.integers(-4, 5, size=(M, N)).astype(np.float32)
    else:
        A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
        C0 = rng.standard_normal((M, N)).astype(np.float32)
    if c_nan:
        assert beta == 0.0
        C0[:] = np.nan
    a_flat, a_off, lda = stored(A, tA, ld_extra[0], lead[0])
    b_flat, b_off, ldb = stored(B, tB, ld_extra[1], lead[1])
    c_flat, c_off, ldc = stored(C0, 0, ld_extra[2], lead[2])
    dA = torch.from_numpy(a_flat).cuda()
    dB = torch.from_numpy(b_flat).cuda()
    dC = torch.from_numpy(c_flat).cuda()
    st = dm.dmath_gemm(tA, tB, M, N, K, alpha, dA[a_off:], lda, dB[b_off:], ldb, beta, dC[c_off:], ldc)
    assert st == dm.OK, (dm.dmath_status_string(st), dm.dmath_last_error_arg())
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    ref, mag = oracle.gemm(tA, tB, M, N, K, alpha, a_flat[a_off:], lda, b_flat[b_off:], ldb, beta,
                           c_flat[c_off:] if beta != 0.0 else None, ldc)
    got = out[c_off:c_off + M * ldc].reshape(M, ldc) if M > 0 else np.zeros((0, ldc), np.float32)
    # guard frame: everything that is not an element of C must still be NaN
    if M > 0:
        assert np.isnan(got[:, N:]).all(), "row padding of C was written"
    assert np.isnan(out[:c_off]).all() and np.isnan(out[c_off + M * ldc:]).all(), "wrote outside C"
    if M == 0 or N == 0:
        return 0.0
    if exact:
        assert np.array_equal(got[:, :N].astype(np.float64), ref), "integer case must be bit-exact"
        return 0.0
    return check_bound(got[:, :N], ref, mag, max(K, 1), "gemm t%d%d %dx%dx%d" % (tA, tB, M, N, K))


def stored_half(op_matrix, trans, ld_extra=0, lead=0, tail=8):
    """Like stored(), for float16 storage."""
    m = np.ascontiguousarray(op_matrix.T if trans else op_matrix, dtype=np.float16)
    rows, cols = m.shape
    ld = max(1, cols + ld_extra)
    flat = np.full(lead + rows * ld + tail, np.nan, dtype=np.float16)
    view = flat[lead:lead + rows * ld].reshape(rows, ld)
    view[:, :cols] = m
    return flat, lead, ld


def run_hgemm_case(dm, torch, tA, tB, M, N, K, alpha=1.0, beta=0.0, ld_extra=(0, 0, 0), lead=(0, 0, 0),
                   seed=0, ints=False, exact=False):
    """One dmath_hgemm call (half-precision storage, FP32 arithmetic) against the oracle."""
    rng = np.random.default_rng(seed)
    if ints:
        A = rng.integers(-2, 3, size=(M, K)).astype(np.float16)
        B = rng.integers(-2, 3, size=(K, N)).astype(np.float16)
        C0 = rng.integers(-4, 5, size=(M, N)).astype(np.float16)
    else:
        A = rng.uniform(-1, 1, (M, K)).astype(np.float16)
        B = rng.uniform(-1, 1, (K, N)).astype(np.float16)
        C0 = rng.standard_normal((M, N)).astype(np.float16)
    if beta == 0.0:
        C0[:] = np.nan
    a_flat, a_off, lda = stored_half(A, tA, ld_extra[0], lead[0])
    b_flat, b_off, ldb = stored_half(B, tB, ld_extra[1], lead[1])
    c_flat, c_off, ldc = stored_half(C0, 0, ld_extra[2], lead[2])
    dA, dB, dC = (torch.from_numpy(f).cuda() for f in (a_flat, b_flat, c_flat))
    st = dm.dmath_hgemm(tA, tB, M, N, K, alpha, dA[a_off:], lda, dB[b_off:], ldb, beta, dC[c_off:], ldc)
    assert st == dm.OK, (dm.dmath_status_string(st), dm.dmath_last_error_arg())
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    ref, mag = oracle.hgemm(tA, tB, M, N, K, alpha, a_flat[a_off:], lda, b_flat[b_off:], ldb, beta,
                            c_flat[c_off:] if beta != 0.0 else None, ldc)
    got = out[c_off:c_off + M * ldc].reshape(M, ldc) if M > 0 else np.zeros((0, ldc), np.float16)
    if M > 0:
        assert np.isnan(got[:, N:]).all(), "row padding of C was written"
    assert np.isnan(out[:c_off]).all() and np.isnan(out[c_off + M * ldc:]).all(), "wrote outside C"
    if M == 0 or N == 0:
        return 0.0
    g = got[:, :N].astype(np.float64)
    if exact:
        assert np.array_equal(g, ref), "integer case must be bit-exact"
        return 0.0
    err = np.abs(g - ref)
    bnd = oracle.half_bound(max(K, 1), mag, ref)
    bad = ~(err <= bnd)
    assert not bad.any(), "hgemm t%d%d %dx%dx%d: %d elements outside the bound, first %s err %s bound %s" % (
        tA, tB, M, N, K, int(bad.sum()), np.argwhere(bad)[:3].tolist(), err[bad][:3], bnd[bad][:3])
    return float((err / bnd).max())


def run_dgemm_case(dm, torch, tA, tB, M, N, K, alpha=1.0, beta=0.0, ld_extra=(0, 0, 0), lead=(0, 0, 0), seed=0,
                   ints=False, exact=False):
    """One dmath_dgemm call against the long-double oracle, NaN guard frames around every operand."""
    rng = np.random.default_rng(seed)
    if ints:
        A = rng.integers(-1000, 1001, size=(M, K)).astype(np.float64)
        B = rng.integers(-1000, 1001, size=(K, N)).astype(np.float64)
        C0 = rng.integers(-1000, 1001, size=(M, N)).astype(np.float64)
    else:
        A = rng.uniform(-1, 1, (M, K))
        B = rng.uniform(-1, 1, (K, N))
        C0 = rng.standard_normal((M, N))
    if beta == 0.0:
        C0[:] = np.nan

    def put(op_matrix, trans, extra, ld0):
        m = np.ascontiguousarray(op_matrix.T if trans else op_matrix)
        rows, cols = m.shape
        ld = max(1, cols + extra)
        flat = np.full(ld0 + rows * ld + 8, np.nan)
        flat[ld0:ld0 + rows * ld].reshape(rows, ld)[:, :cols] = m
        return flat, ld

    a_flat, lda = put(A, tA, ld_extra[0], lead[0])
    b_flat, ldb = put(B, tB, ld_extra[1], lead[1])
    c_flat, ldc = put(C0, 0, ld_extra[2], lead[2])
    dA, dB, dC = (torch.from_numpy(f).cuda() for f in (a_flat, b_flat, c_flat))
    st = dm.dmath_dgemm(tA, tB, M, N, K, alpha, dA[lead[0]:], lda, dB[lead[1]:], ldb, beta, dC[lead[2]:], ldc)
    assert st == dm.OK, (dm.dmath_status_string(st), dm.dmath_last_error_arg())
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    ref, mag = oracle.dgemm(tA, tB, M, N, K, alpha, a_flat[lead[0]:], lda, b_flat[lead[1]:], ldb, beta,
                            c_flat[lead[2]:] if beta != 0.0 else None, ldc)
    c_off = lead[2]
    got = out[c_off:c_off + M * ldc].reshape(M, ldc) if M > 0 else np.zeros((0, ldc))
    if M > 0:
        assert np.isnan(got[:, N:]).all(), "row padding of C was written"
    assert np.isnan(out[:c_off]).all() and np.isnan(out[c_off + M * ldc:]).all(), "wrote outside C"
    if M == 0 or N == 0:
        return 0.0
    g = got[:, :N]
    if exact:
        assert np.array_equal(g, ref), "integer case must be bit-exact"
        return 0.0
    err = np.abs(g - ref)
    bnd = oracle.double_bound(max(K, 1), mag)
    bad = ~(err <= bnd)
    assert not bad.any(), "dgemm t%d%d %dx%dx%d: %d elements outside the bound, first %s err %s bound %s" % (
        tA, tB, M, N, K, int(bad.sum()), np.argwhere(bad)[:3].tolist(), err[bad][:3], bnd[bad][:3])
    return float((err / bnd).max())


def run_gemm_panels_case(dm, torch, tA, tB, M, N, K, P, alpha=1.0, beta=0.0, ld_extra=(0, 0, 0), lead=(0, 0, 0),
                         seed=0, ints=False, exact=False):
    """One dmath_gemm_panels call over P panels against the oracle's sum of products."""
    rng = np.random.default_rng(seed)
    if ints:
        As = [rng.integers(-3, 4, size=(M, K)).astype(np.float32) for _ in range(P)]
        Bs = [rng.integers(-3, 4, size=(K, N)).astype(np.float32) for _ in range(P)]
        C0 = rng.integers(-4, 5, size=(M, N)).astype(np.float32)
    else:
        As = [rng.uniform(-1, 1, (M, K)).astype(np.float32) for _ in range(P)]
        Bs = [rng.uniform(-1, 1, (K, N)).astype(np.float32) for _ in range(P)]
        C0 = rng.standard_normal((M, N)).astype(np.float32)
    if beta == 0.0:
        C0[:] = np.nan
    sa = [stored(a, tA, ld_extra[0], lead[0]) for a in As]
    sb = [stored(b, tB, ld_extra[1], lead[1]) for b in Bs]
    c_flat, c_off, ldc = stored(C0, 0, ld_extra[2], lead[2])
    lda = sa[0][2] if P else max(1, (M if tA else K) + ld_extra[0])
    ldb = sb[0][2] if P else max(1, (K if tB else N) + ld_extra[1])
    dA = [torch.from_numpy(f).cuda() for f, _, _ in sa]
    dB = [torch.from_numpy(f).cuda() for f, _, _ in sb]
    dC = torch.from_numpy(c_flat).cuda()
    st = dm.dmath_gemm_panels(tA, tB, M, N, K, alpha, [t[lead[0]:] for t in dA], lda, [t[lead[1]:] for t in dB], ldb,
                              beta, dC[c_off:], ldc)
    assert st == dm.OK, (dm.dmath_status_string(st), dm.dmath_last_error_arg())
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    ref, mag = oracle.gemm_panels(tA, tB, M, N, K, alpha, [f[o:] for f, o, _ in sa], lda, [f[o:] for f, o, _ in sb],
                                  ldb, beta, c_flat[c_off:] if beta != 0.0 else None, ldc)
    got = out[c_off:c_off + M * ldc].reshape(M, ldc) if M > 0 else np.zeros((0, ldc), np.float32)
    if M > 0:
        assert np.isnan(got[:, N:]).all(), "row padding of C was written"
    assert np.isnan(out[:c_off]).all() and np.isnan(out[c_off + M * ldc:]).all(), "wrote outside C"
    if M == 0 or N == 0:
        return 0.0
    if exact:
        assert np.array_equal(got[:, :N].astype(np.float64), ref), "integer case must be bit-exact"
        return 0.0
    return check_bound(got[:, :N], ref, mag, max(K * P, 1), "gemm_panels t%d%d %dx%dx%d x%d" % (tA, tB, M, N, K, P))


def run_conv_case(dm, torch, N, C, H, W, Kout, R, S, pad, stride, alpha=1.0, beta=0.0, seed=0, ints=False,
                  exact=False, lead=0):
    rng = np.random.default_rng(seed)
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    if ints:
        x = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
        w = rng.integers(-3, 4, size=(Kout, C, R, S)).astype(np.float32)
        y0 = rng.integers(-3, 4, size=(N, Kout, P, Q)).astype(np.float32)
    else:
        x = np.maximum(rng.standard_normal((N, C, H, W)), 0).astype(np.float32)
        w = (rng.standard_normal((Kout, C, R, S)) * np.sqrt(2.0 / max(1, C * R * S))).astype(np.float32)
        y0 = rng.standard_normal((N, Kout, P, Q)).astype(np.float32)
    if beta == 0.0:
        y0[:] = np.nan
    tail = 8

    def flat_of(t):
        f = np.full(lead + t.size + tail, GUARD, dtype=np.float32)
        f[lead:lead + t.size] = t.reshape(-1)
        return f

    xf, wf, yf = flat_of(x), flat_of(w), flat_of(y0)
    dx, dw, dy = (torch.from_numpy(f).cuda() for f in (xf, wf, yf))
    st = dm.dmath_conv2d_fwd(N, C, H, W, Kout, R, S, pad[0], pad[1], stride[0], stride[1], alpha,
                             dx[lead:], dw[lead:], beta, dy[lead:])
    assert st == dm.OK, (dm.dmath_status_string(st), dm.dmath_last_error_arg())
    torch.cuda.synchronize()
    out = dy.cpu().numpy()
    assert np.isnan(out[:lead]).all() and np.isnan(out[lead + y0.size:]).all(), "wrote outside y"
    got = out[lead:lead + y0.size].reshape(y0.shape)
    ref, mag = oracle.conv2d_fwd(x, w, pad=pad, stride=stride, alpha=alpha, beta=beta,
                                 y0=y0 if beta != 0.0 else None)
    if got.size == 0:
        return 0.0
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), "integer case must be bit-exact"
        return 0.0
    return check_bound(got, ref, mag, max(1, C * R * S), "conv %s" % ((N, C, H, W, Kout, R, S, pad, stride),))


def run_conv_bwd_data_case(dm, torch, N, C, H, W, Kout, R, S, pad, stride, alpha=1.0, beta=0.0, seed=0, ints=False,
                           exact=False, lead=0):
    """dmath_conv2d_bwd_data against the oracle's adjoint-of-forward definition."""
    rng = np.random.default_rng(seed)
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    if ints:
        dy = rng.integers(-3, 4, size=(N, Kout, P, Q)).astype(np.float32)
        w = rng.integers(-3, 4, size=(Kout, C, R, S)).astype(np.float32)
        dx0 = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
    else:
        dy = (rng.standard_normal((N, Kout, P, Q)) * 0.1).astype(np.float32)
        w = (rng.standard_normal((Kout, C, R, S)) * np.sqrt(2.0 / max(1, C * R * S))).astype(np.float32)
        dx0 = rng.standard_normal((N, C, H, W)).astype(np.float32)
    if beta == 0.0:
        dx0[:] = np.nan
    tail = 8

    def flat_of(t):
        f = np.full(lead + t.size + tail, GUARD, dtype=np.float32)
        f[lead:lead + t.size] = t.reshape(-1)
        return f

    gf, wf, xf = flat_of(dy), flat_of(w), flat_of(dx0)
    dg, dw, dxd = (torch.from_numpy(f).cuda() for f in (gf, wf, xf))
    st = dm.dmath_conv2d_bwd_data(N, C, H, W, Kout, R, S, pad[0], pad[1], stride[0], stride[1], alpha,
                                  dg[lead:], dw[lead:], beta, dxd[lead:])
    assert st == dm.OK, (dm.dmath_status_string(st), dm.dmath_last_error_arg())
    torch.cuda.synchronize()
    out = dxd.cpu().numpy()
    assert np.isnan(out[:lead]).all() and np.isnan(out[lead + dx0.size:]).all(), "wrote outside dx"
    got = out[lead:lead + dx0.size].reshape(dx0.shape)
    ref, mag = oracle.conv2d_bwd_data(dy, w, (N, C, H, W), pad=pad, stride=stride, alpha=alpha, beta=beta,
                                      dx0=dx0 if beta != 0.0 else None)
    if got.size == 0:
        return 0.0
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), "integer case must be bit-exact"
        return 0.0
    return check_bound(got, ref, mag, max(1, Kout * R * S), "conv bwd-data %s" % ((N, C, H, W, Kout, R, S, pad, stride),))


def run_conv_bwd_filter_case(dm, torch, N, C, H, W, Kout, R, S, pad, stride, alpha=1.0, beta=0.0, seed=0, ints=False,
                             exact=False, lead=0):
    """dmath_conv2d_bwd_filter against the oracle's adjoint-of-forward definition."""
    rng = np.random.default_rng(seed)
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    if ints:
        x = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
        dy = rng.integers(-3, 4, size=(N, Kout, P, Q)).astype(np.float32)
        dw0 = rng.integers(-3, 4, size=(Kout, C, R, S)).astype(np.float32)
    else:
        x = rng.standard_normal((N, C, H, W)).astype(np.float32)
        dy = (rng.standard_normal((N, Kout, P, Q)) * 0.1).astype(np.float32)
        dw0 = rng.standard_normal((Kout, C, R, S)).astype(np.float32)
    if beta == 0.0:
        dw0[:] = np.nan
    tail = 8

    def flat_of(t):
        f = np.full(lead + t.size + tail, GUARD, dtype=np.float32)
        f[lead:lead + t.size] = t.reshape(-1)
        return f

    xf, gf, wf = flat_of(x), flat_of(dy), flat_of(dw0)
    dx, dg, dwd = (torch.from_numpy(f).cuda() for f in (xf, gf, wf))
    st = dm.dmath_conv2d_bwd_filter(N, C, H, W, Kout, R, S, pad[0], pad[1], stride[0], stride[1], alpha,
                                    dx[lead:], dg[lead:], beta, dwd[lead:])
    assert st == dm.OK, (dm.dmath_status_string(st), dm.dmath_last_error_arg())
    torch.cuda.synchronize()
    out = dwd.cpu().numpy()
    assert np.isnan(out[:lead]).all() and np.isnan(out[lead + dw0.size:]).all(), "wrote outside dw"
    got = out[lead:lead + dw0.size].reshape(dw0.shape)
    ref, mag = oracle.conv2d_bwd_filter(x, dy, (Kout, C, R, S), pad=pad, stride=stride, alpha=alpha, beta=beta,
                                        dw0=dw0 if beta != 0.0 else None)
    if got.size == 0:
        return 0.0
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), "integer case must be bit-exact"
        return 0.0
    return check_bound(got, ref, mag, max(1, N * P * Q), "conv bwd-filter %s" % ((N, C, H, W, Kout, R, S, pad, stride),))
