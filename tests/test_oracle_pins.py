"""Pins for the FP64 CPU oracle: none of the expected values below comes from the oracle.

Each test fixes the oracle against something the mathematics fixes: hand-worked
fixtures, exact integer arithmetic, identity / permutation / rank-1 / all-ones
closed forms, transposition identities, padding and NaN conventions, linearity,
the chain invariant of the stage-by-stage block update (dMath paper, section
"Matrix Multiplication"), delta filters, tap counts, brute force written a
second time in Python, and the float64 library routines of numpy / torch.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_fixture(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


def _store(op_matrix, trans, ld_extra=0, fill=np.nan):
    """Store op(X) the way the API expects it: X itself (N) or X^T (T), with padded rows."""
    m = op_matrix.T if trans else op_matrix
    rows, cols = m.shape
    ld = cols + ld_extra
    buf = np.full((rows, ld), fill, dtype=np.float32)
    buf[:, :cols] = m
    return np.ascontiguousarray(buf), ld


# ----------------------------------------------------------------------------- GEMM

def test_gemm_hand_worked_fixture_all_transposes():
    fx = _read_fixture("gemm_hand_worked.txt")
    M, N, K = int(fx["M"][0]), int(fx["N"][0]), int(fx["K"][0])
    A = np.array(fx["A"], dtype=np.float32).reshape(M, K)
    B = np.array(fx["B"], dtype=np.float32).reshape(K, N)
    C0 = np.array(fx["C0"], dtype=np.float32).reshape(M, N)
    want = np.array(fx["ref"]).reshape(M, N)
    want_mag = np.array(fx["mag"]).reshape(M, N)
    for tA, tB in itertools.product((0, 1), (0, 1)):
        a, lda = _store(A, tA)
        b, ldb = _store(B, tB)
        ref, mag = oracle.gemm(tA, tB, M, N, K, fx["alpha"][0], a, lda, b, ldb, fx["beta"][0], C0, N)
        assert np.array_equal(ref, want), (tA, tB)
        assert np.array_equal(mag, want_mag), (tA, tB)


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (17, 33, 64), (64, 31, 256)])
def test_gemm_integer_exact(tA, tB, M, N, K):
    rng = np.random.default_rng(100 + M + 7 * N + 13 * K + 2 * tA + tB)
    Ai = rng.integers(-8, 9, size=(M, K))
    Bi = rng.integers(-8, 9, size=(K, N))
    Ci = rng.integers(-8, 9, size=(M, N))
    alpha, beta = 3, -2
    want = alpha * (Ai.astype(np.int64) @ Bi.astype(np.int64)) + beta * Ci
    want_mag = abs(alpha) * (np.abs(Ai) @ np.abs(Bi)) + abs(beta) * np.abs(Ci)
    a, lda = _store(Ai.astype(np.float32), tA, ld_extra=3)
    b, ldb = _store(Bi.astype(np.float32), tB, ld_extra=2)
    c, ldc = _store(Ci.astype(np.float32), 0, ld_extra=5)
    ref, mag = oracle.gemm(tA, tB, M, N, K, alpha, a, lda, b, ldb, beta, c, ldc)
    assert np.array_equal(ref, want.astype(np.float64))
    assert np.array_equal(mag, want_mag.astype(np.float64))
    # the point-wise routine gives the same numbers
    pi, pj = np.divmod(np.arange(M * N), N)
    rp, mp = oracle.gemm_points(tA, tB, M, N, K, alpha, a, lda, b, ldb, beta, c, ldc, pi, pj)
    assert np.array_equal(rp.reshape(M, N), ref)
    assert np.array_equal(mp.reshape(M, N), mag)


def test_gemm_identity_and_permutation():
    rng = np.random.default_rng(1)
    n, m = 9, 6
    B = rng.standard_normal((n, m)).astype(np.float32)
    C0 = rng.standard_normal((n, m)).astype(np.float32)
    eye = np.eye(n, dtype=np.float32)
    ref, _ = oracle.gemm(0, 0, n, m, n, 0.5, eye, n, B, m, 2.0, C0, m)
    assert np.array_equal(ref, 0.5 * B.astype(np.float64) + 2.0 * C0.astype(np.float64))
    A = rng.standard_normal((m, n)).astype(np.float32)
    ref, _ = oracle.gemm(0, 0, m, n, n, 1.0, A, n, eye, n, 0.0, None, n)
    assert np.array_equal(ref, A.astype(np.float64))
    perm = rng.permutation(n)
    Pm = np.zeros((n, n), dtype=np.float32)
    Pm[np.arange(n), perm] = 1.0          # row i of P*B is row perm[i] of B
    ref, _ = oracle.gemm(0, 0, n, m, n, 1.0, Pm, n, B, m, 0.0, None, m)
    assert np.array_equal(ref, B[perm].astype(np.float64))
    ref, _ = oracle.gemm(0, 0, m, n, n, 1.0, A, n, Pm, n, 0.0, None, n)
    want = np.zeros((m, n))
    want[:, perm] = A                      # column perm[i] of A*P is column i of A
    assert np.array_equal(ref, want)
    # a transposed permutation is its inverse: catches a swapped transpose flag
    ref, _ = oracle.gemm(1, 0, n, m, n, 1.0, Pm, n, B, m, 0.0, None, m)
    want = np.zeros((n, m))
    want[perm] = B
    assert np.array_equal(ref, want)


def test_gemm_rank1_and_all_ones():
    u = np.array([1, -2, 4, 0.5, 8], dtype=np.float32)
    z = np.array([2, 0.25, -1, 16], dtype=np.float32)
    ref, mag = oracle.gemm(0, 0, 5, 4, 1, 1.0, u.reshape(5, 1).copy(), 1, z.reshape(1, 4).copy(), 4)
    assert np.array_equal(ref, np.outer(u, z).astype(np.float64))
    assert np.array_equal(mag, np.abs(np.outer(u, z)).astype(np.float64))
    K = 37
    A = np.repeat(u.reshape(5, 1), K, axis=1).copy()      # u * 1^T
    B = np.repeat(z.reshape(1, 4), K, axis=0).copy()      # 1 * z^T
    ref, _ = oracle.gemm(0, 0, 5, 4, K, 1.0, A, K, B, 4)
    assert np.array_equal(ref, K * np.outer(u, z).astype(np.float64))
    rng = np.random.default_rng(5)
    Bi = rng.integers(-5, 6, size=(K, 4)).astype(np.float32)
    ones = np.ones((3, K), dtype=np.float32)
    ref, _ = oracle.gemm(0, 0, 3, 4, K, 1.0, ones, K, Bi, 4)
    assert np.array_equal(ref, np.tile(Bi.sum(axis=0, dtype=np.float64), (3, 1)))


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_gemm_transposition_identities(tA, tB):
    rng = np.random.default_rng(7)
    M, N, K = 13, 11, 29
    A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    base, base_mag = oracle.gemm(0, 0, M, N, K, 1.0, A, K, B, N)
    a, lda = _store(A, tA, ld_extra=4)
    b, ldb = _store(B, tB, ld_extra=1)
    ref, mag = oracle.gemm(tA, tB, M, N, K, 1.0, a, lda, b, ldb)
    assert np.array_equal(ref, base)      # same products, same k order: identical bits
    assert np.array_equal(mag, base_mag)
    # C^T = B^T A^T: op(B)^T stored as given, roles swapped
    refT, _ = oracle.gemm(1 - tB, 1 - tA, N, M, K, 1.0, b, ldb, a, lda)
    assert np.array_equal(refT, base.T)


def test_gemm_padding_is_never_read_and_nan_conventions():
    rng = np.random.default_rng(11)
    M, N, K = 7, 5, 9
    A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    C0 = rng.uniform(-1, 1, (M, N)).astype(np.float32)
    tight, _ = oracle.gemm(0, 0, M, N, K, 1.5, A, K, B, N, 0.5, C0, N)
    a, lda = _store(A, 0, ld_extra=6)        # padding is NaN
    b, ldb = _store(B, 0, ld_extra=2)
    c, ldc = _store(C0, 0, ld_extra=3)
    ref, mag = oracle.gemm(0, 0, M, N, K, 1.5, a, lda, b, ldb, 0.5, c, ldc)
    assert np.array_equal(ref, tight) and np.isfinite(mag).all()
    # beta == 0: C0 full of NaN must not show up
    nanC = np.full((M, N), np.nan, dtype=np.float32)
    ref0, _ = oracle.gemm(0, 0, M, N, K, 1.0, A, K, B, N, 0.0, nanC, N)
    assert np.isfinite(ref0).all()
    assert np.allclose(ref0, A.astype(np.float64) @ B.astype(np.float64), rtol=1e-14, atol=0)
    # alpha == 0: A, B full of NaN must not show up, result is beta*C0
    nanA = np.full((M, K), np.nan, dtype=np.float32)
    ref1, mag1 = oracle.gemm(0, 0, M, N, K, 0.0, nanA, K, nanA[:K, :N].copy(), N, -2.0, C0, N)
    assert np.array_equal(ref1, -2.0 * C0.astype(np.float64))
    assert np.array_equal(mag1, 2.0 * np.abs(C0.astype(np.float64)))
    # K == 0
    ref2, _ = oracle.gemm(0, 0, M, N, 0, 1.0, A, K, B, N, 3.0, C0, N)
    assert np.array_equal(ref2, 3.0 * C0.astype(np.float64))
    # empty outputs
    r, m = oracle.gemm(0, 0, 0, N, K, 1.0, A, K, B, N)
    assert r.shape == (0, N)


def test_gemm_linearity_power_of_two_alpha():
    rng = np.random.default_rng(13)
    M, N, K = 8, 6, 50
    A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    r1, _ = oracle.gemm(0, 0, M, N, K, 1.0, A, K, B, N)
    r4, _ = oracle.gemm(0, 0, M, N, K, 4.0, A, K, B, N)
    rA, _ = oracle.gemm(0, 0, M, N, K, 1.0, (4 * A).astype(np.float32), K, B, N)
    assert np.array_equal(r4, 4.0 * r1)
    assert np.array_equal(rA, 4.0 * r1)


def test_gemm_matches_brute_force_python_and_numpy():
    rng = np.random.default_rng(17)
    M, N, K = 4, 3, 6
    alpha, beta = 0.75, -1.25
    for tA, tB in itertools.product((0, 1), (0, 1)):
        A = rng.standard_normal((M, K)).astype(np.float32)
        B = rng.standard_normal((K, N)).astype(np.float32)
        C0 = rng.standard_normal((M, N)).astype(np.float32)
        a, lda = _store(A, tA, ld_extra=2)
        b, ldb = _store(B, tB, ld_extra=1)
        ref, mag = oracle.gemm(tA, tB, M, N, K, alpha, a, lda, b, ldb, beta, C0, N)
        for i in range(M):
            for j in range(N):
                s = 0.0
                t = 0.0
                for k in range(K):
                    av = float(a[k, i]) if tA else float(a[i, k])
                    bv = float(b[j, k]) if tB else float(b[k, j])
                    s += av * bv
                    t += abs(av) * abs(bv)
                assert ref[i, j] == alpha * s + beta * float(C0[i, j])
                assert mag[i, j] == abs(alpha) * t + abs(beta) * abs(float(C0[i, j]))
    M, N, K = 40, 50, 300
    A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    ref, _ = oracle.gemm(0, 0, M, N, K, 1.0, A, K, B, N)
    lib = np.matmul(A.astype(np.float64), B.astype(np.float64))
    assert np.max(np.abs(ref - lib)) <= 1e-12 * np.max(np.abs(lib))


def test_chain_of_accumulate_steps_equals_one_product():
    """Summing the per-stage local updates equals the one-shot product (section "Matrix Multiplication")."""
    rng = np.random.default_rng(19)
    m, kp, steps = 24, 8, 16
    C0 = rng.standard_normal((m, m)).astype(np.float32)
    As = [rng.uniform(-1, 1, (m, kp)).astype(np.float32) for _ in range(steps)]
    Bs = [rng.uniform(-1, 1, (kp, m)).astype(np.float32) for _ in range(steps)]
    Acat = np.ascontiguousarray(np.concatenate(As, axis=1))
    Bcat = np.ascontiguousarray(np.concatenate(Bs, axis=0))
    one, one_mag = oracle.gemm(0, 0, m, m, kp * steps, 1.0, Acat, kp * steps, Bcat, m, 1.0, C0, m)
    acc = C0.astype(np.float64)
    acc_mag = np.abs(acc)
    for a, b in zip(As, Bs):
        step, step_mag = oracle.gemm(0, 0, m, m, kp, 1.0, a, kp, b, m)
        acc = acc + step
        acc_mag = acc_mag + step_mag
    assert np.max(np.abs(acc - one)) <= 1e-9 * np.max(np.abs(one))
    assert np.max(np.abs(acc_mag - one_mag)) <= 1e-9 * np.max(np.abs(one_mag))


def test_gemm_points_on_a_window_with_leading_dimensions():
    rng = np.random.default_rng(23)
    big = rng.integers(-4, 5, size=(20, 30)).astype(np.float32)
    # A = big[2:9, 3:14] (7 x 11), B = big[5:16, 10:16] (11 x 6), both windows of one buffer
    A = big.reshape(-1)[2 * 30 + 3:]
    B = big.reshape(-1)[5 * 30 + 10:]
    want = big[2:9, 3:14].astype(np.int64) @ big[5:16, 10:16].astype(np.int64)
    ref, _ = oracle.gemm(0, 0, 7, 6, 11, 1.0, np.ascontiguousarray(A), 30, np.ascontiguousarray(B), 30)
    assert np.array_equal(ref, want.astype(np.float64))


# ----------------------------------------------------------------------------- convolution

# ----------------------------------------------------------------------------- multi-panel update

def test_gemm_panels_hand_worked_fixture_all_transposes():
    fx = _read_fixture("gemm_panels_hand_worked.txt")
    M, N, K, P = (int(fx[k][0]) for k in ("M", "N", "K", "panels"))
    C0 = np.array(fx["C0"], dtype=np.float32).reshape(M, N)
    want = np.array(fx["ref"]).reshape(M, N)
    want_mag = np.array(fx["mag"]).reshape(M, N)
    for tA, tB in itertools.product((0, 1), (0, 1)):
        As, Bs = [], []
        for p in range(P):
            a, lda = _store(np.array(fx["A%d" % p], dtype=np.float32).reshape(M, K), tA, ld_extra=1)
            b, ldb = _store(np.array(fx["B%d" % p], dtype=np.float32).reshape(K, N), tB, ld_extra=2)
            As.append(a)
            Bs.append(b)
        ref, mag = oracle.gemm_panels(tA, tB, M, N, K, fx["alpha"][0], As, lda, Bs, ldb, fx["beta"][0], C0, N)
        assert np.array_equal(ref, want), (tA, tB)
        assert np.array_equal(mag, want_mag), (tA, tB)
        pts, _ = oracle.gemm_panels(tA, tB, M, N, K, fx["alpha"][0], As, lda, Bs, ldb, fx["beta"][0], C0, N,
                                    pi=[1, 0], pj=[0, 1])
        assert np.array_equal(pts, want[[1, 0], [0, 1]])


def test_gemm_panels_closed_forms():
    # panel p holds A_p = (p+1) everywhere, B_p = 1: every element is K * sum_p (p+1); a dropped or repeated
    # panel, or a panel used twice, changes the count
    M, N, K, P = 3, 4, 5, 6
    As = [np.full((M, K), p + 1, dtype=np.float32) for p in range(P)]
    Bs = [np.ones((K, N), dtype=np.float32) for _ in range(P)]
    ref, mag = oracle.gemm_panels(0, 0, M, N, K, 1.0, As, K, Bs, N)
    assert np.array_equal(ref, np.full((M, N), K * P * (P + 1) / 2))
    assert np.array_equal(mag, ref)
    # A_p = e_p e_p^T pattern: panel p contributes only to C[p][p] (pairs A_p with B_p, not B_q)
    P = 4
    As, Bs = [], []
    for p in range(P):
        a = np.zeros((P, 2), dtype=np.float32)
        a[p, 1] = 1.0
        b = np.zeros((2, P), dtype=np.float32)
        b[1, p] = float(p + 2)
        As.append(a)
        Bs.append(b)
    ref, _ = oracle.gemm_panels(0, 0, P, P, 2, 1.0, As, 2, Bs, P)
    assert np.array_equal(ref, np.diag(np.arange(P) + 2.0))
    # no panels, or K == 0: beta * C0 alone; alpha == 0 never reads the panels
    C0 = np.arange(12, dtype=np.float32).reshape(3, 4)
    ref, mag = oracle.gemm_panels(0, 0, 3, 4, 5, 2.0, [], 5, [], 4, beta=-1.0, C0=C0)
    assert np.array_equal(ref, -C0.astype(np.float64)) and np.array_equal(mag, C0.astype(np.float64))
    nanA = [np.full((3, 5), np.nan, dtype=np.float32)]
    nanB = [np.full((5, 4), np.nan, dtype=np.float32)]
    ref, _ = oracle.gemm_panels(0, 0, 3, 4, 5, 0.0, nanA, 5, nanB, 4, beta=1.0, C0=C0)
    assert np.array_equal(ref, C0.astype(np.float64))


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_gemm_panels_matches_numpy_float64_and_brute_force(tA, tB):
    rng = np.random.default_rng(100 + 2 * tA + tB)
    M, N, K, P = 6, 5, 7, 3
    A = [rng.standard_normal((M, K)).astype(np.float32) for _ in range(P)]
    B = [rng.standard_normal((K, N)).astype(np.float32) for _ in range(P)]
    C0 = rng.standard_normal((M, N)).astype(np.float32)
    alpha, beta = -0.75, 1.5
    stA = [_store(a, tA, ld_extra=3) for a in A]
    stB = [_store(b, tB, ld_extra=1) for b in B]
    ref, mag = oracle.gemm_panels(tA, tB, M, N, K, alpha, [s[0] for s in stA], stA[0][1], [s[0] for s in stB],
                                  stB[0][1], beta, C0, N)
    want = alpha * sum(a.astype(np.float64) @ b.astype(np.float64) for a, b in zip(A, B)) + beta * C0.astype(np.float64)
    want_mag = abs(alpha) * sum(np.abs(a).astype(np.float64) @ np.abs(b).astype(np.float64) for a, b in zip(A, B)) \
        + abs(beta) * np.abs(C0).astype(np.float64)
    assert np.allclose(ref, want, rtol=0, atol=1e-12)
    assert np.allclose(mag, want_mag, rtol=0, atol=1e-12)
    brute = np.zeros((M, N))
    for i in range(M):
        for j in range(N):
            acc = 0.0
            for p in range(P):
                for k in range(K):
                    acc += float(A[p][i, k]) * float(B[p][k, j])
            brute[i, j] = alpha * acc + beta * float(C0[i, j])
    assert np.allclose(ref, brute, rtol=0, atol=1e-12)


def test_gemm_panels_integer_exact_equals_product_of_concatenations():
    # [A_0 A_1 ...] * [B_0; B_1; ...] in exact integer arithmetic (int64 numpy, no floating point)
    rng = np.random.default_rng(5)
    M, N, K, P = 9, 11, 16, 5
    A = [rng.integers(-4, 5, size=(M, K)) for _ in range(P)]
    B = [rng.integers(-4, 5, size=(K, N)) for _ in range(P)]
    want = np.concatenate(A, axis=1) @ np.concatenate(B, axis=0)
    ref, _ = oracle.gemm_panels(0, 0, M, N, K, 1.0, [a.astype(np.float32) for a in A], K,
                                [b.astype(np.float32) for b in B], N)
    assert np.array_equal(ref, want.astype(np.float64))


# ----------------------------------------------------------------------------- half-precision storage

def _half(bits):
    return np.array(bits, dtype=np.uint16).view(np.float16)


def test_half_decoder_agrees_with_numpy_on_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)          # numpy's own conversion, not the oracle's
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))     # -0.0 keeps its sign
    # a few values fixed by the format itself
    assert oracle.half_to_double(0x3C00) == 1.0 and oracle.half_to_double(0xC000) == -2.0
    assert oracle.half_to_double(0x0001) == 2.0 ** -24 and oracle.half_to_double(0x0400) == 2.0 ** -14
    assert oracle.half_to_double(0x7BFF) == 65504.0 and oracle.half_to_double(0x7C00) == np.inf


def test_hgemm_hand_worked_fixture_all_transposes():
    raw = {}
    with open(os.path.join(GOLDEN, "hgemm_hand_worked.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                raw[key] = vals
    M, N, K = int(raw["M"][0]), int(raw["N"][0]), int(raw["K"][0])
    A = _half([int(v, 16) for v in raw["A"]]).reshape(M, K)
    B = _half([int(v, 16) for v in raw["B"]]).reshape(K, N)
    C0 = _half([int(v, 16) for v in raw["C0"]]).reshape(M, N)
    want = np.array([float(v) for v in raw["ref"]]).reshape(M, N)
    want_mag = np.array([float(v) for v in raw["mag"]]).reshape(M, N)
    alpha, beta = float(raw["alpha"][0]), float(raw["beta"][0])
    for tA, tB in itertools.product((0, 1), (0, 1)):
        a = np.ascontiguousarray(A.T if tA else A)
        b = np.ascontiguousarray(B.T if tB else B)
        ref, mag = oracle.hgemm(tA, tB, M, N, K, alpha, a, a.shape[1], b, b.shape[1], beta, C0, N)
        assert np.array_equal(ref, want), (tA, tB, ref)
        assert np.array_equal(mag, want_mag), (tA, tB, mag)
        pts, _ = oracle.hgemm(tA, tB, M, N, K, alpha, a, a.shape[1], b, b.shape[1], beta, C0, N, pi=[1, 0], pj=[1, 0])
        assert np.array_equal(pts, want[[1, 0], [1, 0]])


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_hgemm_matches_numpy_float64_of_the_same_halves(tA, tB):
    rng = np.random.default_rng(40 + 2 * tA + tB)
    M, N, K = 7, 9, 33
    A = rng.standard_normal((M, K)).astype(np.float16)
    B = rng.standard_normal((K, N)).astype(np.float16)
    C0 = rng.standard_normal((M, N)).astype(np.float16)
    lda, ldb, ldc = (M if tA else K) + 3, (K if tB else N) + 1, N + 2

    def store(m, ld):
        buf = np.full((m.shape[0], ld), np.nan, dtype=np.float16)
        buf[:, :m.shape[1]] = m
        return buf

    a, b, c = store(A.T if tA else A, lda), store(B.T if tB else B, ldb), store(C0, ldc)
    ref, mag = oracle.hgemm(tA, tB, M, N, K, -1.5, a, lda, b, ldb, 0.25, c, ldc)
    want = -1.5 * (A.astype(np.float64) @ B.astype(np.float64)) + 0.25 * C0.astype(np.float64)
    want_mag = 1.5 * (np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)) + 0.25 * np.abs(C0).astype(np.float64)
    assert np.allclose(ref, want, rtol=0, atol=1e-12)
    assert np.allclose(mag, want_mag, rtol=0, atol=1e-12)
    # the same numbers through the FP32 oracle (halves are exactly representable as floats)
    a32, b32, c32 = (np.nan_to_num(x.astype(np.float32)) for x in (a, b, c))
    ref32, _ = oracle.gemm(tA, tB, M, N, K, -1.5, a32, lda, b32, ldb, 0.25, c32, ldc)
    assert np.array_equal(ref, ref32)


def test_hgemm_integer_exact_and_conventions():
    rng = np.random.default_rng(8)
    M, N, K = 12, 10, 64
    A = rng.integers(-4, 5, size=(M, K))
    B = rng.integers(-4, 5, size=(K, N))
    ref, _ = oracle.hgemm(0, 0, M, N, K, 1.0, A.astype(np.float16), K, B.astype(np.float16), N)
    assert np.array_equal(ref, (A @ B).astype(np.float64))
    # beta == 0 never reads C0 (NaN there), alpha == 0 never reads A, B
    nanC = np.full((M, N), np.nan, dtype=np.float16)
    ref, _ = oracle.hgemm(0, 0, M, N, K, 1.0, A.astype(np.float16), K, B.astype(np.float16), N, 0.0, nanC, N)
    assert np.array_equal(ref, (A @ B).astype(np.float64))
    C0 = rng.integers(-4, 5, size=(M, N)).astype(np.float16)
    nanA = np.full((M, K), np.nan, dtype=np.float16)
    ref, _ = oracle.hgemm(0, 0, M, N, K, 0.0, nanA, K, nanA.reshape(K, M)[:, :N].copy(), N, 2.0, C0, N)
    assert np.array_equal(ref, 2.0 * C0.astype(np.float64))


def test_half_bound_formula():
    ref = np.array([0.0, 1.0, -2048.0, 1e-6])
    mag = np.array([0.0, 1.0, 4096.0, 1e-6])
    got = oracle.half_bound(100, mag, ref)
    base = 4.0 * 100 * 2.0 ** -24 * mag + 1e-6
    want = base + np.array([2.0 ** -25, 2.0 ** -11, 1.0, 2.0 ** -25])
    assert np.allclose(got, want, rtol=1e-15, atol=0)


# ----------------------------------------------------------------------------- double precision

def test_dgemm_hand_worked_fixture():
    raw = {}
    with open(os.path.join(GOLDEN, "dgemm_hand_worked.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                raw[key] = vals
    M, N, K = int(raw["M"][0]), int(raw["N"][0]), int(raw["K"][0])
    A = np.array([float.fromhex(v) for v in raw["A"]]).reshape(M, K)
    B = np.array([float.fromhex(v) for v in raw["B"]]).reshape(K, N)
    want = np.array([float.fromhex(v) for v in raw["ref"]]).reshape(M, N)
    for tA, tB in itertools.product((0, 1), (0, 1)):
        a = np.ascontiguousarray(A.T if tA else A)
        b = np.ascontiguousarray(B.T if tB else B)
        ref, _ = oracle.dgemm(tA, tB, M, N, K, 1.0, a, a.shape[1], b, b.shape[1])
        assert np.array_equal(ref, want), (tA, tB, [x.hex() for x in ref.ravel()])


def test_dgemm_accumulates_wider_than_double():
    assert oracle.long_double_digits() >= 64
    # 2^60 + 1 - 2^60 summed left to right: FP64 accumulation loses the 1, the oracle must not
    A = np.array([[2.0 ** 60, 1.0, -2.0 ** 60]])
    B = np.ones((3, 1))
    ref, mag = oracle.dgemm(0, 0, 1, 1, 3, 1.0, A, 3, B, 1)
    assert ref[0, 0] == 1.0
    assert mag[0, 0] == 2.0 ** 61      # 2^61 + 1 rounded to double
    # products are exact too: (1 + 2^-30)^2 - 1 - 2^-29 = 2^-60, lost by FP64 products
    x = 1.0 + 2.0 ** -30
    A = np.array([[x, -1.0, -2.0 ** -29]])
    B = np.array([[x], [1.0], [1.0]])
    ref, _ = oracle.dgemm(0, 0, 1, 1, 3, 1.0, A, 3, B, 1)
    assert ref[0, 0] == 2.0 ** -60


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_dgemm_matches_exact_rational_arithmetic(tA, tB):
    from fractions import Fraction
    rng = np.random.default_rng(60 + 2 * tA + tB)
    M, N, K = 4, 5, 9
    A = rng.standard_normal((M, K))
    B = rng.standard_normal((K, N))
    C0 = rng.standard_normal((M, N))
    alpha, beta = -1.25, 0.5
    a, lda = np.ascontiguousarray(A.T if tA else A), (M if tA else K)
    b, ldb = np.ascontiguousarray(B.T if tB else B), (K if tB else N)
    ref, mag = oracle.dgemm(tA, tB, M, N, K, alpha, a, lda, b, ldb, beta, C0, N)
    for i in range(M):
        for j in range(N):
            exact = Fraction(alpha) * sum(Fraction(A[i, k]) * Fraction(B[k, j]) for k in range(K)) \
                + Fraction(beta) * Fraction(C0[i, j])
            emag = abs(Fraction(alpha)) * sum(abs(Fraction(A[i, k])) * abs(Fraction(B[k, j])) for k in range(K)) \
                + abs(Fraction(beta)) * abs(Fraction(C0[i, j]))
            # long-double accumulation of 9 terms, then one rounding to double
            tol = float(emag) * (2.0 ** -53 + 12 * 2.0 ** -64)
            assert abs(Fraction(ref[i, j]) - exact) <= Fraction(tol), (i, j)
            assert abs(Fraction(mag[i, j]) - emag) <= Fraction(tol), (i, j)


def test_dgemm_integer_exact_leading_dimensions_and_conventions():
    rng = np.random.default_rng(9)
    M, N, K = 11, 7, 40
    A = rng.integers(-1000, 1001, size=(M, K))
    B = rng.integers(-1000, 1001, size=(K, N))
    want = (A @ B).astype(np.float64)
    a = np.full((M, K + 3), np.nan)
    a[:, :K] = A
    b = np.full((K, N + 2), np.nan)
    b[:, :N] = B
    ref, _ = oracle.dgemm(0, 0, M, N, K, 1.0, a, K + 3, b, N + 2)
    assert np.array_equal(ref, want)
    at = np.ascontiguousarray(A.T.astype(np.float64))
    bt = np.ascontiguousarray(B.T.astype(np.float64))
    ref, _ = oracle.dgemm(1, 1, M, N, K, 2.0, at, M, bt, K, -1.0, want.copy(), N)
    assert np.array_equal(ref, want)                       # 2*AB - AB
    pts, _ = oracle.dgemm(1, 1, M, N, K, 2.0, at, M, bt, K, -1.0, want.copy(), N, pi=[10, 0], pj=[6, 3])
    assert np.array_equal(pts, want[[10, 0], [6, 3]])
    nanC = np.full((M, N), np.nan)
    ref, _ = oracle.dgemm(0, 0, M, N, K, 1.0, A.astype(np.float64), K, B.astype(np.float64), N, 0.0, nanC, N)
    assert np.array_equal(ref, want)
    ref, _ = oracle.dgemm(0, 0, M, N, K, 0.0, np.full((M, K), np.nan), K, np.full((K, N), np.nan), N, 3.0, want, N)
    assert np.array_equal(ref, 3.0 * want)


def test_double_bound_formula():
    mag = np.array([0.0, 1.0, 1e6])
    got = oracle.double_bound(1000, mag)
    assert np.allclose(got, 4000 * 2.0 ** -53 * mag + 2.0 ** -49, rtol=1e-15, atol=0)


def _conv_brute(x, w, pad, stride):
    """Second, independent statement of the definition: python loops in float64."""
    N, C, H, W = x.shape
    Kout, _, R, S = w.shape
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    xp = np.zeros((N, C, H + 2 * pad[0], W + 2 * pad[1]))
    xp[:, :, pad[0]:pad[0] + H, pad[1]:pad[1] + W] = x
    y = np.zeros((N, Kout, P, Q))
    for n in range(N):
        for j in range(Kout):
            for p in range(P):
                for q in range(Q):
                    win = xp[n, :, p * stride[0]:p * stride[0] + R, q * stride[1]:q * stride[1] + S]
                    y[n, j, p, q] = float(np.sum(win * w[j].astype(np.float64)))
    return y


def test_conv_hand_worked_fixture():
    fx = _read_fixture("conv_hand_worked.txt")
    x = np.array(fx["x"], dtype=np.float32).reshape(1, 1, 3, 3)
    w = np.array(fx["w"], dtype=np.float32).reshape(1, 1, 2, 2)
    ref, mag = oracle.conv2d_fwd(x, w, pad=(0, 0), stride=(1, 1))
    assert np.array_equal(ref.reshape(-1), np.array(fx["y_pad0_stride1"]))
    assert np.array_equal(mag, ref)          # all entries positive
    ref, _ = oracle.conv2d_fwd(x, w, pad=(1, 1), stride=(2, 2))
    assert ref.shape == (1, 1, 2, 2)
    assert np.array_equal(ref.reshape(-1), np.array(fx["y_pad1_stride2"]))


def test_conv_1x1_is_a_gemm_per_image():
    rng = np.random.default_rng(29)
    N, C, H, W, Kout = 3, 10, 5, 4, 7
    x = rng.integers(-4, 5, size=(N, C, H, W)).astype(np.float32)
    w = rng.integers(-4, 5, size=(Kout, C, 1, 1)).astype(np.float32)
    ref, _ = oracle.conv2d_fwd(x, w)
    for n in range(N):
        want = w.reshape(Kout, C).astype(np.int64) @ x[n].reshape(C, H * W).astype(np.int64)
        assert np.array_equal(ref[n].reshape(Kout, H * W), want.astype(np.float64))


def test_conv_delta_filters_pin_no_flip():
    rng = np.random.default_rng(31)
    N, C, H, W = 2, 4, 6, 5
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    centre = np.zeros((C, C, 3, 3), dtype=np.float32)
    corner = np.zeros((C, C, 3, 3), dtype=np.float32)
    for c in range(C):
        centre[c, c, 1, 1] = 1.0
        corner[c, c, 0, 0] = 1.0
    ref, _ = oracle.conv2d_fwd(x, centre, pad=(1, 1))
    assert np.array_equal(ref, x.astype(np.float64))
    ref, _ = oracle.conv2d_fwd(x, corner, pad=(1, 1))
    want = np.zeros((N, C, H, W))
    want[:, :, 1:, 1:] = x[:, :, :-1, :-1]     # y[p,q] = x[p-1,q-1], zero border
    assert np.array_equal(ref, want)


def test_conv_all_ones_counts_valid_taps():
    C, H, W, Kout = 5, 6, 7, 3
    x = np.ones((2, C, H, W), dtype=np.float32)
    w = np.ones((Kout, C, 3, 3), dtype=np.float32)
    ref, _ = oracle.conv2d_fwd(x, w, pad=(1, 1))
    want = np.full((H, W), 9.0)
    want[0, :] = want[-1, :] = 6.0
    want[:, 0] = want[:, -1] = 6.0
    want[0, 0] = want[0, -1] = want[-1, 0] = want[-1, -1] = 4.0
    assert np.array_equal(ref, np.broadcast_to(C * want, ref.shape))


@pytest.mark.parametrize("shape", [
    dict(N=2, C=3, H=7, W=5, Kout=4, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=1, C=2, H=9, W=6, Kout=3, R=3, S=2, pad=(0, 0), stride=(2, 2)),
    dict(N=2, C=1, H=8, W=11, Kout=2, R=5, S=3, pad=(2, 1), stride=(2, 3)),
    dict(N=1, C=4, H=4, W=4, Kout=5, R=1, S=1, pad=(0, 0), stride=(1, 1)),
])
def test_conv_matches_brute_force_and_torch(shape):
    import torch
    rng = np.random.default_rng(37 + shape["H"])
    x = rng.standard_normal((shape["N"], shape["C"], shape["H"], shape["W"])).astype(np.float32)
    w = rng.standard_normal((shape["Kout"], shape["C"], shape["R"], shape["S"])).astype(np.float32)
    y0 = rng.standard_normal(1000).astype(np.float32)
    ref, mag = oracle.conv2d_fwd(x, w, pad=shape["pad"], stride=shape["stride"])
    brute = _conv_brute(x, w, shape["pad"], shape["stride"])
    assert ref.shape == brute.shape
    assert np.max(np.abs(ref - brute)) <= 1e-12 * max(1.0, np.max(np.abs(brute)))
    brute_mag = _conv_brute(np.abs(x), np.abs(w), shape["pad"], shape["stride"])
    assert np.max(np.abs(mag - brute_mag)) <= 1e-12 * max(1.0, np.max(np.abs(brute_mag)))
    lib = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     padding=shape["pad"], stride=shape["stride"]).numpy()
    assert np.max(np.abs(ref - lib)) <= 1e-12 * max(1.0, np.max(np.abs(lib)))
    # alpha / beta and the point-wise routine
    y0 = np.ascontiguousarray(y0[:ref.size].reshape(ref.shape))
    ref2, mag2 = oracle.conv2d_fwd(x, w, pad=shape["pad"], stride=shape["stride"], alpha=2.0, beta=-0.5, y0=y0)
    assert np.array_equal(ref2, 2.0 * ref - 0.5 * y0.astype(np.float64))
    assert np.array_equal(mag2, 2.0 * mag + 0.5 * np.abs(y0.astype(np.float64)))
    idx = np.arange(ref.size)[::3]
    rp, mp = oracle.conv2d_fwd_points(x, w, idx, pad=shape["pad"], stride=shape["stride"], alpha=2.0,
                                      beta=-0.5, y0=y0)
    assert np.array_equal(rp, ref2.reshape(-1)[idx])
    assert np.array_equal(mp, mag2.reshape(-1)[idx])


def test_conv_nan_conventions():
    x = np.ones((1, 2, 4, 4), dtype=np.float32)
    w = np.ones((2, 2, 3, 3), dtype=np.float32)
    nan_y = np.full((1, 2, 4, 4), np.nan, dtype=np.float32)
    ref, _ = oracle.conv2d_fwd(x, w, pad=(1, 1), beta=0.0, y0=nan_y)
    assert np.isfinite(ref).all()
    y0 = np.arange(32, dtype=np.float32).reshape(1, 2, 4, 4)
    ref, _ = oracle.conv2d_fwd(np.full_like(x, np.nan), w, pad=(1, 1), alpha=0.0, beta=2.0, y0=y0)
    assert np.array_equal(ref, 2.0 * y0.astype(np.float64))


def test_bound_formula():
    mag = np.array([0.0, 1.0, 2.5])
    got = oracle.bound(4096, mag)
    assert np.array_equal(got, 4.0 * 4096 * 2.0 ** -24 * mag + 1e-6)


# ----------------------------------------------------------------------------- convolution, backward passes

BWD_SHAPES = [
    dict(N=2, C=3, H=7, W=5, Kout=4, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=1, C=2, H=9, W=6, Kout=3, R=3, S=2, pad=(0, 0), stride=(2, 2)),
    dict(N=2, C=1, H=8, W=11, Kout=2, R=5, S=3, pad=(2, 1), stride=(2, 3)),
    dict(N=1, C=4, H=4, W=4, Kout=5, R=1, S=1, pad=(0, 0), stride=(1, 1)),
    dict(N=2, C=2, H=6, W=6, Kout=2, R=3, S=3, pad=(0, 2), stride=(1, 2)),
]


def _bwd_inputs(shape, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((shape["N"], shape["C"], shape["H"], shape["W"])).astype(np.float32)
    w = rng.standard_normal((shape["Kout"], shape["C"], shape["R"], shape["S"])).astype(np.float32)
    P, Q = oracle.conv_out_shape(shape["H"], shape["W"], shape["R"], shape["S"], *shape["pad"], *shape["stride"])
    dy = rng.standard_normal((shape["N"], shape["Kout"], P, Q)).astype(np.float32)
    return x, w, dy


def test_conv_backward_hand_worked_fixture():
    fx = _read_fixture("conv_hand_worked.txt")
    x = np.array(fx["x"], dtype=np.float32).reshape(1, 1, 3, 3)
    w = np.array(fx["w"], dtype=np.float32).reshape(1, 1, 2, 2)
    dy = np.array(fx["dy"], dtype=np.float32).reshape(1, 1, 2, 2)
    dx, mag = oracle.conv2d_bwd_data(dy, w, x.shape)
    assert np.array_equal(dx.reshape(-1), np.array(fx["dx_pad0_stride1"]))
    assert np.array_equal(mag, dx)
    dw, mag = oracle.conv2d_bwd_filter(x, dy, w.shape)
    assert np.array_equal(dw.reshape(-1), np.array(fx["dw_pad0_stride1"]))
    assert np.array_equal(mag, dw)


@pytest.mark.parametrize("shape", BWD_SHAPES)
def test_conv_backward_is_the_adjoint_of_forward(shape):
    """<dy, conv(x, w)> == <bwd_data(dy, w), x> == <bwd_filter(x, dy), w>: fixes both backward oracles
    against the (independently pinned) forward one."""
    x, w, dy = _bwd_inputs(shape, 51)
    y, _ = oracle.conv2d_fwd(x, w, pad=shape["pad"], stride=shape["stride"])
    lhs = float(np.sum(dy.astype(np.float64) * y))
    dx, _ = oracle.conv2d_bwd_data(dy, w, x.shape, pad=shape["pad"], stride=shape["stride"])
    dw, _ = oracle.conv2d_bwd_filter(x, dy, w.shape, pad=shape["pad"], stride=shape["stride"])
    scale = float(np.sum(np.abs(dy.astype(np.float64)) * np.abs(y))) + 1e-30
    assert abs(float(np.sum(dx * x.astype(np.float64))) - lhs) <= 1e-12 * scale
    assert abs(float(np.sum(dw * w.astype(np.float64))) - lhs) <= 1e-12 * scale


@pytest.mark.parametrize("shape", BWD_SHAPES)
def test_conv_backward_matches_brute_force_and_torch(shape):
    import torch
    x, w, dy = _bwd_inputs(shape, 53)
    N, C, H, W = x.shape
    Kout, _, R, S = w.shape
    _, _, P, Q = dy.shape
    ph, pw = shape["pad"]
    sh, sw = shape["stride"]
    # second statement of the definitions: scatter form, python loops, float64
    dx_b = np.zeros((N, C, H, W))
    dw_b = np.zeros((Kout, C, R, S))
    dxm_b = np.zeros_like(dx_b)
    dwm_b = np.zeros_like(dw_b)
    for n in range(N):
        for j in range(Kout):
            for p in range(P):
                for q in range(Q):
                    g = float(dy[n, j, p, q])
                    for c in range(C):
                        for r in range(R):
                            for s in range(S):
                                ih, iw = p * sh + r - ph, q * sw + s - pw
                                if 0 <= ih < H and 0 <= iw < W:
                                    dx_b[n, c, ih, iw] += g * float(w[j, c, r, s])
                                    dxm_b[n, c, ih, iw] += abs(g) * abs(float(w[j, c, r, s]))
                                    dw_b[j, c, r, s] += g * float(x[n, c, ih, iw])
                                    dwm_b[j, c, r, s] += abs(g) * abs(float(x[n, c, ih, iw]))
    dx, dxm = oracle.conv2d_bwd_data(dy, w, x.shape, pad=shape["pad"], stride=shape["stride"])
    dw, dwm = oracle.conv2d_bwd_filter(x, dy, w.shape, pad=shape["pad"], stride=shape["stride"])
    for got, want in ((dx, dx_b), (dxm, dxm_b), (dw, dw_b), (dwm, dwm_b)):
        assert np.max(np.abs(got - want)) <= 1e-12 * max(1.0, np.max(np.abs(want)))
    # library routines in float64
    tx, tw, tdy = (torch.from_numpy(a).double() for a in (x, w, dy))
    lib_dx = torch.nn.grad.conv2d_input(x.shape, tw, tdy, stride=shape["stride"], padding=shape["pad"]).numpy()
    lib_dw = torch.nn.grad.conv2d_weight(tx, w.shape, tdy, stride=shape["stride"], padding=shape["pad"]).numpy()
    assert np.max(np.abs(dx - lib_dx)) <= 1e-12 * max(1.0, np.max(np.abs(lib_dx)))
    assert np.max(np.abs(dw - lib_dw)) <= 1e-12 * max(1.0, np.max(np.abs(lib_dw)))
    # alpha / beta and the sampled form
    rng = np.random.default_rng(3)
    dx0 = rng.standard_normal(x.shape).astype(np.float32)
    dw0 = rng.standard_normal(w.shape).astype(np.float32)
    dx2, dxm2 = oracle.conv2d_bwd_data(dy, w, x.shape, pad=shape["pad"], stride=shape["stride"], alpha=2.0, beta=-0.5,
                                       dx0=dx0)
    assert np.array_equal(dx2, 2.0 * dx - 0.5 * dx0.astype(np.float64))
    assert np.array_equal(dxm2, 2.0 * dxm + 0.5 * np.abs(dx0.astype(np.float64)))
    dw2, dwm2 = oracle.conv2d_bwd_filter(x, dy, w.shape, pad=shape["pad"], stride=shape["stride"], alpha=-1.0, beta=3.0,
                                         dw0=dw0)
    assert np.array_equal(dw2, -dw + 3.0 * dw0.astype(np.float64))
    assert np.array_equal(dwm2, dwm + 3.0 * np.abs(dw0.astype(np.float64)))
    idx = np.arange(dx.size)[::2]
    r, m = oracle.conv2d_bwd_data(dy, w, x.shape, pad=shape["pad"], stride=shape["stride"], alpha=2.0, beta=-0.5,
                                  dx0=dx0, idx=idx)
    assert np.array_equal(r, dx2.reshape(-1)[idx]) and np.array_equal(m, dxm2.reshape(-1)[idx])
    idx = np.arange(dw.size)[::3]
    r, m = oracle.conv2d_bwd_filter(x, dy, w.shape, pad=shape["pad"], stride=shape["stride"], alpha=-1.0, beta=3.0,
                                    dw0=dw0, idx=idx)
    assert np.array_equal(r, dw2.reshape(-1)[idx]) and np.array_equal(m, dwm2.reshape(-1)[idx])


def test_conv_backward_closed_forms():
    # centre-delta filter, pad 1: forward is the identity, so dx = dy; dw[j][c] at the centre = <dy_j, x_c>
    rng = np.random.default_rng(59)
    N, C, H, W = 2, 3, 5, 4
    x = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
    dy = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
    centre = np.zeros((C, C, 3, 3), dtype=np.float32)
    for c in range(C):
        centre[c, c, 1, 1] = 1.0
    dx, _ = oracle.conv2d_bwd_data(dy, centre, x.shape, pad=(1, 1))
    assert np.array_equal(dx, dy.astype(np.float64))
    dw, _ = oracle.conv2d_bwd_filter(x, dy, centre.shape, pad=(1, 1))
    want_centre = np.einsum("njhw,nchw->jc", dy.astype(np.int64), x.astype(np.int64))
    assert np.array_equal(dw[:, :, 1, 1], want_centre.astype(np.float64))
    # corner tap (0,0) sees x shifted by (-1,-1): dw[j][c][0][0] = sum dy[p][q] * x[p-1][q-1]
    want_corner = np.einsum("njhw,nchw->jc", dy[:, :, 1:, 1:].astype(np.int64), x[:, :, :-1, :-1].astype(np.int64))
    assert np.array_equal(dw[:, :, 0, 0], want_corner.astype(np.float64))
    # all ones: every dx element counts the (j, r, s) terms that reach it
    ones_dy = np.ones((1, 2, 4, 4), dtype=np.float32)
    ones_w = np.ones((2, 3, 3, 3), dtype=np.float32)
    dx, _ = oracle.conv2d_bwd_data(ones_dy, ones_w, (1, 3, 4, 4), pad=(1, 1))
    want = np.full((4, 4), 9.0)
    want[0, :] = want[-1, :] = 6.0
    want[:, 0] = want[:, -1] = 6.0
    want[0, 0] = want[0, -1] = want[-1, 0] = want[-1, -1] = 4.0
    assert np.array_equal(dx, np.broadcast_to(2 * want, dx.shape))
    # 1x1: dx = W^T dy per pixel, dw = dy x^T summed over pixels (integer exact)
    w11 = rng.integers(-3, 4, size=(4, 3, 1, 1)).astype(np.float32)
    dy11 = rng.integers(-3, 4, size=(2, 4, 5, 4)).astype(np.float32)
    dx, _ = oracle.conv2d_bwd_data(dy11, w11, (2, 3, 5, 4))
    assert np.array_equal(dx, np.einsum("jc,njhw->nchw", w11[:, :, 0, 0].astype(np.int64), dy11.astype(np.int64)).astype(np.float64))
    dw, _ = oracle.conv2d_bwd_filter(x, dy11, w11.shape)
    assert np.array_equal(dw[:, :, 0, 0], np.einsum("njhw,nchw->jc", dy11.astype(np.int64), x.astype(np.int64)).astype(np.float64))
