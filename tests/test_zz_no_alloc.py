"""GPU test of dmath_gemm_noalloc, the entry point for callers that cannot allocate: it must give the
results of dmath_gemm (same kernels, same plan) while its split-K slices, tail-tile partial sums and
counters live in the library's own device array instead of a caller's workspace.

Two calls in a row on shapes whose plans really use scratch, the second smaller than the first (so it
meets the first call's leftovers in the shared array), each compared bit for bit with dmath_gemm run
with a registered workspace of the same size, and against the FP64 oracle under the contract bound.
This file is named so that pytest collects it last.
"""
import numpy as np
import pytest

import oracle
from parity_util import check_bound

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    return t


@pytest.fixture()
def dm(torch):
    from paper_1604_01416_amd import dmath
    dmath.dmath_set_override(-1, -1)
    ws = torch.empty(dmath.NOALLOC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    dmath.check(dmath.dmath_set_workspace(ws, ws.numel()))
    yield dmath
    torch.cuda.synchronize()
    dmath.dmath_set_override(-1, -1)
    dmath.dmath_set_workspace(None, 0)


def _operands(torch, tA, tB, M, N, K, seed, ints):
    rng = np.random.default_rng(seed)
    if ints:
        A = rng.integers(-4, 5, size=(M, K)).astype(np.float32)
        B = rng.integers(-4, 5, size=(K, N)).astype(np.float32)
        C0 = rng.integers(-4, 5, size=(M, N)).astype(np.float32)
    else:
        A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
        C0 = rng.standard_normal((M, N)).astype(np.float32)
    As = np.ascontiguousarray(A.T if tA else A)
    Bs = np.ascontiguousarray(B.T if tB else B)
    return As, Bs, C0


def _one(dm, torch, tA, tB, M, N, K, alpha, beta, seed, ints=False):
    """dmath_gemm_noalloc against dmath_gemm (bits) and the oracle (bound); returns the split factor."""
    need = dm.dmath_gemm_workspace_bytes(tA, tB, M, N, K)
    assert 0 < need <= dm.NOALLOC_SCRATCH_BYTES, "the case must use scratch, and fit"
    st, cfg, split = dm.dmath_gemm_plan(tA, tB, M, N, K)
    assert st == dm.OK and split > 1, "the plan must really split"
    As, Bs, C0 = _operands(torch, tA, tB, M, N, K, seed, ints)
    lda, ldb, ldc = As.shape[1], Bs.shape[1], N
    dA, dB = torch.from_numpy(As).cuda(), torch.from_numpy(Bs).cuda()
    c_ref = torch.from_numpy(C0).cuda()
    c_new = torch.from_numpy(C0).cuda()
    dm.check(dm.dmath_gemm(tA, tB, M, N, K, alpha, dA, lda, dB, ldb, beta, c_ref, ldc))
    dm.check(dm.dmath_gemm_noalloc(tA, tB, M, N, K, alpha, dA, lda, dB, ldb, beta, c_new, ldc))
    torch.cuda.synchronize()
    got, want = c_new.cpu().numpy(), c_ref.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), "differs from dmath_gemm"
    ref, mag = oracle.gemm(tA, tB, M, N, K, alpha, As, lda, Bs, ldb, beta, C0 if beta != 0.0 else None, ldc)
    if ints:
        assert np.array_equal(got.astype(np.float64), ref), "integer case must be bit-exact"
    else:
        check_bound(got, ref, mag, K, "gemm_noalloc t%d%d %dx%dx%d" % (tA, tB, M, N, K))
    return split


def test_two_calls_in_a_row_second_smaller(dm, torch):
    # 18 x 18 tiles of 128 x 128 = one round over the 256 compute units + a tail of 68 tiles that is cut
    # into K slices and combined in the kernel (partial sums + counters in scratch) ...
    _one(dm, torch, 0, 0, 2304, 2304, 2048, 1.0, 1.0, seed=11)
    # ... then, right behind it, a smaller one of the same kind on another tile size (64 tail tiles) ...
    _one(dm, torch, 1, 0, 1536, 1536, 2048, 1.0, 0.0, seed=12)
    # ... and a skinny product (plain split-K: whole-output slices in scratch)
    _one(dm, torch, 0, 1, 192, 1000, 2048, 0.5, 0.0, seed=13)
    # the same sequence with integer entries, where any summation order is exact
    _one(dm, torch, 1, 0, 2304, 2304, 2048, 1.0, 1.0, seed=14, ints=True)
    _one(dm, torch, 0, 0, 1536, 1536, 2048, 1.0, 0.0, seed=15, ints=True)
    _one(dm, torch, 0, 0, 192, 1000, 1024, 1.0, 0.0, seed=16, ints=True)


def test_scratch_is_reused_without_stale_state(dm, torch):
    """The same tail-split shape twice, then a smaller one with fewer split tiles: counters left by a
    call must not leak into the next (each call clears the ones it uses)."""
    for seed in (21, 22):
        _one(dm, torch, 0, 0, 2304, 2304, 2048, 1.0, 0.0, seed=seed)
    _one(dm, torch, 0, 0, 2176, 2304, 4096, 1.0, 0.0, seed=23)


def test_beyond_the_scratch_is_refused_and_no_workspace_is_needed(dm, torch):
    M = N = K = 6144                      # its tail split wants 64 MiB of partial sums
    assert dm.dmath_gemm_workspace_bytes(0, 0, M, N, K) > dm.NOALLOC_SCRATCH_BYTES
    A = torch.zeros((M, K), device="cuda")
    B = torch.zeros((K, N), device="cuda")
    C = torch.full((M, N), 7.0, device="cuda")
    assert dm.dmath_gemm_noalloc(0, 0, M, N, K, 1.0, A, K, B, N, 0.0, C, N) == dm.ERR_WORKSPACE
    assert dm.dmath_last_error_arg() == 0
    torch.cuda.synchronize()
    assert bool((C == 7.0).all()), "a refused call must not touch C"
    # argument errors are reported as by dmath_gemm, before the scratch question
    assert dm.dmath_gemm_noalloc(0, 0, M, N, K, 1.0, A, K - 1, B, N, 0.0, C, N) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 8
    # the registered workspace plays no part: take it away and a splitting shape still splits and agrees
    small = dm.dmath_gemm_workspace_bytes(0, 0, 192, 1000, 2048)
    assert small > 0
    dm.check(dm.dmath_set_workspace(None, 0))
    rng = np.random.default_rng(31)
    As = rng.uniform(-1, 1, (192, 2048)).astype(np.float32)
    Bs = rng.uniform(-1, 1, (2048, 1000)).astype(np.float32)
    dA, dB = torch.from_numpy(As).cuda(), torch.from_numpy(Bs).cuda()
    out = torch.full((192, 1000), float("nan"), device="cuda")
    dm.check(dm.dmath_gemm_noalloc(0, 0, 192, 1000, 2048, 1.0, dA, 2048, dB, 1000, 0.0, out, 1000))
    torch.cuda.synchronize()
    ref, mag = oracle.gemm(0, 0, 192, 1000, 2048, 1.0, As, 2048, Bs, 1000, 0.0, None, 1000)
    check_bound(out.cpu().numpy(), ref, mag, 2048, "gemm_noalloc without a registered workspace")
