"""GPU parity at the benchmark launch shapes with integer-valued operands.

With entries in {-4..4} every partial sum of these shapes stays below 2^24, so every FP32 summation
order (tile order, K slices, wave-split reductions, panel walks) gives the exact result and the GPU must
match the FP64 oracle bit for bit: a dropped k term, a tile written twice or a misapplied beta cannot
hide inside a rounding bound.  The full-size configurations are compared on sampled outputs the oracle
computes one by one (whole rows, columns and planes plus random points); configuration 4 on every
element.  These are the launch configurations bench.py times (automatic plans, 128 MiB workspace).
"""
import numpy as np
import pytest

import oracle
from paper_1604_01416_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    return t


@pytest.fixture(scope="module")
def dm(torch):
    from paper_1604_01416_amd import dmath
    dmath.dmath_set_override(-1, -1)
    ws = torch.empty(128 << 20, dtype=torch.uint8, device="cuda")
    dmath.check(dmath.dmath_set_workspace(ws, ws.numel()))
    yield dmath
    torch.cuda.synchronize()
    dmath.dmath_set_workspace(None, 0)


def _points(rng, M, N, nrows, ncols, nrand):
    rows = np.unique(np.concatenate([rng.choice(M, size=nrows, replace=False), [0, M // 2 - 1, M // 2, M - 1]]))
    cols = np.unique(np.concatenate([rng.choice(N, size=ncols, replace=False), [0, N // 2 - 1, N // 2, N - 1]]))
    pi = np.concatenate([np.repeat(rows, N), np.tile(np.arange(M), len(cols)), rng.integers(0, M, size=nrand)])
    pj = np.concatenate([np.tile(np.arange(N), len(rows)), np.repeat(cols, M), rng.integers(0, N, size=nrand)])
    return pi, pj


def _config3_integer_operands(seed):
    rng = np.random.default_rng(seed)
    m, kp, steps = 8192, 512, 16
    C0 = workloads.small_ints(rng, (m, m))
    As = [workloads.small_ints(rng, (m, kp)) for _ in range(steps)]
    Bs = [workloads.small_ints(rng, (kp, m)) for _ in range(steps)]
    return m, kp, steps, C0, As, Bs


def test_config3_chain_of_16_calls_integer_exact(dm, torch):
    """|C0 + sum| <= 4 + 16 * 8192 < 2^24: the 16 accumulate calls must land on the exact integers."""
    m, kp, steps, C0, As, Bs = _config3_integer_operands(101)
    dC = torch.from_numpy(C0).cuda()
    for a, b in zip(As, Bs):
        da, db = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
        dm.check(dm.dmath_gemm(0, 0, m, m, kp, 1.0, da, kp, db, m, 1.0, dC, m))
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    pi, pj = _points(np.random.default_rng(1), m, m, 3, 3, 20000)
    ref, _ = oracle.gemm_panels(0, 0, m, m, kp, 1.0, As, kp, Bs, m, 1.0, C0, m, pi=pi, pj=pj)
    assert np.array_equal(got[pi, pj].astype(np.float64), ref)


def test_config3_as_one_fused_call_integer_exact(dm, torch):
    m, kp, steps, C0, As, Bs = _config3_integer_operands(102)
    dC = torch.from_numpy(C0).cuda()
    dAs = [torch.from_numpy(a).cuda() for a in As]
    dBs = [torch.from_numpy(b).cuda() for b in Bs]
    dm.check(dm.dmath_gemm_panels(0, 0, m, m, kp, 1.0, dAs, kp, dBs, m, 1.0, dC, m))
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    pi, pj = _points(np.random.default_rng(2), m, m, 3, 3, 20000)
    ref, _ = oracle.gemm_panels(0, 0, m, m, kp, 1.0, As, kp, Bs, m, 1.0, C0, m, pi=pi, pj=pj)
    assert np.array_equal(got[pi, pj].astype(np.float64), ref)


def test_config4_three_products_integer_exact_every_element(dm, torch):
    rng = np.random.default_rng(103)
    batch, width = 256, 4096
    X = np.maximum(workloads.small_ints(rng, (batch, width)), 0.0).astype(np.float32)   # about half zeros, like ReLU
    W = workloads.small_ints(rng, (width, width))
    dY = workloads.small_ints(rng, (batch, width))
    dX_, dW_, dY_ = (torch.from_numpy(t).cuda() for t in (X, W, dY))
    Y = torch.full((batch, width), float("nan"), device="cuda")
    dXo = torch.full((batch, width), float("nan"), device="cuda")
    dWo = torch.full((width, width), float("nan"), device="cuda")
    dm.check(dm.dmath_gemm(0, 0, batch, width, width, 1.0, dX_, width, dW_, width, 0.0, Y, width))
    dm.check(dm.dmath_gemm(0, 1, batch, width, width, 1.0, dY_, width, dW_, width, 0.0, dXo, width))
    dm.check(dm.dmath_gemm(1, 0, width, width, batch, 1.0, dX_, width, dY_, width, 0.0, dWo, width))
    torch.cuda.synchronize()
    ref, _ = oracle.gemm(0, 0, batch, width, width, 1.0, X, width, W, width)
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), ref), "Y = X W"
    ref, _ = oracle.gemm(0, 1, batch, width, width, 1.0, dY, width, W, width)
    assert np.array_equal(dXo.cpu().numpy().astype(np.float64), ref), "dX = dY W^T"
    ref, _ = oracle.gemm(1, 0, width, width, batch, 1.0, X, width, dY, width)
    assert np.array_equal(dWo.cpu().numpy().astype(np.float64), ref), "dW = X^T dY"


def _config5_integer_operands(seed):
    rng = np.random.default_rng(seed)
    N, C, H, W, Kout = 128, 256, 28, 28, 256
    x = np.maximum(workloads.small_ints(rng, (N, C, H, W)), 0.0).astype(np.float32)
    w = workloads.small_ints(rng, (Kout, C, 3, 3))
    dy = workloads.small_ints(rng, (N, Kout, H, W))
    return N, C, H, W, Kout, x, w, dy


def _sample_tensor(rng, shape, nrand, planes):
    total = int(np.prod(shape))
    plane = shape[2] * shape[3]
    idx = [rng.choice(total, size=nrand, replace=False)]
    for a, b in planes:
        base = (a * shape[1] + b) * plane
        idx.append(np.arange(base, base + plane))
    return np.concatenate(idx)


def test_config5_forward_integer_exact_sampled(dm, torch):
    N, C, H, W, Kout, x, w, _ = _config5_integer_operands(104)      # |sum| <= 16 * 2304
    dx, dw = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    y = torch.full((N, Kout, H, W), float("nan"), device="cuda")
    dm.check(dm.dmath_conv2d_fwd(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, dx, dw, 0.0, y))
    torch.cuda.synchronize()
    got = y.cpu().numpy().reshape(-1)
    idx = _sample_tensor(np.random.default_rng(4), (N, Kout, H, W), 150000,
                         [(0, 0), (N - 1, Kout - 1), (N // 2, 129), (N - 1, 0), (125, 200)])   # 125: inside the tail tiles
    ref, _ = oracle.conv2d_fwd_points(x, w, idx, pad=(1, 1), stride=(1, 1))
    assert np.array_equal(got[idx].astype(np.float64), ref)


def test_config5_backward_data_integer_exact_sampled(dm, torch):
    N, C, H, W, Kout, _, w, dy = _config5_integer_operands(105)
    ddy, dw = torch.from_numpy(dy).cuda(), torch.from_numpy(w).cuda()
    dxo = torch.full((N, C, H, W), float("nan"), device="cuda")
    dm.check(dm.dmath_conv2d_bwd_data(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, ddy, dw, 0.0, dxo))
    torch.cuda.synchronize()
    got = dxo.cpu().numpy().reshape(-1)
    idx = _sample_tensor(np.random.default_rng(5), (N, C, H, W), 150000,
                         [(0, 0), (N - 1, C - 1), (N // 2, 129), (126, 7)])
    ref, _ = oracle.conv2d_bwd_data(dy, w, (N, C, H, W), pad=(1, 1), stride=(1, 1), idx=idx)
    assert np.array_equal(got[idx].astype(np.float64), ref)


def test_config5_backward_filter_integer_exact_sampled(dm, torch):
    N, C, H, W, Kout, x, _, dy = _config5_integer_operands(106)     # |sum| <= 16 * 100352 < 2^24
    dx, ddy = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    dwo = torch.full((Kout, C, 3, 3), float("nan"), device="cuda")
    dm.check(dm.dmath_conv2d_bwd_filter(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, dx, ddy, 0.0, dwo))
    torch.cuda.synchronize()
    got = dwo.cpu().numpy().reshape(-1)
    rng = np.random.default_rng(6)
    idx = np.unique(np.concatenate([rng.choice(got.size, size=40000, replace=False),
                                    np.arange(0, 2304), np.arange(got.size - 2304, got.size)]))   # first and last filter
    ref, _ = oracle.conv2d_bwd_filter(x, dy, (Kout, C, 3, 3), pad=(1, 1), stride=(1, 1), idx=idx)
    assert np.array_equal(got[idx].astype(np.float64), ref)
