"""GPU parity: the HIP library, called through its C ABI, against the FP64 CPU oracle.

Small cases are compared element by element (sizes span several tiles and a ragged tail, every
transpose form, every tile configuration, aligned and unaligned operands, a NaN guard frame around
C); the five benchmark configurations run at full size in the launch configuration bench.py times,
and are compared on every element where the oracle finishes in seconds and on sampled rows /
columns / outputs otherwise.  Bound: |gpu - ref| <= 4*K*2^-24*mag + 1e-6; bit-exact where the
inputs are small integers (every FP32 summation order is then exact).
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_1604_01416_amd import workloads
from parity_util import check_bound, run_conv_bwd_data_case, run_conv_bwd_filter_case, run_conv_case, run_dgemm_case, run_gemm_case, run_gemm_panels_case, run_hgemm_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    return t


@pytest.fixture(scope="module")
def dm(torch):
    from paper_1604_01416_amd import dmath
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")      # 64 MiB split-K scratch
    dmath.check(dmath.dmath_set_workspace(ws, ws.numel()))
    dmath._test_workspace = ws                                       # keep it alive
    yield dmath
    dmath.dmath_set_override(-1, -1)
    dmath.dmath_set_workspace(None, 0)


@pytest.fixture(autouse=True)
def _auto_plan(dm):
    dm.dmath_set_override(-1, -1)
    dm.dmath_set_hgemm_path(-1)
    dm.dmath_set_dgemm_config(-1)
    yield
    dm.dmath_set_override(-1, -1)
    dm.dmath_set_hgemm_path(-1)
    dm.dmath_set_dgemm_config(-1)


TRANS = list(itertools.product((0, 1), (0, 1)))


# ------------------------------------------------------------------ first: does the MFMA layout hold

def test_identity_and_index_matrices_pin_the_tile_layout(dm, torch):
    """A = I gives C = B exactly, B = I gives C = A exactly: any wrong lane/register mapping of the
    MFMA operands or accumulators moves an element and fails this."""
    for cfg in range(dm.dmath_num_configs()):
        dm.dmath_set_override(cfg, 1)
        n = 320
        idx = (np.arange(n * n, dtype=np.float32).reshape(n, n) % 4093) - 2000.0
        eye = np.eye(n, dtype=np.float32)
        for A, B, want in ((eye, idx, idx), (idx, eye, idx)):
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            dC = torch.full((n, n), float("nan"), device="cuda")
            dm.check(dm.dmath_gemm(0, 0, n, n, n, 1.0, dA, n, dB, n, 0.0, dC, n))
            torch.cuda.synchronize()
            assert np.array_equal(dC.cpu().numpy(), want), dm.dmath_config_name(cfg)


# ------------------------------------------------------------------ small cases, element by element

SHAPES = [(1, 1, 1), (3, 5, 7), (17, 33, 19), (64, 64, 64), (127, 129, 65), (255, 257, 130),
          (300, 200, 100), (513, 260, 48)]


@pytest.mark.parametrize("tA,tB", TRANS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_small_auto(dm, torch, tA, tB, M, N, K):
    run_gemm_case(dm, torch, tA, tB, M, N, K, alpha=1.0, beta=0.0, seed=M + N + K, c_nan=True)
    run_gemm_case(dm, torch, tA, tB, M, N, K, alpha=-0.75, beta=1.5, ld_extra=(3, 5, 2), lead=(1, 3, 1),
                  seed=M * 3 + K)


@pytest.mark.parametrize("cfg", range(7))
@pytest.mark.parametrize("tA,tB", TRANS)
def test_gemm_every_config_aligned_and_unaligned(dm, torch, cfg, tA, tB):
    if cfg >= dm.dmath_num_configs():
        pytest.skip("no such configuration")
    dm.dmath_set_override(cfg, 1)
    # multiples of 4 and 16-byte aligned: vector path, ragged tiles in M, N and K
    run_gemm_case(dm, torch, tA, tB, 388, 516, 200, alpha=1.0, beta=0.0, ld_extra=(4, 8, 12), lead=(4, 8, 4),
                  seed=cfg, c_nan=True)
    run_gemm_case(dm, torch, tA, tB, 388, 516, 203, alpha=0.5, beta=-2.0, ld_extra=(5, 0, 4), lead=(0, 4, 0),
                  seed=cfg + 10)
    # odd sizes, odd leading dimensions, misaligned bases: scalar path
    run_gemm_case(dm, torch, tA, tB, 259, 131, 77, alpha=2.0, beta=1.0, ld_extra=(1, 2, 3), lead=(1, 2, 3),
                  seed=cfg + 20)
    # integer entries: bit-exact
    run_gemm_case(dm, torch, tA, tB, 260, 136, 96, alpha=1.0, beta=1.0, seed=cfg + 30, ints=True, exact=True)


@pytest.mark.parametrize("cfg,split", [(0, 2), (3, 4), (4, 8), (4, 3)])
@pytest.mark.parametrize("tA,tB", TRANS)
def test_gemm_split_k(dm, torch, cfg, split, tA, tB):
    dm.dmath_set_override(cfg, split)
    run_gemm_case(dm, torch, tA, tB, 130, 264, 1000, alpha=1.25, beta=0.5, ld_extra=(0, 0, 4), seed=split)
    run_gemm_case(dm, torch, tA, tB, 67, 93, 515, alpha=1.0, beta=0.0, ld_extra=(1, 1, 1), lead=(1, 1, 1),
                  seed=split + 1, c_nan=True)
    run_gemm_case(dm, torch, tA, tB, 64, 128, 512, alpha=1.0, beta=1.0, seed=split + 2, ints=True, exact=True)


def _windowed(torch, mat, ld):
    """mat (rows x cols, numpy) as a window of a device row panel of width ld; the padding is never defined."""
    rows, cols = mat.shape
    flat = torch.empty(rows * ld, dtype=torch.from_numpy(mat).dtype, device="cuda")
    flat.view(rows, ld)[:, :cols] = torch.from_numpy(mat).cuda()
    return flat


@pytest.mark.parametrize("tA,tB", TRANS)
@pytest.mark.parametrize("ld", [1 << 22, (1 << 22) + 4, (1 << 22) + 5])
def test_gemm_block_of_a_very_wide_row_panel(dm, torch, tA, tB, ld):
    """Leading dimensions at and beyond 2^22 elements, where the per-thread byte offsets of the tile loaders
    no longer fit 32 bits and the kernels with 64-bit offsets take over (16-byte and element loads)."""
    M, N, K = 70, 44, 36
    rng = np.random.default_rng(ld % 97 + 2 * tA + tB)
    A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    C0 = rng.standard_normal((M, N)).astype(np.float32)
    As, Bs = (A.T if tA else A).copy(), (B.T if tB else B).copy()
    dA, dB = _windowed(torch, As, ld), _windowed(torch, Bs, ld)
    dC = torch.from_numpy(C0).cuda()
    dm.check(dm.dmath_gemm(tA, tB, M, N, K, 0.5, dA, ld, dB, ld, 2.0, dC, N))
    torch.cuda.synchronize()
    ref, mag = oracle.gemm(tA, tB, M, N, K, 0.5, As, As.shape[1], Bs, Bs.shape[1], 2.0, C0, N)
    check_bound(dC.cpu().numpy(), ref, mag, K, "wide ld %d t%d%d" % (ld, tA, tB))
    # the same product through the panel entry point (it falls back to one call per panel) and in half storage
    dC2 = torch.from_numpy(C0).cuda()
    dm.check(dm.dmath_gemm_panels(tA, tB, M, N, K, 0.5, [dA, dA], ld, [dB, dB], ld, 2.0, dC2, N))
    torch.cuda.synchronize()
    ref2, mag2 = oracle.gemm_panels(tA, tB, M, N, K, 0.5, [As, As], As.shape[1], [Bs, Bs], Bs.shape[1], 2.0, C0, N)
    check_bound(dC2.cpu().numpy(), ref2, mag2, 2 * K, "wide ld panels")
    del dA, dB
    Ah, Bh, Ch = As.astype(np.float16), Bs.astype(np.float16), C0.astype(np.float16)
    dAh, dBh = _windowed(torch, Ah, ld), _windowed(torch, Bh, ld)
    dCh = torch.from_numpy(Ch).cuda()
    dm.check(dm.dmath_hgemm(tA, tB, M, N, K, 1.0, dAh, ld, dBh, ld, 1.0, dCh, N))
    torch.cuda.synchronize()
    refh, magh = oracle.hgemm(tA, tB, M, N, K, 1.0, Ah, Ah.shape[1], Bh, Bh.shape[1], 1.0, Ch, N)
    err = np.abs(dCh.cpu().numpy().astype(np.float64) - refh)
    assert (err <= oracle.half_bound(K, magh, refh)).all()


WAVE_SPLIT = [6]   # configuration indices of the kernels that split K over the waves of a workgroup


@pytest.mark.parametrize("cfg", WAVE_SPLIT)
@pytest.mark.parametrize("tA,tB", TRANS)
def test_gemm_wave_split_k_ranges(dm, torch, cfg, tA, tB):
    """K from less than one K tile (most waves get nothing) through every remainder class of the round
    robin over 8 waves: the partial last tile must land on the wave whose turn it is."""
    assert "wavek" in dm.dmath_config_name(cfg)
    dm.dmath_set_override(cfg, -1)
    for K in (4, 8, 12, 60, 64, 68, 72, 124, 128, 132, 136, 200, 516, 1032):      # 16-byte loads
        run_gemm_case(dm, torch, tA, tB, 72, 132, K, alpha=1.25, beta=0.5, ld_extra=(4, 0, 4), seed=K)
    for K in (1, 7, 9, 63, 65, 127, 129, 135, 137, 515, 1031):                     # element loads
        run_gemm_case(dm, torch, tA, tB, 70, 131, K, alpha=1.0, beta=0.0, ld_extra=(1, 2, 3), lead=(1, 2, 3),
                      seed=K, c_nan=True)
    run_gemm_case(dm, torch, tA, tB, 130, 200, 1096, alpha=1.0, beta=1.0, seed=3, ints=True, exact=True)


def test_gemm_wave_split_is_the_plan_for_skinny_products_and_repeats_its_bits(dm, torch):
    """The fully connected layer's forward and backward-data products get the wave-split kernel by
    themselves (no workspace needed), integer entries come out exact at that launch shape, and two runs
    give the same bits."""
    for tA, tB in ((0, 0), (0, 1)):
        st, cfg, split = dm.dmath_gemm_plan(tA, tB, 256, 4096, 4096)
        assert st == dm.OK and cfg in WAVE_SPLIT and split == 1, (cfg, split)
        assert dm.dmath_gemm_workspace_bytes(tA, tB, 256, 4096, 4096) == 0
        run_gemm_case(dm, torch, tA, tB, 256, 4096, 4096, alpha=1.0, beta=1.0, seed=50 + tB, ints=True, exact=True)
    rng = np.random.default_rng(52)
    A = rng.uniform(-1, 1, (256, 4096)).astype(np.float32)
    B = rng.uniform(-1, 1, (4096, 4096)).astype(np.float32)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    outs = []
    for _ in range(3):
        dC = torch.empty((256, 4096), device="cuda")
        dm.check(dm.dmath_gemm(0, 0, 256, 4096, 4096, 1.0, dA, 4096, dB, 4096, 0.0, dC, 4096))
        torch.cuda.synchronize()
        outs.append(dC.cpu().numpy())
    assert all(np.array_equal(outs[0].view(np.uint32), o.view(np.uint32)) for o in outs[1:])


@pytest.mark.parametrize("tA,tB", [(0, 0), (1, 1)])
def test_gemm_tail_tiles_split(dm, torch, tA, tB):
    """17 x 16 tiles of 128 x 128 on 256 compute units: one full round plus 16 tiles, which the planner
    cuts into K slices combined in-kernel; also the same with ragged edges."""
    st, cfg, split = dm.dmath_gemm_plan(tA, tB, 2176, 2048, 768)
    assert st == dm.OK
    run_gemm_case(dm, torch, tA, tB, 2176, 2048, 768, alpha=1.0, beta=0.0, seed=41, c_nan=True)
    run_gemm_case(dm, torch, tA, tB, 2170, 2044, 771, alpha=0.5, beta=1.0, ld_extra=(2, 4, 4), seed=42)
    dm.dmath_set_override(3, -1)       # fixed 128 x 128 tiles, automatic split: the tail-split plan
    st, cfg, split = dm.dmath_gemm_plan(tA, tB, 2176, 2048, 768)
    assert cfg == 3 and split > 1, (cfg, split)
    run_gemm_case(dm, torch, tA, tB, 2176, 2048, 768, alpha=1.0, beta=1.0, seed=43, ints=True, exact=True)
    outs = []
    for _ in range(2):                 # which slice arrives last may differ between runs; the bits may not
        rng = np.random.default_rng(44)
        A = rng.uniform(-1, 1, (2176, 768)).astype(np.float32)
        B = rng.uniform(-1, 1, (768, 2048)).astype(np.float32)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        dC = torch.empty((2176, 2048), device="cuda")
        dm.check(dm.dmath_gemm(0, 0, 2176, 2048, 768, 1.0, dA, 768, dB, 2048, 0.0, dC, 2048))
        torch.cuda.synchronize()
        outs.append(dC.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


def test_gemm_tail_slices_never_read_stale_partial_sums(dm, torch):
    """The K slices of tail tiles leave their sums in the workspace and the last slice to arrive reads them from
    whichever die it runs on.  Calls with different operands reuse the same workspace addresses back to back, so a
    slice sum served from a cache that still holds the previous call's value would show: integer operands, every
    call bit-exact against the oracle, sizes shrinking and growing so that old sums lie under new ones."""
    dm.dmath_set_override(3, -1)
    shapes = [(2176, 2048, 768), (2176, 2048, 768), (1664, 2688, 768), (2176, 2048, 768), (2304, 2176, 640), (1792, 2560, 1024)]
    for i, (M, N, K) in enumerate(shapes):
        st, cfg, split = dm.dmath_gemm_plan(0, 1, M, N, K)
        assert st == dm.OK and cfg == 3 and split > 1, (M, N, K, cfg, split)   # a split tail
        rng = np.random.default_rng(900 + i)
        A = workloads.small_ints(rng, (M, K))
        B = workloads.small_ints(rng, (N, K))
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        dC = torch.full((M, N), float("nan"), device="cuda")
        for rep in range(2):
            dm.check(dm.dmath_gemm(0, 1, M, N, K, 1.0, dA, K, dB, K, 0.0, dC, N))
        torch.cuda.synchronize()
        ref, _ = oracle.gemm(0, 1, M, N, K, 1.0, A, K, B, K)
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref), (i, M, N, K)


def test_gemm_quick_returns_and_nan_conventions(dm, torch):
    rng = np.random.default_rng(5)
    M, N, K = 70, 50, 40
    C0 = rng.standard_normal((M, N)).astype(np.float32)
    nanA = torch.full((M, K), float("nan"), device="cuda")
    nanB = torch.full((K, N), float("nan"), device="cuda")
    # alpha == 0: A, B not read, C = beta*C
    dC = torch.from_numpy(C0).cuda()
    dm.check(dm.dmath_gemm(0, 0, M, N, K, 0.0, nanA, K, nanB, N, -2.0, dC, N))
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), -2.0 * C0)
    # K == 0, beta == 0: exact zeros even over NaN
    dC = torch.full((M, N), float("nan"), device="cuda")
    dm.check(dm.dmath_gemm(0, 0, M, N, 0, 1.0, None, 1, None, N, 0.0, dC, N))
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), np.zeros((M, N), np.float32))
    # K == 0, beta == 1: untouched; and with a padded C only the M x N window is scaled
    dC = torch.from_numpy(C0).cuda()
    dm.check(dm.dmath_gemm(0, 0, M, N, 0, 1.0, None, 1, None, N, 1.0, dC, N))
    dm.check(dm.dmath_gemm(0, 0, M, N - 10, 0, 1.0, None, 1, None, N, 3.0, dC, N))
    torch.cuda.synchronize()
    want = C0.copy()
    want[:, :N - 10] *= 3.0
    assert np.array_equal(dC.cpu().numpy(), want)
    # empty output
    assert dm.dmath_gemm(0, 0, 0, N, K, 1.0, nanA, K, nanB, N, 0.0, dC, N) == dm.OK


def test_gemm_run_to_run_bits(dm, torch):
    wl = workloads.gemm_square(512, 77, "determinism")
    dA, dB = torch.from_numpy(wl.arrays["A"]).cuda(), torch.from_numpy(wl.arrays["B"]).cuda()
    outs = []
    for cfg, split in [(-1, -1), (-1, -1), (4, 4), (4, 4)]:
        dm.dmath_set_override(cfg, split)
        dC = torch.empty((512, 512), device="cuda")
        dm.check(dm.dmath_gemm(0, 0, 512, 512, 512, 1.0, dA, 512, dB, 512, 0.0, dC, 512))
        torch.cuda.synchronize()
        outs.append(dC.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    assert np.array_equal(outs[2], outs[3])


def test_gemm_on_a_side_stream(dm, torch):
    s = torch.cuda.Stream()
    wl = workloads.gemm_square(256, 3, "stream")
    dA, dB = torch.from_numpy(wl.arrays["A"]).cuda(), torch.from_numpy(wl.arrays["B"]).cuda()
    dC = torch.empty((256, 256), device="cuda")
    torch.cuda.synchronize()
    dm.check(dm.dmath_gemm(0, 0, 256, 256, 256, 1.0, dA, 256, dB, 256, 0.0, dC, 256, stream=s))
    s.synchronize()
    ref, mag = oracle.gemm(0, 0, 256, 256, 256, 1.0, wl.arrays["A"], 256, wl.arrays["B"], 256)
    check_bound(dC.cpu().numpy(), ref, mag, 256, "side stream")


# ------------------------------------------------------------------ the five configurations

def _run_workload(dm, torch, wl):
    dev = {k: torch.from_numpy(v).cuda() for k, v in wl.arrays.items()}
    for c in wl.calls:
        dm.check(dm.dmath_gemm(c.transA, c.transB, c.M, c.N, c.K, c.alpha, dev[c.A], c.lda, dev[c.B], c.ldb,
                               c.beta, dev[c.C], c.ldc))
    torch.cuda.synchronize()
    return {k: dev[k].cpu().numpy() for k in wl.outputs}


def test_config1_gemm_256(dm, torch):
    wl = workloads.config1()
    out = _run_workload(dm, torch, wl)
    c = wl.calls[0]
    ref, mag = oracle.gemm(0, 0, c.M, c.N, c.K, 1.0, wl.arrays["A"], c.lda, wl.arrays["B"], c.ldb)
    r = check_bound(out["C"], ref, mag, c.K, "config 1")
    print("config 1 max err/bound %.3g" % r)


def _sample_rows_cols(rng, M, N, nrows, ncols):
    rows = np.sort(rng.choice(M, size=min(nrows, M), replace=False))
    cols = np.sort(rng.choice(N, size=min(ncols, N), replace=False))
    # always include the corners of the matrix and of the first / last tiles
    rows = np.unique(np.concatenate([rows, [0, 1, M // 2, M - 2, M - 1]]))
    cols = np.unique(np.concatenate([cols, [0, 1, N // 2, N - 2, N - 1]]))
    pi = np.concatenate([np.repeat(rows, N), np.tile(np.arange(M), len(cols))])
    pj = np.concatenate([np.tile(np.arange(N), len(rows)), np.repeat(cols, M)])
    return pi, pj


def test_config2_gemm_4096(dm, torch):
    wl = workloads.config2()
    out = _run_workload(dm, torch, wl)
    c = wl.calls[0]
    pi, pj = _sample_rows_cols(np.random.default_rng(0), c.M, c.N, 24, 24)
    ref, mag = oracle.gemm_points(0, 0, c.M, c.N, c.K, 1.0, wl.arrays["A"], c.lda, wl.arrays["B"], c.ldb,
                                  0.0, None, c.ldc, pi, pj)
    r = check_bound(out["C"][pi, pj], ref, mag, c.K, "config 2 (24+ full rows and columns)")
    print("config 2 max err/bound %.3g" % r)


def test_config2_shape_integer_entries_bit_exact(dm, torch):
    """Same 4096^3 launch, entries in {-4..4}: |sums| <= 65536, so the GPU must match bit for bit."""
    n = 4096
    rng = np.random.default_rng(11)
    A, B = workloads.small_ints(rng, (n, n)), workloads.small_ints(rng, (n, n))
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.empty((n, n), device="cuda")
    dm.check(dm.dmath_gemm(0, 0, n, n, n, 1.0, dA, n, dB, n, 0.0, dC, n))
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    pi, pj = _sample_rows_cols(np.random.default_rng(1), n, n, 16, 16)
    ref, _ = oracle.gemm_points(0, 0, n, n, n, 1.0, A, n, B, n, 0.0, None, n, pi, pj)
    assert np.array_equal(got[pi, pj].astype(np.float64), ref)


def test_config3_summa_chain(dm, torch):
    """16 accumulate steps; the end state is checked against C0 + [A_0..A_15]*[B_0;..;B_15] (K = 8192)."""
    wl = workloads.config3()
    out = _run_workload(dm, torch, wl)
    m, kp, steps = 8192, 512, 16
    Acat = np.ascontiguousarray(np.concatenate([wl.arrays["A%d" % k] for k in range(steps)], axis=1))
    Bcat = np.ascontiguousarray(np.concatenate([wl.arrays["B%d" % k] for k in range(steps)], axis=0))
    pi, pj = _sample_rows_cols(np.random.default_rng(2), m, m, 6, 6)
    ref, mag = oracle.gemm_points(0, 0, m, m, kp * steps, 1.0, Acat, kp * steps, Bcat, m, 1.0, wl.arrays["C"], m,
                                  pi, pj)
    r = check_bound(out["C"][pi, pj], ref, mag, kp * steps, "config 3 chain")
    # The per-step form of the same bound, 16 times tighter: every call rounds a K = 512 product
    # (4*512*2^-24 of its magnitude sum) and rounds C once when it stores it (2^-24 of a value that never
    # exceeds |C0| + sum_k |A_k||B_k|).  A dropped k term (about 0.3 here) or a beta applied twice fails it.
    err = np.abs(out["C"][pi, pj].astype(np.float64) - ref)
    c0 = np.abs(wl.arrays["C"][pi, pj].astype(np.float64))
    mag_ab = mag - c0
    per_step = 4.0 * kp * 2.0 ** -24 * mag_ab + steps * 2.0 ** -24 * (c0 + mag_ab) + 1e-6
    assert (err <= per_step).all(), "config 3 chain outside the per-step bound: %g" % (err / per_step).max()
    print("config 3 max err/contract bound %.3g, max err/per-step bound %.3g, max abs err %.3g"
          % (r, (err / per_step).max(), err.max()))


def test_config4_fc_layer(dm, torch):
    wl = workloads.config4()
    out = _run_workload(dm, torch, wl)
    for c in wl.calls:
        ref, mag = oracle.gemm(c.transA, c.transB, c.M, c.N, c.K, 1.0, wl.arrays[c.A], c.lda, wl.arrays[c.B], c.ldb)
        r = check_bound(out[c.C], ref, mag, c.K, "config 4 %s" % c.C)
        print("config 4 %s max err/bound %.3g" % (c.C, r))


def test_config4_without_workspace(dm, torch):
    """With no scratch registered the skinny products take a path that needs none."""
    ws = dm._test_workspace
    dm.check(dm.dmath_set_workspace(None, 0))
    try:
        wl = workloads.config4(batch=256, width=1024)
        out = _run_workload(dm, torch, wl)
        for c in wl.calls:
            ref, mag = oracle.gemm(c.transA, c.transB, c.M, c.N, c.K, 1.0, wl.arrays[c.A], c.lda, wl.arrays[c.B],
                                   c.ldb)
            check_bound(out[c.C], ref, mag, c.K, "config 4 (no workspace) %s" % c.C)
    finally:
        dm.check(dm.dmath_set_workspace(ws, ws.numel()))


# ------------------------------------------------------------------ convolution

CONV_SMALL = [
    dict(N=2, C=3, H=7, W=5, Kout=4, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=1, C=2, H=9, W=6, Kout=3, R=3, S=2, pad=(0, 0), stride=(2, 2)),
    dict(N=2, C=1, H=8, W=11, Kout=2, R=5, S=3, pad=(2, 1), stride=(2, 3)),
    dict(N=3, C=20, H=14, W=14, Kout=70, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=5, C=16, H=12, W=12, Kout=33, R=1, S=1, pad=(0, 0), stride=(1, 1)),
    dict(N=2, C=7, H=13, W=9, Kout=130, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=1, C=4, H=5, W=5, Kout=6, R=5, S=5, pad=(0, 0), stride=(1, 1)),
]


@pytest.mark.parametrize("shape", CONV_SMALL)
def test_conv_small(dm, torch, shape):
    run_conv_case(dm, torch, seed=shape["H"], **shape)
    run_conv_case(dm, torch, seed=shape["W"], alpha=0.5, beta=-1.5, lead=1, **shape)
    run_conv_case(dm, torch, seed=shape["C"], ints=True, exact=True, beta=1.0, **shape)


@pytest.mark.parametrize("cfg", range(6))
def test_conv_every_config(dm, torch, cfg):
    if cfg >= dm.dmath_num_configs():
        pytest.skip("no such configuration")
    dm.dmath_set_override(cfg, 1)
    run_conv_case(dm, torch, N=3, C=12, H=28, W=28, Kout=72, R=3, S=3, pad=(1, 1), stride=(1, 1), seed=cfg)
    run_conv_case(dm, torch, N=2, C=5, H=11, W=13, Kout=260, R=3, S=3, pad=(1, 1), stride=(2, 1), seed=cfg + 5,
                  alpha=2.0, beta=1.0, lead=3)


CONV_TAP_MAJOR = [
    dict(N=3, C=16, H=9, W=7, Kout=40, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=2, C=32, H=11, W=10, Kout=72, R=5, S=5, pad=(2, 2), stride=(2, 2)),
    dict(N=4, C=48, H=6, W=6, Kout=130, R=1, S=1, pad=(0, 0), stride=(1, 1)),
    dict(N=2, C=64, H=14, W=14, Kout=260, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=1, C=16, H=8, W=9, Kout=8, R=2, S=3, pad=(0, 1), stride=(1, 2)),
]


@pytest.mark.parametrize("shape", CONV_TAP_MAJOR)
def test_conv_tap_major_and_generic_paths(dm, torch, shape):
    """Channel counts that are multiples of the K tile take the tap-major path when a workspace is
    registered (filters re-laid out into it) and the generic path when none is: both must hold."""
    run_conv_case(dm, torch, seed=1, **shape)
    run_conv_case(dm, torch, seed=2, alpha=-1.5, beta=0.5, lead=4, **shape)
    run_conv_case(dm, torch, seed=3, ints=True, exact=True, beta=1.0, **shape)
    for cfg in range(dm.dmath_num_configs()):
        dm.dmath_set_override(cfg, 1)
        run_conv_case(dm, torch, seed=4 + cfg, ints=True, exact=True, **shape)
    dm.dmath_set_override(-1, -1)
    ws = dm._test_workspace
    dm.check(dm.dmath_set_workspace(None, 0))
    try:
        run_conv_case(dm, torch, seed=5, **shape)
        run_conv_case(dm, torch, seed=6, ints=True, exact=True, beta=1.0, **shape)
    finally:
        dm.check(dm.dmath_set_workspace(ws, ws.numel()))


def test_conv_quick_returns(dm, torch):
    y0 = np.arange(2 * 3 * 4 * 4, dtype=np.float32).reshape(2, 3, 4, 4)
    dy = torch.from_numpy(y0).cuda()
    nanx = torch.full((2, 2, 4, 4), float("nan"), device="cuda")
    nanw = torch.full((3, 2, 3, 3), float("nan"), device="cuda")
    dm.check(dm.dmath_conv2d_fwd(2, 2, 4, 4, 3, 3, 3, 1, 1, 1, 1, 0.0, nanx, nanw, 2.0, dy))
    torch.cuda.synchronize()
    assert np.array_equal(dy.cpu().numpy(), 2.0 * y0)
    dm.check(dm.dmath_conv2d_fwd(2, 0, 4, 4, 3, 3, 3, 1, 1, 1, 1, 1.0, None, None, 0.0, dy))
    torch.cuda.synchronize()
    assert np.array_equal(dy.cpu().numpy(), np.zeros_like(y0))


def test_config5_conv_full_size_sampled(dm, torch):
    wl = workloads.config5()
    N, Kout, P, Q = wl.out_shape
    dx, dw = torch.from_numpy(wl.x).cuda(), torch.from_numpy(wl.w).cuda()
    dy = torch.full((N, Kout, P, Q), float("nan"), device="cuda")
    _, C, H, W = wl.x.shape
    dm.check(dm.dmath_conv2d_fwd(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, dx, dw, 0.0, dy))
    torch.cuda.synchronize()
    got = dy.cpu().numpy()
    assert np.isfinite(got).all()
    rng = np.random.default_rng(3)
    total = got.size
    idx = rng.choice(total, size=300000, replace=False)
    # add whole output planes: first and last image / channel, with their borders
    plane = P * Q
    for n, j in [(0, 0), (N - 1, Kout - 1), (N // 2, 129), (1, 255)]:
        base = (n * Kout + j) * plane
        idx = np.concatenate([idx, np.arange(base, base + plane)])
    ref, mag = oracle.conv2d_fwd_points(wl.x, wl.w, idx, pad=wl.pad, stride=wl.stride)
    M, Ng, K = wl.gemm_view
    r = check_bound(got.reshape(-1)[idx], ref, mag, K, "config 5 sampled")
    print("config 5 max err/bound %.3g" % r)


def test_config5_shape_small_batch_every_element(dm, torch):
    wl = workloads.config5(batch=2)
    N, Kout, P, Q = wl.out_shape
    dx, dw = torch.from_numpy(wl.x).cuda(), torch.from_numpy(wl.w).cuda()
    dy = torch.full((N, Kout, P, Q), float("nan"), device="cuda")
    dm.check(dm.dmath_conv2d_fwd(N, 256, 28, 28, Kout, 3, 3, 1, 1, 1, 1, 1.0, dx, dw, 0.0, dy))
    torch.cuda.synchronize()
    ref, mag = oracle.conv2d_fwd(wl.x, wl.w, pad=wl.pad, stride=wl.stride)
    check_bound(dy.cpu().numpy(), ref, mag, 2304, "config 5 shape, batch 2")


# ------------------------------------------------------------------ convolution, backward-data

CONV_BWD_DATA = [
    dict(N=2, C=3, H=7, W=5, Kout=4, R=3, S=3, pad=(1, 1), stride=(1, 1)),       # forward-style path, generic order
    dict(N=1, C=2, H=9, W=6, Kout=3, R=3, S=2, pad=(0, 0), stride=(2, 2)),       # strided gather
    dict(N=2, C=5, H=8, W=11, Kout=2, R=5, S=3, pad=(2, 1), stride=(2, 3)),
    dict(N=3, C=20, H=14, W=14, Kout=32, R=3, S=3, pad=(1, 1), stride=(1, 1)),   # Kout multiple of 16: tap-major
    dict(N=2, C=130, H=9, W=10, Kout=48, R=3, S=3, pad=(1, 1), stride=(1, 1)),
    dict(N=2, C=40, H=6, W=6, Kout=16, R=1, S=1, pad=(1, 1), stride=(1, 1)),     # pad beyond the filter: gather
    dict(N=2, C=33, H=12, W=12, Kout=64, R=3, S=3, pad=(1, 1), stride=(2, 2)),
    dict(N=1, C=4, H=5, W=5, Kout=6, R=5, S=5, pad=(0, 0), stride=(1, 1)),
]


@pytest.mark.parametrize("shape", CONV_BWD_DATA)
def test_conv_bwd_data_small(dm, torch, shape):
    run_conv_bwd_data_case(dm, torch, seed=shape["H"], **shape)
    run_conv_bwd_data_case(dm, torch, seed=shape["W"], alpha=0.5, beta=-1.5, lead=1, **shape)
    run_conv_bwd_data_case(dm, torch, seed=shape["C"], ints=True, exact=True, beta=1.0, **shape)


@pytest.mark.parametrize("cfg", range(6))
def test_conv_bwd_data_every_config(dm, torch, cfg):
    if cfg >= dm.dmath_num_configs():
        pytest.skip("no such configuration")
    dm.dmath_set_override(cfg, 1)
    run_conv_bwd_data_case(dm, torch, N=2, C=72, H=14, W=14, Kout=32, R=3, S=3, pad=(1, 1), stride=(1, 1), seed=cfg,
                           ints=True, exact=True)
    run_conv_bwd_data_case(dm, torch, N=2, C=260, H=11, W=13, Kout=5, R=3, S=3, pad=(1, 1), stride=(2, 1), seed=cfg + 5,
                           alpha=2.0, beta=1.0, lead=3)


def test_conv_bwd_data_needs_a_workspace(dm, torch):
    ws = dm._test_workspace
    dm.check(dm.dmath_set_workspace(None, 0))
    try:
        t = torch.zeros(4096, device="cuda")
        assert dm.dmath_conv2d_bwd_data(1, 2, 4, 4, 3, 3, 3, 1, 1, 1, 1, 1.0, t, t, 0.0, t) == dm.ERR_WORKSPACE
    finally:
        dm.check(dm.dmath_set_workspace(ws, ws.numel()))


def test_config5_shape_bwd_data_full_size_sampled(dm, torch):
    """Data gradient of the config 5 layer: dy 128x256x28x28, w 256x256x3x3 -> dx 128x256x28x28."""
    wl = workloads.config5()
    N, Kout, P, Q = wl.out_shape
    _, C, H, W = wl.x.shape
    rng = np.random.default_rng(7)
    dy = (rng.standard_normal((N, Kout, P, Q)) * 1e-2).astype(np.float32)
    ddy, dw = torch.from_numpy(dy).cuda(), torch.from_numpy(wl.w).cuda()
    ddx = torch.full((N, C, H, W), float("nan"), device="cuda")
    dm.check(dm.dmath_conv2d_bwd_data(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, ddy, dw, 0.0, ddx))
    torch.cuda.synchronize()
    got = ddx.cpu().numpy()
    assert np.isfinite(got).all()
    idx = rng.choice(got.size, size=200000, replace=False)
    plane = H * W
    for n, c in [(0, 0), (N - 1, C - 1), (N // 2, 129)]:
        base = (n * C + c) * plane
        idx = np.concatenate([idx, np.arange(base, base + plane)])
    ref, mag = oracle.conv2d_bwd_data(dy, wl.w, wl.x.shape, pad=wl.pad, stride=wl.stride, idx=idx)
    r = check_bound(got.reshape(-1)[idx], ref, mag, Kout * 9, "config 5 bwd-data sampled")
    print("config 5 bwd-data max err/bound %.3g" % r)


# ------------------------------------------------------------------ convolution, backward-filter

CONV_BWD_FILTER = [
    dict(N=2, C=3, H=7, W=5, Kout=4, R=3, S=3, pad=(1, 1), stride=(1, 1)),       # P*Q = 35: quads straddle images
    dict(N=1, C=2, H=9, W=6, Kout=3, R=3, S=2, pad=(0, 0), stride=(2, 2)),
    dict(N=2, C=5, H=8, W=11, Kout=2, R=5, S=3, pad=(2, 1), stride=(2, 3)),
    dict(N=3, C=20, H=14, W=14, Kout=32, R=3, S=3, pad=(1, 1), stride=(1, 1)),   # P*Q = 196: vector loads of dy
    dict(N=5, C=30, H=9, W=10, Kout=300, R=3, S=3, pad=(1, 1), stride=(1, 1)),   # several row and column tiles
    dict(N=2, C=40, H=6, W=6, Kout=16, R=1, S=1, pad=(1, 1), stride=(1, 1)),     # pad beyond the filter
    dict(N=4, C=33, H=12, W=12, Kout=64, R=3, S=3, pad=(1, 1), stride=(2, 2)),
    dict(N=1, C=4, H=5, W=5, Kout=6, R=5, S=5, pad=(0, 0), stride=(1, 1)),       # one output pixel per image
    dict(N=40, C=8, H=3, W=2, Kout=9, R=2, S=2, pad=(0, 0), stride=(1, 1)),      # images shorter than a K tile
    dict(N=0, C=4, H=5, W=5, Kout=6, R=3, S=3, pad=(1, 1), stride=(1, 1)),       # empty reduction: dw = beta*dw
    dict(N=3, C=21, H=10, W=12, Kout=35, R=3, S=3, pad=(1, 1), stride=(1, 1)),   # Q = 12: quads stay in a row
    dict(N=2, C=18, H=9, W=16, Kout=20, R=5, S=3, pad=(2, 1), stride=(1, 2)),    # Q = 8 with a column stride
    dict(N=7, C=6, H=4, W=4, Kout=10, R=3, S=3, pad=(1, 1), stride=(1, 1)),      # Q = 4: a row per quad
    dict(N=2, C=10, H=5, W=9, Kout=12, R=2, S=2, pad=(0, 0), stride=(3, 1)),     # Q = 8, P*Q = 16 = one K tile
]


@pytest.mark.parametrize("shape", CONV_BWD_FILTER)
def test_conv_bwd_filter_small(dm, torch, shape):
    run_conv_bwd_filter_case(dm, torch, seed=shape["H"], beta=0.25, **shape)
    run_conv_bwd_filter_case(dm, torch, seed=shape["W"], alpha=0.5, beta=-1.5, lead=1, **shape)
    run_conv_bwd_filter_case(dm, torch, seed=shape["C"], ints=True, exact=True, beta=1.0, **shape)
    if shape["N"]:
        run_conv_bwd_filter_case(dm, torch, seed=shape["Kout"], **shape)


@pytest.mark.parametrize("cfg", range(6))
@pytest.mark.parametrize("split", [1, 3])
def test_conv_bwd_filter_every_config(dm, torch, cfg, split):
    if cfg >= dm.dmath_num_configs():
        pytest.skip("no such configuration")
    dm.dmath_set_override(cfg, split)
    if "_l2" in dm.dmath_config_name(cfg):
        t = torch.zeros(4096, device="cuda")
        assert dm.dmath_conv2d_bwd_filter(1, 2, 4, 4, 3, 3, 3, 1, 1, 1, 1, 1.0, t, t, 0.0, t) == dm.ERR_UNSUPPORTED
        return
    run_conv_bwd_filter_case(dm, torch, N=3, C=72, H=14, W=16, Kout=40, R=3, S=3, pad=(1, 1), stride=(1, 1), seed=cfg,
                             ints=True, exact=True)
    run_conv_bwd_filter_case(dm, torch, N=2, C=60, H=11, W=13, Kout=261, R=3, S=3, pad=(1, 1), stride=(2, 1),
                             seed=cfg + 5, alpha=2.0, beta=1.0, lead=3)


def test_conv_bwd_filter_without_workspace(dm, torch):
    ws = dm._test_workspace
    dm.check(dm.dmath_set_workspace(None, 0))
    try:
        run_conv_bwd_filter_case(dm, torch, N=3, C=20, H=14, W=14, Kout=32, R=3, S=3, pad=(1, 1), stride=(1, 1), seed=3)
    finally:
        dm.check(dm.dmath_set_workspace(ws, ws.numel()))


def test_config5_shape_bwd_filter_full_size_sampled(dm, torch):
    """Filter gradient of the config 5 layer: x 128x256x28x28, dy 128x256x28x28 -> dw 256x256x3x3."""
    wl = workloads.config5()
    N, Kout, P, Q = wl.out_shape
    _, C, H, W = wl.x.shape
    rng = np.random.default_rng(11)
    dy = (rng.standard_normal((N, Kout, P, Q)) * 1e-2).astype(np.float32)
    dx, ddy = torch.from_numpy(wl.x).cuda(), torch.from_numpy(dy).cuda()
    ddw = torch.full((Kout, C, 3, 3), float("nan"), device="cuda")
    dm.check(dm.dmath_conv2d_bwd_filter(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, dx, ddy, 0.0, ddw))
    torch.cuda.synchronize()
    got = ddw.cpu().numpy()
    assert np.isfinite(got).all()
    idx = rng.choice(got.size, size=1500, replace=False)
    idx = np.concatenate([idx, np.arange(9 * C), got.size - 1 - np.arange(9 * C)])   # first and last filter rows
    ref, mag = oracle.conv2d_bwd_filter(wl.x, dy, (Kout, C, 3, 3), pad=wl.pad, stride=wl.stride, idx=idx)
    r = check_bound(got.reshape(-1)[idx], ref, mag, N * P * Q, "config 5 bwd-filter sampled")
    print("config 5 bwd-filter max err/bound %.3g" % r)


# ------------------------------------------------------------------ multi-panel update

@pytest.mark.parametrize("tA,tB", TRANS)
def test_gemm_panels_fused_small(dm, torch, tA, tB):
    # K multiple of 16, aligned: the single-launch path; 300 x 260 spans several tiles with ragged edges
    run_gemm_panels_case(dm, torch, tA, tB, 300, 260, 48, 5, seed=1 + 2 * tA + tB, ld_extra=(4, 8, 4))
    run_gemm_panels_case(dm, torch, tA, tB, 300, 260, 16, 7, alpha=-0.5, beta=2.0, seed=7, ld_extra=(0, 0, 4))
    run_gemm_panels_case(dm, torch, tA, tB, 128, 512, 64, 3, ints=True, exact=True, beta=1.0, seed=3)
    run_gemm_panels_case(dm, torch, tA, tB, 64, 64, 32, 40, seed=9)                     # more than one chunk of panels


@pytest.mark.parametrize("tA,tB", TRANS)
def test_gemm_panels_falls_back_to_a_gemm_per_panel(dm, torch, tA, tB):
    run_gemm_panels_case(dm, torch, tA, tB, 45, 37, 19, 4, beta=0.5, seed=2, ld_extra=(1, 3, 2))   # ragged K, odd ld
    run_gemm_panels_case(dm, torch, tA, tB, 64, 64, 32, 3, seed=4, lead=(1, 0, 0))                # unaligned panels
    run_gemm_panels_case(dm, torch, tA, tB, 33, 20, 16, 1, seed=5)


def test_gemm_panels_quick_returns(dm, torch):
    run_gemm_panels_case(dm, torch, 0, 0, 40, 24, 16, 0, beta=0.5, seed=1)      # no panels: C = beta*C
    run_gemm_panels_case(dm, torch, 0, 0, 40, 24, 0, 3, beta=-1.0, seed=2)      # K == 0
    run_gemm_panels_case(dm, torch, 0, 0, 40, 24, 16, 3, alpha=0.0, beta=2.0, seed=3)
    run_gemm_panels_case(dm, torch, 0, 0, 0, 24, 16, 3, seed=4)
    c = torch.zeros(16, device="cuda")
    assert dm.dmath_gemm_panels(0, 0, 4, 4, 16, 1.0, [c, None], 16, [c, c], 4, 0.0, c, 4) == dm.ERR_NULL_PTR
    assert dm.dmath_last_error_arg() == 8
    assert dm.dmath_gemm_panels(0, 0, 4, 4, 16, 1.0, [c], 15, [c], 4, 0.0, c, 4) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 9


@pytest.mark.parametrize("cfg", range(6))
@pytest.mark.parametrize("split", [1, 3])
def test_gemm_panels_every_config(dm, torch, cfg, split):
    if cfg >= dm.dmath_num_configs():
        pytest.skip("no such configuration")
    dm.dmath_set_override(cfg, split)
    run_gemm_panels_case(dm, torch, 0, 0, 270, 520, 32, 6, ints=True, exact=True, beta=1.0, seed=cfg)
    run_gemm_panels_case(dm, torch, 1, 1, 516, 130, 16, 9, alpha=1.5, beta=-1.0, seed=cfg + 10, ld_extra=(4, 4, 0))


def test_gemm_panels_tail_split_and_order_invariance(dm, torch):
    # 17 x 16 = 272 tiles of the 256 x 256 configuration: one full round plus a split tail
    dm.dmath_set_override(2, -1)
    M, N, K, P = 17 * 256, 16 * 256, 64, 4
    rng = np.random.default_rng(12)
    As = [torch.from_numpy(rng.integers(-2, 3, size=(M, K)).astype(np.float32)).cuda() for _ in range(P)]
    Bs = [torch.from_numpy(rng.integers(-2, 3, size=(K, N)).astype(np.float32)).cuda() for _ in range(P)]
    C1 = torch.zeros((M, N), device="cuda")
    C2 = torch.zeros((M, N), device="cuda")
    dm.check(dm.dmath_gemm_panels(0, 0, M, N, K, 1.0, As, K, Bs, N, 0.0, C1, N))
    for p in range(P):
        dm.check(dm.dmath_gemm(0, 0, M, N, K, 1.0, As[p], K, Bs[p], N, 1.0 if p else 0.0, C2, N))
    torch.cuda.synchronize()
    assert torch.equal(C1, C2)          # integer data: exact in any order
    want = sum(a.double() @ b.double() for a, b in zip(As, Bs))
    assert torch.equal(C1.double(), want)


def test_config3_panels_full_size_sampled(dm, torch):
    """Config 3 as one fused call: C(8192 x 8192) += sum of 16 products of 8192 x 512 by 512 x 8192 panels."""
    wl = workloads.config3()
    dev = {k: torch.from_numpy(v).cuda() for k, v in wl.arrays.items()}
    c = wl.calls[0]
    As = [dev[x.A] for x in wl.calls]
    Bs = [dev[x.B] for x in wl.calls]
    dm.check(dm.dmath_gemm_panels(0, 0, c.M, c.N, c.K, 1.0, As, c.lda, Bs, c.ldb, 1.0, dev["C"], c.ldc))
    torch.cuda.synchronize()
    got = dev["C"].cpu().numpy()
    rng = np.random.default_rng(3)
    pi = rng.integers(0, c.M, size=4000)
    pj = rng.integers(0, c.N, size=4000)
    pi[:4], pj[:4] = [0, 0, c.M - 1, c.M - 1], [0, c.N - 1, 0, c.N - 1]
    ref, mag = oracle.gemm_panels(0, 0, c.M, c.N, c.K, 1.0, [wl.arrays[x.A] for x in wl.calls], c.lda,
                                  [wl.arrays[x.B] for x in wl.calls], c.ldb, 1.0, wl.arrays["C"], c.ldc, pi=pi, pj=pj)
    r = check_bound(got[pi, pj], ref, mag, c.K * len(wl.calls), "config 3 fused, sampled")
    print("config 3 fused max err/bound %.3g" % r)


# ------------------------------------------------------------------ half-precision storage

@pytest.mark.parametrize("tA,tB", TRANS)
def test_hgemm_small(dm, torch, tA, tB):
    run_hgemm_case(dm, torch, tA, tB, 300, 260, 150, seed=1 + 2 * tA + tB, ld_extra=(4, 8, 4))          # vector path
    run_hgemm_case(dm, torch, tA, tB, 129, 67, 45, alpha=-0.5, beta=2.0, seed=7, ld_extra=(1, 3, 1))    # scalar path
    run_hgemm_case(dm, torch, tA, tB, 64, 132, 64, seed=9, lead=(1, 2, 3), beta=1.0)                    # 2-byte aligned
    run_hgemm_case(dm, torch, tA, tB, 128, 512, 64, ints=True, exact=True, beta=1.0, seed=3)
    run_hgemm_case(dm, torch, tA, tB, 1, 1, 1, seed=4)
    run_hgemm_case(dm, torch, tA, tB, 33, 20, 0, beta=0.5, seed=5)                                      # K == 0
    run_hgemm_case(dm, torch, tA, tB, 33, 20, 16, alpha=0.0, beta=0.0, seed=6)


@pytest.mark.parametrize("cfg", range(6))
@pytest.mark.parametrize("split", [1, 3])
def test_hgemm_every_config(dm, torch, cfg, split):
    if cfg >= dm.dmath_num_configs():
        pytest.skip("no such configuration")
    dm.dmath_set_override(cfg, split)
    if "_l2" in dm.dmath_config_name(cfg):
        t = torch.zeros(4096, dtype=torch.float16, device="cuda")
        assert dm.dmath_hgemm(0, 0, 16, 16, 16, 1.0, t, 16, t, 16, 0.0, t, 16) == dm.ERR_UNSUPPORTED
        return
    run_hgemm_case(dm, torch, 0, 0, 270, 520, 96, ints=True, exact=True, beta=1.0, seed=cfg)
    run_hgemm_case(dm, torch, 1, 1, 516, 130, 200, alpha=1.5, beta=-1.0, seed=cfg + 10, ld_extra=(4, 4, 0))
    run_hgemm_case(dm, torch, 0, 1, 100, 90, 77, seed=cfg + 20, ld_extra=(1, 1, 1))


def test_hgemm_config4_layer_in_half_storage(dm, torch):
    """The fully connected layer of config 4 with X, W, dY rounded to half and outputs stored as half."""
    wl = workloads.config4()
    half = {k: v.astype(np.float16) for k, v in wl.arrays.items()}
    dev = {k: torch.from_numpy(v).cuda() for k, v in half.items()}
    for c in wl.calls:
        dm.check(dm.dmath_hgemm(c.transA, c.transB, c.M, c.N, c.K, 1.0, dev[c.A], c.lda, dev[c.B], c.ldb, 0.0,
                                dev[c.C], c.ldc))
    torch.cuda.synchronize()
    for c in wl.calls:
        ref, mag = oracle.hgemm(c.transA, c.transB, c.M, c.N, c.K, 1.0, half[c.A], c.lda, half[c.B], c.ldb)
        got = dev[c.C].cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        bnd = oracle.half_bound(c.K, mag, ref)
        assert (err <= bnd).all(), c.C
        print("config 4 half storage %s max err/bound %.3g" % (c.C, (err / bnd).max()))


def test_hgemm_4096_sampled(dm, torch):
    wl = workloads.config2()
    A, B = wl.arrays["A"].astype(np.float16), wl.arrays["B"].astype(np.float16)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.full((4096, 4096), float("nan"), dtype=torch.float16, device="cuda")
    dm.check(dm.dmath_hgemm(0, 0, 4096, 4096, 4096, 1.0, dA, 4096, dB, 4096, 0.0, dC, 4096))
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    assert np.isfinite(got).all()
    rng = np.random.default_rng(2)
    pi = np.concatenate([rng.integers(0, 4096, 20000), np.full(4096, 4095), np.arange(4096)])
    pj = np.concatenate([rng.integers(0, 4096, 20000), np.arange(4096), np.zeros(4096, dtype=np.int64)])
    ref, mag = oracle.hgemm(0, 0, 4096, 4096, 4096, 1.0, A, 4096, B, 4096, pi=pi, pj=pj)
    err = np.abs(got[pi, pj].astype(np.float64) - ref)
    bnd = oracle.half_bound(4096, mag, ref)
    assert (err <= bnd).all()
    print("hgemm 4096 max err/bound %.3g" % (err / bnd).max())


@pytest.mark.parametrize("tA,tB", TRANS)
@pytest.mark.parametrize("K", [32, 64, 96, 128, 160, 192, 224, 256, 288, 320, 384, 448, 512, 640])
@pytest.mark.parametrize("path", [1, 2])
def test_hgemm_fp16_instruction_k_ranges(dm, torch, tA, tB, K, path):
    """The FP16-input matrix-instruction kernels (256 x 256 and 128 x 128 tile; K a multiple of 64: global -> LDS
    loads on the 16x16x32 instruction, else register staging with a K tile of 32) over every prologue / steady /
    drain combination of K tiles."""
    dm.dmath_set_hgemm_path(path)
    run_hgemm_case(dm, torch, tA, tB, 264, 520, K, ints=True, exact=True, beta=1.0, seed=K + tA)
    run_hgemm_case(dm, torch, tA, tB, 264, 520, K, alpha=0.75, beta=-0.5, seed=K + tB, ld_extra=(8, 16, 3))


@pytest.mark.parametrize("tA,tB", TRANS)
@pytest.mark.parametrize("path", [1, 2])
def test_hgemm_fp16_instruction_shapes(dm, torch, tA, tB, path):
    dm.dmath_set_hgemm_path(path)
    m_odd = 37 if tA == 0 else 40          # an operand stored along its own index needs a multiple of 8
    n_odd = 51 if tB == 1 else 56
    run_hgemm_case(dm, torch, tA, tB, m_odd, n_odd, 64, seed=1)
    run_hgemm_case(dm, torch, tA, tB, 1000, 72, 96, beta=2.0, seed=2, ld_extra=(0, 8, 1), lead=(8, 16, 1))
    run_hgemm_case(dm, torch, tA, tB, 8, 8, 32, seed=3)
    run_hgemm_case(dm, torch, tA, tB, 512, 768, 1024, seed=4)
    dm.dmath_set_override(-1, 3)           # forced split-K: FP32 slices in the workspace, reduced in slice order
    run_hgemm_case(dm, torch, tA, tB, 264, 520, 288, ints=True, exact=True, beta=1.0, seed=5)
    run_hgemm_case(dm, torch, tA, tB, 200, 136, 512, alpha=-1.0, beta=0.5, seed=6)
    dm.dmath_set_override(-1, 64)          # more slices than K tiles allow: clamped
    run_hgemm_case(dm, torch, tA, tB, 264, 520, 96, seed=7)


def test_hgemm_fp16_instruction_conditions(dm, torch):
    t = torch.zeros(1 << 16, dtype=torch.float16, device="cuda")
    dm.dmath_set_hgemm_path(1)
    assert dm.dmath_hgemm(0, 0, 64, 64, 48, 1.0, t, 48, t, 64, 0.0, t, 64) == dm.ERR_UNSUPPORTED      # K % 32
    assert dm.dmath_hgemm(0, 0, 64, 60, 64, 1.0, t, 64, t, 64, 0.0, t, 64) == dm.ERR_UNSUPPORTED      # N % 8, B along n
    assert dm.dmath_hgemm(0, 0, 64, 64, 64, 1.0, t[1:], 64, t, 64, 0.0, t, 64) == dm.ERR_UNSUPPORTED  # alignment
    assert dm.dmath_hgemm(0, 0, 64, 64, 64, 1.0, t, 68, t, 64, 0.0, t, 64) == dm.ERR_UNSUPPORTED      # lda % 8
    assert dm.dmath_set_hgemm_path(3) == dm.ERR_INVALID_ARG and dm.dmath_set_hgemm_path(-2) == dm.ERR_INVALID_ARG
    dm.dmath_set_hgemm_path(0)             # the widening kernel takes all of them
    run_hgemm_case(dm, torch, 0, 0, 64, 64, 64, seed=1)
    dm.dmath_set_hgemm_path(-1)
    run_hgemm_case(dm, torch, 0, 0, 64, 60, 48, seed=2)


@pytest.mark.parametrize("K", [320, 352])   # K tile of 64 on the 16x16x32 instruction; K tile of 32 on 32x32x16
def test_hgemm_paths_agree_on_integers(dm, torch, K):
    rng = np.random.default_rng(21)
    M, N = 520, 392
    A = torch.from_numpy(rng.integers(-2, 3, size=(M, K)).astype(np.float16)).cuda()
    B = torch.from_numpy(rng.integers(-2, 3, size=(K, N)).astype(np.float16)).cuda()
    out = []
    for path in (0, 1, 2):
        dm.dmath_set_hgemm_path(path)
        C = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        dm.check(dm.dmath_hgemm(0, 0, M, N, K, 1.0, A, K, B, N, 0.0, C, N))
        out.append(C)
    torch.cuda.synchronize()
    assert all(torch.equal(out[0], o) for o in out[1:])
    assert torch.equal(out[0].double(), A.double() @ B.double())


# ------------------------------------------------------------------ double precision

@pytest.mark.parametrize("tA,tB", TRANS)
@pytest.mark.parametrize("cfg", [0, 1])
def test_dgemm_small(dm, torch, tA, tB, cfg):
    dm.dmath_set_dgemm_config(cfg)
    run_dgemm_case(dm, torch, tA, tB, 300, 260, 150, seed=1 + 2 * tA + tB, ld_extra=(3, 1, 2))      # ragged everything
    run_dgemm_case(dm, torch, tA, tB, 129, 67, 45, alpha=-0.5, beta=2.0, seed=7, lead=(1, 1, 1))      # 8-byte aligned only
    run_dgemm_case(dm, torch, tA, tB, 260, 515, 64, ints=True, exact=True, beta=1.0, seed=3)
    run_dgemm_case(dm, torch, tA, tB, 1, 1, 1, seed=4)
    run_dgemm_case(dm, torch, tA, tB, 17, 9, 5, seed=8)                                             # K below one tile
    run_dgemm_case(dm, torch, tA, tB, 33, 20, 0, beta=0.5, seed=5)                                  # K == 0
    run_dgemm_case(dm, torch, tA, tB, 33, 20, 16, alpha=0.0, beta=0.0, seed=6)
    run_dgemm_case(dm, torch, tA, tB, 0, 20, 16, seed=6)


@pytest.mark.parametrize("K", [16, 32, 48, 64, 80, 100])
def test_dgemm_k_ranges(dm, torch, K):
    run_dgemm_case(dm, torch, 0, 0, 256, 256, K, ints=True, exact=True, seed=K)
    run_dgemm_case(dm, torch, 1, 1, 256, 256, K, beta=-1.0, seed=K + 1)


def test_dgemm_validation(dm, torch):
    t = torch.zeros(64, dtype=torch.float64, device="cuda")
    assert dm.dmath_dgemm(0, 0, 4, 4, 4, 1.0, t, 3, t, 4, 0.0, t, 4) == dm.ERR_INVALID_ARG and dm.dmath_last_error_arg() == 8
    assert dm.dmath_dgemm(0, 0, 4, 4, 4, 1.0, None, 4, t, 4, 0.0, t, 4) == dm.ERR_NULL_PTR and dm.dmath_last_error_arg() == 7
    assert dm.dmath_dgemm(2, 0, 4, 4, 4, 1.0, t, 4, t, 4, 0.0, t, 4) == dm.ERR_INVALID_ARG
    assert dm.dmath_set_dgemm_config(2) == dm.ERR_INVALID_ARG


def test_dgemm_2048_sampled(dm, torch):
    n = 2048
    rng = np.random.default_rng(31)
    A, B = rng.uniform(-1, 1, (n, n)), rng.uniform(-1, 1, (n, n))
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.full((n, n), float("nan"), dtype=torch.float64, device="cuda")
    dm.check(dm.dmath_dgemm(0, 0, n, n, n, 1.0, dA, n, dB, n, 0.0, dC, n))
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    assert np.isfinite(got).all()
    pi = np.concatenate([rng.integers(0, n, 20000), np.full(n, n - 1), np.arange(n)])
    pj = np.concatenate([rng.integers(0, n, 20000), np.arange(n), np.zeros(n, dtype=np.int64)])
    ref, mag = oracle.dgemm(0, 0, n, n, n, 1.0, A, n, B, n, pi=pi, pj=pj)
    err = np.abs(got[pi, pj] - ref)
    bnd = oracle.double_bound(n, mag)
    assert (err <= bnd).all()
    print("dgemm 2048 max err/bound %.3g" % (err / bnd).max())


# ------------------------------------------------------------------ reproducibility and streams, every entry point

def _twice(torch, fn, out):
    """Run fn twice on a NaN-filled output and return both results."""
    res = []
    for _ in range(2):
        out.fill_(float("nan"))
        fn()
        torch.cuda.synchronize()
        res.append(out.clone())
    return res


def test_every_entry_point_is_bit_reproducible(dm, torch):
    """Same call, same data: same bits (no atomics in any reduction; split slices are added in slice order)."""
    g = torch.Generator(device="cuda").manual_seed(5)
    r = lambda *shape, dtype=torch.float32: (torch.rand(shape, device="cuda", generator=g) - 0.5).to(dtype)
    # split-K GEMM (skinny), tail-split GEMM (17 x 16 tiles of 256 x 256)
    A, B, C = r(256, 4096), r(4096, 1024), torch.empty((256, 1024), device="cuda")
    a, b = _twice(torch, lambda: dm.check(dm.dmath_gemm(0, 0, 256, 1024, 4096, 1.0, A, 4096, B, 1024, 0.0, C, 1024)), C)
    assert torch.equal(a, b)
    # multi-panel
    As, Bs, C = [r(512, 64) for _ in range(5)], [r(64, 384) for _ in range(5)], torch.empty((512, 384), device="cuda")
    a, b = _twice(torch, lambda: dm.check(dm.dmath_gemm_panels(0, 0, 512, 384, 64, 1.0, As, 64, Bs, 384, 0.0, C, 384)), C)
    assert torch.equal(a, b)
    # convolution forward (tail split), backward-data, backward-filter (28 slices)
    x, w = r(16, 64, 28, 28), r(64, 64, 3, 3)
    y = torch.empty((16, 64, 28, 28), device="cuda")
    a, b = _twice(torch, lambda: dm.check(dm.dmath_conv2d_fwd(16, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1, 1.0, x, w, 0.0, y)), y)
    assert torch.equal(a, b)
    dx = torch.empty_like(x)
    a, b = _twice(torch, lambda: dm.check(dm.dmath_conv2d_bwd_data(16, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1, 1.0, y, w, 0.0, dx)), dx)
    assert torch.equal(a, b)
    dw = torch.empty_like(w)
    a, b = _twice(torch, lambda: dm.check(dm.dmath_conv2d_bwd_filter(16, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1, 1.0, x, y, 0.0, dw)), dw)
    assert torch.equal(a, b)
    # half storage (FP16-input instruction with split-K) and FP64
    Ah, Bh = r(256, 2048, dtype=torch.float16), r(2048, 512, dtype=torch.float16)
    Ch = torch.empty((256, 512), device="cuda", dtype=torch.float16)
    a, b = _twice(torch, lambda: dm.check(dm.dmath_hgemm(0, 0, 256, 512, 2048, 1.0, Ah, 2048, Bh, 512, 0.0, Ch, 512)), Ch)
    assert torch.equal(a, b)
    Ad, Bd = r(300, 200, dtype=torch.float64), r(200, 260, dtype=torch.float64)
    Cd = torch.empty((300, 260), device="cuda", dtype=torch.float64)
    a, b = _twice(torch, lambda: dm.check(dm.dmath_dgemm(0, 0, 300, 260, 200, 1.0, Ad, 200, Bd, 260, 0.0, Cd, 260)), Cd)
    assert torch.equal(a, b)


def test_other_entry_points_on_a_side_stream(dm, torch):
    """Work goes to the stream that is passed: results are complete after that stream alone is synchronised."""
    s = torch.cuda.Stream()
    rng = np.random.default_rng(77)
    M, N, K = 264, 136, 96
    A, B = rng.integers(-2, 3, size=(M, K)), rng.integers(-2, 3, size=(K, N))
    want = (A @ B).astype(np.float64)
    A16, B16 = (torch.from_numpy(t.astype(np.float16)).cuda() for t in (A, B))
    A64, B64 = (torch.from_numpy(t.astype(np.float64)).cuda() for t in (A, B))
    A32, B32 = (torch.from_numpy(t.astype(np.float32)).cuda() for t in (A, B))
    C16 = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    C64 = torch.zeros((M, N), dtype=torch.float64, device="cuda")
    C32 = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    dm.check(dm.dmath_hgemm(0, 0, M, N, K, 1.0, A16, K, B16, N, 0.0, C16, N, stream=s))
    dm.check(dm.dmath_dgemm(0, 0, M, N, K, 1.0, A64, K, B64, N, 0.0, C64, N, stream=s))
    dm.check(dm.dmath_gemm_panels(0, 0, M, N, K // 2, 1.0, [A32[:, :K // 2], A32[:, K // 2:]], K,
                                  [B32[:K // 2], B32[K // 2:]], N, 0.0, C32, N, stream=s))
    s.synchronize()
    assert np.array_equal(C16.cpu().numpy().astype(np.float64), want)
    assert np.array_equal(C64.cpu().numpy(), want)
    assert np.array_equal(C32.cpu().numpy().astype(np.float64), want)


# ------------------------------------------------------------------ seeded random sweeps of shapes and strides

def _rand_gemm_args(rng, big=False):
    hi = 700 if big else 200
    M, N, K = (int(rng.integers(1, hi)) for _ in range(3))
    tA, tB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
    alpha = float(rng.choice([1.0, -1.0, 0.5, 2.0, 0.0]))
    beta = float(rng.choice([0.0, 1.0, -0.5, 2.0]))
    ld_extra = tuple(int(rng.choice([0, 0, 1, 3, 4, 8])) for _ in range(3))
    lead = tuple(int(rng.choice([0, 0, 0, 1, 2, 4])) for _ in range(3))
    return dict(tA=tA, tB=tB, M=M, N=N, K=K, alpha=alpha, beta=beta, ld_extra=ld_extra, lead=lead)


@pytest.mark.parametrize("seed", range(4))
def test_random_gemm_shapes_every_precision(dm, torch, seed):
    rng = np.random.default_rng(1000 + seed)
    for i in range(12):
        a = _rand_gemm_args(rng, big=(i % 4 == 0))
        run_gemm_case(dm, torch, a["tA"], a["tB"], a["M"], a["N"], a["K"], alpha=a["alpha"], beta=a["beta"],
                      ld_extra=a["ld_extra"], lead=a["lead"], seed=seed * 100 + i, c_nan=(a["beta"] == 0.0))
        run_hgemm_case(dm, torch, a["tA"], a["tB"], a["M"], a["N"], a["K"], alpha=a["alpha"], beta=a["beta"],
                       ld_extra=a["ld_extra"], lead=a["lead"], seed=seed * 100 + i)
        run_dgemm_case(dm, torch, a["tA"], a["tB"], a["M"], a["N"], a["K"], alpha=a["alpha"], beta=a["beta"],
                       ld_extra=a["ld_extra"], lead=a["lead"], seed=seed * 100 + i)


@pytest.mark.parametrize("seed", range(3))
def test_random_hgemm_shapes_on_the_fp16_instruction(dm, torch, seed):
    """Shapes that satisfy the conditions of the FP16-input kernels (multiples of 8, K of 32, aligned)."""
    rng = np.random.default_rng(2000 + seed)
    for i in range(10):
        M, N = 8 * int(rng.integers(1, 90)), 8 * int(rng.integers(1, 90))
        K = 32 * int(rng.integers(1, 20))
        tA, tB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        dm.dmath_set_hgemm_path(int(rng.choice([-1, 1, 2])))
        dm.dmath_set_override(-1, int(rng.choice([-1, -1, 2, 5])))
        run_hgemm_case(dm, torch, tA, tB, M, N, K, alpha=float(rng.choice([1.0, 0.5])), beta=float(rng.choice([0.0, 1.0])),
                       ld_extra=tuple(8 * int(rng.integers(0, 3)) for _ in range(3)),
                       lead=(8 * int(rng.integers(0, 2)), 8 * int(rng.integers(0, 2)), int(rng.integers(0, 3))),
                       seed=seed * 50 + i, ints=(i % 3 == 0), exact=(i % 3 == 0))


@pytest.mark.parametrize("seed", range(3))
def test_random_convolution_shapes_forward_and_gradients(dm, torch, seed):
    rng = np.random.default_rng(3000 + seed)
    for i in range(8):
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        pad = (int(rng.integers(0, R)), int(rng.integers(0, S)))
        stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        H = int(rng.integers(max(1, R - 2 * pad[0]), 20))
        W = int(rng.integers(max(1, S - 2 * pad[1]), 20))
        shape = dict(N=int(rng.integers(1, 5)), C=int(rng.choice([1, 3, 16, 20, 32])), H=H, W=W,
                     Kout=int(rng.choice([1, 5, 16, 40])), R=R, S=S, pad=pad, stride=stride)
        alpha, beta = float(rng.choice([1.0, 0.5])), float(rng.choice([0.0, 1.0, -2.0]))
        run_conv_case(dm, torch, alpha=alpha, beta=beta, seed=seed * 40 + i, lead=int(rng.integers(0, 3)), **shape)
        run_conv_bwd_data_case(dm, torch, alpha=alpha, beta=beta, seed=seed * 40 + i, lead=int(rng.integers(0, 3)), **shape)
        run_conv_bwd_filter_case(dm, torch, alpha=alpha, beta=beta, seed=seed * 40 + i, lead=int(rng.integers(0, 3)), **shape)


@pytest.mark.parametrize("seed", range(2))
def test_random_panel_lists(dm, torch, seed):
    rng = np.random.default_rng(4000 + seed)
    for i in range(8):
        M, N = int(rng.integers(1, 300)), int(rng.integers(1, 300))
        K = int(rng.choice([16, 32, 48, 7, 20]))
        P = int(rng.integers(1, 9))
        if i % 2 == 0:      # the fused path needs multiples of 4 where operands run along their own index
            M, N = 4 * (M // 4 + 1), 4 * (N // 4 + 1)
        run_gemm_panels_case(dm, torch, int(rng.integers(0, 2)), int(rng.integers(0, 2)), M, N, K, P,
                             alpha=float(rng.choice([1.0, -0.5])), beta=float(rng.choice([0.0, 1.0])),
                             ld_extra=tuple(4 * int(rng.integers(0, 2)) for _ in range(3)), seed=seed * 30 + i)


# ------------------------------------------------------------------ operands beyond 2^31 elements

def _sub_check(torch, gpu_sub, A_rows, B_cols, K, alpha, beta, C0_sub, what, kind="f32"):
    """The sums at the sampled rows x sampled columns form a small product of their own: the rows of op(A)
    and the columns of op(B) go to the oracle as that product's operands."""
    A_rows = np.ascontiguousarray(A_rows)
    B_cols = np.ascontiguousarray(B_cols)
    m, n = A_rows.shape[0], B_cols.shape[1]
    C0 = None if C0_sub is None else np.ascontiguousarray(C0_sub)
    if kind == "f16":
        ref, mag = oracle.hgemm(0, 0, m, n, K, alpha, A_rows, K, B_cols, n, beta=beta, C0=C0, ldc=n)
        err = np.abs(gpu_sub.astype(np.float64) - ref)
        assert (err <= oracle.half_bound(K, mag, ref)).all(), what
    elif kind == "f64":
        ref, mag = oracle.dgemm(0, 0, m, n, K, alpha, A_rows, K, B_cols, n, beta=beta, C0=C0, ldc=n)
        err = np.abs(gpu_sub.astype(np.float64) - ref)
        assert (err <= oracle.double_bound(K, mag)).all(), what
    else:
        ref, mag = oracle.gemm(0, 0, m, n, K, alpha, A_rows, K, B_cols, n, beta=beta, C0=C0, ldc=n)
        check_bound(gpu_sub, ref, mag, K, what)


def _uniform(torch, shape, seed, dtype):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    t = torch.rand(shape, generator=g, device="cuda", dtype=torch.float32 if dtype == torch.float16 else dtype)
    t.mul_(2.0).sub_(1.0)
    return t.to(dtype) if dtype == torch.float16 else t


def test_gemm_output_beyond_2_31_elements(dm, torch):
    """C of 49152 x 49152 (9.7 GB): element offsets of its last rows do not fit 31 bits.  K is short, beta = 1:
    the epilogue's addressing, read and write, is what this checks; rows on both sides of offset 2^31."""
    n, K = 49152, 64
    A = _uniform(torch, (n, K), 11, torch.float32)
    B = _uniform(torch, (K, n), 12, torch.float32)
    C = _uniform(torch, (n, n), 13, torch.float32)
    rows = torch.tensor([0, 1, 255, 256, 43689, 43690, 43691, 43692, 49150, 49151], device="cuda")
    cols = torch.tensor([0, 1, 127, 128, 32767, 32768, 40000, 49150, 49151], device="cuda")
    C0 = C[rows][:, cols].cpu().numpy()
    checksum_rows = torch.tensor([2, 30000, 45000], device="cuda")
    before = C[checksum_rows].double().sum(dim=1).cpu().numpy()
    dm.check(dm.dmath_gemm(0, 0, n, n, K, 0.5, A, K, B, n, 1.0, C, n))
    torch.cuda.synchronize()
    got = C[rows][:, cols].cpu().numpy()
    _sub_check(torch, got, A[rows].cpu().numpy(), B[:, cols].cpu().numpy(), K, 0.5, 1.0, C0, "C beyond 2^31")
    # rows that are not sampled changed too (each by 0.5 * sum over the row of A_i . B): not left untouched
    after = C[checksum_rows].double().sum(dim=1).cpu().numpy()
    want = 0.5 * (A[checksum_rows].double() @ B.double().sum(dim=1)).cpu().numpy()
    assert np.allclose(after - before, want, rtol=0, atol=1e-2)


@pytest.mark.parametrize("tA", [0, 1])
def test_gemm_operand_beyond_2_31_elements(dm, torch, tA):
    """A of 40960 x 65536 (10.7 GB; stored transposed for tA = 1): rows past 32768 start beyond element 2^31.
    Long K, so the plan splits it; N is small."""
    M, K, N = 40960, 65536, 256
    A = _uniform(torch, (K, M) if tA else (M, K), 21 + tA, torch.float32)
    B = _uniform(torch, (K, N), 23, torch.float32)
    C = torch.full((M, N), float("nan"), device="cuda")
    dm.check(dm.dmath_gemm(tA, 0, M, N, K, 1.0, A, A.shape[1], B, N, 0.0, C, N))
    torch.cuda.synchronize()
    rows = torch.tensor([0, 255, 32767, 32768, 32769, 40000, 40959], device="cuda")
    A_rows = (A[:, rows].t() if tA else A[rows]).contiguous().cpu().numpy()
    assert not torch.isnan(C).any()
    _sub_check(torch, C[rows].cpu().numpy(), A_rows, B.cpu().numpy(), K, 1.0, 0.0, None, "A beyond 2^31, tA=%d" % tA)


@pytest.mark.parametrize("tA", [0, 1])
def test_hgemm_operand_beyond_2_31_elements(dm, torch, tA):
    """The same for half storage (FP16-input kernels with global -> LDS loads)."""
    M, K, N = 40960, 65536, 256
    A = _uniform(torch, (K, M) if tA else (M, K), 31 + tA, torch.float16)
    B = _uniform(torch, (K, N), 33, torch.float16)
    C = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float16)
    dm.check(dm.dmath_hgemm(tA, 0, M, N, K, 1.0, A, A.shape[1], B, N, 0.0, C, N))
    torch.cuda.synchronize()
    rows = torch.tensor([0, 255, 32767, 32768, 32769, 40000, 40959], device="cuda")
    A_rows = (A[:, rows].t() if tA else A[rows]).contiguous().cpu().numpy()
    assert not torch.isnan(C).any()
    _sub_check(torch, C[rows].cpu().numpy(), A_rows, B.cpu().numpy(), K, 1.0, 0.0, None, "half A beyond 2^31, tA=%d" % tA,
               kind="f16")


def test_dgemm_operand_beyond_2_31_elements(dm, torch):
    """FP64: A of 36864 x 65536 (19.3 GB)."""
    M, K, N = 36864, 65536, 128
    A = _uniform(torch, (M, K), 41, torch.float64)
    B = _uniform(torch, (K, N), 42, torch.float64)
    C = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float64)
    dm.check(dm.dmath_dgemm(0, 0, M, N, K, 1.0, A, K, B, N, 0.0, C, N))
    torch.cuda.synchronize()
    rows = torch.tensor([0, 255, 32767, 32768, 32769, 36863], device="cuda")
    assert not torch.isnan(C).any()
    _sub_check(torch, C[rows].cpu().numpy(), A[rows].cpu().numpy(), B.cpu().numpy(), K, 1.0, 0.0, None, "FP64 A beyond 2^31",
               kind="f64")


@pytest.mark.parametrize("n", [6144, 16384])
def test_paper_table_sizes_sampled(dm, torch, n):
    """Sizes of the paper's table "Matrix Multiplication Performance" beyond config 2, in the launch bench.py
    times for `--workload square`: sampled rows x sampled columns against the oracle."""
    A = _uniform(torch, (n, n), n, torch.float32)
    B = _uniform(torch, (n, n), n + 1, torch.float32)
    C = torch.full((n, n), float("nan"), device="cuda")
    dm.check(dm.dmath_gemm(0, 0, n, n, n, 1.0, A, n, B, n, 0.0, C, n))
    torch.cuda.synchronize()
    rng = np.random.default_rng(n)
    rows = torch.from_numpy(np.unique(np.concatenate([[0, 255, 256, n - 1], rng.integers(0, n, 28)]))).cuda()
    cols = torch.from_numpy(np.unique(np.concatenate([[0, 127, 128, n - 1], rng.integers(0, n, 28)]))).cuda()
    assert not torch.isnan(C).any()
    _sub_check(torch, C[rows][:, cols].cpu().numpy(), A[rows].cpu().numpy(), B[:, cols].cpu().numpy(), n, 1.0, 0.0, None,
               "table size %d" % n)


@pytest.mark.parametrize("tA,tB", TRANS)
@pytest.mark.parametrize("path", [1, 2])
def test_hgemm_epilogue_through_lds(dm, torch, tA, tB, path):
    """16-byte aligned C with ldc a multiple of 8 and tiles wholly inside C: the 16x16x32 kernel stages the tile in LDS
    and stores whole row pieces (beta == 0: rounded halves; beta != 0: FP32 values, old halves added on the way out).
    520 columns leave a ragged tile column on the other path."""
    dm.dmath_set_hgemm_path(path)
    run_hgemm_case(dm, torch, tA, tB, 512, 768, 192, ints=True, exact=True, seed=11 + path)
    run_hgemm_case(dm, torch, tA, tB, 512, 520, 128, alpha=-1.5, seed=12 + path, ld_extra=(8, 8, 8))
    run_hgemm_case(dm, torch, tA, tB, 264, 512, 64, seed=13 + path, ld_extra=(0, 0, 16), lead=(0, 0, 8))
    # beta != 0 on the same tiles: FP32 values staged block row by block row, old halves added, rounded once
    run_hgemm_case(dm, torch, tA, tB, 512, 768, 192, ints=True, exact=True, beta=1.0, seed=14 + path)
    run_hgemm_case(dm, torch, tA, tB, 512, 520, 128, alpha=0.75, beta=-0.5, seed=15 + path, ld_extra=(8, 8, 8))
    run_hgemm_case(dm, torch, tA, tB, 264, 512, 256, alpha=1.0, beta=2.0, seed=16 + path, ld_extra=(0, 0, 16), lead=(0, 0, 8))


@pytest.mark.parametrize("tA,tB", TRANS)
@pytest.mark.parametrize("cfg", [0, 1])
def test_dgemm_split_k(dm, torch, tA, tB, cfg):
    """FP64 products with few tiles are cut into K slices (FP64 slice arrays in the workspace, added in slice order):
    automatic and forced split factors, ragged K, beta != 0, and the unsplit fallback without a workspace."""
    dm.dmath_set_dgemm_config(cfg)
    run_dgemm_case(dm, torch, tA, tB, 130, 264, 1000, alpha=1.25, beta=0.5, seed=1)            # automatic: several slices
    run_dgemm_case(dm, torch, tA, tB, 260, 136, 512, ints=True, exact=True, beta=1.0, seed=2)
    for split in (2, 3, 64):
        dm.dmath_set_override(-1, split)
        run_dgemm_case(dm, torch, tA, tB, 67, 93, 515, seed=split, lead=(1, 1, 1))
        run_dgemm_case(dm, torch, tA, tB, 256, 128, 768, ints=True, exact=True, beta=1.0, seed=split + 10)
    dm.dmath_set_override(-1, -1)
    assert dm.dmath_dgemm_workspace_bytes(tA, tB, 130, 264, 1000) > 0
    assert dm.dmath_dgemm_workspace_bytes(tA, tB, 4096, 4096, 4096) == 0
    ws = dm._test_workspace
    try:
        dm.check(dm.dmath_set_workspace(None, 0))                                               # no room: runs unsplit
        run_dgemm_case(dm, torch, tA, tB, 130, 264, 1000, alpha=-1.0, beta=2.0, seed=3)
    finally:
        dm.check(dm.dmath_set_workspace(ws, ws.numel()))


def test_calls_can_be_captured_in_a_graph(dm, torch):
    """The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, counters cleared
    by a kernel): a fully connected layer's three products (split-K slices and their reduction included) captured
    in a HIP graph replay to the bits of the eager calls, on every replay, with eager work in between."""
    rng = np.random.default_rng(77)
    X = torch.from_numpy(rng.standard_normal((256, 1024)).astype(np.float32)).cuda()
    W = torch.from_numpy((0.01 * rng.standard_normal((1024, 1024))).astype(np.float32)).cuda()
    dY = torch.from_numpy((1e-3 * rng.standard_normal((256, 1024))).astype(np.float32)).cuda()
    Y, dX, dW = (torch.zeros((256, 1024), device="cuda"), torch.zeros((256, 1024), device="cuda"),
                 torch.zeros((1024, 1024), device="cuda"))

    def layer():
        dm.check(dm.dmath_gemm(0, 0, 256, 1024, 1024, 1.0, X, 1024, W, 1024, 0.0, Y, 1024))
        dm.check(dm.dmath_gemm(0, 1, 256, 1024, 1024, 1.0, dY, 1024, W, 1024, 0.0, dX, 1024))
        dm.check(dm.dmath_gemm(1, 0, 1024, 1024, 256, 1.0, X, 1024, dY, 1024, 0.0, dW, 1024))

    layer()
    torch.cuda.synchronize()
    want = [t.clone() for t in (Y, dX, dW)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer()
    for replay in range(3):
        for t in (Y, dX, dW):
            t.fill_(float("nan"))                 # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((Y, dX, dW), want, ("Y", "dX", "dW")):
            assert torch.equal(got, ref), "replay %d: %s differs from the eager result" % (replay, name)
