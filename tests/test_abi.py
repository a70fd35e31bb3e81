"""CPU-side checks of the C-ABI library: it loads, exports every symbol include/dmath.h declares,
and rejects bad arguments before anything is launched (no GPU needed for any call here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dm():
    from paper_1604_01416_amd import build
    build.build(force=False)
    from paper_1604_01416_amd import dmath
    return dmath


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dmath.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dmath_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(dm):
    names = _declared_functions()
    assert "dmath_gemm" in names and "dmath_conv2d_fwd" in names and len(names) >= 10
    lib = ctypes.CDLL(dm.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(dm.EXPORTS) == names


def test_version_and_strings(dm):
    assert "gfx950" in dm.dmath_version()
    assert dm.dmath_status_string(dm.OK) == "ok"
    assert dm.dmath_num_configs() >= 1
    assert dm.dmath_config_name(0)
    assert dm.dmath_config_name(dm.dmath_num_configs()) is None


def test_gemm_argument_validation(dm):
    g = dm.dmath_gemm
    fake = 4096  # never dereferenced: every call below fails validation or returns early
    assert g(2, 0, 4, 4, 4, 1.0, fake, 4, fake, 4, 0.0, fake, 4, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 1
    assert g(0, 7, 4, 4, 4, 1.0, fake, 4, fake, 4, 0.0, fake, 4, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 2
    assert g(0, 0, -1, 4, 4, 1.0, fake, 4, fake, 4, 0.0, fake, 4, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 3
    assert g(0, 0, 4, -1, 4, 1.0, fake, 4, fake, 4, 0.0, fake, 4, stream=0) == dm.ERR_INVALID_ARG
    assert g(0, 0, 4, 4, -1, 1.0, fake, 4, fake, 4, 0.0, fake, 4, stream=0) == dm.ERR_INVALID_ARG
    # leading dimensions: NN needs lda >= K, ldb >= N, ldc >= N
    assert g(0, 0, 4, 5, 6, 1.0, fake, 5, fake, 5, 0.0, fake, 5, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 8
    assert g(0, 0, 4, 5, 6, 1.0, fake, 6, fake, 4, 0.0, fake, 5, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 10
    assert g(0, 0, 4, 5, 6, 1.0, fake, 6, fake, 5, 0.0, fake, 4, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 13
    # transposed: A stored K x M needs lda >= M, B stored N x K needs ldb >= K
    assert g(1, 1, 4, 5, 6, 1.0, fake, 3, fake, 6, 0.0, fake, 5, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 8
    assert g(1, 1, 4, 5, 6, 1.0, fake, 4, fake, 5, 0.0, fake, 5, stream=0) == dm.ERR_INVALID_ARG
    assert dm.dmath_last_error_arg() == 10
    # null pointers
    assert g(0, 0, 4, 4, 4, 1.0, None, 4, fake, 4, 0.0, fake, 4, stream=0) == dm.ERR_NULL_PTR
    assert dm.dmath_last_error_arg() == 7
    assert g(0, 0, 4, 4, 4, 1.0, fake, 4, None, 4, 0.0, fake, 4, stream=0) == dm.ERR_NULL_PTR
    assert g(0, 0, 4, 4, 4, 1.0, fake, 4, fake, 4, 0.0, None, 4, stream=0) == dm.ERR_NULL_PTR
    assert dm.dmath_last_error_arg() == 12
    # empty output: nothing to do, even with null pointers
    assert g(0, 0, 0, 4, 4, 1.0, None, 4, None, 4, 0.0, None, 4, stream=0) == dm.OK
    assert g(0, 0, 4, 0, 4, 1.0, None, 4, None, 1, 0.0, None, 1, stream=0) == dm.OK
    # K == 0 with beta == 1 leaves C alone and needs neither A nor B
    assert g(0, 0, 4, 4, 0, 1.0, None, 1, None, 4, 1.0, fake, 4, stream=0) == dm.OK


def test_conv_argument_validation(dm):
    c = dm.dmath_conv2d_fwd
    fake = 4096
    ok_args = [1, 2, 5, 5, 3, 3, 3, 1, 1, 1, 1]
    for pos, bad in [(0, -1), (1, -1), (2, -1), (3, -1), (4, -1), (5, 0), (6, 0), (7, -1), (8, -1), (9, 0), (10, 0)]:
        args = list(ok_args)
        args[pos] = bad
        assert c(*args, 1.0, fake, fake, 0.0, fake, stream=0) == dm.ERR_INVALID_ARG, pos
        assert dm.dmath_last_error_arg() == pos + 1
    # filter larger than the padded input
    assert c(1, 2, 2, 5, 3, 5, 3, 1, 1, 1, 1, 1.0, fake, fake, 0.0, fake, stream=0) == dm.ERR_INVALID_ARG
    assert c(*ok_args, 1.0, None, fake, 0.0, fake, stream=0) == dm.ERR_NULL_PTR
    assert dm.dmath_last_error_arg() == 13
    assert c(*ok_args, 1.0, fake, None, 0.0, fake, stream=0) == dm.ERR_NULL_PTR
    assert c(*ok_args, 1.0, fake, fake, 0.0, None, stream=0) == dm.ERR_NULL_PTR
    assert dm.dmath_last_error_arg() == 16
    # empty batch: no-op
    assert c(0, 2, 5, 5, 3, 3, 3, 1, 1, 1, 1, 1.0, None, None, 0.0, None, stream=0) == dm.OK


def test_workspace_and_override_api(dm):
    assert dm.dmath_set_workspace(None, 16) == dm.ERR_WORKSPACE
    assert dm.dmath_set_workspace(4100, 64) == dm.ERR_WORKSPACE      # not 16-byte aligned
    assert dm.dmath_set_workspace(None, 0) == dm.OK
    assert dm.dmath_gemm_workspace_bytes(0, 0, 0, 4, 4) == 0
    big = dm.dmath_gemm_workspace_bytes(0, 0, 4096, 4096, 4096)
    assert big == 0                                                  # enough tiles: no split-K
    assert dm.dmath_gemm_workspace_bytes(0, 0, 256, 4096, 4096) == 0 # K is split inside the workgroups
    skinny = dm.dmath_gemm_workspace_bytes(0, 0, 128, 2048, 4096)    # too few tiles for that: slices
    assert skinny >= 2 * 128 * 2048 * 4                              # at least two slices of the output
    assert dm.dmath_set_override(dm.dmath_num_configs(), 1) == dm.ERR_INVALID_ARG
    assert dm.dmath_set_override(0, 0) == dm.ERR_INVALID_ARG
    assert dm.dmath_set_override(0, 4) == dm.OK
    forced = dm.dmath_gemm_workspace_bytes(0, 0, 256, 4096, 4096)
    assert 4 * 256 * 4096 * 4 <= forced <= 4 * 256 * 4096 * 4 + 4096  # 4 slices of every tile + counters
    assert dm.dmath_set_override(-1, -1) == dm.OK


def test_plans_over_random_shapes_are_stable_and_bounded(dm):
    """Host logic of the plan choice: every shape gets a valid configuration, asking twice (the second answer
    comes from the per-thread plan cache) and asking again after other shapes gives the same plan, a forced
    configuration is honoured and forgotten again, and split tails stay at two slices per compute unit."""
    import numpy as np
    rng = np.random.default_rng(11)
    ncfg = dm.dmath_num_configs()
    tile = {0: (256, 128), 1: (128, 256), 2: (256, 256), 3: (128, 128), 4: (64, 64), 5: (256, 256), 6: (64, 64)}
    shapes = [(int(2 ** rng.uniform(3, 14)), int(2 ** rng.uniform(3, 14)), int(2 ** rng.uniform(3, 15))) for _ in range(300)]
    first = {}
    for (M, N, K) in shapes:
        st, cfg, split = dm.dmath_gemm_plan(0, 0, M, N, K)
        assert st == dm.OK and 0 <= cfg < ncfg and 1 <= split <= 64, (M, N, K, cfg, split)
        assert dm.dmath_gemm_plan(0, 0, M, N, K) == (st, cfg, split)
        first[(M, N, K)] = (cfg, split)
        need = dm.dmath_gemm_workspace_bytes(0, 0, M, N, K)
        if cfg == 6:
            assert need == 0 and split == 1          # K is split inside the workgroups
    # without a workspace nothing may be split across workgroups ...
    assert all(s == 1 for (_, s) in first.values())
    # ... and with the room a plan asks for, a split tail is never more than two slices per compute unit
    for (M, N, K) in shapes:
        need = dm.dmath_gemm_workspace_bytes(0, 0, M, N, K)
        if need == 0:
            continue
        assert dm.dmath_set_workspace(1 << 20, need) == dm.OK      # any aligned address: nothing is launched here
        st, cfg, split = dm.dmath_gemm_plan(0, 0, M, N, K)
        assert st == dm.OK and split >= 2 and cfg != 6, (M, N, K, cfg, split)
        bm, bn = tile[cfg]
        tiles = -(-M // bm) * -(-N // bn)
        if tiles > 256 and need < split * M * N * 4:             # only the tail is split
            assert (tiles - tiles // 256 * 256) * split <= 512, (M, N, K, cfg, split, tiles)
        assert dm.dmath_set_workspace(None, 0) == dm.OK
    for (M, N, K) in shapes[:50]:                              # the cache keeps forced and automatic plans apart
        assert dm.dmath_set_override(3, -1) == dm.OK
        assert dm.dmath_gemm_plan(0, 0, M, N, K)[1] == 3
        assert dm.dmath_set_override(-1, -1) == dm.OK
        st, cfg, split = dm.dmath_gemm_plan(0, 0, M, N, K)
        assert (cfg, split) == first[(M, N, K)], (M, N, K)


def test_hgemm_workspace_query_is_host_side_only():
    from paper_1604_01416_amd import dmath as dm
    assert dm.dmath_hgemm_workspace_bytes(0, 0, 0, 16, 16) == 0
    # a ragged K rules the FP16-input kernels out: the widening kernels plan like dmath_gemm
    assert dm.dmath_hgemm_workspace_bytes(0, 0, 256, 4096, 4090) == dm.dmath_gemm_workspace_bytes(0, 0, 256, 4096, 4090)
    # skinny product: FP32 slices of the whole output, a whole number of them
    need = dm.dmath_hgemm_workspace_bytes(0, 0, 256, 4096, 4096)
    assert need > 0 and need % (256 * 4096 * 4) == 0
    assert dm.dmath_hgemm_workspace_bytes(0, 0, 8192, 8192, 8192) == dm.dmath_gemm_workspace_bytes(0, 0, 8192, 8192, 8192)


def test_dgemm_workspace_query_is_host_side_only():
    from paper_1604_01416_amd import dmath as dm
    assert dm.dmath_dgemm_workspace_bytes(0, 0, 0, 16, 16) == 0
    assert dm.dmath_dgemm_workspace_bytes(0, 0, 4096, 4096, 4096) == 0          # enough tiles: no split
    need = dm.dmath_dgemm_workspace_bytes(0, 0, 1024, 1024, 4096)               # 64 tiles: FP64 slices of the whole output
    assert need > 0 and need % (1024 * 1024 * 8) == 0
    assert dm.dmath_dgemm_workspace_bytes(1, 1, 1024, 1024, 64) == 0            # K too short to cut
