// One launch for a whole sequence of accumulating block products
//
//     C = alpha * sum_p op(A_p)[M x K] * op(B_p)[K x N] + beta * C
//
// (the per-stage updates of one C block in the paper's distributed multiply, section "Matrix
// Multiplication", when all the blocks are already resident: the cached-block case of section
// "Memory Management").  The C tile stays in the accumulators over all panels, so C is read and
// written once instead of once per panel.  To the K loop the panels are one long K range: the loaders
// walk a panel tile by tile and jump to the next panel's base pointer at its end, without draining
// the load pipeline.  Needs K to be a multiple of the K tile (no ragged tile in the middle of the sum).
#pragma once
#include "gemm_kernel.h"

namespace dmath {

constexpr int kMaxPanels = 32;  // panels per launch; longer lists are run in chunks

struct GemmPanelArgs {
    GemmArgs g;  // g.A and g.B are unused; g.K is the total npanels * (K of one panel)
    int npanels;
    int tiles_per_panel;  // K of one panel / BK
    const float *A[kMaxPanels];
    const float *B[kMaxPanels];
};

// Wraps a GEMM operand loader: same pieces, but advance() moves to the next panel when the current
// one is used up.  `origin` is the byte offset of this tile row/column inside any panel.
template <class L, int BK>
struct PanelWalker {
    static constexpr int NLOAD = L::NLOAD, NSTORE = L::NSTORE;
    L l;
    const float *const *bases;
    int64_t origin;
    int p, np, left, per;

    __device__ __forceinline__ void init(const float *const *bases_, int np_, int per_, int64_t ld, int64_t r0,
                                         int64_t R, int kt0, int tid)
    {
        bases = bases_;
        np = np_;
        per = per_;
        p = kt0 / per;
        const int tin = kt0 - p * per;
        left = per - tin;
        const int pc = p < np ? p : np - 1;  // a slice without tiles may start past the last panel
        const float *base = bases[pc];
        l.init(base, ld, r0, R, (int64_t)tin * BK, tid);
        origin = (l.tile - reinterpret_cast<const char *>(base)) - L::k_bytes((int64_t)tin * BK, ld);
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        l.template load_piece<I>();
    }
    __device__ __forceinline__ void advance()
    {
        l.advance();
        if (--left == 0) {
            left = per;
            if (++p < np) l.tile = reinterpret_cast<const char *>(bases[p]) + origin;
        }
    }
    template <int I>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        l.template store_piece<I>(S);
    }
    __device__ __forceinline__ void load_tail(int krem) { l.load_tail(krem); }
};

template <class Cfg, bool A_KCONTIG, bool B_KCONTIG>
__global__ __launch_bounds__(Cfg::NT, Cfg::MIN_WAVES) void gemm_panels_tile_kernel(const GemmPanelArgs a)
{
    __shared__ __attribute__((aligned(16))) float smem[Cfg::STAGES * Cfg::STAGE_FLOATS];
    const GemmArgs &g = a.g;

    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 0] = __builtin_readcyclecounter();
        g.clock_probe[blockIdx.x * 4 + 1] = __builtin_amdgcn_s_memrealtime();
    }
    const int tiles = g.tiles_m * g.tiles_n;
    const WorkItem w = work_item(blockIdx.x, tiles, g.split);
    int tm, tn;
    tile_coords<8>(w.tile, g.tiles_m, g.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * Cfg::BM, n0 = (int64_t)tn * Cfg::BN;

    int kt0, T, krem;
    slice_range(a.npanels * a.tiles_per_panel, 0, w.slice, w.nslice, kt0, T, krem);

    PanelWalker<typename RowLoaderSel<Cfg, A_KCONTIG, true>::type, Cfg::BK> rl;
    PanelWalker<typename ColLoaderSel<Cfg, B_KCONTIG, true>::type, Cfg::BK> cl;
    rl.init(a.A, a.npanels, a.tiles_per_panel, g.lda, m0, g.M, kt0, threadIdx.x);
    cl.init(a.B, a.npanels, a.tiles_per_panel, g.ldb, n0, g.N, kt0, threadIdx.x);

    floatx16 acc[Cfg::MB][Cfg::NB];
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.0f;

    mainloop<Cfg>(rl, cl, T, 0, acc, smem);
    if (!combine_slices<Cfg>(acc, g.split, w)) return;

    store_tile_rowmajor<Cfg>(acc, g.C, g.ldc, g.M, g.N, g.alpha, g.beta, g.cvec != 0, m0, n0, g.split, w, g.cvec == 2);
    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 2] = __builtin_readcyclecounter();
        g.clock_probe[blockIdx.x * 4 + 3] = __builtin_amdgcn_s_memrealtime();
    }
}

// Host side.  Operands must allow 16-byte loads (the caller checks).  Returns the hipError_t as int.
template <class Cfg>
int launch_gemm_panels_cfg(const GemmPanelArgs &a, bool a_kcontig, bool b_kcontig, hipStream_t stream)
{
    const int tiles = a.g.tiles_m * a.g.tiles_n;
    const dim3 grid((unsigned)(a.g.split.dp_tiles + (tiles - a.g.split.dp_tiles) * a.g.split.splits)), block(Cfg::NT);
    if (a_kcontig && b_kcontig)
        hipLaunchKernelGGL((gemm_panels_tile_kernel<Cfg, true, true>), grid, block, 0, stream, a);
    else if (a_kcontig)
        hipLaunchKernelGGL((gemm_panels_tile_kernel<Cfg, true, false>), grid, block, 0, stream, a);
    else if (b_kcontig)
        hipLaunchKernelGGL((gemm_panels_tile_kernel<Cfg, false, true>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((gemm_panels_tile_kernel<Cfg, false, false>), grid, block, 0, stream, a);
    return (int)hipGetLastError();
}

}  // namespace dmath
