// Double-precision GEMM on v_mfma_f64_16x16x4_f64 (section "Precisions" of the paper: single and double
// precision are the library's nominal precisions).
//
// Operand layout of the instruction (checked on the device with one-hot operands): lane l holds for A
// the element (row l%16, k = l/16), for B the element (k = l/16, column l%16); of the 16x16 FP64 result,
// register r of lane l is (row 4*r + l/16, column l%16).  One instruction is 16x16x4 = 2048 flop in 64
// cycles, so a K tile of 16 is 64 instructions = 4096 cycles per wave: everything else hides easily,
// and the kernel is written for generality first (8-byte loads with per-element clamping: any
// alignment, any leading dimension, any M, N, K).
//
// LDS image per stage, as in the FP32 kernel: As[BK][LDA], Bs[BK][LDB] doubles (k-major), LD = B + 2.
// (The 16-byte fragment reads still show 4 conflict cycles each on the counters, with this pitch and
// with B + 8 alike; they are hidden: 64 of the 4096 cycles a K tile takes.)
// A wave owns MB x NB blocks of 16x16; block bm covers tile rows wm0 + 32*(bm/2) + 2*i + bm%2 for lane
// row index i, so that a lane's two values of a block pair are adjacent in the image (one 16-byte
// read, 16 lanes reading 256 contiguous bytes) and a lane owns pairs of adjacent columns of C.
#pragma once
#include "gemm_kernel.h"

namespace dmath {

typedef double doublex2 __attribute__((ext_vector_type(2)));
typedef double doublex4 __attribute__((ext_vector_type(4)));

typedef GemmArgsT<double> DGemmArgs;  // alpha and beta travel separately as doubles

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int STAGES_>
struct DTileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = 16;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int MB = WM / 16, NB = WN / 16;
    static constexpr int LDA = BM + 2, LDB = BN + 2;
    static constexpr int A_DOUBLES = BK * LDA, B_DOUBLES = BK * LDB, STAGE_DOUBLES = A_DOUBLES + B_DOUBLES;
    static constexpr int LDS_BYTES = STAGES * STAGE_DOUBLES * 8;
    static constexpr int KSTEPS = BK / 4;
    static constexpr int MIN_WAVES = (NT / 64 + 3) / 4;
    static_assert(WM % 32 == 0 && WN % 32 == 0 && STAGES >= 3, "wave tile is made of pairs of 16x16 blocks; 3+ stages");
};

// Operand contiguous along k: element (r, k) at base[r*ld + k].  Thread (row, k pair); the pair is
// transposed into the image by two 8-byte LDS stores.
template <int BR, int BK, int NT, int LD, bool VEC>
struct DLoaderK {
    static constexpr int PPR = BK / 2;            // pairs per row
    static constexpr int NQ = (BR * PPR) / NT;    // pairs per thread
    static constexpr int NLOAD = VEC ? NQ : 2 * NQ, NSTORE = 2 * NQ;
    static_assert((BR * PPR) % NT == 0 && NQ >= 1, "tile must split evenly over the threads");
    const double *tile;   // &base[r0*ld + k of the tile]
    int64_t off[NQ];      // element offset of (row, first k of the pair)
    double v[NQ][2];
    int row0, kq;

    __device__ __forceinline__ void init(const double *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        // The 16 lanes whose 8-byte stores the LDS serves in one cycle take 4 k pairs x 4 rows: their
        // addresses (2*kq + e)*LD + row with LD = 2 mod 8 then fall on banks 8*(kq%4) + 2*(row%4) + {0, 1},
        // all 32 once.  (With 8 k pairs x 2 rows, pairs kq and kq + 4 met on the same banks: 4 conflict
        // cycles on every store by the counters, a third of all conflict cycles of the kernel.)
        static_assert(PPR == 8 && LD % 8 == 2, "bank layout of the transposing stores");
        kq = (tid & 3) | ((tid >> 2) & 4);
        row0 = ((tid >> 2) & 3) | ((tid >> 3) & ~3);
        tile = base + r0 * ld + k0;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            int64_t lr = row0 + q * (NT / PPR);
            lr = r0 + lr < R ? lr : R - 1 - r0;  // rows past the end re-read the last one; never stored
            off[q] = lr * ld + 2 * kq;
        }
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        if constexpr (VEC) {  // 16-byte aligned pairs: one load
            const doublex2 p = *reinterpret_cast<const doublex2 *>(tile + off[I]);
            v[I][0] = p[0];
            v[I][1] = p[1];
        } else {
            v[I / 2][I % 2] = tile[off[I / 2] + (I % 2)];
        }
    }
    __device__ __forceinline__ void advance() { tile += BK; }
    // last, partial tile: k >= krem does not exist
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int e = 0; e < 2; ++e) v[q][e] = (2 * kq + e < krem) ? tile[off[q] + e] : 0.0;
    }
    template <int I>
    __device__ __forceinline__ void store_piece(double *S) const
    {
        S[(2 * kq + I % 2) * LD + row0 + (I / 2) * (NT / PPR)] = v[I / 2][I % 2];
    }
};

// Operand contiguous along its own index: element (r, k) at base[k*ld + r].  Thread (k row, r pair);
// one 16-byte LDS store per pair.
template <int BR, int BK, int NT, int LD, bool VEC>
struct DLoaderN {
    static constexpr int PPR = BR / 2;            // pairs per k row
    static constexpr int NQ = (BK * PPR) / NT;
    static constexpr int KSTEP = NT / PPR;
    static constexpr int NLOAD = VEC ? NQ : 2 * NQ, NSTORE = NQ;
    static_assert((BK * PPR) % NT == 0 && NQ >= 1 && NT % PPR == 0, "tile must split evenly over the threads");
    const double *tile;   // &base[k of the tile * ld + r0]
    int64_t tstride;
    int64_t off[NQ][2];
    double v[NQ][2];
    int krow, rq;

    __device__ __forceinline__ void init(const double *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        krow = tid / PPR;
        rq = tid % PPR;
        tile = base + k0 * ld + r0;
        tstride = (int64_t)BK * ld;
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                int64_t lr = 2 * rq + e;
                if (VEC)
                    lr = r0 + 2 * rq + 2 <= R ? lr : R - 2 - r0 + e;  // R even: the last whole pair
                else
                    lr = r0 + lr < R ? lr : R - 1 - r0;
                off[q][e] = (int64_t)(krow + q * KSTEP) * ld + lr;
            }
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        if constexpr (VEC) {  // R even and 16-byte aligned rows: the pair is one load, wholly inside or clamped
            const doublex2 p = *reinterpret_cast<const doublex2 *>(tile + off[I][0]);
            v[I][0] = p[0];
            v[I][1] = p[1];
        } else {
            v[I / 2][I % 2] = tile[off[I / 2][I % 2]];
        }
    }
    __device__ __forceinline__ void advance() { tile += tstride; }
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int e = 0; e < 2; ++e) v[q][e] = (krow + q * KSTEP < krem) ? tile[off[q][e]] : 0.0;
    }
    template <int I>
    __device__ __forceinline__ void store_piece(double *S) const
    {
        doublex2 p;
        p[0] = v[I][0];
        p[1] = v[I][1];
        *reinterpret_cast<doublex2 *>(S + (krow + I * KSTEP) * LD + 2 * rq) = p;
    }
};

// (The k-contiguous loader always uses its 8-byte form: the compiler joins the two loads of a pair
// where it can, and the explicit 16-byte form measured 20-40 % slower.)
template <class Cfg, bool KCONTIG, int BR, int LD, bool VEC>
struct DLoaderSel {
    typedef DLoaderK<BR, Cfg::BK, Cfg::NT, LD, false> type;
};
template <class Cfg, int BR, int LD, bool VEC>
struct DLoaderSel<Cfg, false, BR, LD, VEC> {
    typedef DLoaderN<BR, Cfg::BK, Cfg::NT, LD, VEC> type;
};

template <class Cfg>
struct DFrag {
    doublex2 a[Cfg::MB / 2], b[Cfg::NB / 2];
};

// Fragment piece P of k step KS: P < MB/2 is block-row pair P of A, else block-column pair of B.
template <class Cfg, int KS, int P>
__device__ __forceinline__ void dload_frag_piece(DFrag<Cfg> &f, const double *As, const double *Bs, int a_off, int b_off)
{
    if constexpr (P < Cfg::MB / 2)
        f.a[P] = *reinterpret_cast<const doublex2 *>(As + a_off + KS * 4 * Cfg::LDA + P * 32);
    else
        f.b[P - Cfg::MB / 2] = *reinterpret_cast<const doublex2 *>(Bs + b_off + KS * 4 * Cfg::LDB + (P - Cfg::MB / 2) * 32);
}

template <class Cfg, int Q>
__device__ __forceinline__ void dmma_one(const DFrag<Cfg> &f, doublex4 (&acc)[Cfg::MB][Cfg::NB])
{
    constexpr int bm = Q / Cfg::NB, bn = Q % Cfg::NB;
    acc[bm][bn] = __builtin_amdgcn_mfma_f64_16x16x4f64(f.a[bm / 2][bm % 2], f.b[bn / 2][bn % 2], acc[bm][bn], 0, 0, 0);
}

// One K tile: MB*NB matrix instructions per k step; after each, at most one fragment read, LDS store
// of the staged tile or global load of the tile after it.  The flags (workgroup-uniform) say whether
// there is a tile to store, one to load and a next one to read; they guard the memory operations only.
// STEADY: all three hold and nothing is tested.
template <class Cfg, bool STEADY, class RL, class CL>
__device__ __forceinline__ void dtile_iter(RL &rl, CL &cl, DFrag<Cfg> (&fr)[2], doublex4 (&acc)[Cfg::MB][Cfg::NB],
                                           const double *cur, const double *nxt, double *fill, int a_off, int b_off,
                                           bool do_store = true, bool do_load = true, bool has_next = true)
{
    if constexpr (STEADY) {
        do_store = true;
        do_load = true;
        has_next = true;
    }
    constexpr int NMMA = Cfg::MB * Cfg::NB, NFRAG = Cfg::MB / 2 + Cfg::NB / 2, TOTAL = Cfg::KSTEPS * NMMA;
    constexpr int NST = RL::NSTORE + CL::NSTORE, NLD = RL::NLOAD + CL::NLOAD;
    static_assert(NST + NLD <= TOTAL, "one memory operation per matrix instruction");
    static_for<Cfg::KSTEPS>([&](auto ksc) {
        constexpr int ks = decltype(ksc)::value;
        constexpr bool last = ks == Cfg::KSTEPS - 1;
        static_for<NMMA>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            dmma_one<Cfg, q>(fr[ks % 2], acc);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (q < NFRAG) {
                if constexpr (!last)
                    dload_frag_piece<Cfg, ks + 1, q>(fr[(ks + 1) % 2], cur, cur + Cfg::A_DOUBLES, a_off, b_off);
                else if (has_next)
                    dload_frag_piece<Cfg, 0, q>(fr[0], nxt, nxt + Cfg::A_DOUBLES, a_off, b_off);
            } else {
                constexpr int s = ks * (NMMA - NFRAG) + (q - NFRAG);  // index among the free instruction slots
                if constexpr (s < NST) {
                    if (do_store) {
                        if constexpr (s < RL::NSTORE)
                            rl.template store_piece<s>(fill);
                        else
                            cl.template store_piece<s - RL::NSTORE>(fill + Cfg::A_DOUBLES);
                    }
                } else if constexpr (s < NST + NLD) {
                    constexpr int l = s - NST;
                    if (do_load) {
                        if constexpr (l < RL::NLOAD)
                            rl.template load_piece<l>();
                        else
                            cl.template load_piece<l - RL::NLOAD>();
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    });
    if (do_load) {
        rl.advance();
        cl.advance();
    }
}

// Epilogue: lane (j = l%16, h = l/16) holds, for block (bm, bn) and register r, the element in tile
// row wm0 + 32*(bm/2) + 2*(4*r + h) + bm%2 and tile column wn0 + 32*(bn/2) + 2*j + bn%2.
template <class Cfg>
__device__ __forceinline__ void dstore_tile(const doublex4 (&acc)[Cfg::MB][Cfg::NB], double *C, int64_t ldc, int64_t M,
                                            int64_t N, double alpha, double beta, int64_t m0, int64_t n0)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, h = lane >> 4;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    if (beta != 0.0 && m0 + Cfg::BM <= M && n0 + Cfg::BN <= N) {
        // Tile wholly inside C: the old values of a block row are fetched before the first is used, so
        // that the epilogue does not wait out the memory latency once per element.
        double *base = C + (m0 + wm0 + 2 * h) * ldc + (n0 + wn0 + 2 * j);
#pragma unroll
        for (int bm = 0; bm < Cfg::MB; ++bm) {
            double old[4][Cfg::NB];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int bn = 0; bn < Cfg::NB; ++bn)
                    old[r][bn] = base[(32 * (bm / 2) + 8 * r + (bm % 2)) * ldc + 32 * (bn / 2) + (bn % 2)];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int bn = 0; bn < Cfg::NB; ++bn)
                    base[(32 * (bm / 2) + 8 * r + (bm % 2)) * ldc + 32 * (bn / 2) + (bn % 2)] =
                        __builtin_fma(beta, old[r][bn], alpha * acc[bm][bn][r]);
        }
        return;
    }
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = m0 + wm0 + 32 * (bm / 2) + 2 * (4 * r + h) + (bm % 2);
            if (row >= M) continue;
#pragma unroll
            for (int bn = 0; bn < Cfg::NB; ++bn) {
                const int64_t col = n0 + wn0 + 32 * (bn / 2) + 2 * j + (bn % 2);
                if (col >= N) continue;
                double *dst = C + row * ldc + col;
                double o = alpha * acc[bm][bn][r];
                if (beta != 0.0) o += beta * *dst;
                *dst = o;
            }
        }
}

struct DGemmScalars {
    double alpha, beta;
};

// VEC: A and B are 16-byte aligned with even leading dimensions, and an operand stored along its own
// index has an even number of rows / columns: every pair is one 16-byte load.
template <class Cfg, bool A_KCONTIG, bool B_KCONTIG, bool VEC>
__global__ __launch_bounds__(Cfg::NT, Cfg::MIN_WAVES) void dgemm_tile_kernel(const DGemmArgs g, const DGemmScalars sc)
{
    constexpr int S = Cfg::STAGES;
    __shared__ __attribute__((aligned(16))) double smem[S * Cfg::STAGE_DOUBLES];

    const int tiles = g.tiles_m * g.tiles_n;
    const WorkItem w = work_item(blockIdx.x, tiles, g.split);
    int tm, tn;
    tile_coords<8>(w.tile, g.tiles_m, g.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * Cfg::BM, n0 = (int64_t)tn * Cfg::BN;
    // K range of this workgroup: the whole K, or one slice of it (plain split-K: raw sums to the workspace)
    const int ktiles_total = (int)(g.K / Cfg::BK);
    int kt0, T, krem;
    slice_range(ktiles_total, (int)(g.K - (int64_t)ktiles_total * Cfg::BK), w.slice, w.nslice, kt0, T, krem);
    const int64_t k0 = (int64_t)kt0 * Cfg::BK;

    typename DLoaderSel<Cfg, A_KCONTIG, Cfg::BM, Cfg::LDA, VEC>::type rl;
    typename DLoaderSel<Cfg, B_KCONTIG, Cfg::BN, Cfg::LDB, VEC>::type cl;
    rl.init(g.A, g.lda, m0, g.M, k0, threadIdx.x);
    cl.init(g.B, g.ldb, n0, g.N, k0, threadIdx.x);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int a_off = (lane >> 4) * Cfg::LDA + (wave / Cfg::WAVES_N) * Cfg::WM + 2 * (lane & 15);
    const int b_off = (lane >> 4) * Cfg::LDB + (wave % Cfg::WAVES_N) * Cfg::WN + 2 * (lane & 15);

    doublex4 acc[Cfg::MB][Cfg::NB];
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[bm][bn][r] = 0.0;

    auto load_all = [&]() {
        static_for<decltype(rl)::NLOAD>([&](auto ic) { rl.template load_piece<decltype(ic)::value>(); });
        static_for<decltype(cl)::NLOAD>([&](auto ic) { cl.template load_piece<decltype(ic)::value>(); });
        rl.advance();
        cl.advance();
    };
    auto store_all = [&](double *st) {
        static_for<decltype(rl)::NSTORE>([&](auto ic) { rl.template store_piece<decltype(ic)::value>(st); });
        static_for<decltype(cl)::NSTORE>([&](auto ic) { cl.template store_piece<decltype(ic)::value>(st + Cfg::A_DOUBLES); });
    };
    auto stage = [&](int s) { return smem + s * Cfg::STAGE_DOUBLES; };
    auto next_of = [](int s) { return s + 1 == S ? 0 : s + 1; };

    // Tile t lives in stage t % S.  Prologue: tiles 0 .. S-2 into their stages, tile S-1 into the
    // registers; iteration t stores tile t + S - 1 and then loads tile t + S.
#pragma unroll
    for (int s = 0; s < S - 1; ++s) {
        if (s < T) {
            load_all();
            store_all(stage(s));
        }
    }
    if (S - 1 < T) load_all();
    __syncthreads();

    DFrag<Cfg> fr[2];
    auto first_frags = [&](const double *st) {
        static_for<Cfg::MB / 2 + Cfg::NB / 2>([&](auto pc) {
            dload_frag_piece<Cfg, 0, decltype(pc)::value>(fr[0], st, st + Cfg::A_DOUBLES, a_off, b_off);
        });
    };
    if (T > 0) first_frags(smem);

    int cs = 0, fill = S - 1, t = 0;
    for (; t + S < T; ++t) {  // steady state: a tile to store, one to load and a next one to read
        dtile_iter<Cfg, true>(rl, cl, fr, acc, stage(cs), stage(next_of(cs)), stage(fill), a_off, b_off);
        cs = next_of(cs);
        fill = next_of(fill);
        __syncthreads();
    }
    for (; t < T; ++t) {
        dtile_iter<Cfg, false>(rl, cl, fr, acc, stage(cs), stage(next_of(cs)), stage(fill), a_off, b_off, t + S - 1 < T,
                               t + S < T, t + 1 < T);
        cs = next_of(cs);
        fill = next_of(fill);
        __syncthreads();
    }
    if (krem > 0) {
        // the ragged last tile, not pipelined: the loaders stand at tile T after T advances
        rl.load_tail(krem);
        cl.load_tail(krem);
        store_all(smem);
        __syncthreads();
        first_frags(smem);
        dtile_iter<Cfg, false>(rl, cl, fr, acc, smem, smem, smem, a_off, b_off, false, false, false);
    }
    if (w.nslice > 1) {
        // slice `slice` of the tile: its raw FP64 sums go to slice array `slice` (M x N, dense) in the workspace
        double *Z = reinterpret_cast<double *>(g.split.partials) + (int64_t)w.slice * g.split.slice_stride;
        dstore_tile<Cfg>(acc, Z, g.N, g.M, g.N, 1.0, 0.0, m0, n0);
        return;
    }
    dstore_tile<Cfg>(acc, g.C, g.ldc, g.M, g.N, sc.alpha, sc.beta, m0, n0);
}

template <class Cfg>
int launch_dgemm(const DGemmArgs &g, double alpha, double beta, bool a_kcontig, bool b_kcontig, bool vec, hipStream_t stream)
{
    const int tiles = g.tiles_m * g.tiles_n;
    const dim3 grid((unsigned)(g.split.dp_tiles + (tiles - g.split.dp_tiles) * g.split.splits)), block(Cfg::NT);
    const DGemmScalars sc = {alpha, beta};
#define DMATH_DLAUNCH(AK, BK_, V) hipLaunchKernelGGL((dgemm_tile_kernel<Cfg, AK, BK_, V>), grid, block, 0, stream, g, sc)
    if (vec) {
        if (a_kcontig && b_kcontig) DMATH_DLAUNCH(true, true, true);
        else if (a_kcontig) DMATH_DLAUNCH(true, false, true);
        else if (b_kcontig) DMATH_DLAUNCH(false, true, true);
        else DMATH_DLAUNCH(false, false, true);
    } else {
        if (a_kcontig && b_kcontig) DMATH_DLAUNCH(true, true, false);
        else if (a_kcontig) DMATH_DLAUNCH(true, false, false);
        else if (b_kcontig) DMATH_DLAUNCH(false, true, false);
        else DMATH_DLAUNCH(false, false, false);
    }
#undef DMATH_DLAUNCH
    return (int)hipGetLastError();
}

struct DCfgDesc {
    const char *name;
    int BM, BN, BK, NT, lds_bytes;
    int (*launch)(const DGemmArgs &, double alpha, double beta, bool a_kcontig, bool b_kcontig, bool vec, hipStream_t);
};
constexpr int kNumDCfg = 2;
const DCfgDesc &dcfg_desc(int i);  // defined in dgemm_instance.hip

}  // namespace dmath
