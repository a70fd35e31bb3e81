// Device-side core shared by the GEMM and the implicit-GEMM convolution kernels
// (gfx950 only): operand loaders global -> registers -> LDS, the software
// pipeline over K tiles, and the FP32 MFMA macro-tile.
//
// One workgroup computes a BM x BN tile of the product  rows-operand (BM x K)
// times cols-operand (K x BN).  Both operands are staged in LDS in the same
// image, whatever their orientation in memory:
//
//     As[stage][k][LDA]   element (k, r) = rows-operand(r, k),  r in [0, BM)
//     Bs[stage][k][LDB]   element (k, c) = cols-operand(k, c),  c in [0, BN)
//
// so the MFMA loop and the epilogue are the same for every transpose form
// (the local multiply of section "Matrix Multiplication" of the dMath paper and
// its transposed variants) and for the convolution, which only brings its own
// loader for the operand generated from x.
//
// MFMA used: v_mfma_f32_32x32x2_f32.  For lane l (i = l % 32, h = l / 32):
//   A operand register holds A[i][k = h], B operand holds B[k = h][j = i],
//   accumulator register r holds D[8*(r/4) + 4*h + r%4][j = i].
// A wave owns MB x NB such 32x32 blocks.  Block (bm, bn), row i of the MFMA
// block is row  wm0 + MB*i + bm  of the tile and column j is column
// wn0 + NB*j + bn: each lane then reads its MB (NB) operand values for one k
// as one 8- or 16-byte LDS read, and owns NB consecutive columns of C, which
// makes the epilogue a run of 16-byte stores that cover 512 contiguous bytes
// per row across the wave.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dmath {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

template <int N> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef floatx2 type; };
template <> struct VecOf<4> { typedef floatx4 type; };

constexpr int kNumXcd = 8;  // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// Tile configuration.  WM = BM / WAVES_M and WN = BN / WAVES_N are the wave tile.
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_, int MIN_WAVES_PER_SIMD_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    static constexpr int MIN_WAVES = MIN_WAVES_PER_SIMD_;
    static constexpr int NT = WAVES_M * WAVES_N * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int MB = WM / 32, NB = WN / 32;
    // +4 floats of padding: rows stay 16-byte aligned and the transposing
    // 4-byte stores of a K-contiguous operand (4 lanes per row, 16 rows per
    // wave) land in 64 different banks.
    static constexpr int LDA = BM + 4, LDB = BN + 4;
    static constexpr int A_FLOATS = BK * LDA, B_FLOATS = BK * LDB;
    static constexpr int STAGE_FLOATS = A_FLOATS + B_FLOATS;
    static constexpr int LDS_BYTES = STAGES * STAGE_FLOATS * 4;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
    static_assert(MB == 1 || MB == 2 || MB == 4, "operand reads are 4, 8 or 16 bytes");
    static_assert(NB == 1 || NB == 2 || NB == 4, "operand reads are 4, 8 or 16 bytes");
    static_assert(BK % 4 == 0 && BK >= 4, "K tile is a multiple of one 16-byte load");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one compute unit");
};

// ---------------------------------------------------------------------------------------------
// Loader for an operand stored contiguously along k: element (r, k) at base[r*ld + k].
// Used for A when transA == N, for B when transB == T, and for the filters of the convolution.
// Thread t owns 16-byte quads q = t + it*NT of the BR x BK tile, quad q = (row q / (BK/4), k quad
// q % (BK/4)); it keeps them in registers between the global load and the transposing LDS store.
template <int BR, int BK, int NT, int LD, bool VEC>
struct LoaderK {
    static constexpr int QPR = BK / 4;
    static constexpr int NQ = (BR * QPR) / NT;
    static_assert((BR * QPR) % NT == 0 && NQ >= 1, "tile must split evenly over the threads");
    const float *p[NQ];
    floatx4 v[NQ];
    int row0, kq;

    // r0: first row of this tile, R: number of rows of the operand (rows past the end re-read
    // row R-1; their products land in rows/columns of C that are never stored).
    __device__ __forceinline__ void init(const float *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        row0 = tid / QPR;
        kq = tid % QPR;
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            int64_t gr = r0 + row0 + it * (NT / QPR);
            gr = gr < R ? gr : R - 1;
            p[it] = base + gr * ld + k0 + kq * 4;
        }
    }
    __device__ __forceinline__ void load()
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            if (VEC) {
                v[it] = *reinterpret_cast<const floatx4 *>(p[it]);
            } else {
                v[it][0] = p[it][0];
                v[it][1] = p[it][1];
                v[it][2] = p[it][2];
                v[it][3] = p[it][3];
            }
            p[it] += BK;
        }
    }
    // Last, partial K tile: only k < krem exists; the rest of the tile is zero on both operands.
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[it][j] = (kq * 4 + j < krem) ? p[it][j] : 0.0f;
        }
    }
    __device__ __forceinline__ void store(float *S) const
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            const int row = row0 + it * (NT / QPR);
#pragma unroll
            for (int j = 0; j < 4; ++j) S[(kq * 4 + j) * LD + row] = v[it][j];
        }
    }
};

// Loader for an operand stored contiguously along its own index: element (r, k) at base[k*ld + r].
// Used for A when transA == T and for B when transB == N.  Quads run along r; NT is a multiple of
// the quads per k row, so a thread keeps one r quad and walks k.
template <int BR, int BK, int NT, int LD, bool VEC>
struct LoaderMN {
    static constexpr int QPR = BR / 4;
    static constexpr int NQ = (BK * QPR) / NT;
    static constexpr int KSTEP = NT / QPR;
    static_assert((BK * QPR) % NT == 0 && NQ >= 1 && NT % QPR == 0, "tile must split evenly over the threads");
    const float *p;   // row k0 + krow of the operand
    int64_t kstride;  // KSTEP * ld
    int64_t tstride;  // BK * ld
    int c[4];         // column offsets of the four elements (clamped to the last valid one)
    floatx4 v[NQ];
    int krow, rq;

    __device__ __forceinline__ void init(const float *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        krow = tid / QPR;
        rq = tid % QPR;
        p = base + (k0 + krow) * ld;
        kstride = (int64_t)KSTEP * ld;
        tstride = (int64_t)BK * ld;
        if (VEC) {
            // R is a multiple of 4 on this path: a quad is wholly inside or wholly outside.
            int64_t gr = r0 + rq * 4;
            gr = gr + 4 <= R ? gr : R - 4;
            p += gr;
            c[0] = 0; c[1] = 1; c[2] = 2; c[3] = 3;
        } else {
            p += r0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int64_t lr = rq * 4 + j;
                c[j] = (int)(r0 + lr < R ? lr : R - 1 - r0);
            }
        }
    }
    __device__ __forceinline__ void load()
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            const float *q = p + it * kstride;
            if (VEC) {
                v[it] = *reinterpret_cast<const floatx4 *>(q);
            } else {
                v[it][0] = q[c[0]];
                v[it][1] = q[c[1]];
                v[it][2] = q[c[2]];
                v[it][3] = q[c[3]];
            }
        }
        p += tstride;
    }
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            const float *q = p + it * kstride;
            const bool ok = krow + it * KSTEP < krem;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[it][j] = ok ? q[c[j]] : 0.0f;
        }
    }
    __device__ __forceinline__ void store(float *S) const
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it)
            *reinterpret_cast<floatx4 *>(&S[(krow + it * KSTEP) * LD + rq * 4]) = v[it];
    }
};

// ---------------------------------------------------------------------------------------------
// MFMA macro-tile: one K tile (BK deep) from LDS into the accumulators.
template <class Cfg>
__device__ __forceinline__ void mma_stage(const float *As, const float *Bs,
                                          floatx16 (&acc)[Cfg::MB][Cfg::NB], int a_off, int b_off)
{
    typedef typename VecOf<Cfg::MB>::type AV;
    typedef typename VecOf<Cfg::NB>::type BV;
#pragma unroll
    for (int s = 0; s < Cfg::BK / 2; ++s) {
        const AV av = *reinterpret_cast<const AV *>(As + a_off + 2 * s * Cfg::LDA);
        const BV bv = *reinterpret_cast<const BV *>(Bs + b_off + 2 * s * Cfg::LDB);
        float a[Cfg::MB], b[Cfg::NB];
        if constexpr (Cfg::MB == 1) { a[0] = av; } else {
#pragma unroll
            for (int x = 0; x < Cfg::MB; ++x) a[x] = av[x];
        }
        if constexpr (Cfg::NB == 1) { b[0] = bv; } else {
#pragma unroll
            for (int x = 0; x < Cfg::NB; ++x) b[x] = bv[x];
        }
#pragma unroll
        for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
            for (int bn = 0; bn < Cfg::NB; ++bn)
                acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bm], b[bn], acc[bm][bn], 0, 0, 0);
    }
}

// Software pipeline over the K range of one tile.  T full K tiles, then an optional partial one of
// krem (< BK) columns.  LDS holds STAGES tiles; registers hold one more in flight, so a global load
// has a whole K tile of MFMA work to land.  One barrier per K tile: the store of tile t+STAGES-1
// goes to the stage whose readers finished before the previous barrier.
template <class Cfg, class RowLoader, class ColLoader>
__device__ __forceinline__ void mainloop(RowLoader &rl, ColLoader &cl, int T, int krem,
                                         floatx16 (&acc)[Cfg::MB][Cfg::NB], float *smem)
{
    constexpr int S = Cfg::STAGES;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM;
    const int wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const int i = lane & 31, h = lane >> 5;
    const int a_off = h * Cfg::LDA + wm0 + Cfg::MB * i;
    const int b_off = h * Cfg::LDB + wn0 + Cfg::NB * i;

#pragma unroll
    for (int s = 0; s < S - 1; ++s) {
        if (s < T) {
            rl.load();
            cl.load();
            rl.store(smem + s * Cfg::STAGE_FLOATS);
            cl.store(smem + s * Cfg::STAGE_FLOATS + Cfg::A_FLOATS);
        }
    }
    if (S - 1 < T) {
        rl.load();
        cl.load();
    }
    __syncthreads();

    int cur = 0;       // stage holding tile t
    int fill = S - 1;  // stage that receives tile t + S - 1
    for (int t = 0; t < T; ++t) {
        if (t + S - 1 < T) {
            rl.store(smem + fill * Cfg::STAGE_FLOATS);
            cl.store(smem + fill * Cfg::STAGE_FLOATS + Cfg::A_FLOATS);
        }
        if (t + S < T) {
            rl.load();
            cl.load();
        }
        mma_stage<Cfg>(smem + cur * Cfg::STAGE_FLOATS, smem + cur * Cfg::STAGE_FLOATS + Cfg::A_FLOATS, acc,
                       a_off, b_off);
        cur = (cur + 1 == S) ? 0 : cur + 1;
        fill = (fill + 1 == S) ? 0 : fill + 1;
        __syncthreads();
    }
    if (krem > 0) {
        rl.load_tail(krem);
        cl.load_tail(krem);
        rl.store(smem);
        cl.store(smem + Cfg::A_FLOATS);
        __syncthreads();
        mma_stage<Cfg>(smem, smem + Cfg::A_FLOATS, acc, a_off, b_off);
    }
}

// Workgroup id -> tile id.  Workgroups are handed to the 8 dies in turn, each die has its own L2:
// give every die one contiguous run of tile ids, and order tile ids so that a run covers a compact
// block of the tile grid (GROUP tile rows at a time, walking down the rows first), so that the
// A row panels and B column panels a die fetches are shared by the tiles resident on it.
__device__ __forceinline__ int xcd_contiguous_id(int bid, int total)
{
    const int xcd = bid % kNumXcd, loc = bid / kNumXcd;
    const int q = total / kNumXcd, rem = total % kNumXcd;
    return (xcd < rem) ? xcd * (q + 1) + loc : rem * (q + 1) + (xcd - rem) * q + loc;
}

template <int GROUP>
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int per_group = GROUP * tiles_n;
    const int g = pid / per_group;
    const int first = g * GROUP;
    const int rows = (tiles_m - first < GROUP) ? tiles_m - first : GROUP;
    const int in_g = pid - g * per_group;
    tm = first + in_g % rows;
    tn = in_g / rows;
}

}  // namespace dmath
