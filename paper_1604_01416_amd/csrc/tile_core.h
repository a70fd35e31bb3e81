// Device-side core shared by the GEMM and the implicit-GEMM convolution kernels
// (gfx950 only): operand loaders global -> registers -> LDS, the software
// pipeline over K tiles, and the FP32 MFMA macro-tile.
//
// One workgroup computes a BM x BN tile of the product  rows-operand (BM x K)
// times cols-operand (K x BN).  Both operands are staged in LDS in the same
// image, whatever their orientation in memory:
//
//     As[stage][k][LDA]   element (k, col(r, k)) = rows-operand(r, k),  r in [0, BM)
//     Bs[stage][k][LDB]   element (k, col(c, k)) = cols-operand(k, c),  c in [0, BN)
//
// so the MFMA loop and the epilogue are the same for every transpose form
// (the local multiply of section "Matrix Multiplication" of the dMath paper and
// its transposed variants) and for the convolution, which only brings its own
// loader for the operand generated from x.  Two images exist (TileCfg::LKV):
// padded, col(x, k) = x with LDA = BM + 4, and rotated, col(x, k) =
// (x + 8 * (k / 4)) mod extent with LDA = BM, which is free of LDS bank
// conflicts also for the transposing stores of operands contiguous along k.
// The padded image is the faster one on MI355X and is what the product
// configurations use; see LoaderK / LoaderK0.
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

#include <utility>

namespace dmath {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));

// Four consecutive stored elements of type T as one vector, and their values as floats.  T is float, or
// _Float16 for matrices kept in half-precision storage (converted exactly on the way to the LDS image).
template <class T> struct Quad;
template <> struct Quad<float> {
    typedef floatx4 type;
    static __device__ __forceinline__ floatx4 widen(floatx4 q) { return q; }
};
template <> struct Quad<_Float16> {
    typedef halfx4 type;
    static __device__ __forceinline__ floatx4 widen(halfx4 q)
    {
        floatx4 f;
        f[0] = (float)q[0];
        f[1] = (float)q[1];
        f[2] = (float)q[2];
        f[3] = (float)q[3];
        return f;
    }
};

template <int N> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef floatx2 type; };
template <> struct VecOf<4> { typedef floatx4 type; };

constexpr int kNumCU = 256;  // MI355X: compute units
constexpr int kNumXcd = 8;  // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// Tile configuration.  WM = BM / WAVES_M and WN = BN / WAVES_N are the wave tile.
// LKV selects the LDS image: 0 = plain rows padded by 4 floats with 4-byte transposing stores (the faster
// one, used by every product configuration); 2 = rotated rows, no padding, free of bank conflicts (kept
// as the comparison point for the counters).
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_, int MIN_WAVES_PER_SIMD_, int LKV_ = 2>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    static constexpr int MIN_WAVES = MIN_WAVES_PER_SIMD_;
    static constexpr int LKV = LKV_;
    static constexpr int ROT = (LKV_ == 2) ? 8 : 0;
    static constexpr int NT = WAVES_M * WAVES_N * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int MB = WM / 32, NB = WN / 32;
    static constexpr int LDA = BM + (LKV_ == 2 ? 0 : 4), LDB = BN + (LKV_ == 2 ? 0 : 4);
    static constexpr int A_FLOATS = BK * LDA, B_FLOATS = BK * LDB;
    static constexpr int STAGE_FLOATS = A_FLOATS + B_FLOATS;
    static constexpr int LDS_BYTES = STAGES * STAGE_FLOATS * 4;
    static constexpr int KGROUPS = BK / 4;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
    static_assert(MB == 1 || MB == 2 || MB == 4, "operand reads are 4, 8 or 16 bytes");
    static_assert(NB == 1 || NB == 2 || NB == 4, "operand reads are 4, 8 or 16 bytes");
    static_assert(BK % 4 == 0 && BK >= 4, "K tile is a multiple of one 16-byte load");
    static_assert((BM & (BM - 1)) == 0 && (BN & (BN - 1)) == 0 && BM >= 32 && BN >= 32, "rotation wraps with a mask");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one compute unit");
};

// Column of the LDS image that holds element x of k row `k` (extent BR, a power of two).
template <int BR, int ROT>
__device__ __forceinline__ int rot_col(int x, int k)
{
    return ROT == 0 ? x : ((x + ROT * (k >> 2)) & (BR - 1));
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}).
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int U>
__device__ __forceinline__ typename VecOf<U>::type gather_column(const floatx4 (&rows)[U], int j)
{
    typename VecOf<U>::type o;
    if constexpr (U == 1) {
        o = rows[0][j];
    } else {
#pragma unroll
        for (int it = 0; it < U; ++it) o[it] = rows[it][j];
    }
    return o;
}

// All loaders share one interface.  A tile is loaded in NLOAD pieces (load_piece<I>, one 16-byte
// global load each on the fast path) and stored to LDS in NSTORE pieces (store_piece<I>), so that the
// main loop can issue them one at a time between MFMAs; advance() moves to the next K tile.  Global
// addresses are a workgroup-uniform tile pointer (kept in scalar registers, advanced once per tile)
// plus per-thread 32-bit byte offsets that never change, so the K loop spends no vector ALU work on
// addressing.  The host guarantees leading dimensions small enough for those offsets (ld <= 2^22), or
// picks the instantiation with 64-bit offsets.
//
// ---------------------------------------------------------------------------------------------
// Loader for an operand stored contiguously along k: element (r, k) at base[r*ld + k].
// Used for A when transA == N, for B when transB == T, and for the filters of the convolution.
// The BR x BK tile is cut into units of U rows x one 16-byte k quad (U = 4, 2 or 1, as many as the
// tile gives each thread).  Consecutive lanes take the k quads of one row group, so a wave reads
// whole 64-byte row segments.  A thread loads the U quads of a unit, which gives it a U x 4 block of
// the tile in registers, and stores that block transposed: four LDS stores of U consecutive floats,
// one per k.  The lanes the LDS serves together in one cycle (8 lanes of a 16-byte store, 16 of an
// 8-byte one, 32 of a 4-byte one) hold all BK/4 k quads of a few row groups; with the image rows of
// k quad kq rotated by 8*kq floats their addresses fall into distinct banks
// (bank = 8*kq + U*rg + 0..U-1 mod 32), measured as zero SQ_LDS_BANK_CONFLICT cycles.
template <int BR, int BK, int NT, int LD, int ROT, bool VEC>
struct LoaderK {
    static constexpr int QPR = BK / 4;          // k quads per row
    static constexpr int NQ = (BR * QPR) / NT;  // quads per thread
    static constexpr int U = NQ >= 4 ? 4 : NQ;  // rows per unit
    static constexpr int UNITS = NQ / U;        // units per thread
    static constexpr int RG_STEP = NT / QPR;    // row groups between a thread's units
    static constexpr int NLOAD = UNITS * U, NSTORE = UNITS * 4;
    static_assert((BR * QPR) % NT == 0 && NQ >= 1 && NQ % U == 0, "tile must split evenly over the threads");
    static_assert((U == 1 || U == 2 || U == 4) && LD % 4 == 0 && ROT > 0 && ROT % 4 == 0, "layout assumptions");
    typedef typename VecOf<U>::type UV;
    const char *tile;         // &base[r0*ld + k], uniform over the workgroup
    uint32_t off[UNITS][U];   // byte offset of each quad from `tile`
    floatx4 v[UNITS][U];
    int lds[UNITS];           // float offset of the unit's (rotated) column in row kq*4 of the image
    int kq;

    // r0: first row of this tile, R: number of rows of the operand (rows past the end re-read
    // row R-1; their products land in rows/columns of C that are never stored).
    __device__ __forceinline__ void init(const float *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        kq = tid % QPR;
        const int rg0 = tid / QPR;
        tile = reinterpret_cast<const char *>(base + r0 * ld + k0);
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int row = (rg0 + u * RG_STEP) * U;
            lds[u] = kq * 4 * LD + rot_col<BR, ROT>(row, kq * 4);
#pragma unroll
            for (int it = 0; it < U; ++it) {
                int64_t lr = row + it;
                lr = r0 + lr < R ? lr : R - 1 - r0;
                off[u][it] = (uint32_t)((lr * ld + kq * 4) * 4);
            }
        }
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        constexpr int u = I / U, it = I % U;
        const char *q = tile + off[u][it];
        if (VEC) {
            v[u][it] = *reinterpret_cast<const floatx4 *>(q);
        } else {
            const float *f = reinterpret_cast<const float *>(q);
            v[u][it][0] = f[0];
            v[u][it][1] = f[1];
            v[u][it][2] = f[2];
            v[u][it][3] = f[3];
        }
    }
    // byte distance of k elements along K from a tile origin
    static __device__ __forceinline__ int64_t k_bytes(int64_t k, int64_t) { return k * 4; }
    __device__ __forceinline__ void advance() { tile += BK * 4; }
    template <int I>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        constexpr int u = I / 4, j = I % 4;
        *reinterpret_cast<UV *>(&S[lds[u] + j * LD]) = gather_column<U>(v[u], j);
    }
    // Last, partial K tile: only k < krem exists; the rest of the tile is zero on both operands.
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u)
#pragma unroll
            for (int it = 0; it < U; ++it) {
                const float *f = reinterpret_cast<const float *>(tile + off[u][it]);
#pragma unroll
                for (int j = 0; j < 4; ++j) v[u][it][j] = (kq * 4 + j < krem) ? f[j] : 0.0f;
            }
    }
};

// Comparison variant for the unrotated, padded image (LD = BR + 4): 4 consecutive lanes per row,
// 4-byte transposing stores (two-way bank conflicts on every store).
// KADV: K tiles between two consecutive tiles of this loader (1, or the number of waves that share a
// K range tile by tile in the wave-split kernel).
// OffT: type of the per-thread byte offsets: uint32_t (leading dimensions up to 2^22) or uint64_t.
template <int BR, int BK, int NT, int LD, bool VEC, class T = float, int KADV = 1, class OffT = uint32_t>
struct LoaderK0 {
    static constexpr int QPR = BK / 4;
    static constexpr int NQ = (BR * QPR) / NT;
    static constexpr int NLOAD = NQ, NSTORE = NQ * 4;
    static constexpr int ES = (int)sizeof(T);
    static_assert((BR * QPR) % NT == 0 && NQ >= 1, "tile must split evenly over the threads");
    const char *tile;
    OffT off[NQ];
    floatx4 v[NQ];
    int row0, kq;

    __device__ __forceinline__ void init(const T *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        row0 = tid / QPR;
        kq = tid % QPR;
        tile = reinterpret_cast<const char *>(base + r0 * ld + k0);
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            int64_t lr = row0 + it * (NT / QPR);
            lr = r0 + lr < R ? lr : R - 1 - r0;
            off[it] = (OffT)((lr * ld + kq * 4) * ES);
        }
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        const char *q = tile + off[I];
        if (VEC) {
            v[I] = Quad<T>::widen(*reinterpret_cast<const typename Quad<T>::type *>(q));
        } else {
            const T *f = reinterpret_cast<const T *>(q);
            v[I][0] = (float)f[0];
            v[I][1] = (float)f[1];
            v[I][2] = (float)f[2];
            v[I][3] = (float)f[3];
        }
    }
    // byte distance of k elements along K from a tile origin
    static __device__ __forceinline__ int64_t k_bytes(int64_t k, int64_t) { return k * ES; }
    __device__ __forceinline__ void advance() { tile += KADV * BK * ES; }
    template <int I>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        constexpr int it = I / 4, j = I % 4;
        S[(kq * 4 + j) * LD + row0 + it * (NT / QPR)] = v[it][j];
    }
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            const T *f = reinterpret_cast<const T *>(tile + off[it]);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[it][j] = (kq * 4 + j < krem) ? (float)f[j] : 0.0f;
        }
    }
};

template <int LKV, int BR, int BK, int NT, int LD, int ROT, bool VEC, class T = float, class OffT = uint32_t>
struct LoaderKSel {
    typedef LoaderK<BR, BK, NT, LD, ROT, VEC> type;  // FP32 storage, 32-bit offsets only
};
template <int BR, int BK, int NT, int LD, int ROT, bool VEC, class T, class OffT>
struct LoaderKSel<0, BR, BK, NT, LD, ROT, VEC, T, OffT> {
    typedef LoaderK0<BR, BK, NT, LD, VEC, T, 1, OffT> type;
};

// Loader for an operand stored contiguously along its own index: element (r, k) at base[k*ld + r].
// Used for A when transA == T and for B when transB == N.  Quads run along r; NT is a multiple of
// the quads per k row, so a thread keeps one r quad and walks k.  16-byte global loads, 16-byte LDS
// stores; the lanes served together write one contiguous (rotated) run of an image row.
template <int BR, int BK, int NT, int LD, int ROT, bool VEC, class T = float, int KADV = 1, class OffT = uint32_t>
struct LoaderMN {
    static constexpr int QPR = BR / 4;
    static constexpr int NQ = (BK * QPR) / NT;
    static constexpr int KSTEP = NT / QPR;
    static constexpr int NLOAD = NQ, NSTORE = NQ;
    static constexpr int ES = (int)sizeof(T);
    static_assert((BK * QPR) % NT == 0 && NQ >= 1 && NT % QPR == 0, "tile must split evenly over the threads");
    const char *tile;   // &base[k*ld + r0], uniform over the workgroup
    int64_t tstride;    // bytes per K tile: BK * ld * ES
    OffT off[NQ];       // byte offset of k row krow + it*KSTEP, column of the quad (VEC) or 0 (scalar path)
    uint32_t c[4];      // scalar path: byte offsets of the four elements (clamped to the last valid one)
    floatx4 v[NQ];
    int lds[NQ];
    int krow;

    __device__ __forceinline__ void init(const T *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        krow = tid / QPR;
        const int rq = tid % QPR;
        tile = reinterpret_cast<const char *>(base + k0 * ld + r0);
        tstride = (int64_t)KADV * BK * ld * ES;
        int64_t quad = rq * 4;  // VEC: R is a multiple of 4, a quad is wholly inside or wholly outside
        if (VEC) quad = r0 + quad + 4 <= R ? quad : R - 4 - r0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t lr = rq * 4 + j;
            c[j] = (uint32_t)((r0 + lr < R ? lr : R - 1 - r0) * ES);
        }
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            const int k = krow + it * KSTEP;
            off[it] = (OffT)((k * ld + (VEC ? quad : 0)) * ES);
            lds[it] = k * LD + rot_col<BR, ROT>(rq * 4, k);
        }
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        const char *q = tile + off[I];
        if (VEC) {
            v[I] = Quad<T>::widen(*reinterpret_cast<const typename Quad<T>::type *>(q));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[I][j] = (float)*reinterpret_cast<const T *>(q + c[j]);
        }
    }
    static __device__ __forceinline__ int64_t k_bytes(int64_t k, int64_t ld) { return k * ld * ES; }
    __device__ __forceinline__ void advance() { tile += tstride; }
    template <int I>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        *reinterpret_cast<floatx4 *>(&S[lds[I]]) = v[I];
    }
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            const char *q = tile + off[it];
            const bool ok = krow + it * KSTEP < krem;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[it][j] = ok ? (float)*reinterpret_cast<const T *>(q + (VEC ? ES * j : c[j])) : 0.0f;
        }
    }
};

template <class L>
__device__ __forceinline__ void load_tile(L &l)
{
    static_for<L::NLOAD>([&](auto ic) { l.template load_piece<decltype(ic)::value>(); });
    l.advance();
}
template <class L>
__device__ __forceinline__ void store_tile(const L &l, float *S)
{
    static_for<L::NSTORE>([&](auto ic) { l.template store_piece<decltype(ic)::value>(S); });
}

// ---------------------------------------------------------------------------------------------
// MFMA macro-tile.  A K tile is consumed in groups of 4 k (two MFMA k steps).  The operand fragments
// of a group are one LDS read per operand and k step, fetched one group ahead of the MFMAs that use
// them (and the first group of the next K tile during the last group of this one).
template <class Cfg>
struct Frag {
    typename VecOf<Cfg::MB>::type a[2];
    typename VecOf<Cfg::NB>::type b[2];
};

template <int N>
__device__ __forceinline__ float vec_elem(const typename VecOf<N>::type &v, int x)
{
    if constexpr (N == 1) return v; else return v[x];
}

// Fragment read piece R of k group G: R = 2*s2 + (0: rows operand, 1: cols operand).
// a_off[g] / b_off[g]: the lane's float offsets into a k row of k group g (rotation and its k = h row applied).
template <class Cfg, int G, int R>
__device__ __forceinline__ void load_frag_piece(Frag<Cfg> &f, const float *As, const float *Bs,
                                                const int (&a_off)[Cfg::KGROUPS], const int (&b_off)[Cfg::KGROUPS])
{
    typedef typename VecOf<Cfg::MB>::type AV;
    typedef typename VecOf<Cfg::NB>::type BV;
    constexpr int s2 = R / 2;
    if constexpr (R % 2 == 0)
        f.a[s2] = *reinterpret_cast<const AV *>(As + a_off[G] + (4 * G + 2 * s2) * Cfg::LDA);
    else
        f.b[s2] = *reinterpret_cast<const BV *>(Bs + b_off[G] + (4 * G + 2 * s2) * Cfg::LDB);
}
template <class Cfg, int G>
__device__ __forceinline__ void load_frag(Frag<Cfg> &f, const float *As, const float *Bs,
                                          const int (&a_off)[Cfg::KGROUPS], const int (&b_off)[Cfg::KGROUPS])
{
    static_for<4>([&](auto rc) { load_frag_piece<Cfg, G, decltype(rc)::value>(f, As, Bs, a_off, b_off); });
}

// MFMA number M (0 .. 2*MB*NB-1) of a k group.
template <class Cfg, int M>
__device__ __forceinline__ void mma_one(const Frag<Cfg> &f, floatx16 (&acc)[Cfg::MB][Cfg::NB])
{
    constexpr int s2 = M / (Cfg::MB * Cfg::NB), bm = (M / Cfg::NB) % Cfg::MB, bn = M % Cfg::NB;
    acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(vec_elem<Cfg::MB>(f.a[s2], bm), vec_elem<Cfg::NB>(f.b[s2], bn),
                                                       acc[bm][bn], 0, 0, 0);
}

// One K tile, generic form: `cur` holds group 0 on entry.  When next_A is not null, group 0 of that
// stage is left in `cur` on exit (it must already be visible in LDS).
template <class Cfg, int G>
__device__ __forceinline__ void mma_groups_from(Frag<Cfg> &cur, const float *As, const float *Bs, const float *next_A,
                                                const float *next_B, floatx16 (&acc)[Cfg::MB][Cfg::NB],
                                                const int (&a_off)[Cfg::KGROUPS], const int (&b_off)[Cfg::KGROUPS])
{
    Frag<Cfg> nxt;
    if constexpr (G + 1 < Cfg::KGROUPS) {
        load_frag<Cfg, G + 1>(nxt, As, Bs, a_off, b_off);
    } else {
        if (next_A != nullptr) load_frag<Cfg, 0>(nxt, next_A, next_B, a_off, b_off);
    }
    static_for<2 * Cfg::MB * Cfg::NB>([&](auto mc) { mma_one<Cfg, decltype(mc)::value>(cur, acc); });
    if constexpr (G + 1 < Cfg::KGROUPS) {
        cur = nxt;
        mma_groups_from<Cfg, G + 1>(cur, As, Bs, next_A, next_B, acc, a_off, b_off);
    } else {
        if (next_A != nullptr) cur = nxt;
    }
}

// One K tile in the steady state of the pipeline (no conditions: tile t+STAGES-1 is in registers and
// is stored, tile t+STAGES exists and is loaded, tile t+1 is visible in LDS).  CS is the stage of tile
// t, a compile-time constant, so every LDS address is a per-lane base plus an immediate.  A wave's
// MFMA stream only stays dense if the other instructions are issued in the shadow of MFMAs that are
// already running: each MFMA is followed by at most a few of them, in a fixed order pinned with
// scheduling barriers: first the fragment reads of the next k group, then the LDS stores of the
// staged tile, then the global loads of the tile after it.
// What separates the K tiles of a pipeline.  A workgroup that shares its LDS stages needs a barrier; a
// pipeline owned by a single wave needs none: the LDS executes one wave's accesses in program order.
struct BlockSync {
    static __device__ __forceinline__ void sync() { __syncthreads(); }
};
struct WaveSync {
    static __device__ __forceinline__ void sync() { __builtin_amdgcn_wave_barrier(); }
};

template <class Cfg, int CS, class Sync, class RL, class CL>
__device__ __forceinline__ void steady_iter(RL &rl, CL &cl, Frag<Cfg> &cur, floatx16 (&acc)[Cfg::MB][Cfg::NB],
                                            float *smem, const int (&a_off)[Cfg::KGROUPS],
                                            const int (&b_off)[Cfg::KGROUPS])
{
    constexpr int S = Cfg::STAGES, KG = Cfg::KGROUPS, NM = 2 * Cfg::MB * Cfg::NB;
    constexpr int FILL = (CS + S - 1) % S, NS = (CS + 1) % S;
    float *fill_a = smem + FILL * Cfg::STAGE_FLOATS, *fill_b = fill_a + Cfg::A_FLOATS;
    const float *As = smem + CS * Cfg::STAGE_FLOATS, *Bs = As + Cfg::A_FLOATS;
    const float *An = smem + NS * Cfg::STAGE_FLOATS, *Bn = An + Cfg::A_FLOATS;
    constexpr int NWA = RL::NSTORE, NWB = CL::NSTORE, NVA = RL::NLOAD, NVB = CL::NLOAD;
    constexpr int NSIDE = NWA + NWB + NVA + NVB;
    constexpr int SLOTS = KG * NM - (NM >= 4 ? 4 * KG : 0);  // slots not used by fragment reads
    constexpr int PER = (NSIDE + SLOTS - 1) / SLOTS;
    static_for<KG>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        Frag<Cfg> nxt;
        static_for<NM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mma_one<Cfg, m>(cur, acc);
            __builtin_amdgcn_sched_barrier(0);
            // fragment reads of the next group (of the next tile after the last group)
            static_for<4>([&](auto rc) {
                constexpr int r = decltype(rc)::value;
                constexpr int slot = NM >= 4 ? r : (r * NM) / 4;
                if constexpr (slot == m) {
                    if constexpr (g + 1 < KG)
                        load_frag_piece<Cfg, g + 1, r>(nxt, As, Bs, a_off, b_off);
                    else
                        load_frag_piece<Cfg, 0, r>(nxt, An, Bn, a_off, b_off);
                }
            });
            // staged tile -> LDS, then next tile -> registers
            if constexpr (NM < 4 || m >= 4) {
                constexpr int sl = g * (NM >= 4 ? NM - 4 : NM) + (NM >= 4 ? m - 4 : m);
                static_for<PER>([&](auto pc) {
                    constexpr int j = sl * PER + decltype(pc)::value;
                    if constexpr (j < NWA) {
                        rl.template store_piece<j>(fill_a);
                    } else if constexpr (j < NWA + NWB) {
                        cl.template store_piece<j - NWA>(fill_b);
                    } else if constexpr (j < NWA + NWB + NVA) {
                        rl.template load_piece<j - NWA - NWB>();
                        if constexpr (j == NWA + NWB + NVA - 1) rl.advance();
                    } else if constexpr (j < NSIDE) {
                        cl.template load_piece<j - NWA - NWB - NVA>();
                        if constexpr (j == NSIDE - 1) cl.advance();
                    }
                });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        cur = nxt;
    });
    Sync::sync();
}

// Software pipeline over the K range of one tile.  T full K tiles, then an optional partial one of
// krem (< BK) columns.  LDS holds STAGES tiles; registers hold one more in flight, so a global load
// has a whole K tile of MFMA work to land.  One barrier per K tile: the store of tile t+STAGES-1
// goes to the stage whose readers finished before the previous barrier.  With 3 or more stages tile
// t+1 is already visible while tile t is computed, which is what allows the fragment prefetch across
// the barrier and the branch-free steady state (steady_iter, unrolled over the stage ring); the first
// and last tiles, and 2-stage configurations, go through the generic loop with its conditions.
// tid: index of the thread among the Cfg::NT threads that run this pipeline (the workgroup's threads, or
// one wave's lanes when every wave of the workgroup runs a pipeline of its own on a part of K).
template <class Cfg, class RowLoader, class ColLoader, class Sync = BlockSync>
__device__ __forceinline__ void mainloop(RowLoader &rl, ColLoader &cl, int T, int krem,
                                         floatx16 (&acc)[Cfg::MB][Cfg::NB], float *smem, int tid = threadIdx.x)
{
    constexpr int S = Cfg::STAGES;
    constexpr bool kAhead = S >= 3;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM;
    const int wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const int i = lane & 31, h = lane >> 5;
    int a_off[Cfg::KGROUPS], b_off[Cfg::KGROUPS];
#pragma unroll
    for (int g = 0; g < Cfg::KGROUPS; ++g) {
        a_off[g] = h * Cfg::LDA + rot_col<Cfg::BM, Cfg::ROT>(wm0 + Cfg::MB * i, 4 * g);
        b_off[g] = h * Cfg::LDB + rot_col<Cfg::BN, Cfg::ROT>(wn0 + Cfg::NB * i, 4 * g);
    }

#pragma unroll
    for (int s = 0; s < S - 1; ++s) {
        if (s < T) {
            load_tile(rl);
            load_tile(cl);
            store_tile(rl, smem + s * Cfg::STAGE_FLOATS);
            store_tile(cl, smem + s * Cfg::STAGE_FLOATS + Cfg::A_FLOATS);
        }
    }
    if (S - 1 < T) {
        load_tile(rl);
        load_tile(cl);
    }
    Sync::sync();

    Frag<Cfg> cur;
    if (T > 0) load_frag<Cfg, 0>(cur, smem, smem + Cfg::A_FLOATS, a_off, b_off);
    int t = 0;
    if constexpr (kAhead) {
        // S iterations at a time keep the stage of tile t equal to 0 at the top of the loop
        while (t + 2 * S - 1 < T) {
            static_for<S>([&](auto sc) { steady_iter<Cfg, decltype(sc)::value, Sync>(rl, cl, cur, acc, smem, a_off, b_off); });
            t += S;
        }
    }
    int cs = 0;        // stage holding tile t (t is a multiple of S here)
    int fill = S - 1;  // stage that receives tile t + S - 1
    for (; t < T; ++t) {
        if (t + S - 1 < T) {
            store_tile(rl, smem + fill * Cfg::STAGE_FLOATS);
            store_tile(cl, smem + fill * Cfg::STAGE_FLOATS + Cfg::A_FLOATS);
        }
        if (t + S < T) {
            load_tile(rl);
            load_tile(cl);
        }
        const int ns = (cs + 1 == S) ? 0 : cs + 1;
        const float *As = smem + cs * Cfg::STAGE_FLOATS;
        const float *An = smem + ns * Cfg::STAGE_FLOATS;
        const bool more = t + 1 < T;
        mma_groups_from<Cfg, 0>(cur, As, As + Cfg::A_FLOATS, (kAhead && more) ? An : nullptr, An + Cfg::A_FLOATS, acc,
                                a_off, b_off);
        cs = ns;
        fill = (fill + 1 == S) ? 0 : fill + 1;
        Sync::sync();
        if (!kAhead && more) load_frag<Cfg, 0>(cur, An, An + Cfg::A_FLOATS, a_off, b_off);
    }
    if (krem > 0) {
        rl.load_tail(krem);
        cl.load_tail(krem);
        store_tile(rl, smem);
        store_tile(cl, smem + Cfg::A_FLOATS);
        Sync::sync();
        load_frag<Cfg, 0>(cur, smem, smem + Cfg::A_FLOATS, a_off, b_off);
        mma_groups_from<Cfg, 0>(cur, smem, smem + Cfg::A_FLOATS, nullptr, nullptr, acc, a_off, b_off);
    }
}

// ---------------------------------------------------------------------------------------------
// Split tiles.  When the tile grid does not fill the device evenly, the tiles past the last full
// round (or all tiles of a skinny product) are cut into `splits` slices along K, one workgroup each.
// A slice leaves its raw accumulators in the workspace and bumps the tile's counter; whichever slice
// arrives last adds the others to its own registers and runs the epilogue.  Nobody waits (a counter
// is only ever incremented and read by its incrementer), and the slices are always added in slice
// order, block by block, so the result does not depend on which slice finishes last: same bits every
// run, as the paper's remarks on reproducibility ask of a library wherever it is affordable.
struct SplitPlan {
    int dp_tiles;        // tiles [0, dp_tiles) are computed whole by one workgroup each
    int splits;          // every later tile is cut into this many K slices (1: no tile is split)
    float *partials;     // [(tile - dp_tiles) * splits + slice][MB*NB blocks][4][NT][4] floats
    unsigned *counters;  // one per split tile, zero at launch
    // Plain split-K (every tile split, combined by a second kernel): slice z of the whole product is
    // written as a dense M x N array at partials + z * slice_stride; no counters.
    int plain;
    int64_t slice_stride;
};

// Which tile (index in raster order) and which K slice a workgroup owns.
struct WorkItem {
    int tile;    // raster index of the tile
    int slice;   // K slice, 0 when the tile is not split
    int nslice;  // number of slices of this tile (1 or splits)
    int sq;      // index among the split tiles (for partials / counters)
};

__device__ __forceinline__ int xcd_contiguous_id(int bid, int total);

// The K slices of split tiles take the FIRST workgroup ids, the whole tiles the rest.  A slice is short
// (a fraction of the K range, then its partial sums go to the workspace and the last one to arrive adds
// them up): run at the end of the launch its fill, drain and combination would be all a compute unit has
// to do, run at the start they overlap the whole tiles resident beside it.
__device__ __forceinline__ WorkItem work_item(int bid, int tiles, const SplitPlan &sp)
{
    WorkItem w;
    const int nsplit = (tiles - sp.dp_tiles) * sp.splits;   // workgroups that own a slice
    if (bid >= nsplit) {
        // bid - nsplit, not bid: the dies then still get contiguous runs of tile ids (only which die
        // gets which run rotates)
        w.tile = xcd_contiguous_id(bid - nsplit, sp.dp_tiles);
        w.slice = 0;
        w.nslice = 1;
        w.sq = 0;
    } else {
        w.sq = bid / sp.splits;
        w.slice = bid - w.sq * sp.splits;
        w.nslice = sp.splits;
        w.tile = sp.dp_tiles + w.sq;
    }
    return w;
}

// K tiles [first, first + count) and the partial tile (krem columns) of slice `slice` of `nslice`.
__device__ __forceinline__ void slice_range(int ktiles_total, int krem_total, int slice, int nslice, int &first,
                                            int &count, int &krem)
{
    const int per = ktiles_total / nslice;
    first = slice * per;
    const bool last = slice == nslice - 1;
    count = last ? ktiles_total - first : per;
    krem = last ? krem_total : 0;
}

// Returns true when this workgroup has to run the epilogue (its tile is whole, or it is the last
// slice of its tile to arrive, in which case acc holds the sum over all slices on return).
template <class Cfg>
__device__ __forceinline__ bool combine_slices(floatx16 (&acc)[Cfg::MB][Cfg::NB], const SplitPlan &sp, const WorkItem &w)
{
    if (w.nslice == 1 || sp.plain) return true;
    constexpr int NBLK = Cfg::MB * Cfg::NB;
    const size_t slot_floats = (size_t)NBLK * 16 * Cfg::NT;
    float *mine = sp.partials + ((size_t)w.sq * w.nslice + w.slice) * slot_floats;
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                floatx4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = acc[bm][bn][4 * r4 + e];
                *reinterpret_cast<floatx4 *>(mine + ((size_t)((bm * Cfg::NB + bn) * 4 + r4) * Cfg::NT + threadIdx.x) * 4) = o;
            }
    // Publication.  The dies' L2 caches are not coherent with each other: a device-scope release writes
    // back the whole L2 of the die and an acquire invalidates it (and the unit's first-level cache), for
    // every wave that executes one.  One lane does each for the workgroup: every wave waits for its own
    // stores before the barrier, so they are all in L2 when the lane's release fence writes it back
    // before its counter increment; on the other side the lane that saw the last increment acquires, and
    // the barrier after it orders every wave's reads behind that.  A slice that is not the last to arrive
    // invalidates nothing, so the tiles resident beside it keep their operand panels in L2 (with a fence
    // in every wave, 692 slices beside 256 whole tiles ran 909 us against 550 us without the split).
    __shared__ unsigned arrived;
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's stores have been acknowledged by L2
    __syncthreads();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        arrived = atomicAdd(sp.counters + w.sq, 1u);
    }
    __syncthreads();
    if (arrived != (unsigned)(w.nslice - 1)) return false;
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    __syncthreads();
    const float *base = sp.partials + (size_t)w.sq * w.nslice * slot_floats;
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn) {
            floatx16 tot;
            for (int z = 0; z < w.nslice; ++z) {
                floatx16 part;
                if (z == w.slice) {
                    part = acc[bm][bn];
                } else {
                    const float *src = base + (size_t)z * slot_floats;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const floatx4 q = *reinterpret_cast<const floatx4 *>(
                            src + ((size_t)((bm * Cfg::NB + bn) * 4 + r4) * Cfg::NT + threadIdx.x) * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) part[4 * r4 + e] = q[e];
                    }
                }
                if (z == 0) tot = part; else tot += part;
            }
            acc[bm][bn] = tot;
        }
    return true;
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
