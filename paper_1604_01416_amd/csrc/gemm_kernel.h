// GEMM kernel: C = alpha * op(A) * op(B) + beta * C on one BM x BN tile per workgroup, and its
// host-side launcher template.  Included by one translation unit per tile configuration.
#pragma once
#include <type_traits>

#include "tile_core.h"

namespace dmath {

// T: stored element type of A, B and C (float, or _Float16 for half-precision storage; the arithmetic
// is FP32 either way).
template <class T>
struct GemmArgsT {
    const T *A;
    const T *B;
    T *C;
    int64_t lda, ldb, ldc;
    int64_t M, N, K;
    float alpha, beta;
    int tiles_m, tiles_n;
    int cvec;         // C rows allow aligned NB-wide vector access (1), and C is large enough to be streamed (2)
    SplitPlan split;
    unsigned stagger_ticks = 0;  // 0, or how long workgroups 256..511 wait before they start (100 MHz ticks)
    unsigned long long *clock_probe;  // optional: 4 stamps from each of workgroups 0..7 (see dmath_set_clock_probe)
};
typedef GemmArgsT<float> GemmArgs;
typedef GemmArgsT<_Float16> HGemmArgs;

template <class Cfg, bool ROWS_K, bool VEC, class T = float, class OffT = uint32_t>
struct RowLoaderSel {
    typedef typename LoaderKSel<Cfg::LKV, Cfg::BM, Cfg::BK, Cfg::NT, Cfg::LDA, Cfg::ROT, VEC, T, OffT>::type type;
};
template <class Cfg, bool VEC, class T, class OffT>
struct RowLoaderSel<Cfg, false, VEC, T, OffT> {
    typedef LoaderMN<Cfg::BM, Cfg::BK, Cfg::NT, Cfg::LDA, Cfg::ROT, VEC, T, 1, OffT> type;
};
template <class Cfg, bool COLS_K, bool VEC, class T = float, class OffT = uint32_t>
struct ColLoaderSel {
    typedef typename LoaderKSel<Cfg::LKV, Cfg::BN, Cfg::BK, Cfg::NT, Cfg::LDB, Cfg::ROT, VEC, T, OffT>::type type;
};
template <class Cfg, bool VEC, class T, class OffT>
struct ColLoaderSel<Cfg, false, VEC, T, OffT> {
    typedef LoaderMN<Cfg::BN, Cfg::BK, Cfg::NT, Cfg::LDB, Cfg::ROT, VEC, T, 1, OffT> type;
};

// Epilogue of a product whose result is a row-major matrix: out = alpha*acc + beta*out with edge
// predication.  Lane (i, h) owns, for block row bm and accumulator register r, the NB consecutive
// columns n0 + wn0 + NB*i .. of row m0 + wm0 + MB*(8*(r/4) + 4*h + r%4) + bm.  A slice of a plain
// split-K launch writes its raw sums to its M x N array in the workspace instead.
// stream_c: C is large (the host sets it from 32 MiB on, more than the L2 caches hold together): it is read once
// and written once per launch and nobody finds it in a cache afterwards, so the 16-byte accesses of the epilogue
// carry the non-temporal hint and do not push the operand panels out of L2 under the workgroups still multiplying
// (config 3 call 502.8 -> 499.4 us, 4096 x 4096 x 256: 69.1 -> 68.5 us; 4096^3 unchanged).  A smaller result is
// left in the caches for whoever consumes it next.
constexpr int kEpiRows = 8;  // old values of C fetched per batch in the epilogue (4, 8 and 16 measure alike)
template <class Cfg>
__device__ __forceinline__ void store_tile_rowmajor(const floatx16 (&acc)[Cfg::MB][Cfg::NB], float *C, int64_t ldc_,
                                                    int64_t M, int64_t N, float alpha_, float beta_, bool cvec,
                                                    int64_t m0, int64_t n0, const SplitPlan &split, const WorkItem &w,
                                                    bool stream_c = false)
{
    typedef typename VecOf<Cfg::NB>::type CV;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const int64_t col = n0 + wn0 + Cfg::NB * i;
    const bool raw_slice = split.plain && w.nslice > 1;  // plain split-K: raw sums to the workspace
    float *Cz = raw_slice ? split.partials + (int64_t)w.slice * split.slice_stride : C;
    const int64_t ldc = raw_slice ? N : ldc_;
    const float alpha = raw_slice ? 1.0f : alpha_, beta = raw_slice ? 0.0f : beta_;
    const bool full_vec = (raw_slice ? (N % 4 == 0) : cvec) && (col + Cfg::NB <= N);
    if constexpr (Cfg::NB > 1) {
        if (full_vec && beta != 0.0f) {
            // Old values are fetched eight rows at a time before any of them is used: one load per row
            // followed by its use would leave a single 16-byte request per wave in flight and make the
            // epilogue wait out the memory latency 16*MB times.  Rows past M read row M-1 (never stored).
#pragma unroll
            for (int bm = 0; bm < Cfg::MB; ++bm) {
#pragma unroll
                for (int r0 = 0; r0 < 16; r0 += kEpiRows) {
                    CV old[kEpiRows];
#pragma unroll
                    for (int j = 0; j < kEpiRows; ++j) {
                        const int r = r0 + j;
                        const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
                        const CV *src = reinterpret_cast<const CV *>(Cz + (row < M ? row : M - 1) * ldc + col);
                        old[j] = stream_c ? __builtin_nontemporal_load(src) : *src;
                    }
#pragma unroll
                    for (int j = 0; j < kEpiRows; ++j) {
                        const int r = r0 + j;
                        const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
                        CV o;
#pragma unroll
                        for (int bn = 0; bn < Cfg::NB; ++bn) o[bn] = __builtin_fmaf(beta, old[j][bn], alpha * acc[bm][bn][r]);
                        if (row < M) {
                            if (stream_c)
                                __builtin_nontemporal_store(o, reinterpret_cast<CV *>(Cz + row * ldc + col));
                            else
                                *reinterpret_cast<CV *>(Cz + row * ldc + col) = o;
                        }
                    }
                }
            }
            return;
        }
    }
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
            if (row >= M) continue;
            float *dst = Cz + row * ldc + col;
            float out[Cfg::NB];
#pragma unroll
            for (int bn = 0; bn < Cfg::NB; ++bn) out[bn] = alpha * acc[bm][bn][r];
            if (full_vec) {
                CV o;
                if constexpr (Cfg::NB == 1) {
                    o = out[0];
                    if (beta != 0.0f) o += beta * *dst;
                    *dst = o;
                } else {
                    if (beta != 0.0f) {
                        const CV old = *reinterpret_cast<const CV *>(dst);
#pragma unroll
                        for (int bn = 0; bn < Cfg::NB; ++bn) out[bn] += beta * old[bn];
                    }
#pragma unroll
                    for (int bn = 0; bn < Cfg::NB; ++bn) o[bn] = out[bn];
                    if (stream_c && !raw_slice)   // (a raw slice is read back at once by the kernel that adds the slices)
                        __builtin_nontemporal_store(o, reinterpret_cast<CV *>(dst));
                    else
                        *reinterpret_cast<CV *>(dst) = o;
                }
            } else {
#pragma unroll
                for (int bn = 0; bn < Cfg::NB; ++bn) {
                    if (col + bn < N) {
                        float o = out[bn];
                        if (beta != 0.0f) o += beta * dst[bn];
                        dst[bn] = o;
                    }
                }
            }
        }
    }
}

// The same epilogue for C kept in half-precision storage: out = half(alpha*acc + beta*float(out)),
// rounded to nearest even once.  Raw split-K slices stay FP32 and go through the float version.
template <class Cfg>
__device__ __forceinline__ void store_tile_rowmajor(const floatx16 (&acc)[Cfg::MB][Cfg::NB], _Float16 *C, int64_t ldc,
                                                    int64_t M, int64_t N, float alpha, float beta, bool cvec,
                                                    int64_t m0, int64_t n0, const SplitPlan &split, const WorkItem &w,
                                                    bool = false)
{
    if (split.plain && w.nslice > 1) {
        store_tile_rowmajor<Cfg>(acc, static_cast<float *>(nullptr), N, M, N, 1.0f, 0.0f, false, m0, n0, split, w);
        return;
    }
    typedef _Float16 HV __attribute__((ext_vector_type(Cfg::NB)));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const int64_t col = n0 + wn0 + Cfg::NB * i;
    const bool full_vec = cvec && Cfg::NB > 1 && (col + Cfg::NB <= N);
    if constexpr (Cfg::NB > 1) {
        if (full_vec && beta != 0.0f) {
            // old values fetched kEpiRows rows at a time before the first use, as in the FP32 epilogue
#pragma unroll
            for (int bm = 0; bm < Cfg::MB; ++bm) {
#pragma unroll
                for (int r0 = 0; r0 < 16; r0 += kEpiRows) {
                    HV old[kEpiRows];
#pragma unroll
                    for (int j = 0; j < kEpiRows; ++j) {
                        const int r = r0 + j;
                        const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
                        old[j] = *reinterpret_cast<const HV *>(C + (row < M ? row : M - 1) * ldc + col);
                    }
#pragma unroll
                    for (int j = 0; j < kEpiRows; ++j) {
                        const int r = r0 + j;
                        const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
                        HV o;
#pragma unroll
                        for (int bn = 0; bn < Cfg::NB; ++bn)
                            o[bn] = (_Float16)__builtin_fmaf(beta, (float)old[j][bn], alpha * acc[bm][bn][r]);
                        if (row < M) *reinterpret_cast<HV *>(C + row * ldc + col) = o;
                    }
                }
            }
            return;
        }
    }
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
            if (row >= M) continue;
            _Float16 *dst = C + row * ldc + col;
            float out[Cfg::NB];
#pragma unroll
            for (int bn = 0; bn < Cfg::NB; ++bn) out[bn] = alpha * acc[bm][bn][r];
            if constexpr (Cfg::NB > 1) {
                if (full_vec) {
                    if (beta != 0.0f) {
                        const HV old = *reinterpret_cast<const HV *>(dst);
#pragma unroll
                        for (int bn = 0; bn < Cfg::NB; ++bn) out[bn] += beta * (float)old[bn];
                    }
                    HV o;
#pragma unroll
                    for (int bn = 0; bn < Cfg::NB; ++bn) o[bn] = (_Float16)out[bn];
                    *reinterpret_cast<HV *>(dst) = o;
                    continue;
                }
            }
#pragma unroll
            for (int bn = 0; bn < Cfg::NB; ++bn) {
                if (col + bn < N) {
                    float o = out[bn];
                    if (beta != 0.0f) o += beta * (float)dst[bn];
                    dst[bn] = (_Float16)o;
                }
            }
        }
    }
}

// A_KCONTIG: A stored M x K (transA == N).  B_KCONTIG: B stored N x K (transB == T).
// VEC: every 16-byte global load of A and B is aligned and wholly inside the matrix.
// OffT: uint32_t, or uint64_t when a leading dimension is too large for 32-bit per-thread byte offsets
// (a block that is a window of a row panel more than 2^22 elements wide).
template <class Cfg, bool A_KCONTIG, bool B_KCONTIG, bool VEC, class ElemT = float, class OffT = uint32_t>
__global__ __launch_bounds__(Cfg::NT, Cfg::MIN_WAVES) void gemm_tile_kernel(const GemmArgsT<ElemT> g)
{
    __shared__ __attribute__((aligned(16))) float smem[Cfg::STAGES * Cfg::STAGE_FLOATS];

    // Workgroups 0..7 are the first ones handed to each of the 8 dies, which clock independently.
    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 0] = __builtin_readcyclecounter();      // shader-clock counter
        g.clock_probe[blockIdx.x * 4 + 1] = __builtin_amdgcn_s_memrealtime();  // fixed 100 MHz counter
    }
    // Second workgroup of every compute unit (the dispatcher places workgroups 0..255 one per unit and
    // the next 256 beside them): held back so that the two run out of phase and one's epilogue falls
    // into the other's K loop.  The wait is on the free-running 100 MHz counter and always ends.
    if (g.stagger_ticks != 0 && blockIdx.x >= kNumCU && blockIdx.x < 2 * kNumCU) {
        const uint64_t t0 = __builtin_amdgcn_s_memrealtime();
        while (__builtin_amdgcn_s_memrealtime() - t0 < (uint64_t)g.stagger_ticks) __builtin_amdgcn_s_sleep(16);
    }
    const int tiles = g.tiles_m * g.tiles_n;
    const WorkItem w = work_item(blockIdx.x, tiles, g.split);
    int tm, tn;
    tile_coords<8>(w.tile, g.tiles_m, g.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * Cfg::BM, n0 = (int64_t)tn * Cfg::BN;

    // K range of this workgroup: the whole K, or one slice of it
    const int ktiles_total = (int)(g.K / Cfg::BK);
    int kt0, T, krem;
    slice_range(ktiles_total, (int)(g.K - (int64_t)ktiles_total * Cfg::BK), w.slice, w.nslice, kt0, T, krem);
    const int64_t k0 = (int64_t)kt0 * Cfg::BK;

    typename RowLoaderSel<Cfg, A_KCONTIG, VEC, ElemT, OffT>::type rl;
    typename ColLoaderSel<Cfg, B_KCONTIG, VEC, ElemT, OffT>::type cl;
    rl.init(g.A, g.lda, m0, g.M, k0, threadIdx.x);
    cl.init(g.B, g.ldb, n0, g.N, k0, threadIdx.x);

    floatx16 acc[Cfg::MB][Cfg::NB];
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.0f;

    mainloop<Cfg>(rl, cl, T, krem, acc, smem);
    if (!combine_slices<Cfg>(acc, g.split, w)) return;

    store_tile_rowmajor<Cfg>(acc, g.C, g.ldc, g.M, g.N, g.alpha, g.beta, g.cvec != 0, m0, n0, g.split, w, g.cvec == 2);
    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 2] = __builtin_readcyclecounter();
        g.clock_probe[blockIdx.x * 4 + 3] = __builtin_amdgcn_s_memrealtime();
    }
}

// Host side: pick the instantiation for the operand orientations and alignment, and launch.
// wide: a leading dimension of A or B is above 2^22, the kernel needs 64-bit per-thread offsets; only
// the 128 x 128 configuration with the padded LDS image carries those instantiations (the host plans
// such calls on it), every other one answers hipErrorInvalidValue.
// Returns the hipError_t of the launch as int.
template <class Cfg, class T = float>
int launch_gemm_cfg(const GemmArgsT<T> &g, bool a_kcontig, bool b_kcontig, bool vec, bool wide, hipStream_t stream)
{
    constexpr bool kHasWide = Cfg::BM == 128 && Cfg::BN == 128 && Cfg::LKV == 0;
    // half-precision storage is offered on the padded LDS image only
    if constexpr (!std::is_same<T, float>::value && Cfg::LKV != 0) {
        return (int)hipErrorInvalidValue;
    } else {
    if (wide && !kHasWide) return (int)hipErrorInvalidValue;
    const int tiles = g.tiles_m * g.tiles_n;
    const dim3 grid((unsigned)(g.split.dp_tiles + (tiles - g.split.dp_tiles) * g.split.splits)), block(Cfg::NT);
#define DMATH_LAUNCH(AK, BK_, V, OFF) \
    hipLaunchKernelGGL((gemm_tile_kernel<Cfg, AK, BK_, V, T, OFF>), grid, block, 0, stream, g)
#define DMATH_LAUNCH_ALL(OFF) \
    if (vec) { \
        if (a_kcontig && b_kcontig) DMATH_LAUNCH(true, true, true, OFF); \
        else if (a_kcontig) DMATH_LAUNCH(true, false, true, OFF); \
        else if (b_kcontig) DMATH_LAUNCH(false, true, true, OFF); \
        else DMATH_LAUNCH(false, false, true, OFF); \
    } else { \
        if (a_kcontig && b_kcontig) DMATH_LAUNCH(true, true, false, OFF); \
        else if (a_kcontig) DMATH_LAUNCH(true, false, false, OFF); \
        else if (b_kcontig) DMATH_LAUNCH(false, true, false, OFF); \
        else DMATH_LAUNCH(false, false, false, OFF); \
    }
    if constexpr (kHasWide) {
        if (wide) {
            DMATH_LAUNCH_ALL(uint64_t)
            return (int)hipGetLastError();
        }
    }
    DMATH_LAUNCH_ALL(uint32_t)
#undef DMATH_LAUNCH_ALL
#undef DMATH_LAUNCH
    return (int)hipGetLastError();
    }
}

}  // namespace dmath
