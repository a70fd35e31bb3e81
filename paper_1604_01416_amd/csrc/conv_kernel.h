// Forward convolution as an implicit GEMM on the same macro-tile as dmath_gemm:
//
//     y_mat[Kout x (N*P*Q)] = w_mat[Kout x (C*R*S)] * x_unfolded[(C*R*S) x (N*P*Q)]
//
// Rows of the product are output channels (the filters, read in place: w is already a
// Kout x CRS row-major matrix, contiguous along k), columns are output pixels (n, p, q) in memory
// order, so a row of the product is contiguous in y inside one image.  The unfolded matrix is
// never stored: the loaders below generate each of its elements from x with the zero halo applied.
// column = (n*P + p)*Q + q.  Two orders of k are implemented (any order gives the same sums):
//   - generic (LoaderConvX): k = (c*R + r)*S + s, the order of w in memory; works for every shape.
//     Its backward-data form generates the operand of the data gradient instead (see below).
//   - tap-major (LoaderConvTap): k = ((cb*R + r)*S + s)*BK + cc for channel c = cb*BK + cc, with C a
//     multiple of the K tile BK, so a K tile is BK channels of ONE filter tap: the halo test and the
//     tap offset are per tile instead of per element, and a K row is a plain scalar offset H*W away
//     from the previous one.  The R*S taps of a channel block are consecutive K tiles, so the pixels
//     of those channels are re-read while still in cache.  The filters are first re-laid out as
//     w'[j][cb][r][s][cc] into the workspace by a small kernel.
#pragma once
#include "tile_core.h"

namespace dmath {

struct ConvArgs {
    const float *x;
    const float *w;
    float *y;
    int N, C, H, W, Kout, R, S, P, Q;
    int pad_h, pad_w, stride_h, stride_w;
    int RS, PQ;
    int64_t CRS, NPQ;
    uint32_t magic_RS, magic_S;  // ceil(2^32 / d) for d > 1 (see fast_div); unused for d == 1
    uint32_t magic_sh, magic_sw; // the same for the strides (backward-data form of the generic loader)
    float alpha, beta;
    int tiles_m, tiles_n;
    int yvec;  // y is 16-byte aligned and P*Q is a multiple of 4 (1), and y is large enough to be streamed (2)
    int64_t x_bytes;  // size of x, for the buffer descriptor of the tap-major loader
    SplitPlan split;
};

// floor(n / d) for a divisor fixed at launch: with magic = ceil(2^32 / d) the high word of n*magic is
// exact as long as n * d < 2^32, which the host checks for the ranges used (k < C*R*S + BK by R*S, and
// a tap index < R*S by S).  d == 1 has no 32-bit magic and is passed through.
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t magic, int d)
{
    return d == 1 ? n : __umulhi(n, magic);
}

// Loader of the generated operand.  Lanes run along the output pixels (contiguous q in x), each
// thread keeps one column and walks k; k is uniform over a wave, so (c, r, s) and the offset of the
// tap are scalar work, and only the halo test and the load itself are per lane.
//
// BWD = true generates the operand of the data gradient: the columns are the pixels (n, h, w) of dx,
// k = (j*R + r)*S + s runs over output channels and taps, and the element is dy[n][j][p][q] with
// p = (h + pad_h - r) / stride_h, q = (w + pad_w - s) / stride_w when both divisions are exact and
// land inside dy, else 0.  In that form the ConvArgs fields describe the roles, not the names:
// x = dy, C = Kout, H x W = the P x Q extent of dy, P x Q = the H x W extent of dx.
template <int BN, int BK, int NT, int LD, int ROT, bool BWD>
struct LoaderConvX {
    static constexpr int KG = NT / BN;  // k rows loaded side by side
    static constexpr int NQ = BK / KG;  // k rows per thread and tile
    static constexpr int NLOAD = NQ, NSTORE = NQ;
    static_assert(NT % BN == 0 && BK % KG == 0 && BN % 64 == 0 && NQ >= 1, "one column per thread");
    const float *xcol;  // x + n*C*H*W + ih0*W + iw0 (the tap (c=0, r=0, s=0); may lie in the halo)
    int ih0, iw0;
    bool col_ok;
    int col, kg;
    int knext;  // first k of the next tile to load
    int H, W, S, RS, HW;
    int64_t CRS;
    uint32_t magic_RS, magic_S;
    int sh, sw;
    uint32_t magic_sh, magic_sw;
    float v[NQ];

    __device__ __forceinline__ void init(const ConvArgs &a, int64_t c0, int kstart, int tid)
    {
        col = tid % BN;
        kg = __builtin_amdgcn_readfirstlane(tid / BN);
        knext = kstart;
        H = a.H; W = a.W; S = a.S; RS = a.RS; HW = a.H * a.W; CRS = a.CRS;
        magic_RS = a.magic_RS; magic_S = a.magic_S;
        sh = a.stride_h; sw = a.stride_w; magic_sh = a.magic_sh; magic_sw = a.magic_sw;
        int64_t gc = c0 + col;
        col_ok = gc < a.NPQ;
        gc = col_ok ? gc : a.NPQ - 1;
        const int n = (int)(gc / a.PQ);
        const int pq = (int)(gc - (int64_t)n * a.PQ);
        const int p = pq / a.Q, q = pq - p * a.Q;
        if (BWD) {
            ih0 = p + a.pad_h;
            iw0 = q + a.pad_w;
            xcol = a.x + (int64_t)n * a.C * HW;
        } else {
            ih0 = p * a.stride_h - a.pad_h;
            iw0 = q * a.stride_w - a.pad_w;
            xcol = a.x + (int64_t)n * a.C * HW + (int64_t)ih0 * W + iw0;
        }
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        const uint32_t k = (uint32_t)(knext + kg + I * KG);
        const uint32_t c = fast_div(k, magic_RS, RS);
        const uint32_t rs = k - c * (uint32_t)RS;
        const uint32_t r = fast_div(rs, magic_S, S);
        const uint32_t s = rs - r * (uint32_t)S;
        if (BWD) {
            const int th = ih0 - (int)r, tw = iw0 - (int)s;
            const uint32_t p = fast_div((uint32_t)(th < 0 ? 0 : th), magic_sh, sh);
            const uint32_t q = fast_div((uint32_t)(tw < 0 ? 0 : tw), magic_sw, sw);
            const bool ok = col_ok && (int64_t)k < CRS && th >= 0 && tw >= 0 && (int)(p * (uint32_t)sh) == th &&
                            (int)(q * (uint32_t)sw) == tw && p < (uint32_t)H && q < (uint32_t)W;
            v[I] = ok ? xcol[(int)c * HW + (int)p * W + (int)q] : 0.0f;
        } else {
            const int off = (int)c * HW + (int)r * W + (int)s;
            const bool ok = col_ok && (int64_t)k < CRS && (unsigned)(ih0 + (int)r) < (unsigned)H &&
                            (unsigned)(iw0 + (int)s) < (unsigned)W;
            v[I] = ok ? xcol[off] : 0.0f;
        }
    }
    __device__ __forceinline__ void advance() { knext += BK; }
    // the partial last tile needs nothing special: k >= C*R*S is already generated as zero
    __device__ __forceinline__ void load_tail(int)
    {
        static_for<NQ>([&](auto ic) { load_piece<decltype(ic)::value>(); });
    }
    template <int I>
    __device__ __forceinline__ void store_piece(float *Sm) const
    {
        const int k = kg + I * KG;
        Sm[k * LD + rot_col<BN, ROT>(col, k)] = v[I];
    }
};

// Tap-major loader of the generated operand (see the top of the file).  x is read through a buffer
// descriptor whose base is shifted down by pad_h*W + pad_w elements: the lane offset (of the pixel's
// (r=0, s=0) tap) is then never negative, the tap and channel offset is one scalar, and a lane whose
// tap falls into the halo gets an offset beyond the descriptor, which makes the hardware return 0.
template <int BN, int BK, int NT, int LD, int ROT>
struct LoaderConvTap {
    static constexpr int KG = NT / BN;
    static constexpr int NQ = BK / KG;
    static constexpr int NLOAD = NQ, NSTORE = NQ;
    static_assert(NT % BN == 0 && BK % KG == 0 && BN % 64 == 0 && NQ >= 1, "one column per thread");
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t voff;      // byte offset of the lane's (r=0, s=0) tap of channel 0 in the shifted buffer
    uint32_t tapmask;   // bit r*S+s set when that tap of this pixel lies inside x (0 for a column past the end)
    uint32_t tile_voff, tile_soff;
    int col, kg;
    int c0, r, s;       // first channel and tap of the next tile to load
    int HW, W, R, S;
    float v[NQ];

    __device__ __forceinline__ void init(const ConvArgs &a, int64_t col0, int kstart, int tid)
    {
        col = tid % BN;
        kg = __builtin_amdgcn_readfirstlane(tid / BN);
        HW = a.H * a.W; W = a.W; R = a.R; S = a.S;
        const int t0 = kstart / BK;     // kstart is a multiple of the K tile
        const int cb = t0 / a.RS, tap0 = t0 - cb * a.RS;
        c0 = cb * BK;
        r = tap0 / a.S;
        s = tap0 - r * a.S;
        const int shift = a.pad_h * a.W + a.pad_w;
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x) - shift, 0,
                                                 (int)(a.x_bytes + (int64_t)shift * 4), 0x00020000);
        int64_t gc = col0 + col;
        const bool col_ok = gc < a.NPQ;
        gc = col_ok ? gc : a.NPQ - 1;
        const int n = (int)(gc / a.PQ);
        const int pq = (int)(gc - (int64_t)n * a.PQ);
        const int p = pq / a.Q, q = pq - p * a.Q;
        const int ih0 = p * a.stride_h - a.pad_h, iw0 = q * a.stride_w - a.pad_w;
        voff = (uint32_t)(((int64_t)n * a.C * HW + (int64_t)ih0 * W + iw0 + shift) * 4);
        uint32_t m = 0;
        for (int rr = 0; rr < a.R; ++rr)
            for (int ss = 0; ss < a.S; ++ss)
                if ((unsigned)(ih0 + rr) < (unsigned)a.H && (unsigned)(iw0 + ss) < (unsigned)a.W) m |= 1u << (rr * a.S + ss);
        tapmask = col_ok ? m : 0u;
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        if constexpr (I == 0) {
            const bool ok = (tapmask >> (r * S + s)) & 1u;
            tile_voff = ok ? voff : 0x80000000u;
            tile_soff = (uint32_t)(((c0 + kg) * HW + r * W + s) * 4);
        }
        // the builtin returns the loaded dword as an unsigned integer
        v[I] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, tile_voff, tile_soff + (uint32_t)(I * KG * HW * 4), 0));
    }
    __device__ __forceinline__ void advance()
    {
        if (++s == S) {
            s = 0;
            if (++r == R) {
                r = 0;
                c0 += BK;
            }
        }
    }
    __device__ __forceinline__ void load_tail(int) {}  // C is a multiple of BK on this path: no partial tile
    template <int I>
    __device__ __forceinline__ void store_piece(float *Sm) const
    {
        const int k = kg + I * KG;
        Sm[k * LD + rot_col<BN, ROT>(col, k)] = v[I];
    }
};

// Which generator of the unfolded operand a kernel uses.
enum ConvLoaderKind { kConvGeneric = 0, kConvTapMajor = 1, kConvBwdData = 2 };

template <class Cfg, int KIND>
struct ConvColLoaderSel {
    typedef LoaderConvX<Cfg::BN, Cfg::BK, Cfg::NT, Cfg::LDB, Cfg::ROT, KIND == kConvBwdData> type;
};
template <class Cfg>
struct ConvColLoaderSel<Cfg, kConvTapMajor> {
    typedef LoaderConvTap<Cfg::BN, Cfg::BK, Cfg::NT, Cfg::LDB, Cfg::ROT> type;
};

// VEC: 16-byte loads of the filter matrix are aligned.  KIND: generator of the other operand; for the
// tap-major and backward-data kinds a.w is the filter matrix re-laid out in the workspace.
template <class Cfg, bool VEC, int KIND>
__global__ __launch_bounds__(Cfg::NT, Cfg::MIN_WAVES) void conv_tile_kernel(const ConvArgs a)
{
    __shared__ __attribute__((aligned(16))) float smem[Cfg::STAGES * Cfg::STAGE_FLOATS];

    const int tiles = a.tiles_m * a.tiles_n;
    const WorkItem wi = work_item(blockIdx.x, tiles, a.split);
    int tm, tn;
    tile_coords<8>(wi.tile, a.tiles_m, a.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * Cfg::BM, n0 = (int64_t)tn * Cfg::BN;

    const int ktiles_total = (int)(a.CRS / Cfg::BK);
    int kt0, T, krem;
    slice_range(ktiles_total, (int)(a.CRS - (int64_t)ktiles_total * Cfg::BK), wi.slice, wi.nslice, kt0, T, krem);

    typename LoaderKSel<Cfg::LKV, Cfg::BM, Cfg::BK, Cfg::NT, Cfg::LDA, Cfg::ROT, VEC>::type rl;
    typename ConvColLoaderSel<Cfg, KIND>::type cl;
    rl.init(a.w, a.CRS, m0, a.Kout, (int64_t)kt0 * Cfg::BK, threadIdx.x);
    cl.init(a, n0, kt0 * Cfg::BK, threadIdx.x);

    floatx16 acc[Cfg::MB][Cfg::NB];
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.0f;

    mainloop<Cfg>(rl, cl, T, krem, acc, smem);
    if (!combine_slices<Cfg>(acc, a.split, wi)) return;

    // Epilogue: the lane's NB columns are NB consecutive output pixels; when P*Q is a multiple of 4
    // they lie in one image, 16-byte aligned.  Row j of the product is output channel j.
    typedef typename VecOf<Cfg::NB>::type CV;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const int64_t col = n0 + wn0 + Cfg::NB * i;
    int64_t yoff[Cfg::NB];  // offset of (n, channel 0, p, q) for each owned column
#pragma unroll
    for (int bn = 0; bn < Cfg::NB; ++bn) {
        int64_t gc = col + bn;
        gc = gc < a.NPQ ? gc : a.NPQ - 1;
        const int64_t n = gc / a.PQ;
        yoff[bn] = n * a.Kout * a.PQ + (gc - n * a.PQ);
    }
    const bool full_vec = Cfg::NB == 4 && a.yvec && (col + Cfg::NB <= a.NPQ);
    if constexpr (Cfg::NB == 4) {
        if (full_vec && a.beta != 0.0f) {
            // old values fetched kEpiRows rows at a time before the first use (see store_tile_rowmajor)
#pragma unroll
            for (int bm = 0; bm < Cfg::MB; ++bm) {
#pragma unroll
                for (int r0 = 0; r0 < 16; r0 += kEpiRows) {
                    CV old[kEpiRows];
#pragma unroll
                    for (int j = 0; j < kEpiRows; ++j) {
                        const int r = r0 + j;
                        const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
                        const CV *src = reinterpret_cast<const CV *>(a.y + yoff[0] + (row < a.Kout ? row : a.Kout - 1) * a.PQ);
                        old[j] = a.yvec == 2 ? __builtin_nontemporal_load(src) : *src;
                    }
#pragma unroll
                    for (int j = 0; j < kEpiRows; ++j) {
                        const int r = r0 + j;
                        const int64_t row = m0 + wm0 + Cfg::MB * (8 * (r / 4) + 4 * h + (r % 4)) + bm;
                        CV o;
#pragma unroll
                        for (int bn = 0; bn < 4; ++bn) o[bn] = __builtin_fmaf(a.beta, old[j][bn], a.alpha * acc[bm][bn][r]);
                        if (row < a.Kout) {
                            if (a.yvec == 2)
                                __builtin_nontemporal_store(o, reinterpret_cast<CV *>(a.y + yoff[0] + row * a.PQ));
                            else
                                *reinterpret_cast<CV *>(a.y + yoff[0] + row * a.PQ) = o;
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
            if (row >= a.Kout) continue;
            float out[Cfg::NB];
#pragma unroll
            for (int bn = 0; bn < Cfg::NB; ++bn) out[bn] = a.alpha * acc[bm][bn][r];
            if (full_vec) {
                if constexpr (Cfg::NB == 4) {
                    float *dst = a.y + yoff[0] + row * a.PQ;
                    if (a.beta != 0.0f) {
                        const CV old = *reinterpret_cast<const CV *>(dst);
#pragma unroll
                        for (int bn = 0; bn < 4; ++bn) out[bn] += a.beta * old[bn];
                    }
                    CV o;
#pragma unroll
                    for (int bn = 0; bn < 4; ++bn) o[bn] = out[bn];
                    if (a.yvec == 2)   // a large result is streamed (see store_tile_rowmajor)
                        __builtin_nontemporal_store(o, reinterpret_cast<CV *>(dst));
                    else
                        *reinterpret_cast<CV *>(dst) = o;
                }
            } else {
#pragma unroll
                for (int bn = 0; bn < Cfg::NB; ++bn) {
                    if (col + bn < a.NPQ) {
                        float *dst = a.y + yoff[bn] + row * a.PQ;
                        float o = out[bn];
                        if (a.beta != 0.0f) o += a.beta * *dst;
                        *dst = o;
                    }
                }
            }
        }
    }
}

template <class Cfg>
int launch_conv_cfg(const ConvArgs &a, bool vec, int kind, hipStream_t stream)
{
    const int tiles = a.tiles_m * a.tiles_n;
    const dim3 grid((unsigned)(a.split.dp_tiles + (tiles - a.split.dp_tiles) * a.split.splits)), block(Cfg::NT);
    if (kind == kConvTapMajor) {
        if (a.C % Cfg::BK != 0 || !vec) return (int)hipErrorInvalidValue;  // the caller checks this first
        hipLaunchKernelGGL((conv_tile_kernel<Cfg, true, kConvTapMajor>), grid, block, 0, stream, a);
    } else if (kind == kConvBwdData) {
        if (vec)
            hipLaunchKernelGGL((conv_tile_kernel<Cfg, true, kConvBwdData>), grid, block, 0, stream, a);
        else
            hipLaunchKernelGGL((conv_tile_kernel<Cfg, false, kConvBwdData>), grid, block, 0, stream, a);
    } else if (vec) {
        hipLaunchKernelGGL((conv_tile_kernel<Cfg, true, kConvGeneric>), grid, block, 0, stream, a);
    } else {
        hipLaunchKernelGGL((conv_tile_kernel<Cfg, false, kConvGeneric>), grid, block, 0, stream, a);
    }
    return (int)hipGetLastError();
}

}  // namespace dmath
