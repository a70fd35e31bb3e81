// Filter gradient of the convolution as an implicit GEMM on the same macro-tile:
//
//     dw_mat[Kout x (C*R*S)] = dy_mat[Kout x (N*P*Q)] * unfolded(x)^T[(N*P*Q) x (C*R*S)]
//
// The reduction runs over the output pixels k = (n*P + p)*Q + q.  Rows of the product are output
// channels j; dy_mat(j, k) = dy[n][j][p][q] is contiguous along k inside an image and jumps by
// (Kout-1)*P*Q at an image boundary.  Columns are (c, r, s) in the order of dw in memory, so the result
// is a plain row-major matrix with leading dimension C*R*S and the GEMM epilogue is reused.
// unfolded(x)^T(k, (c,r,s)) = x[n][c][p*stride_h + r - pad_h][q*stride_w + s - pad_w], zero in the halo.
// K is long (100352 at the benchmark layer) and the output small (256 x 2304), so the launch is a plain
// split-K over many K slices.
#pragma once
#include <type_traits>

#include "gemm_kernel.h"

namespace dmath {

struct ConvFilterGradArgs {
    const float *x;
    const float *dy;
    float *dw;
    int N, C, H, W, Kout, R, S, P, Q;
    int pad_h, pad_w, stride_h, stride_w;
    int PQ, RS;
    int64_t CRS, NPQ, x_bytes;
    float alpha, beta;
    int tiles_m, tiles_n;
    int cvec;
    SplitPlan split;
};

// Rows operand: BR output channels x BK output pixels of dy.  Thread (row group, k quad) like the
// K-contiguous GEMM loader; the four k of a quad are consecutive pixels.  When P*Q is a multiple of 4
// (QUAD_IN_IMAGE) a quad never straddles an image and is one 16-byte load; otherwise every element
// carries its own (image, pixel) position.  Positions advance by BK pixels per tile without divisions.
template <int BR, int BK, int NT, int LD, bool QUAD_IN_IMAGE>
struct LoaderDyK {
    static constexpr int QPR = BK / 4;
    static constexpr int NQ = (BR * QPR) / NT;
    static constexpr int NLOAD = NQ, NSTORE = NQ * 4;
    static constexpr int NPOS = QUAD_IN_IMAGE ? 1 : 4;
    static_assert((BR * QPR) % NT == 0 && NQ >= 1, "tile must split evenly over the threads");
    const float *dy;
    int64_t rowoff[NQ];   // j * P*Q for the (clamped) output channel of each quad
    int64_t img_stride;   // Kout * P*Q
    int64_t kglob;        // global k of the quad's first element in the next tile to load
    int n[NPOS], pq[NPOS];
    int PQ;
    int64_t Ktot;
    floatx4 v[NQ];
    int row0, kq;

    __device__ __forceinline__ void init(const ConvFilterGradArgs &a, int64_t r0, int64_t kstart, int tid)
    {
        row0 = tid / QPR;
        kq = tid % QPR;
        dy = a.dy;
        PQ = a.PQ;
        Ktot = a.NPQ;
        img_stride = (int64_t)a.Kout * a.PQ;
        kglob = kstart + kq * 4;
#pragma unroll
        for (int e = 0; e < NPOS; ++e) {
            const int64_t k = kglob + e;
            n[e] = (int)(k / a.PQ);
            pq[e] = (int)(k - (int64_t)n[e] * a.PQ);
        }
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            int64_t j = r0 + row0 + it * (NT / QPR);
            j = j < a.Kout ? j : a.Kout - 1;
            rowoff[it] = j * a.PQ;
        }
    }
    __device__ __forceinline__ float elem(int it, int e, int j) const
    {
        return dy[(int64_t)n[e] * img_stride + rowoff[it] + pq[e] + j];
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        if (QUAD_IN_IMAGE) {
            v[I] = *reinterpret_cast<const floatx4 *>(dy + (int64_t)n[0] * img_stride + rowoff[I] + pq[0]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[I][j] = elem(I, j, 0);
        }
    }
    __device__ __forceinline__ void advance()
    {
        kglob += BK;
#pragma unroll
        for (int e = 0; e < NPOS; ++e) {
            pq[e] += BK;
            while (pq[e] >= PQ) {
                pq[e] -= PQ;
                ++n[e];
            }
        }
    }
    // partial last tile: k >= N*P*Q does not exist
    __device__ __forceinline__ void load_tail(int)
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[it][j] = (kglob + j < Ktot) ? (QUAD_IN_IMAGE ? elem(it, 0, j) : elem(it, j, 0)) : 0.0f;
    }
    template <int I>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        constexpr int it = I / 4, j = I % 4;
        S[(kq * 4 + j) * LD + row0 + it * (NT / QPR)] = v[it][j];
    }
};

// Cols operand: BK output pixels x BR filter elements (c, r, s), generated from x.  Thread (column
// group, k quad); each of the quad's four pixels keeps its position as three running values (offset of
// the pixel's window origin in x, row and column of that origin), advanced by BK pixels per tile with
// carries instead of divisions; a column contributes its constant tap offset and halo test.
template <int BR, int BK, int NT, int LD>
struct LoaderXTaps {
    static constexpr int QPR = BK / 4;
    static constexpr int NQ = (BR * QPR) / NT;
    static constexpr int NLOAD = NQ, NSTORE = NQ * 4;
    static_assert((BR * QPR) % NT == 0 && NQ >= 1, "tile must split evenly over the threads");
    const float *x;
    int64_t pix[4];      // n*C*H*W + (p*stride_h)*W + q*stride_w for the four pixels of the quad
    int ihb[4], iwb[4];  // p*stride_h, q*stride_w
    int coff[NQ];        // c*H*W + (r - pad_h)*W + (s - pad_w) for each owned column
    int rph[NQ], spw[NQ];  // r - pad_h, s - pad_w
    bool col_ok[NQ];
    int64_t kglob, Ktot, CHW;
    int H, W, Qsw, Psh, sw, sh, shW;
    floatx4 v[NQ];
    int col0, kq;

    __device__ __forceinline__ void init(const ConvFilterGradArgs &a, int64_t c0, int64_t kstart, int tid)
    {
        col0 = tid / QPR;
        kq = tid % QPR;
        x = a.x;
        H = a.H; W = a.W; sw = a.stride_w; sh = a.stride_h; shW = a.stride_h * a.W;
        Qsw = a.Q * a.stride_w; Psh = a.P * a.stride_h;
        CHW = (int64_t)a.C * a.H * a.W;
        Ktot = a.NPQ;
        kglob = kstart + kq * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t k = kglob + e;
            const int64_t n = k / a.PQ;
            const int pq = (int)(k - n * a.PQ);
            const int p = pq / a.Q, q = pq - p * a.Q;
            ihb[e] = p * a.stride_h;
            iwb[e] = q * a.stride_w;
            pix[e] = n * CHW + (int64_t)ihb[e] * W + iwb[e];
        }
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            int64_t col = c0 + col0 + it * (NT / QPR);
            col_ok[it] = col < a.CRS;
            col = col_ok[it] ? col : a.CRS - 1;
            const int c = (int)(col / a.RS);
            const int rs = (int)(col - (int64_t)c * a.RS);
            const int r = rs / a.S, s = rs - r * a.S;
            rph[it] = r - a.pad_h;
            spw[it] = s - a.pad_w;
            coff[it] = c * a.H * a.W + rph[it] * a.W + spw[it];
        }
    }
    __device__ __forceinline__ float elem(int it, int e) const
    {
        const bool ok = col_ok[it] && kglob + e < Ktot && (unsigned)(ihb[e] + rph[it]) < (unsigned)H &&
                        (unsigned)(iwb[e] + spw[it]) < (unsigned)W;
        return ok ? x[pix[e] + coff[it]] : 0.0f;
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[I][e] = elem(I, e);
    }
    __device__ __forceinline__ void advance()
    {
        kglob += BK;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            iwb[e] += BK * sw;
            pix[e] += BK * sw;
            while (iwb[e] >= Qsw) {   // next output row
                iwb[e] -= Qsw;
                pix[e] += shW - Qsw;
                ihb[e] += sh;
                if (ihb[e] >= Psh) {  // next image
                    ihb[e] -= Psh;
                    pix[e] += CHW - (int64_t)Psh * W;
                }
            }
        }
    }
    __device__ __forceinline__ void load_tail(int)
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it)
#pragma unroll
            for (int e = 0; e < 4; ++e) v[it][e] = elem(it, e);
    }
    template <int I>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        constexpr int it = I / 4, j = I % 4;
        S[(kq * 4 + j) * LD + col0 + it * (NT / QPR)] = v[it][j];
    }
};

// The same operand when Q is a multiple of 4 and x is smaller than 2 GiB: the four pixels of a quad
// then lie in one output row, so a thread keeps ONE running position, the row test is shared by the
// quad, and the loads are raw buffer loads with 32-bit byte offsets whose out-of-range marker returns
// zero for the halo without a branch or a select on the data.
template <int BR, int BK, int NT, int LD>
struct LoaderXRowQuad {
    static constexpr int QPR = BK / 4;
    static constexpr int NQ = (BR * QPR) / NT;
    static constexpr int NLOAD = NQ, NSTORE = NQ * 4;
    static_assert((BR * QPR) % NT == 0 && NQ >= 1, "tile must split evenly over the threads");
    __amdgpu_buffer_rsrc_t rsrc;
    unsigned pix;          // n*C*H*W + (p*stride_h)*W + q*stride_w of the quad's first pixel (element index)
    int ihb, iwb;          // p*stride_h, q*stride_w of the first pixel
    int coff[NQ];          // c*H*W + (r - pad_h)*W + (s - pad_w) for each owned column
    int rph[NQ], spw[NQ];  // r - pad_h (far negative for a column past C*R*S), s - pad_w
    int64_t kglob, Ktot;
    unsigned CHW, PshW;
    int H, W, Qsw, Psh, sw, sh, shW;
    floatx4 v[NQ];
    int col0, kq;

    __device__ __forceinline__ void init(const ConvFilterGradArgs &a, int64_t c0, int64_t kstart, int tid)
    {
        col0 = tid / QPR;
        kq = tid % QPR;
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, (int)a.x_bytes, 0x00020000);
        H = a.H; W = a.W; sw = a.stride_w; sh = a.stride_h; shW = a.stride_h * a.W;
        Qsw = a.Q * a.stride_w; Psh = a.P * a.stride_h;
        CHW = (unsigned)(a.C * a.H * a.W);
        PshW = (unsigned)(Psh * a.W);
        Ktot = a.NPQ;
        kglob = kstart + kq * 4;
        {
            const int64_t n = kglob / a.PQ;
            const int pq = (int)(kglob - n * a.PQ);
            const int p = pq / a.Q, q = pq - p * a.Q;
            ihb = p * a.stride_h;
            iwb = q * a.stride_w;
            pix = (unsigned)n * CHW + (unsigned)(ihb * a.W + iwb);
        }
#pragma unroll
        for (int it = 0; it < NQ; ++it) {
            int64_t col = c0 + col0 + it * (NT / QPR);
            const bool col_ok = col < a.CRS;
            col = col_ok ? col : a.CRS - 1;
            const int c = (int)(col / a.RS);
            const int rs = (int)(col - (int64_t)c * a.RS);
            const int r = rs / a.S, s = rs - r * a.S;
            spw[it] = s - a.pad_w;
            coff[it] = c * a.H * a.W + (r - a.pad_h) * a.W + spw[it];
            rph[it] = col_ok ? r - a.pad_h : -(1 << 30);
        }
    }
    __device__ __forceinline__ void quad(int it, bool live)
    {
        const bool row_ok = live && (unsigned)(ihb + rph[it]) < (unsigned)H;
        const int iw0 = iwb + spw[it];
        const unsigned base = (pix + (unsigned)coff[it]) * 4u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool ok = row_ok && (unsigned)(iw0 + e * sw) < (unsigned)W;
            const unsigned off = ok ? base + (unsigned)(e * sw) * 4u : 0x80000000u;
            v[it][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0));
        }
    }
    template <int I>
    __device__ __forceinline__ void load_piece()
    {
        quad(I, true);
    }
    __device__ __forceinline__ void advance()
    {
        kglob += BK;
        iwb += BK * sw;
        pix += (unsigned)(BK * sw);
        while (iwb >= Qsw) {   // next output row
            iwb -= Qsw;
            pix += (unsigned)(shW - Qsw);
            ihb += sh;
            if (ihb >= Psh) {  // next image
                ihb -= Psh;
                pix += CHW - PshW;
            }
        }
    }
    // N*P*Q and the quad's first k are multiples of 4: a quad is entirely inside or outside the reduction
    __device__ __forceinline__ void load_tail(int)
    {
#pragma unroll
        for (int it = 0; it < NQ; ++it) quad(it, kglob < Ktot);
    }
    template <int I>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        constexpr int it = I / 4, j = I % 4;
        S[(kq * 4 + j) * LD + col0 + it * (NT / QPR)] = v[it][j];
    }
};

template <class Cfg, bool QUAD_IN_IMAGE, bool QUAD_IN_ROW>
__global__ __launch_bounds__(Cfg::NT, Cfg::MIN_WAVES) void conv_bwd_filter_tile_kernel(const ConvFilterGradArgs a)
{
    static_assert(Cfg::LKV == 0, "these loaders write the padded LDS image");
    __shared__ __attribute__((aligned(16))) float smem[Cfg::STAGES * Cfg::STAGE_FLOATS];

    const int tiles = a.tiles_m * a.tiles_n;
    const WorkItem w = work_item(blockIdx.x, tiles, a.split);
    int tm, tn;
    tile_coords<8>(w.tile, a.tiles_m, a.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * Cfg::BM, n0 = (int64_t)tn * Cfg::BN;

    const int ktiles_total = (int)(a.NPQ / Cfg::BK);
    int kt0, T, krem;
    slice_range(ktiles_total, (int)(a.NPQ - (int64_t)ktiles_total * Cfg::BK), w.slice, w.nslice, kt0, T, krem);

    LoaderDyK<Cfg::BM, Cfg::BK, Cfg::NT, Cfg::LDA, QUAD_IN_IMAGE> rl;
    std::conditional_t<QUAD_IN_ROW, LoaderXRowQuad<Cfg::BN, Cfg::BK, Cfg::NT, Cfg::LDB>,
                       LoaderXTaps<Cfg::BN, Cfg::BK, Cfg::NT, Cfg::LDB>> cl;
    rl.init(a, m0, (int64_t)kt0 * Cfg::BK, threadIdx.x);
    cl.init(a, n0, (int64_t)kt0 * Cfg::BK, threadIdx.x);

    floatx16 acc[Cfg::MB][Cfg::NB];
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.0f;

    mainloop<Cfg>(rl, cl, T, krem, acc, smem);
    if (!combine_slices<Cfg>(acc, a.split, w)) return;
    store_tile_rowmajor<Cfg>(acc, a.dw, a.CRS, a.Kout, a.CRS, a.alpha, a.beta, a.cvec != 0, m0, n0, a.split, w);
}

template <class Cfg>
int launch_conv_bwd_filter_cfg(const ConvFilterGradArgs &a, bool quad_in_image, bool quad_in_row, hipStream_t stream)
{
    const int tiles = a.tiles_m * a.tiles_n;
    const dim3 grid((unsigned)(a.split.dp_tiles + (tiles - a.split.dp_tiles) * a.split.splits)), block(Cfg::NT);
    if constexpr (Cfg::LKV == 0) {
        if (quad_in_image && quad_in_row)
            hipLaunchKernelGGL((conv_bwd_filter_tile_kernel<Cfg, true, true>), grid, block, 0, stream, a);
        else if (quad_in_image)
            hipLaunchKernelGGL((conv_bwd_filter_tile_kernel<Cfg, true, false>), grid, block, 0, stream, a);
        else if (quad_in_row)
            hipLaunchKernelGGL((conv_bwd_filter_tile_kernel<Cfg, false, true>), grid, block, 0, stream, a);
        else
            hipLaunchKernelGGL((conv_bwd_filter_tile_kernel<Cfg, false, false>), grid, block, 0, stream, a);
        return (int)hipGetLastError();
    } else {
        return (int)hipErrorInvalidValue;  // the rotated-image comparison configuration has no filter-gradient kernel
    }
}

}  // namespace dmath
