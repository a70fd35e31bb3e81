// GEMM for products with few output tiles and a long K (the skinny products of a fully connected
// layer at a small batch: figure "cyclic_gemm_cache_fwd" of the dMath paper, Y = W^T X and
// grad X = W grad Y): the K range is split INSIDE the workgroup instead of across workgroups.
//
// One workgroup of 8 waves owns one 64 x 64 tile of C and walks K in tiles of 64.  The workgroup
// stages a K tile of both operands in LDS with whole-cache-line loads (64 "rows" of 256 bytes each,
// whatever the orientation); wave w then multiplies only the k columns 8w .. 8w+7 of that tile, for the
// whole 64 x 64 output (2 x 2 blocks of v_mfma_f32_32x32x2_f32).  Every wave therefore keeps a full
// set of accumulators and two waves per SIMD cover each other's stalls, where the tile kernels would
// run such a product as one four-wave workgroup per compute unit plus slices in a workspace.  At the
// end every wave leaves its 64 x 64 partial sums in LDS and the workgroup adds them in wave order: the
// result does not depend on timing (same bits every run), no scratch in device memory, no second
// kernel.
//
// LDS images (per pipeline stage and operand: 64 rows of 64 floats, no padding; the 16-byte chunk c of
// row r sits at position c ^ (r & 15) of the row, which keeps every access below free of bank conflicts):
//   operand stored along k (A for transA == N, B for transB == T): kept as it is in memory,
//     [row or column of the operand][k].  Lane (i, h) of a wave reads, per block b, ONE 16-byte vector
//     at row i + 32*b, k = 8w + 4h .. +3, and feeds element j to the j-th MFMA step.  An MFMA step adds
//     the k of both lane halves, so step j covers k = 8w + j and 8w + 4 + j: the order of the k inside
//     a wave's chunk is permuted, which a sum does not mind, and no transposing store is needed.
//   operand stored along its own index: [k][index], read per step j at k row 8w + 4h + j as one
//     8-byte vector of the interleaved blocks (index 2i + b).
// Both k assignments agree (k = 8w + 4h + j for lane half h and step j), whichever images meet.
//
// When every 16-byte load is aligned (VEC) the tiles go global -> LDS directly
// (global_load_lds_dwordx4: lane l's 16 bytes land at a wave-uniform LDS address + 16*l; each lane
// fetches the chunk that belongs at its position of the swizzled image): no staging registers, no LDS
// store instructions, and a tile is requested two K tiles before its first use.  Otherwise, and for
// the partial last K tile, the tile is staged through registers.
#pragma once
#include "gemm_kernel.h"

namespace dmath {

struct WaveK {
    static constexpr int KW = 8;           // waves per workgroup = k chunks of 8 per K tile
    static constexpr int BM = 64, BN = 64, BK = 64;
    static constexpr int NT = 64 * KW;
    static constexpr int P = 64;           // row pitch of the operand images (floats)
    static constexpr int OPER_FLOATS = 64 * P;
    static constexpr int STAGE_FLOATS = 2 * OPER_FLOATS;
    static constexpr int RP = 68;          // row pitch of a wave's partial sums
    static constexpr int RED_FLOATS = 64 * RP;
    // float offset of 16-byte chunk `chunk` of image row `row`
    static __device__ __forceinline__ int at(int row, int chunk) { return row * P + ((chunk ^ (row & 15)) << 2); }
};

// s_waitcnt immediate: wait until at most n vector-memory operations are outstanding, and for every LDS
// operation (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 left at "no wait", lgkmcnt 11:8 = 0).
constexpr int wavek_waitcnt(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4); }

// Global -> LDS fill of one operand image (16-byte aligned operands only).  The image is 16 blocks of
// 4 rows = 1 KB; wave w fills blocks w and w + 8 with one instruction each.  Lane l writes position
// l % 16 of row 4*block + l / 16 and fetches the chunk that belongs there.
template <bool KC>
struct WaveKDma {
    const char *tile;   // uniform over the workgroup (scalar registers)
    int64_t tstride;
    uint32_t off[2];
    uint32_t wave_lds;

    __device__ __forceinline__ void init(const float *base, int64_t ld, int64_t x0, int64_t X, int tid)
    {
        const int wave = tid >> 6, lane = tid & 63;
        const float *t0 = KC ? base + x0 * ld : base + x0;
        const uint64_t u = reinterpret_cast<uint64_t>(t0);   // the same in every lane
        tile = reinterpret_cast<const char *>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(u >> 32)) << 32) |
                                              (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)u));
        tstride = KC ? 64 * 4 : (int64_t)64 * ld * 4;
        wave_lds = (uint32_t)__builtin_amdgcn_readfirstlane(wave * 1024);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int row = 4 * (wave + 8 * p) + (lane >> 4);
            const int chunk = (lane & 15) ^ (row & 15);
            if (KC) {
                int64_t r = row;
                r = x0 + r < X ? r : X - 1 - x0;   // rows past the end re-read the last one (never stored)
                off[p] = (uint32_t)((r * ld + 4 * chunk) * 4);
            } else {
                int64_t quad = 4 * chunk;           // X is a multiple of 4: a quad is wholly inside or outside
                quad = x0 + quad + 4 <= X ? quad : X - 4 - x0;
                off[p] = (uint32_t)((row * ld + quad) * 4);
            }
        }
    }
    // image_lds: LDS byte address of the operand image being filled.  Assembly on purpose: the compiler
    // cannot tell which LDS bytes such a load writes and would wait for all of them before every later
    // LDS read; the waits are placed by hand in the kernel.  m0 = LDS byte address of lane 0's 16 bytes.
    template <int PIECE>
    __device__ __forceinline__ void fill_piece(uint32_t image_lds) const
    {
        asm volatile("s_add_u32 m0, %2, %3\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(off[PIECE]), "s"(tile), "s"(image_lds + wave_lds), "n"(PIECE * 8 * 1024)
                     : "memory", "scc");
    }
    __device__ __forceinline__ void advance() { tile += tstride; }
};

// Staging of one operand: 64 rows of 64 floats.  natural (KC == true): row = row/column of the
// operand, 64 consecutive k.  k-major (KC == false): row = k, 64 consecutive indices of the operand.
// Thread t owns quads (row t/16 + 32*it, floats 4*(t%16) .. +3), it = 0, 1: 16 consecutive lanes read
// 256 contiguous bytes.
template <bool KC, bool VEC>
struct WaveKLoader {
    const char *tile;   // uniform over the workgroup
    int64_t tstride;    // bytes per K tile
    uint32_t off[2];    // VEC: byte offset of each quad; scalar path: of the quad's row
    uint32_t col[4];    // scalar path: byte offsets of the four elements inside the row (clamped)
    floatx4 v[2];
    int lds[2];
    int q4, row0;

    // base: operand; ld; x0: first row/column of the operand in this tile; X: their number; kt0: first K tile.
    __device__ __forceinline__ void init(const float *base, int64_t ld, int64_t x0, int64_t X, int tid, int64_t kt0 = 0)
    {
        row0 = tid >> 4;
        q4 = (tid & 15) * 4;
        if (KC) {
            tile = reinterpret_cast<const char *>(base + x0 * ld + kt0 * 64);
            tstride = 64 * 4;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                int64_t r = row0 + 32 * it;
                r = x0 + r < X ? r : X - 1 - x0;   // rows past the end re-read the last one (never stored)
                off[it] = (uint32_t)((r * ld + (VEC ? q4 : 0)) * 4);
                lds[it] = WaveK::at(row0 + 32 * it, tid & 15);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) col[e] = (uint32_t)((q4 + e) * 4);
        } else {
            tile = reinterpret_cast<const char *>(base + x0 + kt0 * 64 * ld);
            tstride = (int64_t)64 * ld * 4;
            int64_t quad = q4;  // VEC: X is a multiple of 4, a quad is wholly inside or wholly outside
            if (VEC) quad = x0 + quad + 4 <= X ? quad : X - 4 - x0;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                off[it] = (uint32_t)(((row0 + 32 * it) * ld + (VEC ? quad : 0)) * 4);
                lds[it] = WaveK::at(row0 + 32 * it, tid & 15);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t c = q4 + e;
                col[e] = (uint32_t)((x0 + c < X ? c : X - 1 - x0) * 4);
            }
        }
    }
    template <int IT>
    __device__ __forceinline__ void load_piece()
    {
        const char *p = tile + off[IT];
        if (VEC) {
            v[IT] = *reinterpret_cast<const floatx4 *>(p);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[IT][e] = *reinterpret_cast<const float *>(p + col[e]);
        }
    }
    __device__ __forceinline__ void advance() { tile += tstride; }
    template <int IT>
    __device__ __forceinline__ void store_piece(float *S) const
    {
        *reinterpret_cast<floatx4 *>(S + lds[IT]) = v[IT];
    }
    // Last, partial K tile: only k < krem exists, the rest of the tile is zero on both operands.
    __device__ __forceinline__ void load_tail(int krem)
    {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const char *p = tile + off[it];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = KC ? (q4 + e < krem) : (row0 + 32 * it < krem);
                v[it][e] = ok ? *reinterpret_cast<const float *>(p + (VEC ? 4 * e : col[e])) : 0.0f;
            }
        }
    }
};

// A wave's operand fragments of one K tile (its 8 k): natural image 2 x 16 bytes (blocks), k-major
// image 4 x 8 bytes (steps).
template <bool KC> struct WaveKFrag;
template <> struct WaveKFrag<true> {
    floatx4 v[2];
    static constexpr int PIECES = 2;
    // lane (i, h) of wave w: chunk 2w + h of row i (+ 32 per block; the swizzle only looks at i % 16)
    static __device__ __forceinline__ void offsets(int (&off)[4], int wave, int i, int h)
    {
        off[0] = WaveK::at(i, 2 * wave + h);
        off[1] = off[2] = off[3] = 0;
    }
    template <int I> __device__ __forceinline__ void read(const float *img, const int (&off)[4])
    {
        v[I] = *reinterpret_cast<const floatx4 *>(img + off[0] + I * 32 * WaveK::P);
    }
    template <int J, int B> __device__ __forceinline__ float get() const { return v[B][J]; }
};
template <> struct WaveKFrag<false> {
    floatx2 v[4];
    static constexpr int PIECES = 4;
    // step j: k row 8w + 4h + j, columns 2i and 2i + 1 (chunk i / 2, second half of it for odd i)
    static __device__ __forceinline__ void offsets(int (&off)[4], int wave, int i, int h)
    {
#pragma unroll
        for (int j = 0; j < 4; ++j) off[j] = WaveK::at(8 * wave + 4 * h + j, i >> 1) + 2 * (i & 1);
    }
    template <int I> __device__ __forceinline__ void read(const float *img, const int (&off)[4])
    {
        v[I] = *reinterpret_cast<const floatx2 *>(img + off[I]);
    }
    template <int J, int B> __device__ __forceinline__ float get() const { return v[J][B]; }
};

template <bool A_KCONTIG, bool B_KCONTIG, bool VEC, int STAGES>
__global__ __launch_bounds__(WaveK::NT, 2) void gemm_wavek_kernel(const GemmArgs g)
{
    constexpr int S = STAGES, KW = WaveK::KW, RP = WaveK::RP;
    constexpr int PIPE = S * WaveK::STAGE_FLOATS, RED = KW * WaveK::RED_FLOATS;
    constexpr int SMEM = PIPE > RED ? PIPE : RED;
    static_assert(SMEM * 4 <= 160 * 1024, "LDS of one compute unit");
    static_assert(S >= (VEC ? 4 : 3), "fragments are read one tile ahead; direct loads are requested two tiles ahead");
    __shared__ __attribute__((aligned(1024))) float smem[SMEM];
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(3))) float *lds_ptr;
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lds_ptr)smem;
#else
    const uint32_t smem_lds = 0;
#endif

    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 0] = __builtin_readcyclecounter();
        g.clock_probe[blockIdx.x * 4 + 1] = __builtin_amdgcn_s_memrealtime();
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    const int tiles = g.tiles_m * g.tiles_n;
    int tm, tn;
    tile_coords<8>(xcd_contiguous_id(blockIdx.x, tiles), g.tiles_m, g.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * 64, n0 = (int64_t)tn * 64;

    const int T = (int)(g.K / 64);
    const int krem = (int)(g.K - (int64_t)T * 64);

    typedef WaveKFrag<A_KCONTIG> FA;
    typedef WaveKFrag<B_KCONTIG> FB;
    constexpr int NFA = FA::PIECES, NFB = FB::PIECES;
    int a_off[4], b_off[4];   // the lane's float offsets into an operand image for its fragment reads
    FA::offsets(a_off, wave, i, h);
    FB::offsets(b_off, wave, i, h);

    floatx16 acc[2][2];
#pragma unroll
    for (int bm = 0; bm < 2; ++bm)
#pragma unroll
        for (int bn = 0; bn < 2; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.0f;

    auto read_frags = [&](FA &fa, FB &fb, const float *stage) {
        static_for<NFA>([&](auto pc) { fa.template read<decltype(pc)::value>(stage, a_off); });
        static_for<NFB>([&](auto pc) { fb.template read<decltype(pc)::value>(stage + WaveK::OPER_FLOATS, b_off); });
    };
    // the 16 MFMAs of one K tile: step j (k = 8w + j and 8w + 4 + j), blocks (bm, bn)
    auto mma = [&](const FA &fa, const FB &fb, auto mc) {
        constexpr int m = decltype(mc)::value, j = m / 4, bm = (m / 2) % 2, bn = m % 2;
        acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.template get<j, bm>(), fb.template get<j, bn>(), acc[bm][bn], 0, 0, 0);
    };
    FA fa;
    FB fb;

    if constexpr (VEC) {
        // ---- global -> LDS pipeline.  Tile u lives in stage u % S.  Iteration t requests tile t + S - 1
        // into the stage tile t - 1 has left, reads the fragments of tile t + 1 and, before its barrier,
        // waits for this wave's own loads of tile t + 2 (requested one iteration ago; the 4 loads of this
        // iteration may stay in flight).
        WaveKDma<A_KCONTIG> da;
        WaveKDma<B_KCONTIG> db;
        da.init(g.A, g.lda, m0, g.M, threadIdx.x);
        db.init(g.B, g.ldb, n0, g.N, threadIdx.x);
        auto fill_all = [&](int stage) {
            const uint32_t st = smem_lds + stage * (WaveK::STAGE_FLOATS * 4);
            da.template fill_piece<0>(st);
            da.template fill_piece<1>(st);
            db.template fill_piece<0>(st + WaveK::OPER_FLOATS * 4);
            db.template fill_piece<1>(st + WaveK::OPER_FLOATS * 4);
            da.advance();
            db.advance();
        };
#pragma unroll
        for (int s = 0; s < S - 1; ++s) {
            if (s < T) fill_all(s);
        }
        // tiles 0 and 1 have landed when at most the last tile's 4 loads are outstanding
        if (T >= S - 1)
            __builtin_amdgcn_s_waitcnt(wavek_waitcnt(4 * (S - 3)));
        else
            __builtin_amdgcn_s_waitcnt(wavek_waitcnt(0));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (T > 0) read_frags(fa, fb, smem);
        int t = 0;
        while (t + 2 * S - 2 < T) {   // every iteration of the trip has a tile to request and a next tile
            static_for<S>([&](auto sc) {
                constexpr int CS = decltype(sc)::value, NS = (CS + 1) % S, FILL = (CS + S - 1) % S;
                const float *nxt = smem + NS * WaveK::STAGE_FLOATS;
                const uint32_t fill = smem_lds + FILL * (WaveK::STAGE_FLOATS * 4);
                FA na;
                FB nb;
                static_for<16>([&](auto mc) {
                    constexpr int m = decltype(mc)::value;
                    mma(fa, fb, mc);
                    __builtin_amdgcn_sched_barrier(0);
                    // one other instruction in the shadow of each MFMA: the requests first, then the
                    // next tile's fragments
                    if constexpr (m == 0) {
                        da.template fill_piece<0>(fill);
                    } else if constexpr (m == 1) {
                        da.template fill_piece<1>(fill);
                    } else if constexpr (m == 2) {
                        db.template fill_piece<0>(fill + WaveK::OPER_FLOATS * 4);
                    } else if constexpr (m == 3) {
                        db.template fill_piece<1>(fill + WaveK::OPER_FLOATS * 4);
                        da.advance();
                        db.advance();
                    } else if constexpr (m - 4 < NFA) {
                        na.template read<m - 4>(nxt, a_off);
                    } else if constexpr (m - 4 < NFA + NFB) {
                        nb.template read<m - 4 - NFA>(nxt + WaveK::OPER_FLOATS, b_off);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
                fa = na;
                fb = nb;
                __builtin_amdgcn_s_waitcnt(wavek_waitcnt(4 * (S - 3)));
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            });
            t += S;
        }
        // last tiles (t is a multiple of S here): the same steps under conditions, every load awaited
        for (int cs = 0; t < T; ++t) {
            const int ns = cs + 1 == S ? 0 : cs + 1, fill = cs == 0 ? S - 1 : cs - 1;
            if (t + S - 1 < T) fill_all(fill);
            FA na;
            FB nb;
            const bool more = t + 1 < T;
            if (more) read_frags(na, nb, smem + ns * WaveK::STAGE_FLOATS);
            static_for<16>([&](auto mc) { mma(fa, fb, mc); });
            if (more) {
                fa = na;
                fb = nb;
            }
            cs = ns;
            __builtin_amdgcn_s_waitcnt(wavek_waitcnt(0));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        // ---- register-staged pipeline: LDS holds S tiles, registers one more in flight
        WaveKLoader<A_KCONTIG, false> la;
        WaveKLoader<B_KCONTIG, false> lb;
        la.init(g.A, g.lda, m0, g.M, threadIdx.x);
        lb.init(g.B, g.ldb, n0, g.N, threadIdx.x);
        auto load_all = [&]() {
            la.template load_piece<0>(); la.template load_piece<1>(); la.advance();
            lb.template load_piece<0>(); lb.template load_piece<1>(); lb.advance();
        };
        auto store_all = [&](int stage) {
            float *st = smem + stage * WaveK::STAGE_FLOATS;
            la.template store_piece<0>(st); la.template store_piece<1>(st);
            lb.template store_piece<0>(st + WaveK::OPER_FLOATS); lb.template store_piece<1>(st + WaveK::OPER_FLOATS);
        };
#pragma unroll
        for (int s = 0; s < S - 1; ++s) {
            if (s < T) {
                load_all();
                store_all(s);
            }
        }
        if (S - 1 < T) load_all();
        __syncthreads();
        if (T > 0) read_frags(fa, fb, smem);
        int cs = 0, fill = S - 1;
        for (int t = 0; t < T; ++t) {
            if (t + S - 1 < T) store_all(fill);
            if (t + S < T) load_all();
            const int ns = (cs + 1 == S) ? 0 : cs + 1;
            FA na;
            FB nb;
            const bool more = t + 1 < T;
            if (more) read_frags(na, nb, smem + ns * WaveK::STAGE_FLOATS);
            static_for<16>([&](auto mc) { mma(fa, fb, mc); });
            if (more) {
                fa = na;
                fb = nb;
            }
            cs = ns;
            fill = (fill + 1 == S) ? 0 : fill + 1;
            __syncthreads();
        }
    }
    if (krem > 0) {
        // partial last K tile: through registers, zero beyond K, into stage 0 (every wave is past the
        // last barrier of the loop and no load is outstanding)
        WaveKLoader<A_KCONTIG, VEC> ta;
        WaveKLoader<B_KCONTIG, VEC> tb;
        ta.init(g.A, g.lda, m0, g.M, threadIdx.x, T);
        tb.init(g.B, g.ldb, n0, g.N, threadIdx.x, T);
        ta.load_tail(krem);
        tb.load_tail(krem);
        ta.template store_piece<0>(smem); ta.template store_piece<1>(smem);
        tb.template store_piece<0>(smem + WaveK::OPER_FLOATS); tb.template store_piece<1>(smem + WaveK::OPER_FLOATS);
        __syncthreads();
        read_frags(fa, fb, smem);
        static_for<16>([&](auto mc) { mma(fa, fb, mc); });
        __syncthreads();
    }

    // ---- partial sums of wave w as a plain 64 x 64 matrix (row pitch RP) at smem + w*RED_FLOATS.  The
    // region overlays the pipeline stages; every wave has passed the last barrier of the K loop.
    {
        float *mine = smem + wave * WaveK::RED_FLOATS;
#pragma unroll
        for (int bm = 0; bm < 2; ++bm)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rb = 8 * (r / 4) + 4 * h + (r % 4);          // row inside the 32 x 32 block
                const int row = A_KCONTIG ? rb + 32 * bm : 2 * rb + bm;
                if (B_KCONTIG) {
                    mine[row * RP + i] = acc[bm][0][r];
                    mine[row * RP + i + 32] = acc[bm][1][r];
                } else {
                    floatx2 v;
                    v[0] = acc[bm][0][r];
                    v[1] = acc[bm][1][r];
                    *reinterpret_cast<floatx2 *>(mine + row * RP + 2 * i) = v;
                }
            }
    }
    __syncthreads();

    // ---- fixed-order sum over the waves and the epilogue: a thread owns two quads of four columns
    const int qc = (threadIdx.x & 15) * 4;
    const bool cvec = g.cvec != 0;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int row = (threadIdx.x >> 4) + 32 * q;
        floatx4 sum = *reinterpret_cast<const floatx4 *>(smem + row * RP + qc);
#pragma unroll
        for (int w = 1; w < KW; ++w) sum += *reinterpret_cast<const floatx4 *>(smem + w * WaveK::RED_FLOATS + row * RP + qc);
        const int64_t gr = m0 + row, gc = n0 + qc;
        if (gr >= g.M || gc >= g.N) continue;
        float *dst = g.C + gr * g.ldc + gc;
        if (cvec && gc + 4 <= g.N) {
            floatx4 o = g.alpha * sum;
            if (g.beta != 0.0f) {
                const floatx4 old = *reinterpret_cast<const floatx4 *>(dst);
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = __builtin_fmaf(g.beta, old[e], o[e]);
            }
            *reinterpret_cast<floatx4 *>(dst) = o;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (gc + e < g.N) {
                    float o = g.alpha * sum[e];
                    if (g.beta != 0.0f) o = __builtin_fmaf(g.beta, dst[e], o);
                    dst[e] = o;
                }
            }
        }
    }
    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 2] = __builtin_readcyclecounter();
        g.clock_probe[blockIdx.x * 4 + 3] = __builtin_amdgcn_s_memrealtime();
    }
}

// Host side.  g.tiles_m / g.tiles_n count 64 x 64 tiles; the split plan of g is not used.
template <int STAGES>
int launch_gemm_wavek(const GemmArgs &g, bool a_kcontig, bool b_kcontig, bool vec, hipStream_t stream)
{
    const dim3 grid((unsigned)(g.tiles_m * g.tiles_n)), block(WaveK::NT);
#define DMATH_LAUNCH(AK, BK_, V) hipLaunchKernelGGL((gemm_wavek_kernel<AK, BK_, V, STAGES>), grid, block, 0, stream, g)
    if (vec) {
        if (a_kcontig && b_kcontig) DMATH_LAUNCH(true, true, true);
        else if (a_kcontig) DMATH_LAUNCH(true, false, true);
        else if (b_kcontig) DMATH_LAUNCH(false, true, true);
        else DMATH_LAUNCH(false, false, true);
    } else {
        if (a_kcontig && b_kcontig) DMATH_LAUNCH(true, true, false);
        else if (a_kcontig) DMATH_LAUNCH(true, false, false);
        else if (b_kcontig) DMATH_LAUNCH(false, true, false);
        else DMATH_LAUNCH(false, false, false);
    }
#undef DMATH_LAUNCH
    return (int)hipGetLastError();
}

}  // namespace dmath
