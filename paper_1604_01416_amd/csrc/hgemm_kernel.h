// GEMM on half-precision storage computed on the FP16-input matrix instructions
// (v_mfma_f32_32x32x16_f16, v_mfma_f32_16x16x32_f16): the product of two halves is exact in FP32 and the
// instructions accumulate in FP32, so the arithmetic is the single-precision arithmetic on converted
// operands that section "Precisions" of the paper describes, at the rate of the 16-bit matrix pipe.
//
// Two kernels; the host (gemm_entry in dmath_api.hip) picks by K:
//   hgemm_mi16_dma64_kernel   K % 64 == 0: K tile 64 (whole cache lines), global -> LDS loads, every orientation (an
//                             operand stored along its own index is read back with the transposing LDS read), on the
//                             16x16x32 instruction, which holds a higher clock under the power limit
//   hgemm_mfma16_kernel       K % 32 == 0 otherwise: K tile 32, operands staged through registers, 32x32x16 instruction
// The text below describes the second; the first is described where it is defined.
//
// Operand layout of the instruction (checked on the device with one-hot operands): lane l holds, for
// A, row l%32 and the 8 consecutive k = 8*(l/32) .. +7; for B, column l%32 and the same k; the 32x32
// FP32 result is laid out like that of the FP32 instruction.  Both operands therefore want 8
// consecutive k per lane, and the LDS image of a K tile is k-contiguous for both:
//
//     As[BM][LD], Bs[BN][LD] halves.  For an operand that is transposed on the way in, LD = BK + 8
//     (80-byte rows: the 16 lanes served together by a 16-byte LDS read hit 16 different 16-byte bank
//     groups when they read 16 consecutive rows).  For an operand copied with 16-byte stores that
//     padding makes the stores collide (4 rows x 4 chunks of a 16-lane group overlap by 48 bytes: 8
//     conflict cycles per store by the counters), so its rows are unpadded (64 bytes) and the four
//     16-byte chunks of row r are stored in the order c ^ ((r >> 2) & 3): stores of 4 rows x 4 chunks
//     and reads of 16 consecutive rows at one logical chunk both cover all banks exactly once.
//
// An operand stored contiguously along k (A for transA == N, B for transB == T) is copied with 16-byte
// loads and 16-byte LDS stores.  An operand stored along its own index (A^T, B) is transposed on the
// way: a thread loads the same 8 columns of two consecutive k rows, pairs them up in registers and
// writes eight 4-byte (k, k+1) pairs.
//
// A wave owns MB x NB blocks of 32x32; block (bm, bn) covers tile rows wm0 + 32*bm .. +31 and tile
// columns wn0 + 32*bn .. +31 (contiguous blocks, unlike the FP32 kernel's interleaved ones, because
// consecutive lanes must read consecutive image rows to stay conflict-free).
#pragma once
#include "gemm_kernel.h"

namespace dmath {

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int STAGES_>
struct HTileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = 32;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int MB = WM / 32, NB = WN / 32;
    static constexpr int LDK = BK + 8;
    static constexpr int A_HALVES = BM * LDK, B_HALVES = BN * LDK, STAGE_HALVES = A_HALVES + B_HALVES;
    static constexpr int LDS_BYTES = STAGES * STAGE_HALVES * 2;
    static constexpr int KSTEPS = BK / 16;
    static constexpr int MIN_WAVES = (NT / 64 + 3) / 4;
    static_assert(WM % 32 == 0 && WN % 32 == 0 && STAGES >= 3, "wave tile is made of 32x32 blocks; 3+ stages");
};

// Operand contiguous along k: element (r, k) at base[r*ld + k].  Thread (row, 8-element chunk).
// SLOTS register sets hold tiles in flight between the global load and the LDS store.
template <int BR, int BK, int NT, int LDK, int SLOTS>
struct HLoaderK {
    static constexpr int CPR = BK / 8;             // 16-byte chunks per row
    static constexpr int NP = (BR * CPR) / NT;     // chunks per thread
    static constexpr int NLOAD = NP, NSTORE = NP;
    static constexpr int LD = BK;                  // unpadded image rows, chunks swizzled
    static_assert((BR * CPR) % NT == 0 && NP >= 1 && CPR == 4 && (NT / CPR) % 16 == 0, "tile must split evenly over the threads");
    const char *tile;
    uint32_t off[NP];
    halfx8 v[SLOTS][NP];
    int lds0;

    __device__ __forceinline__ void init(const _Float16 *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        const int row0 = tid / CPR, ch = tid % CPR;
        tile = reinterpret_cast<const char *>(base + r0 * ld + k0);
        lds0 = row0 * LD + ((ch ^ ((row0 >> 2) & 3)) * 8);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            int64_t lr = row0 + p * (NT / CPR);
            lr = r0 + lr < R ? lr : R - 1 - r0;  // rows past the end re-read the last one; never stored
            off[p] = (uint32_t)((lr * ld + ch * 8) * 2);
        }
    }
    // image offset (halves) of the fragment of k step ks for the lane reading tile row `row` (a
    // multiple of 32 plus lane % 32) with k half h = lane / 32
    static __device__ __forceinline__ int frag_off(int row, int ks, int h)
    {
        return row * LD + (((2 * ks + h) ^ ((row >> 2) & 3)) * 8);
    }
    template <int SLOT, int I>
    __device__ __forceinline__ void load_piece()
    {
        v[SLOT][I] = *reinterpret_cast<const halfx8 *>(tile + off[I]);
    }
    __device__ __forceinline__ void advance() { tile += BK * 2; }
    template <int SLOT, int I>
    __device__ __forceinline__ void store_piece(_Float16 *S) const
    {
        *reinterpret_cast<halfx8 *>(S + lds0 + I * (NT / CPR) * LD) = v[SLOT][I];
    }
};

// Operand contiguous along its own index: element (r, k) at base[k*ld + r].  A thread owns the 8
// consecutive r of one chunk for the k pair (2*kp, 2*kp + 1): lanes 0..15 of a 16-lane group take the
// 16 k pairs of one chunk, so that their 4-byte LDS stores fall into 16 consecutive dwords of a row.
// (Image rows 8 apart share their banks, so the four 16-lane groups of a wave collide two by two:
// 4 conflict cycles per store by the counters.  Exchanging the halves of every other chunk, fetched as
// two 8-byte loads, halved the conflicts but doubled the vector-memory instructions and was 20-35 %
// slower; the 16-byte loads stay.)
template <int BR, int BK, int NT, int LDK, int SLOTS>
struct HLoaderN {
    static constexpr int KP = BK / 2;                     // k pairs per tile
    static constexpr int ITEMS = KP * (BR / 8);           // (k pair, chunk) items
    static constexpr int NP = ITEMS / NT;
    static constexpr int NLOAD = 2 * NP, NSTORE = 8 * NP;
    static constexpr int LD = LDK;                        // padded image rows
    static_assert(ITEMS % NT == 0 && NP >= 1 && NT % KP == 0, "tile must split evenly over the threads");
    static __device__ __forceinline__ int frag_off(int row, int ks, int h) { return row * LD + ks * 16 + 8 * h; }
    const char *tile;
    int64_t tstride, row_bytes;
    uint32_t off[NP];
    halfx8 v[SLOTS][NP][2];
    int lds0;

    __device__ __forceinline__ void init(const _Float16 *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid)
    {
        const int kp = tid % KP, c0 = tid / KP;
        tile = reinterpret_cast<const char *>(base + k0 * ld + r0);
        tstride = (int64_t)BK * ld * 2;
        row_bytes = ld * 2;
        lds0 = c0 * 8 * LDK + 2 * kp;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            int64_t col = (c0 + p * (NT / KP)) * 8;
            col = r0 + col + 8 <= R ? col : R - 8 - r0;  // R is a multiple of 8: the last whole chunk
            off[p] = (uint32_t)(((int64_t)2 * kp * ld + col) * 2);
        }
    }
    template <int SLOT, int I>
    __device__ __forceinline__ void load_piece()
    {
        constexpr int p = I / 2, which = I % 2;
        v[SLOT][p][which] = *reinterpret_cast<const halfx8 *>(tile + off[p] + (which ? row_bytes : 0));
    }
    __device__ __forceinline__ void advance() { tile += tstride; }
    template <int SLOT, int I>
    __device__ __forceinline__ void store_piece(_Float16 *S) const
    {
        constexpr int p = I / 8, j = I % 8;
        halfx2 pr;
        pr[0] = v[SLOT][p][0][j];
        pr[1] = v[SLOT][p][1][j];
        *reinterpret_cast<halfx2 *>(S + lds0 + (p * (NT / KP) * 8 + j) * LDK) = pr;
    }
};

template <class Cfg, bool KCONTIG, int BR, int SLOTS>
struct HLoaderSel {
    typedef HLoaderK<BR, Cfg::BK, Cfg::NT, Cfg::LDK, SLOTS> type;
};
template <class Cfg, int BR, int SLOTS>
struct HLoaderSel<Cfg, false, BR, SLOTS> {
    typedef HLoaderN<BR, Cfg::BK, Cfg::NT, Cfg::LDK, SLOTS> type;
};

template <class Cfg>
struct HFrag {
    halfx8 a[Cfg::MB], b[Cfg::NB];
};

// Fragment piece P of k step KS: P < MB is block row P of A, else block column P - MB of B.
// a_off / b_off: the lane's image offsets for k steps 0 and 1 (see frag_off of the loaders); LDA / LDB:
// row strides of the two images.
template <class Cfg, int LDA, int LDB, int KS, int P>
__device__ __forceinline__ void hload_frag_piece(HFrag<Cfg> &f, const _Float16 *As, const _Float16 *Bs,
                                                 const int (&a_off)[2], const int (&b_off)[2])
{
    if constexpr (P < Cfg::MB)
        f.a[P] = *reinterpret_cast<const halfx8 *>(As + a_off[KS] + P * 32 * LDA);
    else
        f.b[P - Cfg::MB] = *reinterpret_cast<const halfx8 *>(Bs + b_off[KS] + (P - Cfg::MB) * 32 * LDB);
}

template <class Cfg, int Q>
__device__ __forceinline__ void hmma_one(const HFrag<Cfg> &f, floatx16 (&acc)[Cfg::MB][Cfg::NB])
{
    constexpr int bm = Q / Cfg::NB, bn = Q % Cfg::NB;
    acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.a[bm], f.b[bn], acc[bm][bn], 0, 0, 0);
}

// One K tile (including its barrier): MB*NB matrix instructions per k step.  Between them: the fragment
// reads of the next k step (or of the next tile's first step), the LDS stores of the staged tile
// (DO_STORE) and the global loads of a later tile (DO_LOAD).  SLOT is the register set both use: the
// tile stored now was loaded SLOTS iterations ago.
//
// STEADY: everything happens, no conditions.  Otherwise (first and last tiles of a K range) the
// workgroup-uniform flags say whether there is a tile to store, one to load and a next one to read;
// the conditions guard the memory operations only, the matrix instructions are common code.
template <class Cfg, int SLOT, bool STEADY, class RL, class CL>
__device__ __forceinline__ void htile_iter(RL &rl, CL &cl, HFrag<Cfg> (&fr)[2], floatx16 (&acc)[Cfg::MB][Cfg::NB],
                                           const _Float16 *cur, const _Float16 *nxt, _Float16 *fill, const int (&a_off)[2],
                                           const int (&b_off)[2],
                                           bool DO_STORE = true, bool DO_LOAD = true, bool NEXT = true)
{
    if constexpr (STEADY) {
        DO_STORE = true;
        DO_LOAD = true;
        NEXT = true;
    }
    constexpr int NMMA = Cfg::MB * Cfg::NB, NFRAG = Cfg::MB + Cfg::NB;
    constexpr int NST = RL::NSTORE + CL::NSTORE, NLD = RL::NLOAD + CL::NLOAD;
    constexpr int PER = (NST + NMMA - 1) / NMMA;  // LDS stores after each matrix instruction of k step 0
    static_assert(Cfg::KSTEPS == 2 && NFRAG <= NMMA && NLD <= NMMA, "two k steps: stores in the first, loads in the second");
    // k step 0: fragments of k step 1, and the staged tile goes to LDS
    static_for<NMMA>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
        hmma_one<Cfg, q>(fr[0], acc);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (q < NFRAG) hload_frag_piece<Cfg, RL::LD, CL::LD, 1, q>(fr[1], cur, cur + Cfg::A_HALVES, a_off, b_off);
        if (DO_STORE) {
            static_for<PER>([&](auto ec) {
                constexpr int st = q * PER + decltype(ec)::value;
                if constexpr (st < RL::NSTORE)
                    rl.template store_piece<SLOT, st>(fill);
                else if constexpr (st < NST)
                    cl.template store_piece<SLOT, st - RL::NSTORE>(fill + Cfg::A_HALVES);
            });
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    // The one barrier of the iteration sits here, between the k steps: what it has to wait for (the
    // LDS stores above, the fragment reads the next instructions need anyway) was issued at the start
    // of k step 0, so the wait is short; at the end of the iteration it would expose the latency of
    // the next tile's fragment reads on every K tile.  Hazards: the stage written above was last read
    // by fragment reads issued before the previous iteration's barrier; the tile written above is
    // first read after the next iteration's barrier.
    __syncthreads();
    // k step 1: fragments of the next tile's k step 0, and the global loads of a later tile into the
    // register set that was just stored
    static_for<NMMA>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
        hmma_one<Cfg, q>(fr[1], acc);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (q < NFRAG) {
            if (NEXT) hload_frag_piece<Cfg, RL::LD, CL::LD, 0, q>(fr[0], nxt, nxt + Cfg::A_HALVES, a_off, b_off);
        }
        if constexpr (q < NLD) {
            if (DO_LOAD) {
                if constexpr (q < RL::NLOAD)
                    rl.template load_piece<SLOT, q>();
                else
                    cl.template load_piece<SLOT, q - RL::NLOAD>();
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    if (DO_LOAD) {
        rl.advance();
        cl.advance();
    }
}

// Epilogue: lane (i, h) holds, for block (bm, bn) and register r, the element in tile row
// wm0 + 32*bm + 8*(r/4) + 4*h + r%4, tile column wn0 + 32*bn + i.  out = half(alpha*acc + beta*out);
// a slice of a plain split-K launch writes raw FP32 sums to its M x N array in the workspace.
template <class Cfg>
__device__ __forceinline__ void hstore_tile(const floatx16 (&acc)[Cfg::MB][Cfg::NB], _Float16 *C, int64_t ldc, int64_t M,
                                            int64_t N, float alpha, float beta, int64_t m0, int64_t n0,
                                            const SplitPlan &split, const WorkItem &w)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const bool raw = split.plain && w.nslice > 1;
    float *Z = raw ? split.partials + (int64_t)w.slice * split.slice_stride : nullptr;
    if (!raw && beta != 0.0f && m0 + Cfg::BM <= M && n0 + Cfg::BN <= N) {
        // Tile wholly inside C: the old values of eight rows are fetched before the first is used, so
        // that the epilogue does not wait out the memory latency once per row.
        _Float16 *base = C + (m0 + wm0 + 4 * h) * ldc + (n0 + wn0 + i);
#pragma unroll
        for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
            for (int r0 = 0; r0 < 16; r0 += 8) {
                _Float16 old[8][Cfg::NB];
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int bn = 0; bn < Cfg::NB; ++bn)
                        old[j][bn] = base[(32 * bm + 8 * ((r0 + j) / 4) + ((r0 + j) % 4)) * ldc + 32 * bn];
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int bn = 0; bn < Cfg::NB; ++bn)
                        base[(32 * bm + 8 * ((r0 + j) / 4) + ((r0 + j) % 4)) * ldc + 32 * bn] =
                            (_Float16)__builtin_fmaf(beta, (float)old[j][bn], alpha * acc[bm][bn][r0 + j]);
            }
        return;
    }
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + wm0 + 32 * bm + 8 * (r / 4) + 4 * h + (r % 4);
            if (row >= M) continue;
#pragma unroll
            for (int bn = 0; bn < Cfg::NB; ++bn) {
                const int64_t col = n0 + wn0 + 32 * bn + i;
                if (col >= N) continue;
                if (raw) {
                    Z[row * N + col] = acc[bm][bn][r];
                } else {
                    _Float16 *dst = C + row * ldc + col;
                    float o = alpha * acc[bm][bn][r];
                    if (beta != 0.0f) o += beta * (float)*dst;
                    *dst = (_Float16)o;
                }
            }
        }
}

// Needs: K a multiple of BK, 16-byte aligned A and B with leading dimensions that are multiples of 8,
// and an operand stored along its own index to have a multiple of 8 rows/columns (the host checks).
template <class Cfg, bool A_KCONTIG, bool B_KCONTIG>
__global__ __launch_bounds__(Cfg::NT, Cfg::MIN_WAVES) void hgemm_mfma16_kernel(const HGemmArgs g)
{
    constexpr int S = Cfg::STAGES, SLOTS = 2;
    __shared__ __attribute__((aligned(16))) _Float16 smem[S * Cfg::STAGE_HALVES];

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
    slice_range((int)(g.K / Cfg::BK), 0, w.slice, w.nslice, kt0, T, krem);
    const int64_t k0 = (int64_t)kt0 * Cfg::BK;

    typename HLoaderSel<Cfg, A_KCONTIG, Cfg::BM, SLOTS>::type rl;
    typename HLoaderSel<Cfg, B_KCONTIG, Cfg::BN, SLOTS>::type cl;
    rl.init(g.A, g.lda, m0, g.M, k0, threadIdx.x);
    cl.init(g.B, g.ldb, n0, g.N, k0, threadIdx.x);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    typedef decltype(rl) RLT;
    typedef decltype(cl) CLT;
    const int a_row = (wave / Cfg::WAVES_N) * Cfg::WM + (lane & 31), b_row = (wave % Cfg::WAVES_N) * Cfg::WN + (lane & 31);
    const int a_off[2] = {RLT::frag_off(a_row, 0, lane >> 5), RLT::frag_off(a_row, 1, lane >> 5)};
    const int b_off[2] = {CLT::frag_off(b_row, 0, lane >> 5), CLT::frag_off(b_row, 1, lane >> 5)};

    floatx16 acc[Cfg::MB][Cfg::NB];
#pragma unroll
    for (int bm = 0; bm < Cfg::MB; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::NB; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.0f;

    // Prologue: tiles 0 .. S-2 go to LDS stages 0 .. S-2 through register set 0; then tiles S-1 and S
    // are loaded into register sets 0 and 1 and stay in flight.  Tile t lives in stage t % S; iteration
    // t stores tile t + S - 1 (register set t % 2) and then loads tile t + S + 1 into the same set.
    auto load_all = [&](auto slotc) {
        constexpr int SL = decltype(slotc)::value;
        static_for<decltype(rl)::NLOAD>([&](auto ic) { rl.template load_piece<SL, decltype(ic)::value>(); });
        static_for<decltype(cl)::NLOAD>([&](auto ic) { cl.template load_piece<SL, decltype(ic)::value>(); });
        rl.advance();
        cl.advance();
    };
    auto store_all = [&](_Float16 *st) {
        static_for<decltype(rl)::NSTORE>([&](auto ic) { rl.template store_piece<0, decltype(ic)::value>(st); });
        static_for<decltype(cl)::NSTORE>([&](auto ic) { cl.template store_piece<0, decltype(ic)::value>(st + Cfg::A_HALVES); });
    };
    typedef std::integral_constant<int, 0> Slot0;
    typedef std::integral_constant<int, 1> Slot1;
    HFrag<Cfg> fr[2];
    auto first_frags = [&]() {
        static_for<Cfg::MB + Cfg::NB>([&](auto pc) {
            hload_frag_piece<Cfg, RLT::LD, CLT::LD, 0, decltype(pc)::value>(fr[0], smem, smem + Cfg::A_HALVES, a_off, b_off);
        });
    };
    int cs = 0, fill = S - 1;
    auto stage = [&](int s) { return smem + s * Cfg::STAGE_HALVES; };
    auto next_of = [](int s) { return s + 1 == S ? 0 : s + 1; };
    int t = 0;
    if (T > S + 2) {
        // Long K range.  Everything in the prologue is unconditional, so that on every path into the
        // steady loop the loads in flight are the same two groups in the same order and the waits
        // before the LDS stores can leave the younger group in flight.
#pragma unroll
        for (int s = 0; s < S - 1; ++s) {
            load_all(Slot0());
            store_all(smem + s * Cfg::STAGE_HALVES);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_all(Slot0());
        __builtin_amdgcn_sched_barrier(0);  // keep the two groups in issue order
        load_all(Slot1());
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        first_frags();
        // Two tiles per trip (register sets 0 and 1); LDS stages by pointer.
        while (t + S + 2 < T) {
            htile_iter<Cfg, 0, true>(rl, cl, fr, acc, stage(cs), stage(next_of(cs)), stage(fill), a_off, b_off);
            cs = next_of(cs);
            fill = next_of(fill);
            htile_iter<Cfg, 1, true>(rl, cl, fr, acc, stage(cs), stage(next_of(cs)), stage(fill), a_off, b_off);
            cs = next_of(cs);
            fill = next_of(fill);
            t += 2;
        }
    } else {
#pragma unroll
        for (int s = 0; s < S - 1; ++s) {
            if (s < T) {
                load_all(Slot0());
                store_all(smem + s * Cfg::STAGE_HALVES);
            }
        }
        if (S - 1 < T) load_all(Slot0());
        if (S < T) load_all(Slot1());
        __syncthreads();
        if (T > 0) first_frags();
    }
    // first and last tiles of the range: the same iterations with their conditions
    for (; t < T; t += 2) {
        htile_iter<Cfg, 0, false>(rl, cl, fr, acc, stage(cs), stage(next_of(cs)), stage(fill), a_off, b_off,
                                  t + S - 1 < T, t + S + 1 < T, t + 1 < T);
        cs = next_of(cs);
        fill = next_of(fill);
        if (t + 1 < T) {
            htile_iter<Cfg, 1, false>(rl, cl, fr, acc, stage(cs), stage(next_of(cs)), stage(fill), a_off, b_off,
                                      t + S < T, t + S + 2 < T, t + 2 < T);
            cs = next_of(cs);
            fill = next_of(fill);
        }
    }
    if (!combine_slices<Cfg>(acc, g.split, w)) return;
    hstore_tile<Cfg>(acc, g.C, g.ldc, g.M, g.N, g.alpha, g.beta, m0, n0, g.split, w);
    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 2] = __builtin_readcyclecounter();
        g.clock_probe[blockIdx.x * 4 + 3] = __builtin_amdgcn_s_memrealtime();
    }
}

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0
// and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "no wait") or for vector memory and LDS both.
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
constexpr int waitcnt_vm_lds0(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4); }

// ---------------------------------------------------------------------------------------------
// The same product with a K tile of 64.  A row of a 32-wide K tile is 64 bytes, half a 128-byte
// cache line: each line is then requested twice, by consecutive K tiles, and by the time of the
// second request the 32 KB first-level cache has seen 64 KB of other lines, so the line comes from
// L2 again (counters at 8192^3: 133.8 M line requests to L2 against 67.1 M for the vendor kernel,
// whose K tile is 64).  That doubled traffic, not the load instructions' latency, issue slots or
// scalar bookkeeping, is what the loads cost here (a timing-only variant without them: +26 %).
// With 128-byte rows every line is requested once.  Two stages of 64 KB; four k steps per tile.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_>
struct HTile64Cfg {
    static constexpr int BM = BM_, BN = BN_, BK = 64;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = 2;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int MB = WM / 32, NB = WN / 32;
    static constexpr int A_HALVES = BM * BK, B_HALVES = BN * BK, STAGE_HALVES = A_HALVES + B_HALVES;
    static constexpr int LDS_BYTES = STAGES * STAGE_HALVES * 2;
    static constexpr int KSTEPS = BK / 16;
    // waves per SIMD the register budget is sized for: as many workgroups as the LDS holds
    static constexpr int MIN_WAVES = ((NT / 64 + 3) / 4) * ((160 * 1024 / LDS_BYTES) < 2 ? 1 : 2);
    static_assert(WM % 32 == 0 && WN % 32 == 0 && LDS_BYTES <= 160 * 1024, "wave tile is made of 32x32 blocks");
};

// Global -> LDS loader for an operand stored along k, 128-byte image rows: one instruction fills 8
// consecutive rows; lane l writes position l%8 of row l/8 and fetches the logical chunk
// pos ^ ((row >> 1) & 7), so that the 16 lanes of a fragment read (16 consecutive rows, one logical
// chunk) fall into 16 different 16-byte bank groups of the 256-byte LDS line.
// NBLK blocks of 16 rows per wave; fragments of 16 rows, two k steps of 32 per tile (16x16x32 instruction).
template <int BR, int NT, int NBLK>
struct HLoaderKDma64 {
    static constexpr int NW = NT / 64;
    static constexpr int NP = BR / (8 * NW);  // instructions per thread and tile
    static constexpr int NFILL = NP;
    static constexpr int READS = 1;           // LDS instructions per fragment
    static_assert(BR % (8 * NW) == 0 && NP >= 1, "8 rows of 128 bytes per wave instruction");
    const char *tile;   // workgroup-uniform, kept in scalar registers
    uint32_t off[NP];   // this lane's byte offsets from it
    uint32_t wave_lds;  // byte offset of this wave's first row group inside the image
    uint32_t foff[2];   // byte offset of the lane's fragment of block 0, per k step

    // w0: first row of this wave's part of the tile
    __device__ __forceinline__ void init(const _Float16 *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int tid, int w0)
    {
        const int wave = tid / 64, lane = tid % 64;
        const uint64_t t0 = reinterpret_cast<uint64_t>(base + r0 * ld + k0);  // the same in every lane
        tile = reinterpret_cast<const char *>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(t0 >> 32)) << 32) |
                                              (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)t0));
        wave_lds = (uint32_t)__builtin_amdgcn_readfirstlane(wave * 8 * 128);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int row = (wave + p * NW) * 8 + lane / 8;  // image row
            const int ch = (lane & 7) ^ ((row >> 1) & 7);   // logical chunk stored at this lane's position
            int64_t lr = row;
            lr = r0 + lr < R ? lr : R - 1 - r0;
            off[p] = (uint32_t)((lr * ld + ch * 8) * 2);
        }
        const int row = w0 + (lane & 15), q = lane >> 4;  // lane holds k = 32*ks + 8*q .. +7 of its row
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) foff[ks] = (uint32_t)(row * 128 + (((4 * ks + q) ^ ((row >> 1) & 7)) * 16));
    }
    template <int I>
    __device__ __forceinline__ void fill_piece(uint32_t image_lds) const
    {
        // Written as assembly on purpose: for the builtin form the compiler, which cannot tell which LDS
        // bytes a global -> LDS load writes, waits for all of them (vmcnt(0)) before every later LDS
        // read, which serialises the very loads this path is meant to keep in flight.  The waits are
        // placed by hand instead (htile_iter_mi16).  m0 = LDS byte address of lane 0's 16 bytes (the 16
        // bytes of lane l land at that address + 16*l, checked on the device); the global address is the
        // tile pointer in scalar registers plus the lane's 32-bit offset.  LDS addresses are handled as
        // integers: through generic pointers every load paid a null check and a 64-bit add in scalar
        // instructions, a dozen of them between two matrix instructions.
        asm volatile("s_add_u32 m0, %2, %3\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(off[I]), "s"(tile), "s"(image_lds + wave_lds), "n"(I * NW * 8 * 128)
                     : "memory", "scc");
    }
    __device__ __forceinline__ void advance_fill(int64_t) { tile += 64 * 2; }
    // the lane's 8 halves of block BLK (16 rows), k step KS: 8 consecutive k of one row
    template <int KS, int BLK>
    __device__ __forceinline__ halfx8 read_frag(uint32_t image_lds) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        typedef const __attribute__((address_space(3))) halfx8 *lp;
        return *(lp)(uintptr_t)(image_lds + foff[KS] + BLK * 16 * 128);
#else
        (void)image_lds;
        return halfx8{};
#endif
    }
};

// Global -> LDS loader for an operand stored along its own index (element (k, x) at base[k*ld + x]),
// read back with the transposing LDS read.  ds_read_b64_tr_b16 (checked on the device with an image
// whose element i holds i): in a group of 16 lanes, lane s supplies the address of 4 consecutive
// 16-bit elements, taken as row s/4, columns 4*(s%4)..+3 of a 4 x 16 block, and lane j receives
// column j of the 4 rows.  With rows = k and columns = x a lane gets 4 consecutive k of one x, which
// is what the matrix instruction wants, from an image that keeps the operand's own layout.
// The image is made of 1 KB units of 4 k rows x 128 x (one load instruction each: lane l = 16-byte
// position l of the unit); position r*16 + (c ^ 4r) holds chunk c (8 x) of row r, so that the 4 rows x
// 32 bytes of a 16-lane group, and the two groups that share a pass, use different banks.
// Unit (k/4, x/128) is unit number (k/4)*(BR/128) + x/128.
// For the 16x16x32 instruction the two 16-lane groups that share a pass read k rows 8 apart: the chunk
// position is also XORed with 2*((k >> 3) & 1) to keep them on different banks.
template <int BR, int NT, int NBLK>
struct HLoaderNDma64 {
    static constexpr int NW = NT / 64;
    static constexpr int XH = BR / 128;             // units per row group
    static constexpr int NP = (16 * XH) / NW;       // instructions per thread and tile
    static constexpr int NFILL = NP;
    static constexpr int READS = 2;
    static_assert(BR % 128 == 0 && (16 * XH) % NW == 0 && NP >= 1, "whole units per wave");
    const char *tile;
    uint32_t off[NP];
    uint32_t wave_lds;
    uint32_t foff[NBLK];  // byte offset of the lane's source address for block b, k step 0, first half

    __device__ __forceinline__ void init(const _Float16 *base, int64_t ld, int64_t x0, int64_t X, int64_t k0, int tid, int w0)
    {
        const int wave = tid / 64, lane = tid % 64;
        const uint64_t t0 = reinterpret_cast<uint64_t>(base + k0 * ld + x0);
        tile = reinterpret_cast<const char *>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(t0 >> 32)) << 32) |
                                              (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)t0));
        wave_lds = (uint32_t)__builtin_amdgcn_readfirstlane(wave * 1024);
        const int r = lane / 16;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int u = wave + p * NW;
            const int k = (u / XH) * 4 + r;
            const int c = (lane % 16) ^ (4 * r) ^ (2 * ((k >> 3) & 1));
            int64_t x = (u % XH) * 128 + c * 8;
            x = x0 + x + 8 <= X ? x : X - 8 - x0;  // past the edge: the last whole chunk (never used)
            off[p] = (uint32_t)((k * ld + x) * 2);
        }
        // source address this lane supplies to the transposing read of block b (k step 0, k 0..3 of its 8)
        // the group of 16 lanes l/16 reads k = 8*(l/16) .. +3 (then +4 .. +7) of 16 columns
        const int kk = 8 * (lane / 16) + (lane % 16) / 4;
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const int x = w0 + b * 16 + 4 * (lane % 4);
            const int u = (kk / 4) * XH + x / 128, rr = kk % 4, cc = (x % 128) / 8;
            foff[b] = (uint32_t)(u * 1024 + (rr * 16 + (cc ^ (4 * rr) ^ (2 * ((kk >> 3) & 1)))) * 16 + (x % 8) * 2);
        }
    }
    template <int I>
    __device__ __forceinline__ void fill_piece(uint32_t image_lds) const
    {
        asm volatile("s_add_u32 m0, %2, %3\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(off[I]), "s"(tile), "s"(image_lds + wave_lds), "n"(I * NW * 1024)
                     : "memory", "scc");
    }
    __device__ __forceinline__ void advance_fill(int64_t ld) { tile += 64 * ld * 2; }
    template <int KS, int BLK>
    __device__ __forceinline__ halfx8 read_frag(uint32_t image_lds) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        typedef short shortx4 __attribute__((ext_vector_type(4)));
        typedef short shortx8 __attribute__((ext_vector_type(8)));
        typedef __attribute__((address_space(3))) shortx4 *lp;
        // k step KS starts 8 row groups further, the second half of the lane's 8 k one row group further
        const uint32_t a = image_lds + foff[BLK] + KS * 8 * XH * 1024;
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(uintptr_t)a);
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(uintptr_t)(a + XH * 1024));
        const shortx8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(halfx8, both);
#else
        (void)image_lds;
        return halfx8{};
#endif
    }
};

template <bool KCONTIG, int BR, int NT, int NBLK>
struct HLoader64Sel {
    typedef HLoaderKDma64<BR, NT, NBLK> type;
};
template <int BR, int NT, int NBLK>
struct HLoader64Sel<false, BR, NT, NBLK> {
    typedef HLoaderNDma64<BR, NT, NBLK> type;
};

// ---------------------------------------------------------------------------------------------
// The K = 64 kernel on v_mfma_f32_16x16x32_f16.  Same tile, loads and LDS images (the image of an operand
// stored along its own index with one more XOR, see HLoaderNDma64); a wave tile is MB16 x NB16 blocks
// of 16 x 16, a k step is 32 wide, two per tile.  Operand layout of the instruction: lane l holds row
// (column) l%16 and k = 8*(l/16) .. +7; result register r of lane l is row 4*(l/16) + r, column l%16.
// Why: a stream of this instruction sustains a higher clock than 32x32x16 under the power limit
// (2155 against 1875 TFLOP/s for nothing but matrix instructions with lane-varying operands), and a
// timing-only variant of the 32x32 kernel with each instruction replaced by two of these ran 7-12 %
// faster.  Fragments are single-buffered and replaced as they die: block row bm of A after the last
// instruction of row bm, block column bn of B after its last use in the last row.
template <class Cfg>
struct HFrag16 {
    halfx8 a[Cfg::WM / 16], b[Cfg::WN / 16];
};

// Slot program of one tile (NMMA matrix instructions per k step, numbered q):
//   k step 0: operands of k step 1 replace those of k step 0 as they die (read from the current stage);
//             the last loads of tile t + 1 (those that did not fit k step 1 of the previous iteration).
//   k step 1: after the first pair of rows the one barrier of the iteration: by then the wave has used
//             every fragment it read from the current stage and has waited for its own loads of tile
//             t + 1, so after it the current stage is free and the next stage complete.  The rest of
//             the step reads the next tile's first operands from the next stage and issues the loads
//             of tile t + 2 into the current stage, one every SP instructions.
// Block rows go in pairs, alternating along the block columns: a B operand then dies 2*NB16 - 1
// instructions before its replacement is first used (NB16 with the rows one after the other).
template <class Cfg, bool STEADY, class RL, class CL>
__device__ __forceinline__ void htile_iter_mi16(RL &rl, CL &cl, HFrag16<Cfg> &fr, floatx4 (&acc)[Cfg::WM / 16][Cfg::WN / 16],
                                                uint32_t cur_lds, uint32_t nxt_lds, int64_t lda, int64_t ldb,
                                                bool do_fill = true, bool has_next = true)
{
    if constexpr (STEADY) {
        do_fill = true;
        has_next = true;
    }
    constexpr int MB16 = Cfg::WM / 16, NB16 = Cfg::WN / 16, NMMA = MB16 * NB16;
    constexpr int NFILL = RL::NFILL + CL::NFILL;
    constexpr int SP = NMMA / NFILL;                       // matrix instructions between two loads (2 to 6 measure within 3 %)
    constexpr int BAR = 2 * NB16 - 1;                      // the barrier follows this instruction of k step 1
    constexpr int N1 = (NMMA - BAR - 1 + SP - 1) / SP < NFILL ? (NMMA - BAR - 1 + SP - 1) / SP : NFILL;  // loads issued in k step 1
    constexpr int Q0 = BAR + 1 + SP * N1 - NMMA;           // slot of k step 0 (next iteration) of the first load left over
    constexpr uint32_t B_IMG = Cfg::A_HALVES * 2;
    static_assert(MB16 % 2 == 0 && Q0 >= 0 && Q0 + (NFILL - N1 - 1) * SP < NMMA, "loads fit their slots");
    auto fill_one = [&](auto stc, uint32_t stage_lds) {
        constexpr int st = decltype(stc)::value;
        if constexpr (st < RL::NFILL)
            rl.template fill_piece<st>(stage_lds);
        else
            cl.template fill_piece<st - RL::NFILL>(stage_lds + B_IMG);
    };
    static_for<2>([&](auto kc) {
        constexpr int ks = decltype(kc)::value;
        const uint32_t src = ks == 0 ? cur_lds : nxt_lds;   // stage the replacement operands come from
        const bool rd = ks == 0 ? true : has_next;
        static_for<NMMA>([&](auto qc) {
            // block rows are taken in pairs, the two rows of a pair alternating along the block columns
            constexpr int q = decltype(qc)::value, pair = q / (2 * NB16), wi = q % (2 * NB16);
            constexpr int bm = 2 * pair + wi % 2, bn = wi / 2;
            acc[bm][bn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fr.a[bm], fr.b[bn], acc[bm][bn], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (ks == 1 && q == BAR) {
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds0(0));
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (wi == 2 * NB16 - 1) {    // pair done: both its A operands are dead (after the barrier, if any)
                if (rd) {
                    fr.a[bm - 1] = rl.template read_frag<1 - ks, bm - 1>(src);
                    fr.a[bm] = rl.template read_frag<1 - ks, bm>(src);
                }
            }
            if constexpr (bm == MB16 - 1) {        // last pair, second row: this B operand is dead
                if (rd) fr.b[bn] = cl.template read_frag<1 - ks, bn>(src + B_IMG);
            }
            if constexpr (ks == 1 && q > BAR && (q - BAR - 1) % SP == 0) {
                if (do_fill) fill_one(std::integral_constant<int, (q - BAR - 1) / SP>{}, cur_lds);
            }
            if constexpr (ks == 0 && q >= Q0 && (q - Q0) % SP == 0 && N1 + (q - Q0) / SP < NFILL) {
                if (has_next) fill_one(std::integral_constant<int, N1 + (q - Q0) / SP>{}, nxt_lds);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (ks == 0) {
            if (has_next) {
                rl.advance_fill(lda);
                cl.advance_fill(ldb);
            }
        }
    });
}

// Epilogue of the 16x16 blocks: lane l holds, for block (bm, bn) and register r, tile row
// wm0 + 16*bm + 4*(l/16) + r and tile column wn0 + 16*bn + l%16.
template <class Cfg>
__device__ __forceinline__ void hstore_tile16(const floatx4 (&acc)[Cfg::WM / 16][Cfg::WN / 16], _Float16 *C, int64_t ldc,
                                              int64_t M, int64_t N, float alpha, float beta, int64_t m0, int64_t n0,
                                              const SplitPlan &split, const WorkItem &w)
{
    constexpr int MB16 = Cfg::WM / 16, NB16 = Cfg::WN / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const bool raw = split.plain && w.nslice > 1;
    float *Z = raw ? split.partials + (int64_t)w.slice * split.slice_stride : nullptr;
    if (!raw && beta != 0.0f && m0 + Cfg::BM <= M && n0 + Cfg::BN <= N) {
        // tile wholly inside C: old values of a block row are fetched before the first is used
        _Float16 *base = C + (m0 + wm0 + 4 * g) * ldc + (n0 + wn0 + i);
#pragma unroll
        for (int bm = 0; bm < MB16; ++bm) {
            _Float16 old[4][NB16];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int bn = 0; bn < NB16; ++bn) old[r][bn] = base[(16 * bm + r) * ldc + 16 * bn];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int bn = 0; bn < NB16; ++bn)
                    base[(16 * bm + r) * ldc + 16 * bn] = (_Float16)__builtin_fmaf(beta, (float)old[r][bn], alpha * acc[bm][bn][r]);
        }
        return;
    }
#pragma unroll
    for (int bm = 0; bm < MB16; ++bm)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = m0 + wm0 + 16 * bm + 4 * g + r;
            if (row >= M) continue;
#pragma unroll
            for (int bn = 0; bn < NB16; ++bn) {
                const int64_t col = n0 + wn0 + 16 * bn + i;
                if (col >= N) continue;
                if (raw) {
                    Z[row * N + col] = acc[bm][bn][r];
                } else {
                    _Float16 *dst = C + row * ldc + col;
                    float o = alpha * acc[bm][bn][r];
                    if (beta != 0.0f) o += beta * (float)*dst;
                    *dst = (_Float16)o;
                }
            }
        }
}

// Epilogue through LDS for beta == 0 and a tile wholly inside an aligned C: in the accumulator layout a
// store instruction writes 32-byte pieces of four rows (2 bytes per lane), 128 of them per lane, and at
// 4096^3 that epilogue was 11 % of the kernel.  Each wave instead rounds its WM x WN block to half into
// a region of its own in LDS (the stages are dead by then: every wave has passed the last barrier of
// the K loop, after its last fragment read) and copies it out with 16-byte stores of whole 256-byte row
// pieces.  Rows are padded by 16 bytes so that the four row groups of a 2-byte write and the rows of a
// 16-byte read fall on different banks.
template <class Cfg>
struct HEpilogueLds {
    static constexpr int ROWB = Cfg::WN * 2 + 16;                          // bytes per staged row
    static constexpr int BYTES = (Cfg::NT / 64) * Cfg::WM * ROWB;          // all waves
    static constexpr int CH = Cfg::WN * 2 / 16, RPI = 64 / CH;             // 16-byte chunks per row, rows per instruction
};

template <class Cfg>
__device__ __forceinline__ void hstore_tile16_lds(const floatx4 (&acc)[Cfg::WM / 16][Cfg::WN / 16], _Float16 *C, int64_t ldc,
                                                  float alpha, int64_t m0, int64_t n0, uint32_t smem_lds, bool nt)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef HEpilogueLds<Cfg> E;
    constexpr int MB16 = Cfg::WM / 16, NB16 = Cfg::WN / 16;
    typedef __attribute__((address_space(3))) _Float16 *lp16;
    typedef __attribute__((address_space(3))) const halfx8 *lp128;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const uint32_t region = smem_lds + (uint32_t)wave * (Cfg::WM * E::ROWB);
    const uint32_t wr = region + (uint32_t)(4 * g) * E::ROWB + (uint32_t)i * 2;
#pragma unroll
    for (int bm = 0; bm < MB16; ++bm)
#pragma unroll
        for (int bn = 0; bn < NB16; ++bn)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                *(lp16)(uintptr_t)(wr + (16 * bm + r) * E::ROWB + 32 * bn) = (_Float16)(alpha * acc[bm][bn][r]);
    // the region is this wave's own: its writes only have to have landed
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds0(63));
    const int row = lane / E::CH, ch = lane % E::CH;
    const uint32_t rd = region + (uint32_t)row * E::ROWB + (uint32_t)ch * 16;
    _Float16 *dst = C + (m0 + wm0 + row) * ldc + (n0 + wn0 + ch * 8);
#pragma unroll
    for (int it = 0; it < Cfg::WM / E::RPI; ++it) {
        const halfx8 v = *(lp128)(uintptr_t)(rd + it * E::RPI * E::ROWB);
        if (nt)
            __builtin_nontemporal_store(v, reinterpret_cast<halfx8 *>(dst + (int64_t)it * E::RPI * ldc));
        else
            *reinterpret_cast<halfx8 *>(dst + (int64_t)it * E::RPI * ldc) = v;
    }
#endif
}

// The same for beta != 0: the result must be rounded once, from alpha*acc + beta*old, so the wave stages
// FP32 values, one block row (16 rows of its tile) at a time, in the same region of its own, and the copy
// loop reads 8 of them per lane, adds the 8 old halves it fetched with one 16-byte load before the
// staging began, rounds and stores 16 bytes.  The arithmetic is that of the direct epilogue, bit for bit.
// FP32 rows are padded by 16 bytes: the four row groups of a 4-byte write fall on different banks.
template <class Cfg>
struct HEpilogueLdsBeta {
    static constexpr int ROWB = Cfg::WN * 4 + 16;                 // bytes per staged row
    static constexpr int BYTES = (Cfg::NT / 64) * 16 * ROWB;      // all waves, one block row each
    static constexpr int CH = Cfg::WN / 8, RPI = 64 / CH;         // 8-element chunks per row, rows per instruction
    static constexpr int IT = 16 / RPI;                           // copy instructions per block row
    static_assert(64 % CH == 0 && 16 % RPI == 0, "whole rows per instruction");
};

template <class Cfg>
__device__ __forceinline__ void hstore_tile16_lds_beta(const floatx4 (&acc)[Cfg::WM / 16][Cfg::WN / 16], _Float16 *C,
                                                       int64_t ldc, float alpha, float beta, int64_t m0, int64_t n0,
                                                       uint32_t smem_lds, bool nt)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef HEpilogueLdsBeta<Cfg> E;
    constexpr int MB16 = Cfg::WM / 16, NB16 = Cfg::WN / 16;
    typedef __attribute__((address_space(3))) float *lp32;
    typedef __attribute__((address_space(3))) const floatx4 *lp128;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int wm0 = (wave / Cfg::WAVES_N) * Cfg::WM, wn0 = (wave % Cfg::WAVES_N) * Cfg::WN;
    const uint32_t region = smem_lds + (uint32_t)wave * (16 * E::ROWB);
    const uint32_t wr = region + (uint32_t)(4 * g) * E::ROWB + (uint32_t)i * 4;
    const int row = lane / E::CH, ch = lane % E::CH;
    const uint32_t rd = region + (uint32_t)row * E::ROWB + (uint32_t)ch * 32;
    _Float16 *dst = C + (m0 + wm0 + row) * ldc + (n0 + wn0 + ch * 8);
#pragma unroll
    for (int bm = 0; bm < MB16; ++bm) {
        halfx8 old[E::IT];
#pragma unroll
        for (int it = 0; it < E::IT; ++it)
            old[it] = *reinterpret_cast<const halfx8 *>(dst + (int64_t)(16 * bm + it * E::RPI) * ldc);
#pragma unroll
        for (int bn = 0; bn < NB16; ++bn)
#pragma unroll
            for (int r = 0; r < 4; ++r) *(lp32)(uintptr_t)(wr + r * E::ROWB + 64 * bn) = alpha * acc[bm][bn][r];
        // the region is this wave's own and the LDS serves one wave's accesses in order: its writes only
        // have to have landed before its reads, and the next block row's writes follow this one's reads
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds0(63));
#pragma unroll
        for (int it = 0; it < E::IT; ++it) {
            const floatx4 lo = *(lp128)(uintptr_t)(rd + it * E::RPI * E::ROWB);
            const floatx4 hi = *(lp128)(uintptr_t)(rd + it * E::RPI * E::ROWB + 16);
            halfx8 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[j] = (_Float16)__builtin_fmaf(beta, (float)old[it][j], lo[j]);
                o[4 + j] = (_Float16)__builtin_fmaf(beta, (float)old[it][4 + j], hi[j]);
            }
            if (nt)
                __builtin_nontemporal_store(o, reinterpret_cast<halfx8 *>(dst + (int64_t)(16 * bm + it * E::RPI) * ldc));
            else
                *reinterpret_cast<halfx8 *>(dst + (int64_t)(16 * bm + it * E::RPI) * ldc) = o;
        }
    }
#endif
}

// Needs K a multiple of 64, the alignment of hgemm_mfma16_kernel, and a plain split-K plan (raw slices).
template <class Cfg, bool A_KCONTIG, bool B_KCONTIG>
__global__ __launch_bounds__(Cfg::NT, Cfg::MIN_WAVES) void hgemm_mi16_dma64_kernel(const HGemmArgs g)
{
    constexpr int MB16 = Cfg::WM / 16, NB16 = Cfg::WN / 16;
    typedef typename HLoader64Sel<A_KCONTIG, Cfg::BM, Cfg::NT, MB16>::type RLT;
    typedef typename HLoader64Sel<B_KCONTIG, Cfg::BN, Cfg::NT, NB16>::type CLT;
    constexpr int A_H = Cfg::A_HALVES, STAGE_H = Cfg::STAGE_HALVES;
    constexpr uint32_t STAGE_B = STAGE_H * 2;
    constexpr int NMMA = MB16 * NB16, NFILL = RLT::NFILL + CLT::NFILL, SP = NMMA / NFILL;
    constexpr int N1 = (NMMA - 2 * NB16 + SP - 1) / SP < NFILL ? (NMMA - 2 * NB16 + SP - 1) / SP : NFILL;  // as in htile_iter_mi16
    constexpr int SMEM_H = 2 * STAGE_H > HEpilogueLds<Cfg>::BYTES / 2 ? 2 * STAGE_H : HEpilogueLds<Cfg>::BYTES / 2;
    static_assert(SMEM_H * 2 <= 160 * 1024, "LDS of one compute unit");
    __shared__ __attribute__((aligned(1024))) _Float16 smem[SMEM_H];
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(3))) _Float16 *lds_ptr;
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lds_ptr)smem;
#else
    const uint32_t smem_lds = 0;  // host pass: the body is never run
    (void)smem;
#endif

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
    slice_range((int)(g.K / Cfg::BK), 0, w.slice, w.nslice, kt0, T, krem);
    const int64_t k0 = (int64_t)kt0 * Cfg::BK;

    const int wave = threadIdx.x >> 6;
    RLT rl;
    CLT cl;
    rl.init(g.A, g.lda, m0, g.M, k0, threadIdx.x, (wave / Cfg::WAVES_N) * Cfg::WM);
    cl.init(g.B, g.ldb, n0, g.N, k0, threadIdx.x, (wave % Cfg::WAVES_N) * Cfg::WN);

    floatx4 acc[MB16][NB16];
#pragma unroll
    for (int bm = 0; bm < MB16; ++bm)
#pragma unroll
        for (int bn = 0; bn < NB16; ++bn)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[bm][bn][r] = 0.0f;

    auto fill_range = [&](auto loc, auto hic, uint32_t stage_lds) {  // pieces LO .. HI-1 of the tile at the fill pointers
        constexpr int LO = decltype(loc)::value, HI = decltype(hic)::value;
        static_for<HI - LO>([&](auto ic) {
            constexpr int st = LO + decltype(ic)::value;
            if constexpr (st < RLT::NFILL)
                rl.template fill_piece<st>(stage_lds);
            else
                cl.template fill_piece<st - RLT::NFILL>(stage_lds + A_H * 2);
        });
    };
    typedef std::integral_constant<int, 0> I0;

    // Prologue: tile 0 landed in stage 0 and visible to all waves; the first N1 loads of tile 1 on their way
    // into stage 1 (iteration 0 issues the rest and moves the pointers on).
    if (T > 0) {
        fill_range(I0(), std::integral_constant<int, NFILL>(), smem_lds);
        rl.advance_fill(g.lda);
        cl.advance_fill(g.ldb);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds0(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (T > 1) fill_range(I0(), std::integral_constant<int, N1>(), smem_lds + STAGE_B);

    HFrag16<Cfg> fr;
    if (T > 0) {
        static_for<MB16>([&](auto bc) { fr.a[decltype(bc)::value] = rl.template read_frag<0, decltype(bc)::value>(smem_lds); });
        static_for<NB16>([&](auto bc) { fr.b[decltype(bc)::value] = cl.template read_frag<0, decltype(bc)::value>(smem_lds + A_H * 2); });
    }

    int t = 0;
    while (t + 3 < T) {   // steady state, two tiles per trip (stage addresses are constants)
        htile_iter_mi16<Cfg, true>(rl, cl, fr, acc, smem_lds, smem_lds + STAGE_B, g.lda, g.ldb);
        htile_iter_mi16<Cfg, true>(rl, cl, fr, acc, smem_lds + STAGE_B, smem_lds, g.lda, g.ldb);
        t += 2;
    }
    for (; t < T; ++t) {  // the last tiles (t is even here): the same iteration with its conditions
        const uint32_t cs = (uint32_t)(t & 1);
        htile_iter_mi16<Cfg, false>(rl, cl, fr, acc, smem_lds + cs * STAGE_B, smem_lds + (cs ^ 1u) * STAGE_B, g.lda, g.ldb,
                                    t + 2 < T, t + 1 < T);
    }

    // cvec here: C 16-byte aligned with ldc a multiple of 8 (set by the host for this kernel)
    const bool raw = g.split.plain && w.nslice > 1;
    static_assert(HEpilogueLdsBeta<Cfg>::BYTES <= SMEM_H * 2, "the staging regions fit into the stages");
    const bool through_lds = !raw && g.cvec >= 2 && T > 0 && m0 + Cfg::BM <= g.M && n0 + Cfg::BN <= g.N;
    const bool nt = g.cvec == 3;   // large result: stores with the non-temporal hint (set by the host)
    if (through_lds && g.beta == 0.0f)
        hstore_tile16_lds<Cfg>(acc, g.C, g.ldc, g.alpha, m0, n0, smem_lds, nt);
    else if (through_lds)
        hstore_tile16_lds_beta<Cfg>(acc, g.C, g.ldc, g.alpha, g.beta, m0, n0, smem_lds, nt);
    else
        hstore_tile16<Cfg>(acc, g.C, g.ldc, g.M, g.N, g.alpha, g.beta, m0, n0, g.split, w);
    if (g.clock_probe != nullptr && blockIdx.x < kNumXcd && threadIdx.x == 0) {
        g.clock_probe[blockIdx.x * 4 + 2] = __builtin_readcyclecounter();
        g.clock_probe[blockIdx.x * 4 + 3] = __builtin_amdgcn_s_memrealtime();
    }
}

template <class Cfg>
int launch_hgemm_mi16_dma64(const HGemmArgs &g, bool a_kcontig, bool b_kcontig, hipStream_t stream)
{
    const int tiles = g.tiles_m * g.tiles_n;
    if (g.K % Cfg::BK != 0 || (g.split.splits > 1 && (!g.split.plain || g.split.dp_tiles != 0))) return (int)hipErrorInvalidValue;
    const dim3 grid((unsigned)(g.split.dp_tiles + (tiles - g.split.dp_tiles) * g.split.splits)), block(Cfg::NT);
    if (a_kcontig && b_kcontig)
        hipLaunchKernelGGL((hgemm_mi16_dma64_kernel<Cfg, true, true>), grid, block, 0, stream, g);
    else if (a_kcontig)
        hipLaunchKernelGGL((hgemm_mi16_dma64_kernel<Cfg, true, false>), grid, block, 0, stream, g);
    else if (b_kcontig)
        hipLaunchKernelGGL((hgemm_mi16_dma64_kernel<Cfg, false, true>), grid, block, 0, stream, g);
    else
        hipLaunchKernelGGL((hgemm_mi16_dma64_kernel<Cfg, false, false>), grid, block, 0, stream, g);
    return (int)hipGetLastError();
}

template <class Cfg>
int launch_hgemm_mfma16(const HGemmArgs &g, bool a_kcontig, bool b_kcontig, hipStream_t stream)
{
    const int tiles = g.tiles_m * g.tiles_n;
    const dim3 grid((unsigned)(g.split.dp_tiles + (tiles - g.split.dp_tiles) * g.split.splits)), block(Cfg::NT);
    if (a_kcontig && b_kcontig)
        hipLaunchKernelGGL((hgemm_mfma16_kernel<Cfg, true, true>), grid, block, 0, stream, g);
    else if (a_kcontig)
        hipLaunchKernelGGL((hgemm_mfma16_kernel<Cfg, true, false>), grid, block, 0, stream, g);
    else if (b_kcontig)
        hipLaunchKernelGGL((hgemm_mfma16_kernel<Cfg, false, true>), grid, block, 0, stream, g);
    else
        hipLaunchKernelGGL((hgemm_mfma16_kernel<Cfg, false, false>), grid, block, 0, stream, g);
    return (int)hipGetLastError();
}

struct HCfgDesc {
    const char *name;
    int BM, BN, BK, NT, lds_bytes;
    int (*launch)(const HGemmArgs &, bool a_kcontig, bool b_kcontig, hipStream_t);       // K tile of 32, loads through registers
    int (*launch_mi16)(const HGemmArgs &, bool a_kcontig, bool b_kcontig, hipStream_t);  // K % 64 == 0: K tile of 64, global -> LDS
};
constexpr int kNumHCfg = 2;
const HCfgDesc &hcfg_desc(int i);  // defined in hgemm_instance.hip

}  // namespace dmath
