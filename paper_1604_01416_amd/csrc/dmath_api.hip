// C ABI of the library (see include/dmath.h): argument validation, the choice of tile
// configuration / split-K factor from the problem shape, and the two small helper kernels
// (scaling C when no product is needed, and the fixed-order reduction of split-K slices).
#include "../../include/dmath.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstdlib>

#include "configs.h"

namespace dmath {
namespace {


struct ThreadState {
    void *ws = nullptr;
    size_t ws_bytes = 0;
    int force_cfg = -1;
    int force_split = -1;
    int hgemm_path = -1;  // -1 automatic, 0 FP32 matrix instruction on widened operands, 1 / 2 a tile of the FP16-input kernels
    int dgemm_cfg = -1;   // -1 automatic, else index of the FP64 tile configuration
    int last_error_arg = 0;
    unsigned long long *clock_probe = nullptr;
};
thread_local ThreadState g_state;

const CfgDesc &desc(int i)
{
    switch (i) {
        case 0: return cfg_desc<0>();
        case 1: return cfg_desc<1>();
        case 2: return cfg_desc<2>();
        case 3: return cfg_desc<3>();
        case 4: return cfg_desc<4>();
        default: return cfg_desc<5>();
    }
}

dmath_status fail(dmath_status s, int arg)
{
    g_state.last_error_arg = arg;
    return s;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// C[row*ldc + col] = beta * C[...] (exact zero when beta == 0, whatever C held).
__global__ void scale_kernel(float *C, int64_t ldc, int64_t M, int64_t N, float beta)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / N, col = e - row * N;
        float *dst = C + row * ldc + col;
        *dst = (beta == 0.0f) ? 0.0f : beta * *dst;
    }
}

__global__ void scale_kernel_f64(double *C, int64_t ldc, int64_t M, int64_t N, double beta)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / N, col = e - row * N;
        double *dst = C + row * ldc + col;
        *dst = (beta == 0.0) ? 0.0 : beta * *dst;
    }
}

// C = alpha * (slice 0 + slice 1 + ...) + beta * C for the FP64 product, slices added in slice order.
__global__ void splitk_reduce_kernel_f64(const double *ws, int splits, int64_t slice_stride, double *C, int64_t ldc, int64_t M,
                                         int64_t N, double alpha, double beta)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        double sum = ws[e];
        for (int z = 1; z < splits; ++z) sum += ws[(int64_t)z * slice_stride + e];
        const int64_t row = e / N, col = e - row * N;
        double *dst = C + row * ldc + col;
        double o = alpha * sum;
        if (beta != 0.0) o += beta * *dst;
        *dst = o;
    }
}

__global__ void scale_kernel(_Float16 *C, int64_t ldc, int64_t M, int64_t N, float beta)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / N, col = e - row * N;
        _Float16 *dst = C + row * ldc + col;
        *dst = (beta == 0.0f) ? (_Float16)0.0f : (_Float16)(beta * (float)*dst);
    }
}

// C = alpha * (slice 0 + slice 1 + ... in that order) + beta * C.  Slices are dense M x N FP32; C is
// FP32 or half-precision storage (rounded once, at the store).
template <class T>
__global__ void splitk_reduce_kernel(const float *ws, int splits, int64_t slice_stride, T *C, int64_t ldc,
                                     int64_t M, int64_t N, float alpha, float beta)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / N, col = e - row * N;
        float s = ws[e];
        for (int z = 1; z < splits; ++z) s += ws[e + z * slice_stride];
        T *dst = C + row * ldc + col;
        float o = alpha * s;
        if (beta != 0.0f) o += beta * (float)*dst;
        *dst = (T)o;
    }
}

// Vectorised form for N % 4 == 0 and C rows that allow aligned 4-element accesses.
template <class T>
__global__ void splitk_reduce_kernel_v4(const float *ws, int splits, int64_t slice_stride, T *C, int64_t ldc,
                                        int64_t M, int64_t N, float alpha, float beta)
{
    typedef typename Quad<T>::type QT;
    const int64_t nq = N / 4, total = M * nq;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / nq, col = (e - row * nq) * 4;
        const float *src = ws + row * N + col;
        floatx4 s = *reinterpret_cast<const floatx4 *>(src);
        for (int z = 1; z < splits; ++z) s += *reinterpret_cast<const floatx4 *>(src + z * slice_stride);
        T *dst = C + row * ldc + col;
        floatx4 o = alpha * s;
        if (beta != 0.0f) o += beta * Quad<T>::widen(*reinterpret_cast<const QT *>(dst));
        QT q;
        q[0] = (T)o[0];
        q[1] = (T)o[1];
        q[2] = (T)o[2];
        q[3] = (T)o[3];
        *reinterpret_cast<QT *>(dst) = q;
    }
}

__global__ void zero_u32_kernel(unsigned *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Copies the filters into the workspace as the rows x (chans*RS) matrix a convolution kernel reads.
// Forward (transposed == 0): rows = Kout, chans = C, source w[row][ch][tap].  Backward-data
// (transposed == 1): rows = C, chans = Kout, source w[ch][row][tap].  flip reverses the tap index
// (r, s) -> (R-1-r, S-1-s).  tap_major: destination k = ((cb*RS + tap)*BK + cc) for channel cb*BK + cc
// (the order LoaderConvTap walks); else k = ch*RS + tap.
// Also clears the ncounters tile counters of a split plan (or none), which saves that plan its own
// clearing launch.
__global__ void conv_filter_copy_kernel(const float *w, float *wt, int64_t rows, int chans, int RS, int BK,
                                        int transposed, int flip, int tap_major, unsigned *counters, int ncounters)
{
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < ncounters; c += gridDim.x * blockDim.x) counters[c] = 0u;
    const int64_t KK = (int64_t)chans * RS, total = rows * KK;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / KK;
        const int rem = (int)(e - row * KK);
        int ch, tap;
        if (tap_major) {
            const int t = rem / BK, cc = rem - t * BK;
            const int cb = t / RS;
            tap = t - cb * RS;
            ch = cb * BK + cc;
        } else {
            ch = rem / RS;
            tap = rem - ch * RS;
        }
        if (flip) tap = RS - 1 - tap;
        wt[e] = transposed ? w[((int64_t)ch * rows + row) * RS + tap] : w[(row * chans + ch) * RS + tap];
    }
}

constexpr int kMaxSplits = 64;
// A result of this many FP32 elements (32 MiB) or more is accessed with the non-temporal hint in the epilogue: it
// is more than the eight L2 caches hold together, so no consumer would find it there anyway.
constexpr int64_t kStreamElems = (int64_t)1 << 23;

struct Plan {
    int cfg;
    int dp_tiles;  // tiles computed whole; the remaining tiles - dp_tiles are cut into `splits` slices
    int splits;    // 1: nothing is split (dp_tiles == tiles)
};
// dp_tiles == 0 with splits > 1 (every tile split: skinny products) is run as plain split-K: each slice
// writes an M x N array of raw sums to the workspace and a second kernel adds the slices in order;
// measured faster than combining in the tile kernel when every workgroup has to publish its slice.
// A split tail (dp_tiles > 0) is combined in the tile kernel by the last slice to arrive.

// Shape-based choice (the paper's outlook names choosing the multiply algorithm from the shape as
// future work; this is its one-GPU form).  A small time model in microseconds, fitted to measurements
// on MI355X: a compute unit works through its share of the tiles at the MFMA rate it sustains under
// load (about 2.39 GHz), scaled by how well the configuration keeps the MFMA pipe fed, and pays a
// fixed fill/drain time per batch of co-resident workgroups (first loads, last stores; hidden behind
// the other resident workgroup when there is one).  Tiles past the last full round over the 256
// compute units, or all tiles of a product with few of them, can be cut into K slices (see
// combine_slices); slices pay for writing and re-reading their accumulators.
struct CfgModel {
    double eff;        // fraction of the MFMA rate sustained in the K loop with a full compute unit
    double eff_alone;  // the same with a single workgroup on the compute unit (less latency hiding)
    double fill_us;    // fill + drain per batch of resident workgroups
    int wg_per_cu;     // workgroups resident on a compute unit
};
const CfgModel kModel[kNumCfg] = {
    {0.935, 0.93, 9.0, 2},  // 256x128
    {0.938, 0.93, 8.0, 2},  // 128x256
    {0.989, 0.989, 36.0, 1}, // 256x256
    {0.930, 0.92, 9.0, 3},  // 128x128
    {0.800, 0.60, 8.0, 6},   // 64x64
    {0.970, 0.97, 36.0, 1},  // 256x256, rotated image (measured slower than 2; offered, never preferred)
};

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// Workspace a plan needs: slice accumulators, then one counter per split tile.
size_t plan_bytes(const Plan &p, int64_t tiles, int64_t M, int64_t N)
{
    if (p.splits <= 1) return 0;
    const CfgDesc &d = desc(p.cfg);
    if (p.dp_tiles == 0) return (size_t)p.splits * (size_t)M * (size_t)N * sizeof(float);  // plain split-K
    const size_t split_tiles = (size_t)(tiles - p.dp_tiles);
    return align256(split_tiles * p.splits * (size_t)d.BM * d.BN * sizeof(float)) + align256(split_tiles * sizeof(unsigned));
}

double plan_cost(int c, int64_t tiles, int64_t dp, int s, int64_t K)
{
    const double flop_per_us_cu = 256.0 * 2390.0;  // flop per microsecond per compute unit at the sustained clock
    const CfgDesc &d = desc(c);
    const CfgModel &m = kModel[c];
    const int64_t items = (tiles - dp) * s;
    const int64_t per_cu_whole = ceil_div(dp, kNumCU), per_cu_items = ceil_div(items, kNumCU);
    const bool alone = per_cu_whole + per_cu_items < 2 && m.wg_per_cu > 1;
    const double tile_us = 2.0 * d.BM * d.BN * (double)K / flop_per_us_cu / (alone ? m.eff_alone : m.eff);
    double cost = per_cu_whole * tile_us + (double)ceil_div(per_cu_whole, m.wg_per_cu) * m.fill_us;
    if (items > 0) {
        cost += per_cu_items * (tile_us / s) + (double)ceil_div(per_cu_items, m.wg_per_cu) * m.fill_us;
        // slices out and back at ~5 TB/s; a second launch (plain split-K) or the publication fences (split tail)
        cost += (double)items * d.BM * d.BN * 8.0 / 5.0e6 + (dp == 0 ? 5.0 : 8.0);
    }
    return cost;
}

// only_cfg >= 0 restricts the search to that configuration; forced_split >= 1 fixes the split factor
// (then every tile is split); allow_split == false forbids splitting; plans whose scratch would not
// fit into avail bytes are not considered.
Plan choose_plan(int64_t M, int64_t N, int64_t K, bool allow_split, int only_cfg = -1, int forced_split = -1,
                 size_t avail = ~(size_t)0)
{
    Plan best = {only_cfg >= 0 ? only_cfg : 0, 0, 1};
    double best_cost = 1e300;
    for (int c = 0; c < kNumCfg; ++c) {
        if (only_cfg >= 0 && c != only_cfg) continue;
        const CfgDesc &d = desc(c);
        const int64_t tiles = ceil_div(M, d.BM) * ceil_div(N, d.BN);
        if (tiles > 0x7fffffff / 64) continue;
        const int64_t ktiles = K / d.BK;
        const int64_t full = (tiles / kNumCU) * kNumCU;
        if (forced_split >= 1) {
            const int s = (allow_split && ktiles >= forced_split) ? forced_split : 1;
            const double cost = plan_cost(c, tiles, s > 1 ? 0 : tiles, s, K);
            if (cost < best_cost) {
                best_cost = cost;
                best = {c, (int)(s > 1 ? 0 : tiles), s};
            }
            continue;
        }
        // Split factors tried: powers of two, and the factors that make the slices of all tiles fill
        // one to four rounds over the compute units exactly (long reductions into few tiles, as in the
        // filter gradient of a convolution, want more than 16 slices).
        int cand[9] = {1, 2, 4, 8, 16, 0, 0, 0, 0};
        int ncand = allow_split ? 5 : 1;
        for (int r = 1; allow_split && r <= 4; ++r) {
            const int64_t f = (int64_t)r * kNumCU / tiles;
            if (f >= 3 && f <= kMaxSplits && (f & (f - 1)) != 0) cand[ncand++] = (int)f;
        }
        for (int ci = 0; ci < ncand; ++ci) {
            const int s = cand[ci];
            if (s > 1 && ktiles / s < 8) continue;
            // s == 1: no split.  s > 1: all tiles split, and (if there is a full round) only the tail split.
            const int64_t dps[2] = {s == 1 ? tiles : 0, full};
            for (int v = 0; v < (s > 1 && full > 0 && full < tiles ? 2 : 1); ++v) {
                const Plan cand_plan = {c, (int)dps[v], s};
                if (s > 1 && plan_bytes(cand_plan, tiles, M, N) > avail) continue;
                // A split tail is combined inside the launch, and every combination invalidates the L2 of
                // its die under the whole tiles resident there: fine for a tail of a few dozen tiles, ruinous
                // for one of most of a round (173 tail tiles in 4 slices each: 807 us against 548 us unsplit).
                if (s > 1 && dps[v] > 0 && (tiles - dps[v]) * s > 2 * kNumCU) continue;
                const double cost = plan_cost(c, tiles, dps[v], s, K);
                if (cost < best_cost) {
                    best_cost = cost;
                    best = {c, (int)dps[v], s};
                }
            }
        }
    }
    return best;
}

// Start delay of workgroups 256..511 (100 MHz ticks; 0 = none).  When two workgroups share a compute
// unit and the launch runs for several rounds, all of them reach their epilogues together and the
// memory system sees the whole C traffic of a round in one burst while the matrix pipes idle.  Holding
// the second workgroup of each unit back by 20 us keeps the pairs out of phase for the rest of the
// launch: config 3 (8192 x 8192 x 512, beta = 1) 133.8 -> 135.9 TFLOP/s, K = 256 likewise +2 %; 15 to
// 55 us measure alike, 80 us loses, beta = 0 and long K are neutral.
unsigned stagger_ticks(const CfgDesc &d, int64_t tiles, int splits)
{
    const bool two_per_cu = d.lds_bytes * 2 <= 160 * 1024 && d.lds_bytes * 3 > 160 * 1024;
    return (two_per_cu && splits == 1 && tiles >= 4 * kNumCU) ? 2000u : 0u;
}

// The plan a call will really use: the automatic one, or the forced configuration / split factor, and
// always one whose scratch fits into `avail` bytes (measure_only: as if the workspace were unlimited).
// wide: a leading dimension needs the kernels with 64-bit per-thread offsets, which exist for one tile
// configuration only (it overrides a forced one).
// The search costs a few microseconds of host time, which is as long as a small product runs on the
// device, and a caller repeats its shapes: each thread remembers the plans of the last shapes it asked for.
struct PlanKey {
    int64_t M, N, K;
    size_t avail;
    int only, force_split;
    bool operator==(const PlanKey &o) const
    {
        return M == o.M && N == o.N && K == o.K && avail == o.avail && only == o.only && force_split == o.force_split;
    }
};
struct PlanCache {
    static constexpr int kSlots = 32;
    PlanKey key[kSlots];
    Plan plan[kSlots];
    bool used[kSlots] = {};
};
thread_local PlanCache g_plan_cache;

Plan resolve_plan(int64_t M, int64_t N, int64_t K, size_t avail, bool measure_only, bool wide = false)
{
    const ThreadState &st = g_state;
    // a forced wave-split kernel only concerns dmath_gemm
    const int only = wide ? kWideCfg : (st.force_cfg < kNumCfg ? st.force_cfg : -1);
    if (measure_only) avail = ~(size_t)0;
    const PlanKey key = {M, N, K, avail, only, st.force_split};
    const uint64_t hash = ((uint64_t)M * 0x9e3779b97f4a7c15ull) ^ ((uint64_t)N * 0xc2b2ae3d27d4eb4full) ^
                          ((uint64_t)K * 0x165667b19e3779f9ull) ^ (uint64_t)avail ^ ((uint64_t)(only + 1) << 40) ^
                          ((uint64_t)(st.force_split + 1) << 48);
    const int slot = (int)((hash ^ (hash >> 29) ^ (hash >> 47)) % PlanCache::kSlots);
    PlanCache &pc = g_plan_cache;
    if (pc.used[slot] && pc.key[slot] == key) return pc.plan[slot];
    Plan p = choose_plan(M, N, K, true, only, st.force_split, avail);
    const CfgDesc &d = desc(p.cfg);
    if (plan_bytes(p, ceil_div(M, d.BM) * ceil_div(N, d.BN), M, N) > avail)
        p = choose_plan(M, N, K, false, only, -1);  // no room: best plan that needs no scratch
    pc.key[slot] = key;
    pc.plan[slot] = p;
    pc.used[slot] = true;
    return p;
}

// Fills the SplitPlan of a launch from a plan and the scratch area [ws, ws + plan_bytes), and resets
// the counters on the stream (clear_counters == false: the caller has a kernel of its own in front of
// the launch that clears out.counters[0 .. tiles - dp_tiles)).  Returns false if the reset could not be
// launched.
bool prepare_split(const Plan &p, int64_t tiles, int64_t M, int64_t N, void *ws, hipStream_t stream, SplitPlan &out,
                   bool clear_counters = true)
{
    out.dp_tiles = p.dp_tiles;
    out.splits = p.splits;
    out.partials = nullptr;
    out.counters = nullptr;
    out.plain = 0;
    out.slice_stride = 0;
    if (p.splits > 1 && p.dp_tiles == 0) {
        out.plain = 1;
        out.partials = static_cast<float *>(ws);
        out.slice_stride = M * N;
        return true;
    }
    if (p.splits <= 1) {
        out.dp_tiles = (int)tiles;
        out.splits = 1;
        return true;
    }
    const CfgDesc &d = desc(p.cfg);
    const size_t split_tiles = (size_t)(tiles - p.dp_tiles);
    out.partials = static_cast<float *>(ws);
    out.counters = reinterpret_cast<unsigned *>(static_cast<char *>(ws) +
                                                align256(split_tiles * p.splits * (size_t)d.BM * d.BN * sizeof(float)));
    if (!clear_counters) return true;
    hipLaunchKernelGGL(zero_u32_kernel, dim3((unsigned)ceil_div((int64_t)split_tiles, 256)), dim3(256), 0, stream,
                       out.counters, (int)split_tiles);
    return hipGetLastError() == hipSuccess;
}

}  // namespace
}  // namespace dmath

using namespace dmath;

// Scratch of dmath_gemm_noalloc: split-K slices and tile counters live here instead of in a caller's
// workspace.  Every device the library runs on holds its own copy of this array, at its own address,
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress: kernels,
// fills and copies are given the per-device address kept in g_scratch_ptr, never the name.
static __device__ __align__(256) unsigned char scratch[DMATH_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Address of `scratch` on the current device, looked up once per device (threads that race here all
// store the same value).  nullptr if the runtime cannot tell.
static void *noalloc_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p != nullptr) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

// Tile configuration and split-K factor of the FP16-input kernels for a shape (this thread's forced path
// and split included).  Automatic: the 256 x 256 tile once it fills a good part of the device, else the
// 128 x 128 tile; few tiles: K is cut so that the slices fill the compute units (plain split-K with FP32
// slices), as far as `avail` bytes of workspace allow.
int hgemm_tile_choice(int64_t M, int64_t N)
{
    if (g_state.hgemm_path >= 1) return g_state.hgemm_path - 1;
    return ceil_div(M, 256) * ceil_div(N, 256) < 96 ? 1 : 0;
}

int64_t hgemm_split_choice(int hidx, int64_t M, int64_t N, int64_t K, size_t avail)
{
    const HCfgDesc &h = hcfg_desc(hidx);
    const int64_t tiles = ceil_div(M, h.BM) * ceil_div(N, h.BN), ktiles = K / h.BK;
    int64_t s = 1;
    if (g_state.force_split >= 1)
        s = g_state.force_split;
    else if (tiles < kNumCU / 2)
        s = kNumCU / tiles;
    else if (hidx == 1 && tiles < kNumCU)
        s = 2 * kNumCU / tiles;  // two of the small workgroups fit a compute unit
    if (s > kMaxSplits) s = kMaxSplits;
    if (s > ktiles / 2) s = ktiles / 2;
    const size_t slice_bytes = (size_t)M * (size_t)N * sizeof(float);
    if (s > 1 && (size_t)s * slice_bytes > avail) s = (int64_t)(avail / slice_bytes);
    return s < 2 ? 1 : s;
}

// Wave-split kernel (gemm_wavek_kernel.h) for this FP32 product, or -1.  Forced: configuration index
// kNumCfg + v of dmath_set_override.  Automatic: one workgroup of 8 waves per compute unit and 64 x 64 tile,
// so it pays when the 64 x 64 tiles fill whole rounds over the 256 compute units well (measured on
// MI355X against the best tile configuration with its automatic split: 256 tiles 0.78-0.91 of its time
// for K from 512 to 8192, 512 and 768 tiles 0.93-0.94, 1024 tiles equal; 192 of 256 equal at K = 4096, 320
// and 384 of 512 slower; with K up to 256 any tile count up to 256 is 0.94-0.98 of the 64 x 64 tile kernel,
// at K = 512 from 100 tiles on 0.90, at K = 1024 from 144 tiles on 0.90, 196 tiles 0.64; K = 1540 - 1728 with
// 209 - 219 tiles 0.79 - 0.83).  Such products
// used to be cut into K slices across workgroups, with the slices written to and re-read from a workspace
// by a second kernel.
int wavek_choice(int64_t M, int64_t N, int64_t K)
{
    if (g_state.force_cfg >= kNumCfg) return g_state.force_cfg - kNumCfg;
    if (g_state.force_cfg >= 0 || g_state.force_split >= 1) return -1;
    const int64_t tiles = ceil_div(M, 64) * ceil_div(N, 64);
    const int64_t rounds = ceil_div(tiles, kNumCU);
    if (rounds == 1) {
        // Less than a round: the fewer tiles, the sooner cutting K across workgroups (more compute units
        // at work) beats cutting it across the waves of few workgroups.  Measured thresholds.
        const int64_t min_tiles = K <= 256 ? 1 : K <= 512 ? 96 : K <= 1024 ? 144 : K <= 2048 ? 192 : 224;
        return tiles >= min_tiles ? 0 : -1;
    }
    return (rounds <= 3 && tiles * 8 >= rounds * kNumCU * 7 && K >= 512) ? 0 : -1;
}

// Body of dmath_gemm (T = float) and dmath_hgemm (T = _Float16: same kernels, operands widened on the
// way into LDS, result rounded once on the way out).
// ws / ws_bytes: the scratch split plans may use (the thread's registered workspace, or the library's
// own array for dmath_gemm_noalloc).  strict: refuse (WORKSPACE) instead of falling back to a plan without
// scratch when the plan this shape would get with unlimited scratch does not fit.
template <class T>
dmath_status gemm_entry(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K, float alpha, const T *A,
                        int64_t lda, const T *B, int64_t ldb, float beta, T *C, int64_t ldc, void *stream_, void *ws,
                        size_t ws_bytes, bool strict)
{
    constexpr bool kHalf = !std::is_same<T, float>::value;
    constexpr uintptr_t kQuadAlign = 4 * sizeof(T) - 1;  // alignment of a 4-element vector access
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (transA != DMATH_OP_N && transA != DMATH_OP_T) return fail(DMATH_ERR_INVALID_ARG, 1);
    if (transB != DMATH_OP_N && transB != DMATH_OP_T) return fail(DMATH_ERR_INVALID_ARG, 2);
    if (M < 0) return fail(DMATH_ERR_INVALID_ARG, 3);
    if (N < 0) return fail(DMATH_ERR_INVALID_ARG, 4);
    if (K < 0) return fail(DMATH_ERR_INVALID_ARG, 5);
    const bool a_k = (transA == DMATH_OP_N);  // A contiguous along k
    const bool b_k = (transB == DMATH_OP_T);  // B contiguous along k
    const int64_t a_cols = a_k ? K : M, b_cols = b_k ? K : N;
    if (lda < (a_cols > 1 ? a_cols : 1)) return fail(DMATH_ERR_INVALID_ARG, 8);
    if (ldb < (b_cols > 1 ? b_cols : 1)) return fail(DMATH_ERR_INVALID_ARG, 10);
    if (ldc < (N > 1 ? N : 1)) return fail(DMATH_ERR_INVALID_ARG, 13);
    if (M == 0 || N == 0) return DMATH_OK;
    if (C == nullptr) return fail(DMATH_ERR_NULL_PTR, 12);
    const bool no_product = (K == 0 || alpha == 0.0f);
    if (!no_product) {
        if (A == nullptr) return fail(DMATH_ERR_NULL_PTR, 7);
        if (B == nullptr) return fail(DMATH_ERR_NULL_PTR, 9);
    }
    // tile counts and in-kernel K tile counters are 32-bit
    if (M > (int64_t)1 << 40 || N > (int64_t)1 << 40 || K > (int64_t)1 << 33) return fail(DMATH_ERR_UNSUPPORTED, 3);

    if (no_product) {
        if (beta == 1.0f) return DMATH_OK;
        const int64_t total = M * N;
        const int blocks = (int)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
        hipLaunchKernelGGL((void (*)(T *, int64_t, int64_t, int64_t, float))scale_kernel, dim3(blocks), dim3(256), 0,
                           stream, C, ldc, M, N, beta);
        return hipGetLastError() == hipSuccess ? DMATH_OK : fail(DMATH_ERR_LAUNCH, 0);
    }

    // The tile loaders keep 32-bit per-thread byte offsets (up to 256 rows of ld elements of 4 bytes); a
    // block that is a window of a wider row panel runs on the instantiations with 64-bit offsets.
    const bool wide = lda > ((int64_t)1 << 22) || ldb > ((int64_t)1 << 22);
    if constexpr (kHalf) {
        // The FP16-input matrix instruction computes the same FP32 sums of exact products 16 times
        // faster; its kernel needs whole K tiles and 16-byte chunks everywhere.
        const int hidx = hgemm_tile_choice(M, N);
        const HCfgDesc &h = hcfg_desc(hidx);
        const bool fits = aligned16(A) && aligned16(B) && lda % 8 == 0 && ldb % 8 == 0 && K % h.BK == 0 &&
                          (a_k || M % 8 == 0) && (b_k || N % 8 == 0);
        if (g_state.hgemm_path >= 1 && (!fits || wide)) return fail(DMATH_ERR_UNSUPPORTED, 0);
        if (fits && !wide && g_state.hgemm_path != 0 && g_state.force_cfg < 0) {
            const int64_t tiles_m = ceil_div(M, h.BM), tiles_n = ceil_div(N, h.BN), tiles = tiles_m * tiles_n;
            if (tiles * 64 > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 3);
            const int64_t s = hgemm_split_choice(hidx, M, N, K, ws ? ws_bytes : 0);
            HGemmArgs g;
            g.A = A;
            g.B = B;
            g.C = C;
            g.lda = lda;
            g.ldb = ldb;
            g.ldc = ldc;
            g.M = M;
            g.N = N;
            g.K = K;
            g.alpha = alpha;
            g.beta = beta;
            g.tiles_m = (int)tiles_m;
            g.tiles_n = (int)tiles_n;
            g.clock_probe = g_state.clock_probe;
            g.cvec = ((reinterpret_cast<uintptr_t>(C) & 7u) == 0 && ldc % 4 == 0) ? 1 : 0;
            if (aligned16(C) && ldc % 8 == 0) g.cvec = 2;  // 16-byte stores of whole row pieces are possible
            // ... with the non-temporal hint when the result is large (64 MB and more): it would push the operand
            // panels out of L2 (8192^3: 784 -> 756 us NN, 800 -> 742 us NT; at 4096^3 the hint costs 1 %)
            if (g.cvec == 2 && M * N >= ((int64_t)1 << 25)) g.cvec = 3;
            g.split.dp_tiles = s > 1 ? 0 : (int)tiles;
            g.split.splits = (int)s;
            g.split.partials = s > 1 ? static_cast<float *>(ws) : nullptr;
            g.split.counters = nullptr;
            g.split.plain = s > 1 ? 1 : 0;
            g.split.slice_stride = M * N;
            // K a multiple of 64: whole 128-byte lines per tile row, global -> LDS loads, the 16x16x32 form of
            // the instruction (it sustains a higher clock under the power limit); else the K tile of 32
            if ((K % 64 == 0 ? h.launch_mi16 : h.launch)(g, a_k, b_k, stream) != (int)hipSuccess)
                return fail(DMATH_ERR_LAUNCH, 0);
            if (s > 1) {
                const bool v4 = (N % 4 == 0) && g.cvec;
                const int64_t items = v4 ? M * (N / 4) : M * N;
                const int blocks = (int)(ceil_div(items, 256) < 8192 ? ceil_div(items, 256) : 8192);
                if (v4)
                    hipLaunchKernelGGL(splitk_reduce_kernel_v4<_Float16>, dim3(blocks), dim3(256), 0, stream,
                                       static_cast<const float *>(ws), (int)s, M * N, C, ldc, M, N, alpha, beta);
                else
                    hipLaunchKernelGGL(splitk_reduce_kernel<_Float16>, dim3(blocks), dim3(256), 0, stream,
                                       static_cast<const float *>(ws), (int)s, M * N, C, ldc, M, N, alpha, beta);
                if (hipGetLastError() != hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
            }
            return DMATH_OK;
        }
    }

    if constexpr (!kHalf) {
        const int wk = wide ? -1 : wavek_choice(M, N, K);
        if (wk >= 0) {
            const int64_t tiles_m = ceil_div(M, 64), tiles_n = ceil_div(N, 64);
            if (tiles_m * tiles_n > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 3);
            bool vec = aligned16(A) && aligned16(B) && lda % 4 == 0 && ldb % 4 == 0;
            if (!a_k && M % 4 != 0) vec = false;
            if (!b_k && N % 4 != 0) vec = false;
            GemmArgs g;
            g.A = A;
            g.B = B;
            g.C = C;
            g.lda = lda;
            g.ldb = ldb;
            g.ldc = ldc;
            g.M = M;
            g.N = N;
            g.K = K;
            g.alpha = alpha;
            g.beta = beta;
            g.tiles_m = (int)tiles_m;
            g.tiles_n = (int)tiles_n;
            g.clock_probe = g_state.clock_probe;
            g.cvec = (aligned16(C) && ldc % 4 == 0) ? 1 : 0;
            g.split = SplitPlan{(int)(tiles_m * tiles_n), 1, nullptr, nullptr, 0, 0};
            g.stagger_ticks = 0;
            if (wavek_desc(wk).gemm(g, a_k, b_k, vec, stream) != (int)hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
            return DMATH_OK;
        }
    }
    if (strict) {
        const Plan want = resolve_plan(M, N, K, 0, true, wide);
        const CfgDesc &wd = desc(want.cfg);
        if (plan_bytes(want, ceil_div(M, wd.BM) * ceil_div(N, wd.BN), M, N) > (ws ? ws_bytes : 0))
            return fail(DMATH_ERR_WORKSPACE, 0);
    }
    const Plan plan = resolve_plan(M, N, K, ws ? ws_bytes : 0, false, wide);
    const CfgDesc &d = desc(plan.cfg);
    const int64_t tiles_m = ceil_div(M, d.BM), tiles_n = ceil_div(N, d.BN);
    if (tiles_m * tiles_n * plan.splits > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 3);

    // 16-byte loads need aligned bases and rows; along the operand's own index also a whole number of quads.
    auto quad_aligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & kQuadAlign) == 0; };
    bool vec = quad_aligned(A) && quad_aligned(B) && lda % 4 == 0 && ldb % 4 == 0;
    if (!a_k && M % 4 != 0) vec = false;
    if (!b_k && N % 4 != 0) vec = false;

    GemmArgsT<T> g;
    g.A = A;
    g.B = B;
    g.C = C;
    g.lda = lda;
    g.ldb = ldb;
    g.ldc = ldc;
    g.M = M;
    g.N = N;
    g.K = K;
    g.alpha = alpha;
    g.beta = beta;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    g.clock_probe = g_state.clock_probe;
    g.cvec = (quad_aligned(C) && ldc % 4 == 0) ? 1 : 0;
    if (g.cvec && !kHalf && M * N >= kStreamElems) g.cvec = 2;
    if (!prepare_split(plan, tiles_m * tiles_n, M, N, ws, stream, g.split)) return fail(DMATH_ERR_LAUNCH, 0);
    g.stagger_ticks = stagger_ticks(d, tiles_m * tiles_n, plan.splits);
    int rc;
    if constexpr (kHalf)
        rc = d.hgemm(g, a_k, b_k, vec, wide, stream);
    else
        rc = d.gemm(g, a_k, b_k, vec, wide, stream);
    if (rc == (int)hipErrorInvalidValue) return fail(DMATH_ERR_UNSUPPORTED, 0);
    if (rc != (int)hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
    if (g.split.plain) {
        const bool v4 = (N % 4 == 0) && g.cvec;
        const int64_t items = v4 ? M * (N / 4) : M * N;
        const int blocks = (int)(ceil_div(items, 256) < 8192 ? ceil_div(items, 256) : 8192);
        if (v4)
            hipLaunchKernelGGL(splitk_reduce_kernel_v4<T>, dim3(blocks), dim3(256), 0, stream,
                               static_cast<const float *>(ws), plan.splits, M * N, C, ldc, M, N, alpha, beta);
        else
            hipLaunchKernelGGL(splitk_reduce_kernel<T>, dim3(blocks), dim3(256), 0, stream,
                               static_cast<const float *>(ws), plan.splits, M * N, C, ldc, M, N, alpha, beta);
        if (hipGetLastError() != hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
    }
    return DMATH_OK;
}

// FP64 product: tile configuration and K split.  Few tiles (fewer than 3/4 of the compute units with
// the 128x128 tile) are cut into K slices, as many as fill the device, each at least 8 K tiles long;
// the slices are FP64 arrays of M x N in the workspace, added in slice order by a second kernel.
int dgemm_cfg_choice(int64_t M, int64_t N)
{
    if (g_state.dgemm_cfg >= 0) return g_state.dgemm_cfg;
    return ceil_div(M, dcfg_desc(0).BM) * ceil_div(N, dcfg_desc(0).BN) >= (kNumCU * 3) / 4 ? 0 : 1;
}

int64_t dgemm_split_choice(int cfg, int64_t M, int64_t N, int64_t K, size_t avail)
{
    const DCfgDesc &d = dcfg_desc(cfg);
    const int64_t tiles = ceil_div(M, d.BM) * ceil_div(N, d.BN), ktiles = K / d.BK;
    int64_t s = 1;
    if (g_state.force_split >= 1)
        s = g_state.force_split;
    else if (tiles < (kNumCU * 3) / 4)
        s = kNumCU / tiles;
    if (s > kMaxSplits) s = kMaxSplits;
    if (s > ktiles / 8) s = ktiles / 8;
    while (s > 1 && (size_t)s * (size_t)M * (size_t)N * sizeof(double) > avail) --s;
    return s < 1 ? 1 : s;
}

extern "C" {

const char *dmath_version(void) { return "dmath-mi355x 0.1 (gfx950, fp32 mfma)"; }

const char *dmath_status_string(dmath_status s)
{
    switch (s) {
        case DMATH_OK: return "ok";
        case DMATH_ERR_INVALID_ARG: return "invalid argument";
        case DMATH_ERR_NULL_PTR: return "null pointer";
        case DMATH_ERR_UNSUPPORTED: return "unsupported";
        case DMATH_ERR_LAUNCH: return "kernel launch failed";
        case DMATH_ERR_WORKSPACE: return "bad workspace";
    }
    return "unknown status";
}

int dmath_last_error_arg(void) { return g_state.last_error_arg; }

int dmath_num_configs(void) { return kNumCfg + kNumWaveK; }

const char *dmath_config_name(int i)
{
    if (i >= kNumCfg && i < kNumCfg + kNumWaveK) return wavek_desc(i - kNumCfg).name;
    return (i >= 0 && i < kNumCfg) ? desc(i).name : nullptr;
}

dmath_status dmath_set_override(int tile_config, int split_k)
{
    if (tile_config >= kNumCfg + kNumWaveK) return fail(DMATH_ERR_INVALID_ARG, 1);
    if (split_k == 0 || split_k > 64) return fail(DMATH_ERR_INVALID_ARG, 2);
    g_state.force_cfg = tile_config < 0 ? -1 : tile_config;
    g_state.force_split = split_k < 0 ? -1 : split_k;
    return DMATH_OK;
}

dmath_status dmath_set_hgemm_path(int path)
{
    if (path < -1 || path > kNumHCfg) return fail(DMATH_ERR_INVALID_ARG, 1);
    g_state.hgemm_path = path;
    return DMATH_OK;
}

dmath_status dmath_set_clock_probe(void *device_ptr)
{
    if ((reinterpret_cast<uintptr_t>(device_ptr) & 7u) != 0) return fail(DMATH_ERR_INVALID_ARG, 1);
    g_state.clock_probe = static_cast<unsigned long long *>(device_ptr);
    return DMATH_OK;
}

dmath_status dmath_set_workspace(void *device_ptr, size_t bytes)
{
    if (device_ptr == nullptr && bytes != 0) return fail(DMATH_ERR_WORKSPACE, 1);
    if (!aligned16(device_ptr)) return fail(DMATH_ERR_WORKSPACE, 1);
    g_state.ws = device_ptr;
    g_state.ws_bytes = device_ptr ? bytes : 0;
    return DMATH_OK;
}

size_t dmath_gemm_workspace_bytes(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K)
{
    (void)transA;
    (void)transB;
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    if (wavek_choice(M, N, K) >= 0) return 0;  // K is split inside the workgroups: no scratch
    const Plan p = resolve_plan(M, N, K, 0, true);
    const CfgDesc &d = desc(p.cfg);
    return plan_bytes(p, ceil_div(M, d.BM) * ceil_div(N, d.BN), M, N);
}

size_t dmath_hgemm_workspace_bytes(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    size_t need = dmath_gemm_workspace_bytes(transA, transB, M, N, K);  // the widening kernels plan like dmath_gemm
    if (g_state.hgemm_path != 0 && K % 32 == 0) {
        const int64_t s = hgemm_split_choice(hgemm_tile_choice(M, N), M, N, K, ~(size_t)0);
        const size_t fast = s > 1 ? (size_t)s * (size_t)M * (size_t)N * sizeof(float) : 0;
        if (fast > need) need = fast;
    }
    return need;
}

size_t dmath_dgemm_workspace_bytes(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K)
{
    (void)transA;
    (void)transB;
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const int64_t s = dgemm_split_choice(dgemm_cfg_choice(M, N), M, N, K, ~(size_t)0);
    return s > 1 ? (size_t)s * (size_t)M * (size_t)N * sizeof(double) : 0;
}

dmath_status dmath_gemm_plan(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K, int *tile_config,
                             int *split_k)
{
    (void)transA;
    (void)transB;
    if (M < 0) return fail(DMATH_ERR_INVALID_ARG, 3);
    if (N < 0) return fail(DMATH_ERR_INVALID_ARG, 4);
    if (K < 0) return fail(DMATH_ERR_INVALID_ARG, 5);
    Plan p = (M == 0 || N == 0 || K == 0) ? Plan{-1, 0, 1} : resolve_plan(M, N, K, g_state.ws ? g_state.ws_bytes : 0, false);
    if (p.cfg >= 0 && wavek_choice(M, N, K) >= 0) p = Plan{kNumCfg + wavek_choice(M, N, K), 0, 1};
    if (tile_config) *tile_config = p.cfg;
    if (split_k) *split_k = p.splits;
    return DMATH_OK;
}

dmath_status dmath_gemm(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K, float alpha,
                        const float *A, int64_t lda, const float *B, int64_t ldb, float beta, float *C,
                        int64_t ldc, void *stream_)
{
    return gemm_entry<float>(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream_, g_state.ws,
                             g_state.ws_bytes, false);
}

dmath_status dmath_gemm_noalloc(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K, float alpha,
                                const float *A, int64_t lda, const float *B, int64_t ldb, float beta, float *C,
                                int64_t ldc, void *stream_)
{
    void *ptr = noalloc_scratch();
    if (ptr == nullptr) return fail(DMATH_ERR_LAUNCH, 0);
    return gemm_entry<float>(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream_, ptr,
                             (size_t)DMATH_NOALLOC_SCRATCH_BYTES, true);
}

dmath_status dmath_hgemm(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K, float alpha,
                         const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, float beta, uint16_t *C,
                         int64_t ldc, void *stream_)
{
    return gemm_entry<_Float16>(transA, transB, M, N, K, alpha, reinterpret_cast<const _Float16 *>(A), lda,
                                reinterpret_cast<const _Float16 *>(B), ldb, beta, reinterpret_cast<_Float16 *>(C), ldc,
                                stream_, g_state.ws, g_state.ws_bytes, false);
}

dmath_status dmath_dgemm(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K, double alpha,
                         const double *A, int64_t lda, const double *B, int64_t ldb, double beta, double *C,
                         int64_t ldc, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (transA != DMATH_OP_N && transA != DMATH_OP_T) return fail(DMATH_ERR_INVALID_ARG, 1);
    if (transB != DMATH_OP_N && transB != DMATH_OP_T) return fail(DMATH_ERR_INVALID_ARG, 2);
    if (M < 0) return fail(DMATH_ERR_INVALID_ARG, 3);
    if (N < 0) return fail(DMATH_ERR_INVALID_ARG, 4);
    if (K < 0) return fail(DMATH_ERR_INVALID_ARG, 5);
    const bool a_k = (transA == DMATH_OP_N), b_k = (transB == DMATH_OP_T);
    const int64_t a_cols = a_k ? K : M, b_cols = b_k ? K : N;
    if (lda < (a_cols > 1 ? a_cols : 1)) return fail(DMATH_ERR_INVALID_ARG, 8);
    if (ldb < (b_cols > 1 ? b_cols : 1)) return fail(DMATH_ERR_INVALID_ARG, 10);
    if (ldc < (N > 1 ? N : 1)) return fail(DMATH_ERR_INVALID_ARG, 13);
    if (M == 0 || N == 0) return DMATH_OK;
    if (C == nullptr) return fail(DMATH_ERR_NULL_PTR, 12);
    const bool no_product = (K == 0 || alpha == 0.0);
    if (!no_product) {
        if (A == nullptr) return fail(DMATH_ERR_NULL_PTR, 7);
        if (B == nullptr) return fail(DMATH_ERR_NULL_PTR, 9);
    }
    if (M > (int64_t)1 << 40 || N > (int64_t)1 << 40 || K > (int64_t)1 << 33) return fail(DMATH_ERR_UNSUPPORTED, 3);
    if (no_product) {
        if (beta == 1.0) return DMATH_OK;
        const int64_t total = M * N;
        const int blocks = (int)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
        hipLaunchKernelGGL(scale_kernel_f64, dim3(blocks), dim3(256), 0, stream, C, ldc, M, N, beta);
        return hipGetLastError() == hipSuccess ? DMATH_OK : fail(DMATH_ERR_LAUNCH, 0);
    }
    // the large tile once it fills the compute units most of a round, else the small one
    const int cfg = dgemm_cfg_choice(M, N);
    const DCfgDesc &d = dcfg_desc(cfg);
    const int64_t tiles_m = ceil_div(M, d.BM), tiles_n = ceil_div(N, d.BN);
    if (tiles_m * tiles_n > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 3);
    DGemmArgs g;
    g.A = A;
    g.B = B;
    g.C = C;
    g.lda = lda;
    g.ldb = ldb;
    g.ldc = ldc;
    g.M = M;
    g.N = N;
    g.K = K;
    g.alpha = 0.0f;  // the FP64 scalars travel in their own argument
    g.beta = 0.0f;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    g.cvec = 0;
    const int64_t s = dgemm_split_choice(cfg, M, N, K, g_state.ws ? g_state.ws_bytes : 0);
    if (tiles_m * tiles_n * s > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 3);
    g.split.dp_tiles = s > 1 ? 0 : (int)(tiles_m * tiles_n);
    g.split.splits = (int)s;
    g.split.partials = s > 1 ? static_cast<float *>(g_state.ws) : nullptr;   // FP64 slices; the kernel casts
    g.split.counters = nullptr;
    g.split.plain = s > 1 ? 1 : 0;
    g.split.slice_stride = M * N;
    g.clock_probe = nullptr;
    const bool vec = aligned16(A) && aligned16(B) && lda % 2 == 0 && ldb % 2 == 0 && (a_k || M % 2 == 0) && (b_k || N % 2 == 0);
    if (d.launch(g, alpha, beta, a_k, b_k, vec, stream) != (int)hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
    if (s > 1) {
        const int64_t total = M * N;
        const int blocks = (int)(ceil_div(total, 256) < 8192 ? ceil_div(total, 256) : 8192);
        hipLaunchKernelGGL(splitk_reduce_kernel_f64, dim3(blocks), dim3(256), 0, stream, static_cast<const double *>(g_state.ws),
                           (int)s, M * N, C, ldc, M, N, alpha, beta);
        if (hipGetLastError() != hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
    }
    return DMATH_OK;
}

dmath_status dmath_set_dgemm_config(int tile_config)
{
    if (tile_config < -1 || tile_config >= kNumDCfg) return fail(DMATH_ERR_INVALID_ARG, 1);
    g_state.dgemm_cfg = tile_config;
    return DMATH_OK;
}

dmath_status dmath_gemm_panels(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K, int64_t npanels,
                               float alpha, const float *const *A, int64_t lda, const float *const *B, int64_t ldb,
                               float beta, float *C, int64_t ldc, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (transA != DMATH_OP_N && transA != DMATH_OP_T) return fail(DMATH_ERR_INVALID_ARG, 1);
    if (transB != DMATH_OP_N && transB != DMATH_OP_T) return fail(DMATH_ERR_INVALID_ARG, 2);
    if (M < 0) return fail(DMATH_ERR_INVALID_ARG, 3);
    if (N < 0) return fail(DMATH_ERR_INVALID_ARG, 4);
    if (K < 0) return fail(DMATH_ERR_INVALID_ARG, 5);
    if (npanels < 0) return fail(DMATH_ERR_INVALID_ARG, 6);
    const bool a_k = (transA == DMATH_OP_N), b_k = (transB == DMATH_OP_T);
    const int64_t a_cols = a_k ? K : M, b_cols = b_k ? K : N;
    if (lda < (a_cols > 1 ? a_cols : 1)) return fail(DMATH_ERR_INVALID_ARG, 9);
    if (ldb < (b_cols > 1 ? b_cols : 1)) return fail(DMATH_ERR_INVALID_ARG, 11);
    if (ldc < (N > 1 ? N : 1)) return fail(DMATH_ERR_INVALID_ARG, 14);
    if (M == 0 || N == 0) return DMATH_OK;
    if (C == nullptr) return fail(DMATH_ERR_NULL_PTR, 13);
    const bool no_product = (K == 0 || npanels == 0 || alpha == 0.0f);
    bool vec = lda % 4 == 0 && ldb % 4 == 0 && (a_k || M % 4 == 0) && (b_k || N % 4 == 0);
    if (!no_product) {
        if (A == nullptr) return fail(DMATH_ERR_NULL_PTR, 8);
        if (B == nullptr) return fail(DMATH_ERR_NULL_PTR, 10);
        for (int64_t p = 0; p < npanels; ++p) {
            if (A[p] == nullptr) return fail(DMATH_ERR_NULL_PTR, 8);
            if (B[p] == nullptr) return fail(DMATH_ERR_NULL_PTR, 10);
            vec = vec && aligned16(A[p]) && aligned16(B[p]);
        }
    }
    if (M > (int64_t)1 << 40 || N > (int64_t)1 << 40 || K > (int64_t)1 << 33 || npanels > (int64_t)1 << 24)
        return fail(DMATH_ERR_UNSUPPORTED, 3);

    if (no_product) {
        if (beta == 1.0f) return DMATH_OK;
        const int64_t total = M * N;
        const int blocks = (int)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
        hipLaunchKernelGGL((void (*)(float *, int64_t, int64_t, int64_t, float))scale_kernel, dim3(blocks), dim3(256), 0, stream, C, ldc, M, N, beta);
        return hipGetLastError() == hipSuccess ? DMATH_OK : fail(DMATH_ERR_LAUNCH, 0);
    }
    // Every tile configuration uses the same K tile; a panel with a ragged last K tile, operands that
    // rule out 16-byte loads, or leading dimensions beyond the 32-bit per-thread offsets of the fused
    // kernel are run as one accumulating dmath_gemm per panel instead.
    const int bk = desc(0).BK;
    const bool wide = lda > ((int64_t)1 << 22) || ldb > ((int64_t)1 << 22);
    if (K % bk != 0 || !vec || npanels == 1 || wide) {
        for (int64_t p = 0; p < npanels; ++p) {
            const dmath_status st = dmath_gemm(transA, transB, M, N, K, alpha, A[p], lda, B[p], ldb, p == 0 ? beta : 1.0f,
                                               C, ldc, stream_);
            if (st != DMATH_OK) return st;
        }
        return DMATH_OK;
    }

    for (int64_t p0 = 0; p0 < npanels; p0 += kMaxPanels) {
        const int np = (int)(npanels - p0 < kMaxPanels ? npanels - p0 : kMaxPanels);
        const int64_t Ktot = K * np;
        if (Ktot > (int64_t)1 << 33) return fail(DMATH_ERR_UNSUPPORTED, 5);
        const Plan plan = resolve_plan(M, N, Ktot, g_state.ws ? g_state.ws_bytes : 0, false);
        const CfgDesc &d = desc(plan.cfg);
        const int64_t tiles_m = ceil_div(M, d.BM), tiles_n = ceil_div(N, d.BN);
        if (tiles_m * tiles_n * plan.splits > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 3);
        GemmPanelArgs a;
        GemmArgs &g = a.g;
        g.A = nullptr;
        g.B = nullptr;
        g.C = C;
        g.lda = lda;
        g.ldb = ldb;
        g.ldc = ldc;
        g.M = M;
        g.N = N;
        g.K = Ktot;
        g.alpha = alpha;
        g.beta = p0 == 0 ? beta : 1.0f;
        g.tiles_m = (int)tiles_m;
        g.tiles_n = (int)tiles_n;
        g.clock_probe = g_state.clock_probe;
        g.cvec = (aligned16(C) && ldc % 4 == 0) ? 1 : 0;
        if (g.cvec && M * N >= kStreamElems) g.cvec = 2;
        a.npanels = np;
        a.tiles_per_panel = (int)(K / d.BK);
        for (int p = 0; p < kMaxPanels; ++p) {
            a.A[p] = p < np ? A[p0 + p] : nullptr;
            a.B[p] = p < np ? B[p0 + p] : nullptr;
        }
        if (!prepare_split(plan, tiles_m * tiles_n, M, N, g_state.ws, stream, g.split)) return fail(DMATH_ERR_LAUNCH, 0);
        if (d.gemm_panels(a, a_k, b_k, stream) != (int)hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
        if (g.split.plain) {
            const bool v4 = (N % 4 == 0) && g.cvec;
            const int64_t items = v4 ? M * (N / 4) : M * N;
            const int blocks = (int)(ceil_div(items, 256) < 8192 ? ceil_div(items, 256) : 8192);
            if (v4)
                hipLaunchKernelGGL(splitk_reduce_kernel_v4<float>, dim3(blocks), dim3(256), 0, stream,
                                   static_cast<const float *>(g_state.ws), plan.splits, M * N, C, ldc, M, N, alpha, g.beta);
            else
                hipLaunchKernelGGL(splitk_reduce_kernel<float>, dim3(blocks), dim3(256), 0, stream,
                                   static_cast<const float *>(g_state.ws), plan.splits, M * N, C, ldc, M, N, alpha, g.beta);
            if (hipGetLastError() != hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
        }
    }
    return DMATH_OK;
}

// Shared body of the convolution entry points.  The kernel computes  out_mat[rows x cols] =
// filt_mat[rows x KK] * unfolded(in)[KK x cols]  where, forward: rows = Kout, cols = N*P*Q pixels of y,
// KK = C*R*S, in = x; backward-data: rows = C, cols = N*H*W pixels of dx, KK = Kout*R*S, in = dy.
static dmath_status run_conv(bool bwd_data, int64_t N, int64_t C, int64_t H, int64_t W, int64_t Kout, int64_t R,
                             int64_t S, int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, float alpha,
                             const float *in, const float *w, float beta, float *out, hipStream_t stream)
{
    if (N < 0) return fail(DMATH_ERR_INVALID_ARG, 1);
    if (C < 0) return fail(DMATH_ERR_INVALID_ARG, 2);
    if (H < 0) return fail(DMATH_ERR_INVALID_ARG, 3);
    if (W < 0) return fail(DMATH_ERR_INVALID_ARG, 4);
    if (Kout < 0) return fail(DMATH_ERR_INVALID_ARG, 5);
    if (R < 1) return fail(DMATH_ERR_INVALID_ARG, 6);
    if (S < 1) return fail(DMATH_ERR_INVALID_ARG, 7);
    if (pad_h < 0) return fail(DMATH_ERR_INVALID_ARG, 8);
    if (pad_w < 0) return fail(DMATH_ERR_INVALID_ARG, 9);
    if (stride_h < 1) return fail(DMATH_ERR_INVALID_ARG, 10);
    if (stride_w < 1) return fail(DMATH_ERR_INVALID_ARG, 11);
    if (H + 2 * pad_h < R) return fail(DMATH_ERR_INVALID_ARG, 6);
    if (W + 2 * pad_w < S) return fail(DMATH_ERR_INVALID_ARG, 7);
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1;
    const int64_t Q = (W + 2 * pad_w - S) / stride_w + 1;
    const int64_t RS = R * S;
    // roles
    const int64_t rows = bwd_data ? C : Kout;          // rows of the product = channels of the output tensor
    const int64_t chans = bwd_data ? Kout : C;         // channels of the input tensor
    const int64_t in_h = bwd_data ? P : H, in_w = bwd_data ? Q : W;
    const int64_t out_h = bwd_data ? H : P, out_w = bwd_data ? W : Q;
    const int64_t out_pix = out_h * out_w, cols = N * out_pix, KK = chans * RS;
    if (cols == 0 || rows == 0) return DMATH_OK;
    if (out == nullptr) return fail(DMATH_ERR_NULL_PTR, 16);
    const bool no_product = (KK == 0 || in_h * in_w == 0 || alpha == 0.0f);
    if (!no_product) {
        if (in == nullptr) return fail(DMATH_ERR_NULL_PTR, 13);
        if (w == nullptr) return fail(DMATH_ERR_NULL_PTR, 14);
    }
    // in-kernel tap offsets, magic divisions and tile counters are 32-bit
    const int64_t lim = (int64_t)1 << 31;
    if (chans * in_h * in_w >= lim || out_pix >= lim || (KK + 64) * RS >= ((int64_t)1 << 32) || RS * S >= lim ||
        rows * out_pix >= ((int64_t)1 << 40) || pad_h >= (1 << 15) || pad_w >= (1 << 15) || stride_h >= (1 << 15) ||
        stride_w >= (1 << 15) || H >= (1 << 15) || W >= (1 << 15) || N >= lim || rows >= lim || KK > ((int64_t)1 << 22))
        return fail(DMATH_ERR_UNSUPPORTED, 2);

    if (no_product) {
        if (beta == 1.0f) return DMATH_OK;
        const int64_t total = cols * rows;
        const int blocks = (int)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
        hipLaunchKernelGGL((void (*)(float *, int64_t, int64_t, int64_t, float))scale_kernel, dim3(blocks), dim3(256), 0, stream, out, total, (int64_t)1, total, beta);
        return hipGetLastError() == hipSuccess ? DMATH_OK : fail(DMATH_ERR_LAUNCH, 0);
    }

    // The filter copy (tap-major forward, every backward-data call) sits at the start of the workspace;
    // the slices of split tiles come after it.
    const size_t wt_bytes = align256((size_t)rows * (size_t)KK * sizeof(float));
    const size_t ws_total = g_state.ws ? g_state.ws_bytes : 0;
    const bool room = ws_total >= wt_bytes;
    if (bwd_data && !room) return fail(DMATH_ERR_WORKSPACE, 0);
    // backward-data as a forward convolution of dy with the flipped filters: stride 1 and pads inside the filter
    const bool as_forward = bwd_data && stride_h == 1 && stride_w == 1 && pad_h <= R - 1 && pad_w <= S - 1;
    // padding the kernel sees; the tap-major loader shifts its buffer descriptor down by pad_h*W + pad_w
    // elements and needs the whole shifted range below 2^31 bytes (its halo sentinel is offset 2^31)
    const int64_t kpad_h = as_forward ? R - 1 - pad_h : pad_h, kpad_w = as_forward ? S - 1 - pad_w : pad_w;
    const bool tap_shape = (!bwd_data || as_forward) && room && RS <= 32 && chans % 16 == 0 &&
                           N * chans * in_h * in_w * 4 + (kpad_h * in_w + kpad_w) * 4 + (R * in_w + S) * 4 < lim;
    const bool copy_filters = bwd_data || tap_shape;
    const size_t split_off = copy_filters ? wt_bytes : 0;
    Plan plan = resolve_plan(rows, cols, KK, ws_total - split_off, false);
    if (plan.splits > 1 && plan.dp_tiles == 0)  // the convolution has no plain split-K path: tail splits only
        plan = choose_plan(rows, cols, KK, false, g_state.force_cfg < kNumCfg ? g_state.force_cfg : -1, -1);
    const CfgDesc &d = desc(plan.cfg);
    const int64_t tiles_m = ceil_div(rows, d.BM), tiles_n = ceil_div(cols, d.BN);
    if (tiles_m * tiles_n * plan.splits > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 1);
    const bool tap = tap_shape && chans % d.BK == 0;
    const int kind = tap ? kConvTapMajor : (bwd_data && !as_forward ? kConvBwdData : kConvGeneric);

    ConvArgs a;
    a.x = in;
    a.w = w;
    a.y = out;
    a.N = (int)N; a.C = (int)chans; a.H = (int)in_h; a.W = (int)in_w; a.Kout = (int)rows;
    a.R = (int)R; a.S = (int)S; a.P = (int)out_h; a.Q = (int)out_w;
    if (as_forward) {
        a.pad_h = (int)(R - 1 - pad_h); a.pad_w = (int)(S - 1 - pad_w); a.stride_h = 1; a.stride_w = 1;
    } else {
        a.pad_h = (int)pad_h; a.pad_w = (int)pad_w; a.stride_h = (int)stride_h; a.stride_w = (int)stride_w;
    }
    a.RS = (int)RS;
    a.PQ = (int)out_pix;
    a.CRS = KK;
    a.NPQ = cols;
    a.magic_RS = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)RS - 1) / (uint64_t)RS);
    a.magic_S = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)S - 1) / (uint64_t)S);
    a.magic_sh = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)stride_h - 1) / (uint64_t)stride_h);
    a.magic_sw = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)stride_w - 1) / (uint64_t)stride_w);
    a.alpha = alpha;
    a.beta = beta;
    a.tiles_m = (int)tiles_m;
    a.tiles_n = (int)tiles_n;
    a.yvec = (aligned16(out) && out_pix % 4 == 0) ? 1 : 0;
    if (a.yvec && rows * cols >= kStreamElems) a.yvec = 2;
    a.x_bytes = N * chans * in_h * in_w * 4;
    bool vec = aligned16(w) && KK % 4 == 0;
    // the filter copy, when there is one, also clears the counters of the split tail tiles
    if (!prepare_split(plan, tiles_m * tiles_n, rows, cols, static_cast<char *>(g_state.ws) + split_off, stream, a.split,
                       !copy_filters))
        return fail(DMATH_ERR_LAUNCH, 0);
    if (copy_filters) {
        float *wt = static_cast<float *>(g_state.ws);
        const int64_t total = rows * KK;
        const int blocks = (int)(ceil_div(total, 256) < 2048 ? ceil_div(total, 256) : 2048);
        const int ncounters = a.split.counters != nullptr ? (int)(tiles_m * tiles_n - a.split.dp_tiles) : 0;
        hipLaunchKernelGGL(conv_filter_copy_kernel, dim3(blocks), dim3(256), 0, stream, w, wt, rows, (int)chans, (int)RS,
                           d.BK, bwd_data ? 1 : 0, as_forward ? 1 : 0, tap ? 1 : 0, a.split.counters, ncounters);
        if (hipGetLastError() != hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
        a.w = wt;
        vec = KK % 4 == 0;  // the workspace is 16-byte aligned
    }
    if (d.conv(a, vec, kind, stream) != (int)hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
    return DMATH_OK;
}

dmath_status dmath_conv2d_fwd(int64_t N, int64_t C, int64_t H, int64_t W, int64_t Kout, int64_t R, int64_t S,
                              int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, float alpha,
                              const float *x, const float *w, float beta, float *y, void *stream)
{
    return run_conv(false, N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, x, w, beta, y,
                    static_cast<hipStream_t>(stream));
}

dmath_status dmath_conv2d_bwd_data(int64_t N, int64_t C, int64_t H, int64_t W, int64_t Kout, int64_t R, int64_t S,
                                   int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, float alpha,
                                   const float *dy, const float *w, float beta, float *dx, void *stream)
{
    return run_conv(true, N, C, H, W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, alpha, dy, w, beta, dx,
                    static_cast<hipStream_t>(stream));
}

dmath_status dmath_conv2d_bwd_filter(int64_t N, int64_t C, int64_t H, int64_t W, int64_t Kout, int64_t R, int64_t S,
                                     int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, float alpha,
                                     const float *x, const float *dy, float beta, float *dw, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (N < 0) return fail(DMATH_ERR_INVALID_ARG, 1);
    if (C < 0) return fail(DMATH_ERR_INVALID_ARG, 2);
    if (H < 0) return fail(DMATH_ERR_INVALID_ARG, 3);
    if (W < 0) return fail(DMATH_ERR_INVALID_ARG, 4);
    if (Kout < 0) return fail(DMATH_ERR_INVALID_ARG, 5);
    if (R < 1) return fail(DMATH_ERR_INVALID_ARG, 6);
    if (S < 1) return fail(DMATH_ERR_INVALID_ARG, 7);
    if (pad_h < 0) return fail(DMATH_ERR_INVALID_ARG, 8);
    if (pad_w < 0) return fail(DMATH_ERR_INVALID_ARG, 9);
    if (stride_h < 1) return fail(DMATH_ERR_INVALID_ARG, 10);
    if (stride_w < 1) return fail(DMATH_ERR_INVALID_ARG, 11);
    if (H + 2 * pad_h < R) return fail(DMATH_ERR_INVALID_ARG, 6);
    if (W + 2 * pad_w < S) return fail(DMATH_ERR_INVALID_ARG, 7);
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1;
    const int64_t Q = (W + 2 * pad_w - S) / stride_w + 1;
    const int64_t RS = R * S, CRS = C * RS, PQ = P * Q, NPQ = N * PQ;
    if (Kout == 0 || CRS == 0) return DMATH_OK;
    if (dw == nullptr) return fail(DMATH_ERR_NULL_PTR, 16);
    const bool no_product = (NPQ == 0 || alpha == 0.0f);
    if (!no_product) {
        if (x == nullptr) return fail(DMATH_ERR_NULL_PTR, 13);
        if (dy == nullptr) return fail(DMATH_ERR_NULL_PTR, 14);
    }
    const int64_t lim = (int64_t)1 << 31;
    if (C * H * W >= lim || PQ >= lim || CRS >= lim || Kout >= lim || H >= (1 << 15) || W >= (1 << 15) ||
        pad_h >= (1 << 15) || pad_w >= (1 << 15) || stride_h >= (1 << 15) || stride_w >= (1 << 15) || NPQ >= ((int64_t)1 << 33))
        return fail(DMATH_ERR_UNSUPPORTED, 2);
    if (no_product) {
        if (beta == 1.0f) return DMATH_OK;
        const int64_t total = Kout * CRS;
        const int blocks = (int)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
        hipLaunchKernelGGL((void (*)(float *, int64_t, int64_t, int64_t, float))scale_kernel, dim3(blocks), dim3(256), 0, stream, dw, total, (int64_t)1, total, beta);
        return hipGetLastError() == hipSuccess ? DMATH_OK : fail(DMATH_ERR_LAUNCH, 0);
    }

    const Plan plan = resolve_plan(Kout, CRS, NPQ, g_state.ws ? g_state.ws_bytes : 0, false);
    const CfgDesc &d = desc(plan.cfg);
    const int64_t tiles_m = ceil_div(Kout, d.BM), tiles_n = ceil_div(CRS, d.BN);
    if (tiles_m * tiles_n * plan.splits > (int64_t)0x7fffffff) return fail(DMATH_ERR_UNSUPPORTED, 1);

    ConvFilterGradArgs a;
    a.x = x;
    a.dy = dy;
    a.dw = dw;
    a.N = (int)N; a.C = (int)C; a.H = (int)H; a.W = (int)W; a.Kout = (int)Kout;
    a.R = (int)R; a.S = (int)S; a.P = (int)P; a.Q = (int)Q;
    a.pad_h = (int)pad_h; a.pad_w = (int)pad_w; a.stride_h = (int)stride_h; a.stride_w = (int)stride_w;
    a.PQ = (int)PQ;
    a.RS = (int)RS;
    a.CRS = CRS;
    a.NPQ = NPQ;
    a.alpha = alpha;
    a.beta = beta;
    a.tiles_m = (int)tiles_m;
    a.tiles_n = (int)tiles_n;
    a.cvec = (aligned16(dw) && CRS % 4 == 0) ? 1 : 0;
    if (!prepare_split(plan, tiles_m * tiles_n, Kout, CRS, g_state.ws, stream, a.split)) return fail(DMATH_ERR_LAUNCH, 0);
    const bool x_small = C * H * W <= (lim / 4 - 1) / N;  // x below 2 GiB: 32-bit byte offsets reach all of it
    a.x_bytes = x_small ? N * C * H * W * (int64_t)sizeof(float) : 0;
    const bool quad_in_image = PQ % 4 == 0 && aligned16(dy);
    const bool quad_in_row = Q % 4 == 0 && x_small;
    const int rc = d.conv_bwd_filter(a, quad_in_image, quad_in_row, stream);
    if (rc == (int)hipErrorInvalidValue) return fail(DMATH_ERR_UNSUPPORTED, 0);
    if (rc != (int)hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
    if (a.split.plain) {
        const bool v4 = a.cvec != 0;
        const int64_t items = v4 ? Kout * (CRS / 4) : Kout * CRS;
        const int blocks = (int)(ceil_div(items, 256) < 8192 ? ceil_div(items, 256) : 8192);
        if (v4)
            hipLaunchKernelGGL(splitk_reduce_kernel_v4<float>, dim3(blocks), dim3(256), 0, stream,
                               static_cast<const float *>(g_state.ws), plan.splits, Kout * CRS, dw, CRS, Kout, CRS, alpha, beta);
        else
            hipLaunchKernelGGL(splitk_reduce_kernel<float>, dim3(blocks), dim3(256), 0, stream,
                               static_cast<const float *>(g_state.ws), plan.splits, Kout * CRS, dw, CRS, Kout, CRS, alpha, beta);
        if (hipGetLastError() != hipSuccess) return fail(DMATH_ERR_LAUNCH, 0);
    }
    return DMATH_OK;
}

}  // extern "C"
