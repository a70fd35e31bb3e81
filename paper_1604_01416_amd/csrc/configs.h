// Table of tile configurations.  Each entry is compiled in its own translation unit
// (tile_instance.hip with -DDMATH_CFG_INDEX=<i>) and reached through the function table below.
#pragma once
#include "conv_bwd_filter_kernel.h"
#include "conv_kernel.h"
#include "gemm_kernel.h"
#include "gemm_panels_kernel.h"
#include "hgemm_kernel.h"
#include "dgemm_kernel.h"

namespace dmath {

template <int I> struct CfgAt;
//                                        BM   BN  BK  waves  stages  min waves per SIMD, LDS image
template <> struct CfgAt<0> { typedef TileCfg<256, 128, 16, 4, 1, 3, 2, 0> type; };  // wave tile 64 x 128, 2 workgroups per CU
template <> struct CfgAt<1> { typedef TileCfg<128, 256, 16, 2, 2, 3, 2, 0> type; };  // wave tile 64 x 128, 2 workgroups per CU
template <> struct CfgAt<2> { typedef TileCfg<256, 256, 16, 4, 2, 3, 2, 0> type; };  // 512 threads, one workgroup per CU
template <> struct CfgAt<3> { typedef TileCfg<128, 128, 16, 2, 2, 3, 2, 0> type; };  // wave tile 64 x 64
template <> struct CfgAt<4> { typedef TileCfg<64, 64, 16, 2, 2, 3, 2, 0> type; };    // wave tile 32 x 32, small problems
// Same tile as 2 with the rotated, bank-conflict-free LDS image: the comparison point for the counters.
template <> struct CfgAt<5> { typedef TileCfg<256, 256, 16, 4, 2, 3, 2, 2> type; };
constexpr int kNumCfg = 6;
constexpr int kWideCfg = 3;   // the configuration that also has kernels with 64-bit per-thread offsets

struct CfgDesc {
    const char *name;
    int BM, BN, BK, NT, lds_bytes;
    int (*gemm)(const GemmArgs &, bool a_kcontig, bool b_kcontig, bool vec, bool wide, hipStream_t);
    int (*conv)(const ConvArgs &, bool vec, int loader_kind, hipStream_t);
    int (*hgemm)(const HGemmArgs &, bool a_kcontig, bool b_kcontig, bool vec, bool wide, hipStream_t);  // fails on the rotated-image entry
    int (*gemm_panels)(const GemmPanelArgs &, bool a_kcontig, bool b_kcontig, hipStream_t);
    int (*conv_bwd_filter)(const ConvFilterGradArgs &, bool quad_in_image, bool quad_in_row, hipStream_t);  // fails on the rotated-image entry
};

// Defined one per translation unit.
template <int I> const CfgDesc &cfg_desc();
template <> const CfgDesc &cfg_desc<0>();
template <> const CfgDesc &cfg_desc<1>();
template <> const CfgDesc &cfg_desc<2>();
template <> const CfgDesc &cfg_desc<3>();
template <> const CfgDesc &cfg_desc<4>();
template <> const CfgDesc &cfg_desc<5>();


// Wave-split kernels for products with few tiles and a long K (gemm_wavek_kernel.h), compiled in
// wavek_instance.hip.  For dmath_set_override they are the configurations kNumCfg, kNumCfg + 1, ...
constexpr int kNumWaveK = 1;
struct WaveKDesc {
    const char *name;
    int (*gemm)(const GemmArgs &, bool a_kcontig, bool b_kcontig, bool vec, hipStream_t);
};
const WaveKDesc &wavek_desc(int i);

}  // namespace dmath
