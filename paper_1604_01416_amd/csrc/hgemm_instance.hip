// The FP16-input matrix-instruction GEMM kernels, in a translation unit of their own.
#include "hgemm_kernel.h"

namespace dmath {

typedef HTileCfg<256, 256, 4, 2, 3> HCfg0;  // 8 waves, wave tile 64 x 128, two waves per SIMD
typedef HTileCfg<256, 256, 2, 2, 3> HCfg1;  // 4 waves, wave tile 128 x 128, one wave per SIMD
typedef HTileCfg<128, 128, 2, 2, 3> HCfg2;  // 4 waves, wave tile 64 x 64: products with few tiles

// the same tiles with 4 LDS stages for the kernels that load global -> LDS
typedef HTileCfg<256, 256, 4, 2, 4> HCfg0D;
typedef HTileCfg<256, 256, 2, 2, 4> HCfg1D;
typedef HTileCfg<128, 128, 2, 2, 4> HCfg2D;
// K tile of 64 (128-byte rows), two stages
typedef HTile64Cfg<256, 256, 4, 2> HCfg0K64;
typedef HTile64Cfg<256, 256, 2, 2> HCfg1K64;
typedef HTile64Cfg<128, 128, 2, 2> HCfg2K64;  // 64 KB of LDS: two workgroups per compute unit

const HCfgDesc &hcfg_desc(int i)
{
    static const HCfgDesc d[kNumHCfg] = {
        {"h256x256x32_w4x2_s3", HCfg0::BM, HCfg0::BN, HCfg0::BK, HCfg0::NT, HCfg0::LDS_BYTES, &launch_hgemm_mfma16<HCfg0>, &launch_hgemm_mfma16_dma<HCfg0D>, &launch_hgemm_mfma16_dma64<HCfg0K64>, &launch_hgemm_mi16_dma64<HCfg0K64>},
        {"h256x256x32_w2x2_s3", HCfg1::BM, HCfg1::BN, HCfg1::BK, HCfg1::NT, HCfg1::LDS_BYTES, &launch_hgemm_mfma16<HCfg1>, &launch_hgemm_mfma16_dma<HCfg1D>, &launch_hgemm_mfma16_dma64<HCfg1K64>, nullptr},
        {"h128x128x32_w2x2_s3", HCfg2::BM, HCfg2::BN, HCfg2::BK, HCfg2::NT, HCfg2::LDS_BYTES, &launch_hgemm_mfma16<HCfg2>, &launch_hgemm_mfma16_dma<HCfg2D>, &launch_hgemm_mfma16_dma64<HCfg2K64>, &launch_hgemm_mi16_dma64<HCfg2K64>},
    };
    return d[i < 0 || i >= kNumHCfg ? 0 : i];
}

}  // namespace dmath
