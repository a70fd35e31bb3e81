// The FP16-input matrix-instruction GEMM kernels, in a translation unit of their own.
#include "hgemm_kernel.h"

namespace dmath {

// K tile of 32, operands staged through registers (K a multiple of 32 but not of 64)
typedef HTileCfg<256, 256, 4, 2, 3> HCfg0;  // 8 waves, wave tile 64 x 128, two waves per SIMD
typedef HTileCfg<128, 128, 2, 2, 3> HCfg1;  // 4 waves, wave tile 64 x 64: products with few tiles
// K tile of 64 (128-byte rows), two stages, global -> LDS loads, 16x16x32 instruction
typedef HTile64Cfg<256, 256, 4, 2> HCfg0K64;
typedef HTile64Cfg<128, 128, 2, 2> HCfg1K64;  // 64 KB of LDS: two workgroups per compute unit

const HCfgDesc &hcfg_desc(int i)
{
    static const HCfgDesc d[kNumHCfg] = {
        {"h256x256_w4x2", HCfg0::BM, HCfg0::BN, HCfg0::BK, HCfg0::NT, HCfg0::LDS_BYTES, &launch_hgemm_mfma16<HCfg0>, &launch_hgemm_mi16_dma64<HCfg0K64>},
        {"h128x128_w2x2", HCfg1::BM, HCfg1::BN, HCfg1::BK, HCfg1::NT, HCfg1::LDS_BYTES, &launch_hgemm_mfma16<HCfg1>, &launch_hgemm_mi16_dma64<HCfg1K64>},
    };
    return d[i < 0 || i >= kNumHCfg ? 0 : i];
}

}  // namespace dmath
