// The double-precision GEMM kernels, in a translation unit of their own.
#include "dgemm_kernel.h"

namespace dmath {

typedef DTileCfg<256, 128, 4, 2, 3> DCfg0;  // 8 waves of 64 x 64
typedef DTileCfg<128, 128, 4, 2, 3> DCfg1;  // 8 waves of 32 x 64, for products with few tiles

const DCfgDesc &dcfg_desc(int i)
{
    static const DCfgDesc d[kNumDCfg] = {
        {"d256x128x16_w4x2_s3", DCfg0::BM, DCfg0::BN, DCfg0::BK, DCfg0::NT, DCfg0::LDS_BYTES, &launch_dgemm<DCfg0>},
        {"d128x128x16_w4x2_s3", DCfg1::BM, DCfg1::BN, DCfg1::BK, DCfg1::NT, DCfg1::LDS_BYTES, &launch_dgemm<DCfg1>},
    };
    return d[i < 0 || i >= kNumDCfg ? 0 : i];
}

}  // namespace dmath
