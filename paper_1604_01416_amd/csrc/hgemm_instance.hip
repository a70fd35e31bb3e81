// The FP16-input matrix-instruction GEMM kernels (one tile configuration), in a translation unit of
// their own.
#include "hgemm_kernel.h"

namespace dmath {

typedef HTileCfg<256, 256, 4, 2, 3> HCfg0;

const HCfgDesc &hcfg_desc()
{
    static const HCfgDesc d = {"h256x256x32_w4x2_s3", HCfg0::BM, HCfg0::BN, HCfg0::BK, HCfg0::NT, HCfg0::LDS_BYTES,
                               &launch_hgemm_mfma16<HCfg0>};
    return d;
}

}  // namespace dmath
