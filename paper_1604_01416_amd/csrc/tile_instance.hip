// One tile configuration: instantiates its GEMM and convolution kernels.
// Compile with -DDMATH_CFG_INDEX=<index into the table of configs.h>.
#include <cstdio>

#include "configs.h"

#ifndef DMATH_CFG_INDEX
#error "compile with -DDMATH_CFG_INDEX=<n>"
#endif

namespace dmath {

typedef CfgAt<DMATH_CFG_INDEX>::type ThisCfg;

template <>
const CfgDesc &cfg_desc<DMATH_CFG_INDEX>()
{
    static char name[64];
    std::snprintf(name, sizeof(name), "%dx%dx%d_w%dx%d_s%d_l%d", ThisCfg::BM, ThisCfg::BN, ThisCfg::BK,
                  ThisCfg::WAVES_M, ThisCfg::WAVES_N, ThisCfg::STAGES, ThisCfg::LKV);
    static const CfgDesc d = {
        name,
        ThisCfg::BM, ThisCfg::BN, ThisCfg::BK, ThisCfg::NT, ThisCfg::LDS_BYTES,
        &launch_gemm_cfg<ThisCfg, float>,
        &launch_conv_cfg<ThisCfg>,
        &launch_gemm_cfg<ThisCfg, _Float16>,
        &launch_gemm_panels_cfg<ThisCfg>,
        &launch_conv_bwd_filter_cfg<ThisCfg>,
    };
    return d;
}

}  // namespace dmath
