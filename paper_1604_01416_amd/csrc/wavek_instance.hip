// Instantiates the wave-split GEMM kernels (gemm_wavek_kernel.h) and their table.
#include "configs.h"
#include "gemm_wavek_kernel.h"

namespace dmath {

const WaveKDesc &wavek_desc(int i)
{
    static const WaveKDesc table[kNumWaveK] = {
        {"wavek_64x64x64_w8_s4", &launch_gemm_wavek<4>},
    };
    return table[i < 0 || i >= kNumWaveK ? 0 : i];
}

}  // namespace dmath
