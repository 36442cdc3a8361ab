// binary32 instantiations of the add-bias-LayerNorm kernels.
#include "layernorm_kernels.h"

namespace turbo {

hipError_t launch_layernorm_f32(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    switch (p.vec) {
        case 4: return launch_layernorm_v<float, 4, true>(p, a, lc, s);
        case 2: return launch_layernorm_v<float, 2>(p, a, lc, s);
        case 1: return launch_layernorm_v<float, 1>(p, a, lc, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace turbo
