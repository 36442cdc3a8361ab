// binary16-storage instantiations of the add-bias-LayerNorm kernels (binary32 arithmetic).
#include "layernorm_kernels.h"

namespace turbo {

hipError_t launch_layernorm_f16(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    switch (p.vec) {
        case 8: return launch_layernorm_v<_Float16, 8, true>(p, a, lc, s);
        case 4: return launch_layernorm_v<_Float16, 4>(p, a, lc, s);
        case 2: return launch_layernorm_v<_Float16, 2>(p, a, lc, s);
        case 1: return launch_layernorm_v<_Float16, 1>(p, a, lc, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace turbo
