// libga, gfx950: persistent multi-arrival kernel with in-kernel quadratic-plus-noise gradients.

#include "ga_persistent.h"

namespace ga {

hipError_t launch_persistent(const StatePtrs& st, uint64_t N, int family, const ga_arrival* dev_table,
                             const AdamRow* dev_adam_table, uint32_t T, uint64_t k0, const float* a,
                             const float* theta_star, int mode, bool nesterov, bool keep_m, const RunConst& rc,
                             hipStream_t stream) {
    return launch_persistent_from<kSrcQuadratic>(st, N, family, dev_table, dev_adam_table, T, k0, a, theta_star,
                                                 nullptr, mode, nesterov, keep_m, rc, stream);
}

}  // namespace ga
