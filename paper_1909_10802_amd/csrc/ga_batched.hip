// libga, gfx950: persistent multi-arrival kernel fed from gradient buffers (a queue of arrivals
// whose gradients are already in device memory is applied by one launch).

#include "ga_persistent.h"

namespace ga {

hipError_t launch_batched(const StatePtrs& st, uint64_t N, int family, const ga_arrival* dev_table,
                          const AdamRow* dev_adam_table, uint32_t T, uint64_t k0, const void* const* dev_grads,
                          int grad_dtype, int mode, bool nesterov, bool keep_m, const RunConst& rc,
                          hipStream_t stream) {
    if (grad_dtype == GA_F32)
        return launch_persistent_from<kSrcF32>(st, N, family, dev_table, dev_adam_table, T, k0, nullptr, nullptr,
                                               dev_grads, mode, nesterov, keep_m, rc, stream);
    if (grad_dtype == GA_BF16)
        return launch_persistent_from<kSrcBf16>(st, N, family, dev_table, dev_adam_table, T, k0, nullptr, nullptr,
                                                dev_grads, mode, nesterov, keep_m, rc, stream);
    return hipErrorInvalidValue;
}

}  // namespace ga
