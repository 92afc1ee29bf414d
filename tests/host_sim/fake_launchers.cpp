// Test scaffolding (CPU only): stand-ins for the kernel launchers that ga_host.cpp uses (the HIP runtime's are in
// fake_runtime.cpp), so that the host side of the library -- argument checks, the bookkeeping of Alg. 3 / Alg. 5
// (k, iter[], tau), the per-arrival scalars, the chunking of a schedule into arrival tables, the delay log,
// checkpoints -- runs on a CPU under AddressSanitizer and UndefinedBehaviorSanitizer.  A launch does no arithmetic
// and only records the scalars it was given (one line per arrival) in g_rows.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ga_internal.h"

struct LoggedArrival {
    uint32_t worker;
    float tau, lr, inv_bc_prev;
    int path;   // 0 fused update, 1 persistent table, 2 table with gradient buffers, 3 DANA, 4 Adam, 5 layer-wise
};
std::vector<LoggedArrival> g_rows;
uint64_t g_first_k_of_last_table = 0;

namespace ga {

static void log_step(uint32_t worker, const StepConst& c, int path) {
    g_rows.push_back({worker, c.tau, c.lr, c.inv_bc_prev, path});
}
static void log_table(const ga_arrival* table, uint32_t T, uint64_t k0, int path) {
    g_first_k_of_last_table = k0 + 1;
    for (uint32_t t = 0; t < T; ++t) g_rows.push_back({table[t].worker, table[t].tau, table[t].lr, table[t].inv_bc_prev, path});
}

hipError_t launch_apply(const StatePtrs&, uint64_t, uint32_t worker, const void*, int, int, bool, bool, bool,
                        const StepConst& c, hipStream_t) {
    log_step(worker, c, 0);
    return hipSuccess;
}
hipError_t launch_apply_dana(const StatePtrs&, uint64_t, uint32_t worker, const void*, int, int, bool, bool,
                             const StepConst& c, hipStream_t) {
    log_step(worker, c, 3);
    return hipSuccess;
}
hipError_t launch_apply_adam(const StatePtrs&, uint64_t, uint32_t worker, const void*, int, int, bool, bool,
                             const StepConst& c, hipStream_t) {
    log_step(worker, c, 4);
    return hipSuccess;
}
hipError_t launch_apply_layerwise(const StatePtrs&, uint64_t, uint32_t worker, const void*, int, int, bool,
                                  const LayerTables&, const StepConst& c, bool, int64_t, hipStream_t) {
    log_step(worker, c, 5);
    return hipSuccess;
}
hipError_t launch_persistent(const StatePtrs&, uint64_t, int, const ga_arrival* table, const AdamRow*, uint32_t T,
                             uint64_t k0, const float*, const float*, int, bool, bool, const RunConst&, hipStream_t) {
    log_table(table, T, k0, 1);
    return hipSuccess;
}
hipError_t launch_batched(const StatePtrs&, uint64_t, int, const ga_arrival* table, const AdamRow*, uint32_t T,
                          uint64_t k0, const void* const* dev_grads, int, int, bool, bool, const RunConst&,
                          hipStream_t) {
    for (uint32_t t = 0; t < T; ++t)
        if (!dev_grads[t]) return hipErrorInvalidValue;
    log_table(table, T, k0, 2);
    return hipSuccess;
}
hipError_t launch_quadratic_gradient(const StatePtrs&, uint64_t, uint32_t, const float*, const float*, uint64_t,
                                     const RunConst&, float*, hipStream_t) {
    return hipSuccess;
}
hipError_t launch_diagnostics(const StatePtrs&, uint64_t, uint32_t, float, float, float, DiagPartial* partials,
                              ga_diag* report, hipStream_t) {
    if (report) std::memset(report, 0, sizeof *report);
    else std::memset(partials + kDiagMaxBlocks, 0, sizeof(DiagPartial));
    return hipSuccess;
}
hipError_t launch_diagnostics_static(const float*, const float*, const float*, uint64_t, float, float, float,
                                     ga_diag* report, hipStream_t) {
    std::memset(report, 0, sizeof *report);
    return hipSuccess;
}
hipError_t static_scratch_address(DiagPartial** out) {
    static DiagPartial scratch[kDiagMaxBlocks];
    *out = scratch;
    return hipSuccess;
}
hipError_t launch_box_muller_raw(const uint32_t*, const uint32_t*, uint64_t, float*, float*, hipStream_t) { return hipSuccess; }
hipError_t launch_noise_fill(uint64_t, uint64_t, uint64_t, uint64_t, float*, hipStream_t) { return hipSuccess; }
hipError_t launch_probe_streams(uint32_t, uint32_t, uint32_t, bool, uint64_t, const float* const*, float* const*, hipStream_t) { return hipSuccess; }
hipError_t launch_probe_valu(int, uint32_t, uint32_t, uint32_t*, hipStream_t) { return hipSuccess; }
static uint64_t tiled(int rows, uint64_t i) {
    return rows == 4 ? state_index<1, 4>(i) : rows == 2 ? state_index<1, 2>(i) : rows == 3 ? state_index<1, 3>(i) : i;
}
hipError_t launch_state_get(const float* state, int rows, float* dst, uint64_t n, hipStream_t) {
    for (uint64_t i = 0; i < n; ++i) dst[i] = state[tiled(rows, i)];
    return hipSuccess;
}
hipError_t launch_state_put(float* state, int rows, const float* src, uint64_t n, hipStream_t) {
    for (uint64_t i = 0; i < n; ++i) state[tiled(rows, i)] = src[i];
    return hipSuccess;
}
hipError_t launch_fill(float* dst, uint64_t n, float value, hipStream_t) {
    for (uint64_t i = 0; i < n; ++i) dst[i] = value;
    return hipSuccess;
}
hipError_t launch_broadcast_rows(float* dst, uint64_t stride, uint32_t rows, int snap_rows, const float* src, uint64_t n, hipStream_t) {
    for (uint32_t r = 0; r < rows; ++r)
        for (uint64_t i = 0; i < n; ++i) dst[(uint64_t)r * stride + tiled(snap_rows, i)] = src[i];
    return hipSuccess;
}

}  // namespace ga
