// Internal interface between the host bookkeeping (ga_host.cpp) and the
// gfx950 kernels (ga_apply.hip, ga_persistent.hip, ga_layerwise.hip, ga_aux.hip).  Not part of the public ABI.
#ifndef GA_INTERNAL_H
#define GA_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

#include "ga.h"

namespace ga {

// Scalars that are uniform over one arrival.
struct StepConst {
    float gamma;           // momentum coefficient
    float lr;              // eta_k, or eta_k / tau_k (Alg. 3)
    float tau;             // (float) tau_k
    float inv_bc_prev;     // (float)(1 / (1 - beta^(k-1))), 0 at k = 1
    float eta_max;         // Alg. 14
    float eps;             // Alg. 14
    float beta;            // Alg. 14
    float one_minus_beta;  // 1.0f - beta
    float eta_gamma;       // DANA: eta_k * gamma (float product)
    // ADAM (Alg. 9-11)
    float beta1, omb1, beta2, omb2, adam_eps;
    float inv_bc1, inv_bc2;  // (float)(1 / (1 - beta1^k)), (float)(1 / (1 - beta2^k))
};

// Scalars that are uniform over a whole schedule chunk.
struct RunConst {
    float gamma, eta_max, eps, beta, one_minus_beta;
    float beta1, omb1, beta2, omb2, adam_eps;   // ADAM
    float sigma;       // noise scale of the quadratic source
    uint32_t seed_lo, seed_hi;
};

// Per-arrival Adam bias corrections, parallel to the arrival table.
struct AdamRow {
    float inv_bc1, inv_bc2;   // (float)(1 / (1 - beta1^k)), (float)(1 / (1 - beta2^k))
};

// Reduction partial of the diagnostics kernel (one per block, then one total).
struct DiagPartial {
    double sum_graw;
    unsigned long long n_gt1, n_gt0, n_bad;
};

// Layer-wise Gap: layers are cut into chunks of at most kLayerChunk parameters; one block per chunk.
constexpr uint32_t kLayerChunk = 4096;   // a multiple of 64
struct LayerChunk {
    uint64_t start;   // first parameter
    uint32_t len;     // parameters in the chunk
    uint32_t layer;
};
struct LayerSpan {
    uint32_t first_chunk, n_chunks;
};
struct LayerPartial {
    double dist2;     // sum of (theta - snap)^2
    double msum;      // sum of m
};
struct LayerTables {
    const LayerChunk* chunks;
    const LayerSpan* spans;
    LayerPartial* partials;
    float* gaps;
    uint32_t n_chunks, n_layers;
};

constexpr uint32_t kTableCap = 8192;       // arrivals per persistent launch
constexpr uint64_t kDelayLog = (uint64_t)1 << 20;   // delays of this many most recent arrivals are kept on the host
constexpr uint32_t kDiagMaxBlocks = 2048;  // partials in the workspace

// Bytes of theta, v, m that the update kernels keep in the 256 MiB memory-side cache unless the caller sets another
// budget (ga_set_resident_bytes); the reasons for the value are at Residency in ga_device.h.
constexpr uint64_t kResidentBytes = (uint64_t)240 << 20;

// theta, v and m -- the three arrays that every arrival reads and rewrites -- are stored interleaved by tiles of
// kStateTile floats: [theta tile 0 | v tile 0 | m tile 0 | theta tile 1 | ...], so that one block's accesses to the
// three fall into one contiguous 96 KiB region instead of three places N floats apart.  Measured on the update's
// traffic (five arrays read, four written): 32 KiB tiles move 6 - 11 % more bytes per second from HBM than separate
// arrays at 151 M and 350 M parameters (16 and 64 KiB tiles less, 128 KiB and more nothing).  Element j of one of
// the arrays is at state_index<1>(j) floats from that array's pointer in StatePtrs; a group of four (an aligned pair)
// at state_index<4> (state_index<2>) such units.  The snapshots and the other per-worker arrays are plain rows.
// The Adam master has a fourth array of that kind, the second moment v2: its tiles follow m's (ROWS = 4; measured
// with the same stand-alone kernel at 151 M parameters: 5.99 TB/s with v2 as a separate array, 6.40 TB/s as the
// fourth tiled one).
constexpr uint64_t kStateTile = 8192;
template <int UNIT, int ROWS = 3>
__host__ __device__ inline uint64_t state_index(uint64_t i) {
    constexpr uint64_t per_tile = kStateTile / UNIT;
    return (i / per_tile) * (ROWS * per_tile) + (i % per_tile);
}
constexpr int state_rows(int family) { return family == GA_FAMILY_ADAM ? 4 : 3; }

// The per-worker arrays.  A worker's snapshot is a plain row of N floats, except in the DANA master, whose arrival
// reads and rewrites two arrays of the arriving worker, the snapshot and the momentum v_i: there the two are a tiled
// pair, [snapshot tile 0 | v_i tile 0 | snapshot tile 1 | ...] (stand-alone kernel with DANA's traffic at 151 M
// parameters: 5.98 TB/s with two rows, 6.37 TB/s with the pair).  row_index<UNIT, ROWS> is the index inside one
// worker's region: the identity for ROWS = 1.
constexpr int snapshot_rows(int family) { return family == GA_FAMILY_DANA ? 2 : 1; }
template <int UNIT, int ROWS>
__host__ __device__ inline uint64_t row_index(uint64_t i) {
    if constexpr (ROWS == 1) return i;
    else return state_index<UNIT, ROWS>(i);
}

// State pointers inside the workspace.  snaps is W rows of `stride` floats.
struct StatePtrs {
    float* theta;     // tile 0 of theta; index with state_index
    float* v;         // tile 0 of: MOMENTUM: v;  DANA: vsum;  ADAM: m1 (= theta + kStateTile)
    float* m;         // tile 0 of the Alg. 14 state (= theta + 2 kStateTile)
    float* snaps;     // worker 0's snapshot (DANA: tile 0 of it); worker w's is `stride` floats further per w
    float* worker_v;  // DANA: tile 0 of worker 0's v_i (= snaps + kStateTile), else null
    int snap_rows;    // snapshot_rows(family)
    float* v2;        // ADAM: tile 0 of the second moment (= theta + 3 kStateTile; index with state_index<.., 4>), else null
    int rows;         // tiled arrays per tile: state_rows(family)
    uint64_t stride;  // floats between consecutive workers' regions (N rounded up to 64; DANA: 2 x N rounded up to a tile)
    uint64_t resident_bytes;  // budget of the cache-resident leading part of theta, v, m
};

// Fused update of one arrival.  g: N values of grad_dtype.  In the GA modes m
// and the snapshot are always maintained; elsewhere keep_m / write_snap decide.
hipError_t launch_apply(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype, int mode,
                        bool nesterov, bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream);

// DANA (Alg. 6-8) and Adam (Alg. 9-11) fused updates of one arrival; mode is ASGD, SA, GA or GA_HINGE.
hipError_t launch_apply_dana(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype, int mode,
                             bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream);
hipError_t launch_apply_adam(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype, int mode,
                             bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream);

// Layer-wise / global Gap arrival: per-chunk reduction, per-layer Gap, update with one Gap per layer.
// sums_ready: lt.partials already hold this arrival's chunk sums (left by the previous call), so the
// reduction pass is skipped.  next_worker >= 0: the update pass also leaves the chunk sums of the
// arrival that follows, which must be that worker's, with no change to the state in between.
hipError_t launch_apply_layerwise(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype,
                                  int mode, bool nesterov, const LayerTables& lt, const StepConst& c,
                                  bool sums_ready, int64_t next_worker, hipStream_t stream);

// T arrivals replayed inside one launch, gradients generated in the kernel.
// table: device array of T rows; k0: master step before the first row.
hipError_t launch_persistent(const StatePtrs& st, uint64_t N, int family, const ga_arrival* dev_table,
                             const AdamRow* dev_adam_table, uint32_t T, uint64_t k0, const float* a,
                             const float* theta_star, int mode, bool nesterov, bool keep_m, const RunConst& rc,
                             hipStream_t stream);

// The same with the gradient of row t read from the buffer dev_grads[t] (N values of grad_dtype,
// each buffer aligned to four values); dev_grads is a device array of T pointers.
hipError_t launch_batched(const StatePtrs& st, uint64_t N, int family, const ga_arrival* dev_table,
                          const AdamRow* dev_adam_table, uint32_t T, uint64_t k0, const void* const* dev_grads,
                          int grad_dtype, int mode, bool nesterov, bool keep_m, const RunConst& rc,
                          hipStream_t stream);

// g_out = a * (snap_w - theta_star) + sigma * z(seed, k, j)
hipError_t launch_quadratic_gradient(const StatePtrs& st, uint64_t N, uint32_t worker, const float* a,
                                     const float* theta_star, uint64_t k, const RunConst& rc, float* g_out,
                                     hipStream_t stream);

// Gap statistics of one worker: per-block partials, then a fixed-order total, written as a DiagPartial to
// dev_partials[kDiagMaxBlocks] (dev_report null) or as the finished report to dev_report.
hipError_t launch_diagnostics(const StatePtrs& st, uint64_t N, uint32_t worker, float inv_bc, float eta_max,
                              float eps, DiagPartial* dev_partials, ga_diag* dev_report, hipStream_t stream);

// The same statistics of (theta, snap, m) with the partials in the library's static device array.
hipError_t launch_diagnostics_static(const float* theta, const float* snap, const float* m, uint64_t N, float inv_bc,
                                     float eta_max, float eps, ga_diag* dev_report, hipStream_t stream);

// Device address of that array on the current GPU (resolved once per GPU).
hipError_t static_scratch_address(DiagPartial** out);

hipError_t launch_box_muller_raw(const uint32_t* xa, const uint32_t* xb, uint64_t n, float* zc, float* zs,
                                 hipStream_t stream);
hipError_t launch_noise_fill(uint64_t seed, uint64_t k, uint64_t j0, uint64_t n, float* out, hipStream_t stream);

// Measurement aids (ga_probe.hip): n_read arrays read and n_write arrays written at once (n floats each); blocks x 256
// threads each issuing iterations x 8 independent instructions of kind op (ga_probe_op).
hipError_t launch_probe_streams(uint32_t n_read, uint32_t n_write, uint32_t n_resident, bool tiled, uint64_t n,
                                const float* const* reads, float* const* writes, hipStream_t stream);
hipError_t launch_probe_valu(int op, uint32_t blocks, uint32_t iterations, uint32_t* dev_out, hipStream_t stream);

// One tiled array (the theta, v, m or v2 pointer of StatePtrs with rows = state_rows(family); in the DANA master a
// worker's snapshot or v_i with rows = 2) read into / written from a plain array of n floats.
hipError_t launch_state_get(const float* state, int rows, float* dst, uint64_t n, hipStream_t stream);
hipError_t launch_state_put(float* state, int rows, const float* src, uint64_t n, hipStream_t stream);

// dst[0..n) = value;  worker r's snapshot = src[0..n) for r < rows (stride in floats between workers; snap_rows as in
// StatePtrs).
hipError_t launch_fill(float* dst, uint64_t n, float value, hipStream_t stream);
hipError_t launch_broadcast_rows(float* dst, uint64_t stride, uint32_t rows, int snap_rows, const float* src, uint64_t n,
                                 hipStream_t stream);

}  // namespace ga

#endif
