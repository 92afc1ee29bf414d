// libga, gfx950: fused update of one arrival.
//   apply_kernel         MOMENTUM family (Alg. 2-5 + Alg. 14), gradient from HBM
//   family_apply_kernel  DANA (Alg. 6-8) and Adam (Alg. 9-11) masters
// The path is elementwise (Sec. 4.3: every parameter is penalised independently), bound by HBM
// traffic; there is no contraction and therefore no MFMA.

#include "ga_device.h"

namespace ga {
namespace {

// ---------------------------------------------------------------------------
// Fused update of one arrival.  Each thread owns U groups of four consecutive
// parameters, 256 groups apart, so that every wavefront issues 1 KiB
// contiguous 128-bit loads and stores per array.  All loads of a thread are
// issued before the first dependent operation.
//
// The gradient, the snapshot and, by default, every other array are accessed with the non-temporal
// hint.  The leading blocks of the grid (thresholds in `keep`) access theta, v and m without it, so that
// this part of the state is served by the memory-side cache at the next arrival (ga_device.h).
// ---------------------------------------------------------------------------
template <int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED, int U, bool NT_TH, bool NT_V, bool NT_M>
__device__ __forceinline__ void apply_tile(float* __restrict__ theta, float* __restrict__ v, float* __restrict__ m,
                                           float* __restrict__ snap, const void* __restrict__ g, uint64_t n4,
                                           uint64_t base, const StepConst& c) {
    constexpr bool GAP = is_gap(MODE);
    static_assert((kStateTile / 4) % (kBlock * U) == 0, "a block's groups lie in one tile of the state arrays");
    const uint64_t base_s = state_index<4>(base);   // the same groups in theta, v, m (tiled; ga_internal.h)
    f32x4 th[U], vv[U], mm[U], ss[U], gg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock, qs = base_s + (uint64_t)u * kBlock;
        mm[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        ss[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (q < n4) {
            th[u] = load4<NT_TH>(theta, qs);
            vv[u] = load4<NT_V>(v, qs);
            if constexpr (KEEP_M) mm[u] = load4<NT_M>(m, qs);
            if constexpr (GAP) ss[u] = load4<true>(snap, q);
            gg[u] = load_g4<DT, ALIGNED>(g, q);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock, qs = base_s + (uint64_t)u * kBlock;
        if (q < n4) {
            update4<MODE, KEEP_M>(th[u], vv[u], mm[u], ss[u], gg[u], c);
            store4<NT_TH>(theta, qs, th[u]);
            store4<NT_V>(v, qs, vv[u]);
            if constexpr (KEEP_M) store4<NT_M>(m, qs, mm[u]);
            if constexpr (SNAP) store4<true>(snap, q, th[u]);
        }
    }
}

template <int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED, int U>
__global__ __launch_bounds__(kBlock) void apply_kernel(float* __restrict__ theta, float* __restrict__ v,
                                                       float* __restrict__ m, float* __restrict__ snap,
                                                       const void* __restrict__ g, uint64_t N, StepConst c,
                                                       Residency keep) {
    constexpr bool GAP = is_gap(MODE);
    const uint64_t n4 = N >> 2;
    const uint32_t b = blockIdx.x;
    const uint64_t base = (uint64_t)b * (kBlock * U) + threadIdx.x;
#define GA_APPLY_TILE(NT_TH, NT_V, NT_M) \
    apply_tile<MODE, DT, KEEP_M, SNAP, ALIGNED, U, NT_TH, NT_V, NT_M>(theta, v, m, snap, g, n4, base, c)
    if (b >= keep.theta) GA_HINT_PATH("all streamed", GA_APPLY_TILE(true, true, true));
    else if (b >= keep.v) GA_HINT_PATH("theta kept", GA_APPLY_TILE(false, true, true));
    else if (!KEEP_M || b >= keep.m) GA_HINT_PATH("theta and v kept", GA_APPLY_TILE(false, false, true));
    else GA_HINT_PATH("theta, v and m kept", GA_APPLY_TILE(false, false, false));
#undef GA_APPLY_TILE

    // ragged tail: the last N % 4 parameters, one per thread of block 0
    if (b == 0 && threadIdx.x < (N & 3)) {
        const uint64_t j = 4 * n4 + threadIdx.x, js = state_index<1>(j);
        float t1 = theta[js], v1 = v[js], m1 = 0.0f, s1 = 0.0f;
        if constexpr (KEEP_M) m1 = m[js];
        if constexpr (GAP) s1 = snap[j];
        update_one<MODE, KEEP_M>(t1, v1, m1, s1, load_g1<DT>(g, j), c);
        theta[js] = t1;
        v[js] = v1;
        if constexpr (KEEP_M) m[js] = m1;
        if constexpr (SNAP) snap[j] = t1;
    }
}

// ---------------------------------------------------------------------------
// Fused update of one arrival for the DANA and ADAM families: the same launch
// shape as apply_kernel with one more state array.  x: vsum | m1 (touched at
// every arrival); y: the arriving worker's v_i (always streamed) | v2.  The
// leading blocks keep theta, then x, in the memory-side cache.
// ---------------------------------------------------------------------------
template <int FAMILY, int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED, int U, bool NT_TH, bool NT_X>
__device__ __forceinline__ void family_tile(float* __restrict__ theta, float* __restrict__ x, float* __restrict__ y,
                                            float* __restrict__ m, float* __restrict__ snap,
                                            const void* __restrict__ g, uint64_t n4, uint64_t base,
                                            const StepConst& c) {
    constexpr bool GAP = is_gap(MODE);
    static_assert((kStateTile / 4) % (kBlock * U) == 0, "a block's groups lie in one tile of the state arrays");
    // the same groups in theta, x, m (tiled, ga_internal.h); Adam's y = v2 is the fourth tiled array, DANA's y = v_i
    // and the snapshot are rows
    constexpr int ROWS = state_rows(FAMILY), SROWS = snapshot_rows(FAMILY);
    constexpr bool ADAM = (FAMILY == GA_FAMILY_ADAM);
    const uint64_t base_s = state_index<4, ROWS>(base);
    const uint64_t base_r = row_index<4, SROWS>(base);   // the same groups in the worker's snapshot (DANA: and in its v_i)
    f32x4 th[U], xx[U], yy[U], mm[U], ss[U], gg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock, qs = base_s + (uint64_t)u * kBlock, qr = base_r + (uint64_t)u * kBlock;
        mm[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        ss[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (q < n4) {
            th[u] = load4<NT_TH>(theta, qs);
            xx[u] = load4<NT_X>(x, qs);
            yy[u] = load4<true>(y, ADAM ? qs : qr);
            if constexpr (KEEP_M) mm[u] = load4<true>(m, qs);
            if constexpr (GAP) ss[u] = load4<true>(snap, qr);
            gg[u] = load_g4<DT, ALIGNED>(g, q);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock, qs = base_s + (uint64_t)u * kBlock, qr = base_r + (uint64_t)u * kBlock;
        if (q < n4) {
            f32x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float t1 = th[u][e], x1 = xx[u][e], y1 = yy[u][e], m1 = mm[u][e];
                if constexpr (FAMILY == GA_FAMILY_DANA) out[e] = dana_one<MODE, KEEP_M>(t1, x1, y1, m1, ss[u][e], gg[u][e], c);
                else out[e] = adam_one<MODE, KEEP_M>(t1, x1, y1, m1, ss[u][e], gg[u][e], c);
                th[u][e] = t1; xx[u][e] = x1; yy[u][e] = y1; mm[u][e] = m1;
            }
            store4<NT_TH>(theta, qs, th[u]);
            store4<NT_X>(x, qs, xx[u]);
            store4<true>(y, ADAM ? qs : qr, yy[u]);
            if constexpr (KEEP_M) store4<true>(m, qs, mm[u]);
            if constexpr (SNAP) store4<true>(snap, qr, out);
        }
    }
}

template <int FAMILY, int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED, int U>
__global__ __launch_bounds__(kBlock) void family_apply_kernel(float* __restrict__ theta, float* __restrict__ x,
                                                              float* __restrict__ y, float* __restrict__ m,
                                                              float* __restrict__ snap,
                                                              const void* __restrict__ g, uint64_t N, StepConst c,
                                                              Residency keep) {
    constexpr bool GAP = is_gap(MODE);
    const uint64_t n4 = N >> 2;
    const uint32_t b = blockIdx.x;
    const uint64_t base = (uint64_t)b * (kBlock * U) + threadIdx.x;
#define GA_FAMILY_TILE(NT_TH, NT_X) \
    family_tile<FAMILY, MODE, DT, KEEP_M, SNAP, ALIGNED, U, NT_TH, NT_X>(theta, x, y, m, snap, g, n4, base, c)
    if (b >= keep.theta) GA_HINT_PATH("all streamed", GA_FAMILY_TILE(true, true));
    else if (b >= keep.v) GA_HINT_PATH("theta kept", GA_FAMILY_TILE(false, true));
    else GA_HINT_PATH("theta and x kept", GA_FAMILY_TILE(false, false));
#undef GA_FAMILY_TILE

    if (b == 0 && threadIdx.x < (N & 3)) {
        const uint64_t j = 4 * n4 + threadIdx.x, js = state_index<1, state_rows(FAMILY)>(j);
        const uint64_t jr = row_index<1, snapshot_rows(FAMILY)>(j);
        const uint64_t jy = (FAMILY == GA_FAMILY_ADAM) ? js : jr;
        float t1 = theta[js], x1 = x[js], y1 = y[jy], m1 = 0.0f, s1 = 0.0f, out;
        if constexpr (KEEP_M) m1 = m[js];
        if constexpr (GAP) s1 = snap[jr];
        if constexpr (FAMILY == GA_FAMILY_DANA) out = dana_one<MODE, KEEP_M>(t1, x1, y1, m1, s1, load_g1<DT>(g, j), c);
        else out = adam_one<MODE, KEEP_M>(t1, x1, y1, m1, s1, load_g1<DT>(g, j), c);
        theta[js] = t1;
        x[js] = x1;
        y[jy] = y1;
        if constexpr (KEEP_M) m[js] = m1;
        if constexpr (SNAP) snap[jr] = out;
    }
}

// ---------------------------------------------------------------------------
// Dispatch of the apply kernel over (mode, dtype, keep_m, aligned).
// ---------------------------------------------------------------------------
// One group of four per thread (U = 1).  With separate state arrays two groups per thread were 1 - 2 % faster up to
// 10^8 parameters; with the tiled state arrays one group is faster at every size (cfg3 129.0 against 130.4 us,
// 100 M 527 against 545 us, 128 M 689 against 715 us).
constexpr int kApplyU = 1;

template <int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED, int U>
hipError_t launch_apply_u(const StatePtrs& st, float* snap, const void* g, uint64_t N, const StepConst& c,
                          hipStream_t stream) {
    const uint64_t n4 = N >> 2;
    const uint64_t per_block = (uint64_t)kBlock * U;
    const uint64_t blocks = (n4 + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid(blocks == 0 ? 1u : (uint32_t)blocks), block(kBlock);
    const Residency keep = residency_for(st.resident_bytes, grid.x, per_block * sizeof(f32x4), true, KEEP_M);
    hipLaunchKernelGGL((apply_kernel<MODE, DT, KEEP_M, SNAP, ALIGNED, U>), grid, block, 0, stream, st.theta, st.v,
                       st.m, snap, g, N, c, keep);
    return hipGetLastError();
}

template <int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED>
hipError_t launch_apply_t(const StatePtrs& st, float* snap, const void* g, uint64_t N, const StepConst& c,
                          hipStream_t stream) {
    return launch_apply_u<MODE, DT, KEEP_M, SNAP, ALIGNED, kApplyU>(st, snap, g, N, c, stream);
}

template <int MODE, bool KEEP_M, bool SNAP>
hipError_t launch_apply_m(const StatePtrs& st, float* snap, const void* g, int dt, uint64_t N, const StepConst& c,
                          hipStream_t stream) {
    const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
    if (dt == GA_F32) {
        if ((addr & 15u) == 0) return launch_apply_t<MODE, GA_F32, KEEP_M, SNAP, true>(st, snap, g, N, c, stream);
        return launch_apply_t<MODE, GA_F32, KEEP_M, SNAP, false>(st, snap, g, N, c, stream);
    }
    if ((addr & 7u) == 0) return launch_apply_t<MODE, GA_BF16, KEEP_M, SNAP, true>(st, snap, g, N, c, stream);
    return launch_apply_t<MODE, GA_BF16, KEEP_M, SNAP, false>(st, snap, g, N, c, stream);
}

// non-GA modes: m and the snapshot are optional
template <int MODE>
hipError_t launch_apply_opt(const StatePtrs& st, float* snap, const void* g, int dt, uint64_t N, const StepConst& c,
                            bool keep_m, bool write_snap, hipStream_t stream) {
    if (keep_m) {
        return write_snap ? launch_apply_m<MODE, true, true>(st, snap, g, dt, N, c, stream)
                          : launch_apply_m<MODE, true, false>(st, snap, g, dt, N, c, stream);
    }
    return write_snap ? launch_apply_m<MODE, false, true>(st, snap, g, dt, N, c, stream)
                      : launch_apply_m<MODE, false, false>(st, snap, g, dt, N, c, stream);
}

// ---------------------------------------------------------------------------
// Dispatch of the DANA / ADAM kernel.
// ---------------------------------------------------------------------------
constexpr int kFamilyU = 1;

template <int FAMILY, int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED>
hipError_t launch_family_t(float* theta, float* x, float* y, float* m, float* snap, const void* g, uint64_t N,
                           const StepConst& c, uint64_t resident_bytes, hipStream_t stream) {
    const uint64_t n4 = N >> 2;
    const uint64_t per_block = (uint64_t)kBlock * kFamilyU;
    const uint64_t blocks = (n4 + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid(blocks == 0 ? 1u : (uint32_t)blocks), block(kBlock);
    const Residency keep = residency_for(resident_bytes, grid.x, per_block * sizeof(f32x4), true, false);
    hipLaunchKernelGGL((family_apply_kernel<FAMILY, MODE, DT, KEEP_M, SNAP, ALIGNED, kFamilyU>), grid, block, 0,
                       stream, theta, x, y, m, snap, g, N, c, keep);
    return hipGetLastError();
}

template <int FAMILY, int MODE, bool KEEP_M, bool SNAP>
hipError_t launch_family_m(float* theta, float* x, float* y, float* m, float* snap, const void* g, int dt,
                           uint64_t N, const StepConst& c, uint64_t resident_bytes, hipStream_t stream) {
    const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
    if (dt == GA_F32) {
        if ((addr & 15u) == 0)
            return launch_family_t<FAMILY, MODE, GA_F32, KEEP_M, SNAP, true>(theta, x, y, m, snap, g, N, c, resident_bytes, stream);
        return launch_family_t<FAMILY, MODE, GA_F32, KEEP_M, SNAP, false>(theta, x, y, m, snap, g, N, c, resident_bytes, stream);
    }
    if ((addr & 7u) == 0)
        return launch_family_t<FAMILY, MODE, GA_BF16, KEEP_M, SNAP, true>(theta, x, y, m, snap, g, N, c, resident_bytes, stream);
    return launch_family_t<FAMILY, MODE, GA_BF16, KEEP_M, SNAP, false>(theta, x, y, m, snap, g, N, c, resident_bytes, stream);
}

template <int FAMILY>
hipError_t launch_family(float* theta, float* x, float* y, float* m, float* snap, const void* g, int dt, uint64_t N,
                         int mode, bool keep_m, bool write_snap, const StepConst& c, uint64_t resident_bytes,
                         hipStream_t stream) {
#define GA_FAM(MODE, KEEP, SNAP) \
    launch_family_m<FAMILY, MODE, KEEP, SNAP>(theta, x, y, m, snap, g, dt, N, c, resident_bytes, stream)
    switch (mode) {
        case GA_MODE_GA: return GA_FAM(GA_MODE_GA, true, true);
        case GA_MODE_GA_HINGE: return GA_FAM(GA_MODE_GA_HINGE, true, true);
        case GA_MODE_SA:
            if (keep_m) return write_snap ? GA_FAM(GA_MODE_SA, true, true) : GA_FAM(GA_MODE_SA, true, false);
            return write_snap ? GA_FAM(GA_MODE_SA, false, true) : GA_FAM(GA_MODE_SA, false, false);
        case GA_MODE_ASGD:
            if (keep_m) return write_snap ? GA_FAM(GA_MODE_ASGD, true, true) : GA_FAM(GA_MODE_ASGD, true, false);
            return write_snap ? GA_FAM(GA_MODE_ASGD, false, true) : GA_FAM(GA_MODE_ASGD, false, false);
        default: return hipErrorInvalidValue;
    }
#undef GA_FAM
}

}  // namespace

hipError_t launch_apply_dana(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype, int mode,
                             bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream) {
    return launch_family<GA_FAMILY_DANA>(st.theta, st.v, st.worker_v + (uint64_t)worker * st.stride, st.m,
                                         st.snaps + (uint64_t)worker * st.stride, g, grad_dtype, N, mode, keep_m,
                                         write_snap, c, st.resident_bytes, stream);
}

hipError_t launch_apply_adam(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype, int mode,
                             bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream) {
    return launch_family<GA_FAMILY_ADAM>(st.theta, st.v, st.v2, st.m, st.snaps + (uint64_t)worker * st.stride, g,
                                         grad_dtype, N, mode, keep_m, write_snap, c, st.resident_bytes, stream);
}

hipError_t launch_apply(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype, int mode,
                        bool nesterov, bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream) {
    float* snap = st.snaps + (uint64_t)worker * st.stride;
    if (mode == GA_MODE_SA_STEP) mode = GA_MODE_ASGD;   // the step-size penalty is already folded into c.lr
    switch (mode | (nesterov ? kNesterov : 0)) {
        case GA_MODE_GA:
            return launch_apply_m<GA_MODE_GA, true, true>(st, snap, g, grad_dtype, N, c, stream);
        case GA_MODE_GA_HINGE:
            return launch_apply_m<GA_MODE_GA_HINGE, true, true>(st, snap, g, grad_dtype, N, c, stream);
        case GA_MODE_SA:
            return launch_apply_opt<GA_MODE_SA>(st, snap, g, grad_dtype, N, c, keep_m, write_snap, stream);
        case GA_MODE_ASGD:
            return launch_apply_opt<GA_MODE_ASGD>(st, snap, g, grad_dtype, N, c, keep_m, write_snap, stream);
        case GA_MODE_GA | kNesterov:
            return launch_apply_m<GA_MODE_GA | kNesterov, true, true>(st, snap, g, grad_dtype, N, c, stream);
        case GA_MODE_GA_HINGE | kNesterov:
            return launch_apply_m<GA_MODE_GA_HINGE | kNesterov, true, true>(st, snap, g, grad_dtype, N, c, stream);
        case GA_MODE_SA | kNesterov:
            return launch_apply_opt<GA_MODE_SA | kNesterov>(st, snap, g, grad_dtype, N, c, keep_m, write_snap, stream);
        case GA_MODE_ASGD | kNesterov:
            return launch_apply_opt<GA_MODE_ASGD | kNesterov>(st, snap, g, grad_dtype, N, c, keep_m, write_snap, stream);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace ga
