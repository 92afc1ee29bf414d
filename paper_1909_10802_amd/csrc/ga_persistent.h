// libga, gfx950: the persistent multi-arrival kernel and its dispatch, shared by the translation
// units that instantiate it for the in-kernel quadratic-plus-noise gradients and for gradient buffers.
#ifndef GA_PERSISTENT_H
#define GA_PERSISTENT_H

#include "ga_device.h"

namespace ga {
namespace {

// where the persistent kernel takes the gradient of an arrival from
constexpr int kSrcQuadratic = 0;   // computed from the arriving worker's snapshot, noise generated in the kernel
constexpr int kSrcF32 = 1;         // read from the float buffer named by the arrival's row of the pointer table
constexpr int kSrcBf16 = 2;        // the same with bfloat16 buffers

// below this many parameters the persistent kernel gives each thread 2 instead of 4 of them
constexpr uint64_t kPersistWideMinN = (uint64_t)1 << 21;

// Gradients j0 .. j0+E-1 of one buffer (N values, base aligned to E values); a pack that reaches
// past N is read element by element.
template <int E, int SRC>
__device__ __forceinline__ Pack<E> grad_pack(const void* __restrict__ g, uint64_t p, uint32_t n_valid) {
    Pack<E> r = pack_zero<E>();
    if constexpr (SRC == kSrcF32) {
        const float* base = static_cast<const float*>(g);
        if (n_valid == (uint32_t)E) {
            if constexpr (E == 4) {
                const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(base) + p);
                r.x[0] = t.x; r.x[1] = t.y; r.x[2] = t.z; r.x[3] = t.w;
            } else {
                const f32x2 t = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(base) + p);
                r.x[0] = t.x; r.x[1] = t.y;
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e)
                if ((uint32_t)e < n_valid) r.x[e] = base[(uint64_t)E * p + e];
        }
    } else if constexpr (SRC == kSrcBf16) {
        const uint16_t* base = static_cast<const uint16_t*>(g);
        if (n_valid == (uint32_t)E) {
            if constexpr (E == 4) {
                const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(base) + p);
                r.x[0] = bf16_bits_to_float(w.x & 0xFFFFu); r.x[1] = bf16_bits_to_float(w.x >> 16);
                r.x[2] = bf16_bits_to_float(w.y & 0xFFFFu); r.x[3] = bf16_bits_to_float(w.y >> 16);
            } else {
                const uint32_t w = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(base) + p);
                r.x[0] = bf16_bits_to_float(w & 0xFFFFu); r.x[1] = bf16_bits_to_float(w >> 16);
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e)
                if ((uint32_t)e < n_valid) r.x[e] = bf16_bits_to_float(base[(uint64_t)E * p + e]);
        }
    }
    return r;
}

// ---------------------------------------------------------------------------
// Persistent multi-arrival kernel.  Thread = one group of E parameters.
// theta, v, m (and a, theta* of the quadratic source) stay in registers for the
// whole chunk; per arrival the thread reads and rewrites only its part of the
// arriving worker's snapshot (DANA: and of that worker's momentum; Adam keeps
// m1 and v2 in registers too) and, with gradient buffers, reads its part of
// the arrival's buffer.  No thread ever needs another thread's data, so there
// is no grid-wide or block-wide synchronisation.  The rows of the next arrival
// are requested before the arithmetic of the current one.
//
// Gradient buffers without Gap tracking (KEEP_M false: ASGD / SA penalties) do
// not touch the snapshots at all, as in the per-arrival kernel.
// ---------------------------------------------------------------------------
template <int FAMILY, int MODE, bool KEEP_M, int E, int SRC>
__global__ __launch_bounds__(kBlock) void persistent_kernel(float* __restrict__ theta, float* __restrict__ x,
                                                            float* __restrict__ m, float* snaps, float* worker_v,
                                                            float* __restrict__ v2, uint64_t stride,
                                                            const float* __restrict__ a,
                                                            const float* __restrict__ ts,
                                                            const void* const* __restrict__ grads,
                                                            const ga_arrival* __restrict__ table,
                                                            const AdamRow* __restrict__ adam_table, uint32_t T,
                                                            uint64_t k0, uint64_t N, RunConst rc) {
    constexpr bool DANA = (FAMILY == GA_FAMILY_DANA);
    constexpr bool ADAM = (FAMILY == GA_FAMILY_ADAM);
    constexpr bool QUAD = (SRC == kSrcQuadratic);
    constexpr bool SNAP = QUAD || KEEP_M;                      // the snapshot rows are read and rewritten
    const uint64_t p = (uint64_t)blockIdx.x * kBlock + threadIdx.x;   // pack index
    const uint64_t j0 = (uint64_t)E * p;
    if (j0 >= N || T == 0) return;
    const uint32_t n_valid = (N - j0 >= (uint64_t)E) ? (uint32_t)E : (uint32_t)(N - j0);

    // every array is padded so that the vector access is always in bounds; theta, x and m are tiled (ga_internal.h)
    const uint64_t ps = state_index<E, state_rows(FAMILY)>(p);
    const uint64_t pr = row_index<E, snapshot_rows(FAMILY)>(p);   // this pack in a worker's snapshot (DANA: and in its v_i)
    Pack<E> th = pack_load<E>(theta, ps);
    Pack<E> xx = pack_load<E>(x, ps);                          // v | sum_j v_j | m1
    Pack<E> mm = pack_zero<E>();
    if constexpr (KEEP_M) mm = pack_load<E>(m, ps);
    Pack<E> yy = pack_zero<E>();                               // ADAM: v2 (registers); DANA: v_i of the arriving worker
    if constexpr (ADAM) yy = pack_load<E>(v2, ps);           // the fourth tiled array
    Pack<E> a4 = pack_zero<E>(), t4 = pack_zero<E>();
    if constexpr (QUAD) {
        if (n_valid == (uint32_t)E) {
            a4 = pack_load<E>(a, p);
            t4 = pack_load<E>(ts, p);
        } else {   // caller arrays hold exactly N floats
#pragma unroll
            for (int e = 0; e < E; ++e) {
                if ((uint32_t)e < n_valid) {
                    a4.x[e] = a[j0 + e];
                    t4.x[e] = ts[j0 + e];
                }
            }
        }
    }

    StepConst c = {};
    c.gamma = rc.gamma; c.eta_max = rc.eta_max; c.eps = rc.eps; c.beta = rc.beta;
    c.one_minus_beta = rc.one_minus_beta;
    c.beta1 = rc.beta1; c.omb1 = rc.omb1; c.beta2 = rc.beta2; c.omb2 = rc.omb2; c.adam_eps = rc.adam_eps;

    ga_arrival row = table[0];
    Pack<E> s = pack_zero<E>();                                // this thread's part of the arriving worker's snapshot
    if constexpr (SNAP) s = pack_load<E>(snaps + (uint64_t)row.worker * stride, pr);
    if constexpr (DANA) yy = pack_load<E>(worker_v + (uint64_t)row.worker * stride, pr);
    Pack<E> gb = pack_zero<E>();
    if constexpr (!QUAD) gb = grad_pack<E, SRC>(grads[0], p, n_valid);

    for (uint32_t t = 0; t < T; ++t) {
        const bool more = (t + 1 < T);
        ga_arrival next = row;
        Pack<E> s_next = s, y_next = yy, g_next = gb;
        if (more) {
            next = table[t + 1];
            if constexpr (SNAP) s_next = pack_load<E>(snaps + (uint64_t)next.worker * stride, pr);
            if constexpr (DANA) y_next = pack_load<E>(worker_v + (uint64_t)next.worker * stride, pr);
            if constexpr (!QUAD) g_next = grad_pack<E, SRC>(grads[t + 1], p, n_valid);
        }
        const uint64_t k = k0 + t + 1;
        c.lr = row.lr; c.tau = row.tau; c.inv_bc_prev = row.inv_bc_prev;
        if constexpr (DANA) c.eta_gamma = row.lr * rc.gamma;
        if constexpr (ADAM) {
            const AdamRow ar = adam_table[t];
            c.inv_bc1 = ar.inv_bc1;
            c.inv_bc2 = ar.inv_bc2;
        }
        Pack<E> z = pack_zero<E>();
        if constexpr (QUAD) z = noise_pack<E>(rc.seed_lo, rc.seed_hi, j0, k);

        Pack<E> out = s;                                     // what the worker is sent; padding lanes unchanged
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if ((uint32_t)e < n_valid) {
                float g;
                if constexpr (QUAD) g = quadratic_g(s.x[e], a4.x[e], t4.x[e], rc.sigma, z.x[e]);
                else g = gb.x[e];
                float t1 = th.x[e], x1 = xx.x[e], y1 = yy.x[e], m1 = mm.x[e];
                if constexpr (DANA) {
                    out.x[e] = dana_one<MODE, KEEP_M>(t1, x1, y1, m1, s.x[e], g, c);
                } else if constexpr (ADAM) {
                    out.x[e] = adam_one<MODE, KEEP_M>(t1, x1, y1, m1, s.x[e], g, c);
                } else {
                    update_one<MODE, KEEP_M>(t1, x1, m1, s.x[e], g, c);
                    out.x[e] = t1;
                }
                th.x[e] = t1; xx.x[e] = x1; yy.x[e] = y1; mm.x[e] = m1;
            }
        }

        if constexpr (SNAP) pack_store<E>(snaps + (uint64_t)row.worker * stride, pr, out);
        if constexpr (DANA) pack_store<E>(worker_v + (uint64_t)row.worker * stride, pr, yy);
        // same worker twice in a row: its rows are what was just written
        const bool same = (next.worker == row.worker);
#pragma unroll
        for (int e = 0; e < E; ++e) {                        // element by element: the packs stay in registers
            s.x[e] = same ? out.x[e] : s_next.x[e];
            if constexpr (DANA) yy.x[e] = same ? yy.x[e] : y_next.x[e];
        }
        gb = g_next;
        row = next;
    }

    pack_store<E>(theta, ps, th);
    pack_store<E>(x, ps, xx);
    if constexpr (KEEP_M) pack_store<E>(m, ps, mm);
    if constexpr (ADAM) pack_store<E>(v2, ps, yy);
}

// Picks the instantiation for the family, penalty and vector length and launches it.
template <int SRC>
hipError_t launch_persistent_from(const StatePtrs& st, uint64_t N, int family, const ga_arrival* dev_table,
                                  const AdamRow* dev_adam_table, uint32_t T, uint64_t k0, const float* a,
                                  const float* theta_star, const void* const* dev_grads, int mode, bool nesterov,
                                  bool keep_m, const RunConst& rc, hipStream_t stream) {
    // Four parameters per thread share one Philox block; short vectors use two per thread (the block is
    // then computed twice) so that every SIMD still has several wavefronts to switch between.
    const int ept = (N >= kPersistWideMinN) ? 4 : 2;
    const uint64_t packs = (N + ept - 1) / ept;
    const uint64_t blocks = (packs + kBlock - 1) / kBlock;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)blocks), block(kBlock);
#define GA_LAUNCH_PERSIST(FAM, MODE, KEEP)                                                                          \
    do {                                                                                                            \
        if (ept == 4)                                                                                               \
            hipLaunchKernelGGL((persistent_kernel<FAM, MODE, KEEP, 4, SRC>), grid, block, 0, stream, st.theta,      \
                               st.v, st.m, st.snaps, st.worker_v, st.v2, st.stride, a, theta_star, dev_grads,       \
                               dev_table, dev_adam_table, T, k0, N, rc);                                            \
        else                                                                                                        \
            hipLaunchKernelGGL((persistent_kernel<FAM, MODE, KEEP, 2, SRC>), grid, block, 0, stream, st.theta,      \
                               st.v, st.m, st.snaps, st.worker_v, st.v2, st.stride, a, theta_star, dev_grads,       \
                               dev_table, dev_adam_table, T, k0, N, rc);                                            \
    } while (0)
#define GA_PERSIST_MODES(FAM, NAG)                                                                                  \
    switch (mode) {                                                                                                 \
        case GA_MODE_GA: GA_LAUNCH_PERSIST(FAM, GA_MODE_GA | NAG, true); break;                                     \
        case GA_MODE_GA_HINGE: GA_LAUNCH_PERSIST(FAM, GA_MODE_GA_HINGE | NAG, true); break;                         \
        case GA_MODE_SA:                                                                                            \
            if (keep_m) GA_LAUNCH_PERSIST(FAM, GA_MODE_SA | NAG, true);                                             \
            else GA_LAUNCH_PERSIST(FAM, GA_MODE_SA | NAG, false);                                                   \
            break;                                                                                                  \
        case GA_MODE_ASGD:                                                                                          \
        case GA_MODE_SA_STEP:                                                                                       \
            if (keep_m) GA_LAUNCH_PERSIST(FAM, GA_MODE_ASGD | NAG, true);                                           \
            else GA_LAUNCH_PERSIST(FAM, GA_MODE_ASGD | NAG, false);                                                 \
            break;                                                                                                  \
        default: return hipErrorInvalidValue;                                                                       \
    }
    if (family == GA_FAMILY_DANA) { GA_PERSIST_MODES(GA_FAMILY_DANA, 0) }
    else if (family == GA_FAMILY_ADAM) { GA_PERSIST_MODES(GA_FAMILY_ADAM, 0) }
    else if (nesterov) { GA_PERSIST_MODES(GA_FAMILY_MOMENTUM, kNesterov) }
    else { GA_PERSIST_MODES(GA_FAMILY_MOMENTUM, 0) }
#undef GA_PERSIST_MODES
#undef GA_LAUNCH_PERSIST
    return hipGetLastError();
}

}  // namespace
}  // namespace ga

#endif
