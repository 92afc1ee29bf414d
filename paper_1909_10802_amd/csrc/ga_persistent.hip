// libga, gfx950: persistent multi-arrival kernel with in-kernel quadratic-plus-noise gradients.

#include "ga_device.h"

namespace ga {
namespace {

// below this many parameters the persistent kernel gives each thread 2 instead of 4 of them
#ifndef GA_PERSIST_WIDE_MIN_N
#define GA_PERSIST_WIDE_MIN_N (1ull << 21)
#endif
constexpr uint64_t kPersistWideMinN = GA_PERSIST_WIDE_MIN_N;

// ---------------------------------------------------------------------------
// Persistent multi-arrival kernel.  Thread = one group of four parameters.
// theta, v, m, a, theta* stay in registers for the whole chunk; per arrival
// the thread reads and rewrites only its 16 bytes of the arriving worker's
// snapshot (DANA: and of that worker's momentum; Adam keeps m1 and v2 in
// registers too).  No thread ever needs another thread's data, so there is no
// grid-wide or block-wide synchronisation.  The snapshot of the next arrival
// is requested before the arithmetic of the current one.
// ---------------------------------------------------------------------------
template <int FAMILY, int MODE, bool KEEP_M, int E>
__global__ __launch_bounds__(kBlock) void persistent_kernel(float* __restrict__ theta, float* __restrict__ x,
                                                            float* __restrict__ m, float* snaps, float* worker_v,
                                                            float* __restrict__ v2, uint64_t stride,
                                                            const float* __restrict__ a,
                                                            const float* __restrict__ ts,
                                                            const ga_arrival* __restrict__ table,
                                                            const AdamRow* __restrict__ adam_table, uint32_t T,
                                                            uint64_t k0, uint64_t N, RunConst rc) {
    constexpr bool DANA = (FAMILY == GA_FAMILY_DANA);
    constexpr bool ADAM = (FAMILY == GA_FAMILY_ADAM);
    const uint64_t p = (uint64_t)blockIdx.x * kBlock + threadIdx.x;   // pack index
    const uint64_t j0 = (uint64_t)E * p;
    if (j0 >= N || T == 0) return;
    const uint32_t n_valid = (N - j0 >= (uint64_t)E) ? (uint32_t)E : (uint32_t)(N - j0);

    // state arrays are padded to a multiple of 64 floats: the vector access is always in bounds
    Pack<E> th = pack_load<E>(theta, p);
    Pack<E> xx = pack_load<E>(x, p);                           // v | sum_j v_j | m1
    Pack<E> mm = pack_zero<E>();
    if constexpr (KEEP_M) mm = pack_load<E>(m, p);
    Pack<E> yy = pack_zero<E>();                               // ADAM: v2 (registers); DANA: v_i of the arriving worker
    if constexpr (ADAM) yy = pack_load<E>(v2, p);
    Pack<E> a4 = pack_zero<E>(), t4 = pack_zero<E>();
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

    StepConst c = {};
    c.gamma = rc.gamma; c.eta_max = rc.eta_max; c.eps = rc.eps; c.beta = rc.beta;
    c.one_minus_beta = rc.one_minus_beta;
    c.beta1 = rc.beta1; c.omb1 = rc.omb1; c.beta2 = rc.beta2; c.omb2 = rc.omb2; c.adam_eps = rc.adam_eps;

    ga_arrival row = table[0];
    Pack<E> s = pack_load<E>(snaps + (uint64_t)row.worker * stride, p);   // this thread's column of the snapshots
    if constexpr (DANA) yy = pack_load<E>(worker_v + (uint64_t)row.worker * stride, p);

    for (uint32_t t = 0; t < T; ++t) {
        const bool more = (t + 1 < T);
        ga_arrival next = row;
        Pack<E> s_next = s, y_next = yy;
        if (more) {
            next = table[t + 1];
            s_next = pack_load<E>(snaps + (uint64_t)next.worker * stride, p);
            if constexpr (DANA) y_next = pack_load<E>(worker_v + (uint64_t)next.worker * stride, p);
        }
        const uint64_t k = k0 + t + 1;
        c.lr = row.lr; c.tau = row.tau; c.inv_bc_prev = row.inv_bc_prev;
        if constexpr (DANA) c.eta_gamma = row.lr * rc.gamma;
        if constexpr (ADAM) {
            const AdamRow ar = adam_table[t];
            c.inv_bc1 = ar.inv_bc1;
            c.inv_bc2 = ar.inv_bc2;
        }
        const Pack<E> z = noise_pack<E>(rc.seed_lo, rc.seed_hi, j0, k);

        Pack<E> out = s;                                     // what the worker is sent; padding lanes unchanged
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if ((uint32_t)e < n_valid) {
                const float g = quadratic_g(s.x[e], a4.x[e], t4.x[e], rc.sigma, z.x[e]);
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

        pack_store<E>(snaps + (uint64_t)row.worker * stride, p, out);
        if constexpr (DANA) pack_store<E>(worker_v + (uint64_t)row.worker * stride, p, yy);
        // same worker twice in a row: its rows are what was just written
        const bool same = (next.worker == row.worker);
        s = same ? out : s_next;
        if constexpr (DANA) yy = same ? yy : y_next;
        row = next;
    }

    pack_store<E>(theta, p, th);
    pack_store<E>(x, p, xx);
    if constexpr (KEEP_M) pack_store<E>(m, p, mm);
    if constexpr (ADAM) pack_store<E>(v2, p, yy);
}

}  // namespace

hipError_t launch_persistent(const StatePtrs& st, uint64_t N, int family, const ga_arrival* dev_table,
                             const AdamRow* dev_adam_table, uint32_t T, uint64_t k0, const float* a,
                             const float* theta_star, int mode, bool nesterov, bool keep_m, const RunConst& rc,
                             hipStream_t stream) {
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
            hipLaunchKernelGGL((persistent_kernel<FAM, MODE, KEEP, 4>), grid, block, 0, stream, st.theta, st.v,     \
                               st.m, st.snaps, st.worker_v, st.v2, st.stride, a, theta_star, dev_table,             \
                               dev_adam_table, T, k0, N, rc);                                                       \
        else                                                                                                        \
            hipLaunchKernelGGL((persistent_kernel<FAM, MODE, KEEP, 2>), grid, block, 0, stream, st.theta, st.v,     \
                               st.m, st.snaps, st.worker_v, st.v2, st.stride, a, theta_star, dev_table,             \
                               dev_adam_table, T, k0, N, rc);                                                       \
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

}  // namespace ga
