// Device-side building blocks shared by the gfx950 kernels of libga: vector accesses with cache
// hints, the per-parameter arithmetic of the three master families, and the counter-based noise
// generator.  Included by every .hip file of the library; everything here is inline device code
// (or constexpr) in an unnamed namespace.
//
// Floating point: every operation is a separately rounded IEEE float operation in the order
// given in include/ga.h.  The including file must be compiled with -ffp-contract=off; '/' and
// sqrtf are correctly rounded (hipcc default).
#ifndef GA_DEVICE_H
#define GA_DEVICE_H

#include <hip/hip_runtime.h>

#include "ga_internal.h"

#pragma clang fp contract(off)

namespace ga {
namespace {

constexpr int kBlock = 256;

// native 128-bit / 64-bit vectors (one dwordx4 / dwordx2 access each)
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// 128-bit accesses with or without the non-temporal hint.  The MI355X has a
// 256 MB memory-side cache in front of HBM: arrays that are touched once per
// arrival (gradient, the arriving worker's snapshot) are streamed around it so
// that a leading part of the arrays touched at every arrival (theta, then v, then m) stays in it (Residency below).
template <bool NT>
__device__ __forceinline__ f32x4 load4(const float* __restrict__ base, uint64_t q) {
    const f32x4* p = reinterpret_cast<const f32x4*>(base) + q;
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void store4(float* __restrict__ base, uint64_t q, const f32x4& x) {
    f32x4* p = reinterpret_cast<f32x4*>(base) + q;
    if constexpr (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}

// ---------------------------------------------------------------------------
// One parameter, one arrival.
// ---------------------------------------------------------------------------
// Template parameter MODE: the ga_mode in the low four bits, bit 4 selects the Nesterov form of
// the momentum master.
constexpr int kNesterov = 16;
constexpr int penalty_mode(int mode) { return mode & 15; }
constexpr bool is_nesterov(int mode) { return (mode & kNesterov) != 0; }
constexpr bool is_gap(int mode) { return penalty_mode(mode) == GA_MODE_GA || penalty_mode(mode) == GA_MODE_GA_HINGE; }

// The factor the gradient is divided by: the Gap G (Eq. 5, with C from the Alg. 14 state
// as arrival k-1 left it), the delay (Alg. 5 / 7 / 10), or 1.
template <int MODE>
__device__ __forceinline__ float penalty_of(float th, float s, float cstate, const StepConst& c) {
    if constexpr (is_gap(MODE)) {
        const float diff = th - s;
        const float delta = fabsf(diff);
        const float mhat = cstate * c.inv_bc_prev;
        const float root = sqrtf(mhat);
        const float sum = root + c.eps;
        const float C = c.eta_max * sum;
        const float graw = delta / C;
        return (penalty_mode(MODE) == GA_MODE_GA) ? 1.0f + graw : fmaxf(1.0f, graw);
    } else if constexpr (penalty_mode(MODE) == GA_MODE_SA) {
        return c.tau;
    } else {
        return 1.0f;
    }
}

// Alg. 14: m <- beta m + (1 - beta) x^2
__device__ __forceinline__ float second_moment(float m, float x, const StepConst& c) {
    const float bm = c.beta * m;
    const float xx = x * x;
    const float add = c.one_minus_beta * xx;
    return bm + add;
}

// MOMENTUM family (Alg. 2-5), one parameter, one arrival.  Nesterov form: the step uses
// d = ghat + gamma * v_new instead of v_new, and Alg. 14 follows d.
template <int MODE, bool KEEP_M>
__device__ __forceinline__ void update_one(float& th, float& v, float& m, float s, float g, const StepConst& c) {
    float ghat = g;
    if constexpr (penalty_mode(MODE) != GA_MODE_ASGD) ghat = g / penalty_of<MODE>(th, s, m, c);
    const float gv = c.gamma * v;
    const float vn = gv + ghat;
    float dir = vn;
    if constexpr (is_nesterov(MODE)) {
        const float look = c.gamma * vn;
        dir = ghat + look;
    }
    const float step = c.lr * dir;
    const float tn = th - step;
    v = vn;
    th = tn;
    if constexpr (KEEP_M) m = second_moment(m, dir, c);
}

// DANA family (Alg. 6-8).  x = sum_j v_j, y = v_i of the arriving worker; returns the look-ahead snapshot.
template <int MODE, bool KEEP_M>
__device__ __forceinline__ float dana_one(float& th, float& x, float& y, float& m, float s, float g,
                                          const StepConst& c) {
    float ghat = g;
    if constexpr (penalty_mode(MODE) != GA_MODE_ASGD) ghat = g / penalty_of<MODE>(th, s, m, c);
    const float v_old = y;
    const float gv = c.gamma * v_old;
    const float vn = gv + ghat;
    const float step = c.lr * vn;
    const float tn = th - step;
    const float less = x - v_old;
    const float sn = less + vn;
    y = vn;
    th = tn;
    x = sn;
    if constexpr (KEEP_M) m = second_moment(m, vn, c);
    const float ahead = c.eta_gamma * sn;
    return tn - ahead;
}

// ADAM family (Alg. 9-11).  x = m1, y = v2; m is the Alg. 14 state of the update vector u.
template <int MODE, bool KEEP_M>
__device__ __forceinline__ float adam_one(float& th, float& x, float& y, float& m, float s, float g,
                                          const StepConst& c) {
    float coef = c.omb1;
    if constexpr (penalty_mode(MODE) != GA_MODE_ASGD) coef = c.omb1 / penalty_of<MODE>(th, s, m, c);
    const float b1m = c.beta1 * x;
    const float cg = coef * g;
    const float m1n = b1m + cg;
    const float b2v = c.beta2 * y;
    const float gg = g * g;
    const float add2 = c.omb2 * gg;
    const float v2n = b2v + add2;
    const float m1h = m1n * c.inv_bc1;
    const float v2h = v2n * c.inv_bc2;
    const float root = sqrtf(v2h);
    const float den = root + c.adam_eps;
    const float u = m1h / den;
    const float step = c.lr * u;
    const float tn = th - step;
    x = m1n;
    y = v2n;
    th = tn;
    if constexpr (KEEP_M) m = second_moment(m, u, c);
    return tn;
}

// Four parameters; lanes >= n_valid (padding past N) are left untouched.
template <int MODE, bool KEEP_M>
__device__ __forceinline__ void update4(f32x4& th, f32x4& v, f32x4& m, const f32x4& s, const f32x4& g,
                                        const StepConst& c, uint32_t n_valid = 4) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if ((uint32_t)e < n_valid) {
            float t1 = th[e], v1 = v[e], m1 = m[e];
            update_one<MODE, KEEP_M>(t1, v1, m1, s[e], g[e], c);
            th[e] = t1;
            v[e] = v1;
            m[e] = m1;
        }
    }
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }

// Four gradient values of group q (elements 4q..4q+3).
template <int DT, bool ALIGNED>
__device__ __forceinline__ f32x4 load_g4(const void* __restrict__ g, uint64_t q) {
    f32x4 r;
    if constexpr (DT == GA_F32) {
        const float* p = static_cast<const float*>(g) + 4 * q;
        if constexpr (ALIGNED) {
            r = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        } else {
            r.x = __builtin_nontemporal_load(p);
            r.y = __builtin_nontemporal_load(p + 1);
            r.z = __builtin_nontemporal_load(p + 2);
            r.w = __builtin_nontemporal_load(p + 3);
        }
    } else {
        const uint16_t* p = static_cast<const uint16_t*>(g) + 4 * q;
        if constexpr (ALIGNED) {
            const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
            r.x = bf16_bits_to_float(w.x & 0xFFFFu);
            r.y = bf16_bits_to_float(w.x >> 16);
            r.z = bf16_bits_to_float(w.y & 0xFFFFu);
            r.w = bf16_bits_to_float(w.y >> 16);
        } else {
            r.x = bf16_bits_to_float(__builtin_nontemporal_load(p));
            r.y = bf16_bits_to_float(__builtin_nontemporal_load(p + 1));
            r.z = bf16_bits_to_float(__builtin_nontemporal_load(p + 2));
            r.w = bf16_bits_to_float(__builtin_nontemporal_load(p + 3));
        }
    }
    return r;
}

template <int DT>
__device__ __forceinline__ float load_g1(const void* __restrict__ g, uint64_t j) {
    if constexpr (DT == GA_F32) return static_cast<const float*>(g)[j];
    else return bf16_bits_to_float(static_cast<const uint16_t*>(g)[j]);
}

// The memory-side cache in front of HBM holds 256 MiB, and lines brought in by accesses with the non-temporal
// hint do not displace lines brought in without it.  The arrays a kernel touches at every arrival (theta, v, m)
// therefore keep a leading part in that cache from one arrival to the next: the blocks below a threshold access it
// without the hint, all other accesses carry it.  Measured with the fused update on 70 M - 250 M parameters: the
// time falls linearly with the kept bytes up to about 224 MiB, is flat to 256 MiB and is back at the all-streamed
// time from 288 MiB on (the kept lines then evict each other), so the budget stays clear of that edge.  For the same bytes, keeping more
// of theta beats keeping the same parameters' theta and v.  The default budget is kResidentBytes (ga_internal.h): a
// master that shares the GPU with other tenants of that cache is given a smaller one.

// Leading blocks of a launch whose theta / v / m accesses go without the hint (theta >= v >= m).
struct Residency {
    uint32_t theta, v, m;
};

// blocks: grid size; block_bytes: bytes of ONE array that a block covers.  theta first, then v, then m.
inline Residency residency_for(uint64_t resident_bytes, uint64_t blocks, uint64_t block_bytes, bool with_v, bool with_m) {
    uint64_t budget = resident_bytes / block_bytes;
    Residency r = {0u, 0u, 0u};
    r.theta = (uint32_t)(blocks < budget ? blocks : budget);
    budget -= r.theta;
    if (with_v) r.v = (uint32_t)(blocks < budget ? blocks : budget);
    budget -= r.v;
    if (with_m) r.m = (uint32_t)(blocks < budget ? blocks : budget);
    return r;
}

// Two block-uniform paths that differ only in cache hints are one path to the optimiser, which merges them and
// drops the hints.  An empty asm statement at both ends of each path keeps them apart.
#ifndef GA_HINT_PATH   // a build of these sources for another target (the CPU build of the tests) brings its own
#define GA_HINT_PATH(name, ...)                          \
    do {                                                 \
        asm volatile("; " name " begin" ::: "memory");   \
        __VA_ARGS__;                                     \
        asm volatile("; " name " end" ::: "memory");     \
    } while (0)
#endif

inline uint32_t blocks_for(uint64_t items, uint64_t per_block, uint32_t cap) {
    const uint64_t b = (items + per_block - 1) / per_block;
    return (uint32_t)(b < 1 ? 1 : (b > cap ? cap : b));
}

// ---------------------------------------------------------------------------
// Noise of the quadratic source: Philox4x32-10 (Salmon et al., SC'11) and a
// Box-Muller transform in float operations only.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&x)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32x32->64 multiply gives the high and the low word (v_mad_u64_u32)
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    x[0] = c0; x[1] = c1; x[2] = c2; x[3] = c3;
}

// Correctly rounded a / b and sqrt(x) for operands that are known to be normal, far from the
// ends of the exponent range (a may be zero).  Same iteration as the general expansion of '/'
// and sqrtf (reciprocal, two residual corrections; root, +-1 ulp residual test) without its
// operand scaling and special-case fix-up, which cannot trigger in that range.
__device__ __forceinline__ float div_normal_range(float a, float b) {
    float r = __builtin_amdgcn_rcpf(b);
    const float e0 = fmaf(-b, r, 1.0f);
    r = fmaf(e0, r, r);
    float q = a * r;
    const float e1 = fmaf(-b, q, a);
    q = fmaf(e1, r, q);
    const float e2 = fmaf(-b, q, a);
    return fmaf(e2, r, q);
}

__device__ __forceinline__ float sqrt_normal_range(float x) {
    const float s = __builtin_amdgcn_sqrtf(x);
    const float s_dn = __uint_as_float(__float_as_uint(s) - 1u);
    const float s_up = __uint_as_float(__float_as_uint(s) + 1u);
    const float r_dn = fmaf(-s_dn, s, x);
    const float r_up = fmaf(-s_up, s, x);
    float out = (r_dn <= 0.0f) ? s_dn : s;
    out = (r_up > 0.0f) ? s_up : out;
    return out;
}

// (xa, xb) -> (r cos(angle), r sin(angle)); see ga_noise_fill in include/ga.h.
__device__ __forceinline__ void box_muller_pair(uint32_t xa, uint32_t xb, float& zc, float& zs) {
    // radius: ln(u1), u1 = M 2^-24 with M odd below 2^24, M = t 2^e, t in [sqrt(1/2), sqrt(2))
    const uint32_t M = 2u * (xa >> 9) + 1u;
    const uint32_t bits = __float_as_uint((float)M);           // exact conversion
    int e = (int)(bits >> 23) - 126;
    float t = __uint_as_float((bits & 0x007FFFFFu) | 0x3F000000u);   // [1/2, 1)
    if (t < 0.70710678f) {
        t = 2.0f * t;
        e -= 1;
    }
    const float E = (float)(e - 24);
    const float num = t - 1.0f;                                 // in [-0.293, 0.415], zero or at least 2^-24
    const float den = t + 1.0f;                                 // in [1.707, 2.415]
    const float s = div_normal_range(num, den);
    const float s2 = s * s;
    float P = fmaf(s2, 1.0f / 9.0f, 1.0f / 7.0f);
    P = fmaf(s2, P, 1.0f / 5.0f);
    P = fmaf(s2, P, 1.0f / 3.0f);
    const float s3 = s * s2;
    const float L = fmaf(s3, P, s);                             // atanh(s)
    const float twoL = 2.0f * L;
    const float lnu = fmaf(E, 0.693147180559945f, twoL);
    const float r = sqrt_normal_range(-2.0f * lnu);             // argument in [1.1e-7, 33.3]

    // angle = quad * pi/2 + phi, phi in (-pi/4, pi/4)
    const uint32_t quad = xb >> 30;
    const int hi = (int)(2u * ((xb >> 7) & 0x7FFFFFu) + 1u) - (1 << 23);
    const float h = (float)hi * 5.9604644775390625e-8f;         // 2^-24
    const float phi = h * 1.5707963267948966f;
    const float p2 = phi * phi;
    float S = fmaf(p2, 1.0f / 362880.0f, -1.0f / 5040.0f);
    S = fmaf(p2, S, 1.0f / 120.0f);
    S = fmaf(p2, S, -1.0f / 6.0f);
    const float p3 = phi * p2;
    const float sn = fmaf(p3, S, phi);
    float Cc = fmaf(p2, -1.0f / 3628800.0f, 1.0f / 40320.0f);
    Cc = fmaf(p2, Cc, -1.0f / 720.0f);
    Cc = fmaf(p2, Cc, 1.0f / 24.0f);
    Cc = fmaf(p2, Cc, -0.5f);
    const float cs = fmaf(p2, Cc, 1.0f);

    // quarter-turn rotation: quad 0 (c, s), 1 (-s, c), 2 (-c, -s), 3 (s, -c)
    const float ca0 = (quad & 1u) ? sn : cs;
    const float sa0 = (quad & 1u) ? cs : sn;
    const float ca = (quad == 1u || quad == 2u) ? -ca0 : ca0;
    const float sa = (quad >= 2u) ? -sa0 : sa0;
    zc = r * ca;
    zs = r * sa;
}

// z for parameters 4q..4q+3 at master step k.
__device__ __forceinline__ f32x4 noise4(uint32_t seed_lo, uint32_t seed_hi, uint64_t q, uint64_t k) {
    uint32_t x[4];
    philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), (uint32_t)k, (uint32_t)(k >> 32), seed_lo, seed_hi, x);
    float z0, z1, z2, z3;
    box_muller_pair(x[0], x[1], z0, z1);
    box_muller_pair(x[2], x[3], z2, z3);
    return f32x4{z0, z1, z2, z3};
}

__device__ __forceinline__ float quadratic_g(float s, float a, float ts, float sigma, float z) {
    const float off = s - ts;
    const float pull = a * off;
    const float noise = sigma * z;
    return pull + noise;
}

// E consecutive floats held in registers; E = 4, 2 or 1 (one 128-, 64- or 32-bit access).
template <int E>
struct Pack {
    float x[E];
};
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int E>
__device__ __forceinline__ Pack<E> pack_load(const float* base, uint64_t idx) {   // idx counts packs
    Pack<E> r;
    if constexpr (E == 4) {
        const f32x4 t = reinterpret_cast<const f32x4*>(base)[idx];
        r.x[0] = t.x; r.x[1] = t.y; r.x[2] = t.z; r.x[3] = t.w;
    } else if constexpr (E == 2) {
        const f32x2 t = reinterpret_cast<const f32x2*>(base)[idx];
        r.x[0] = t.x; r.x[1] = t.y;
    } else {
        r.x[0] = base[idx];
    }
    return r;
}

template <int E>
__device__ __forceinline__ void pack_store(float* base, uint64_t idx, const Pack<E>& r) {
    if constexpr (E == 4) reinterpret_cast<f32x4*>(base)[idx] = f32x4{r.x[0], r.x[1], r.x[2], r.x[3]};
    else if constexpr (E == 2) reinterpret_cast<f32x2*>(base)[idx] = f32x2{r.x[0], r.x[1]};
    else base[idx] = r.x[0];
}

template <int E>
__device__ __forceinline__ Pack<E> pack_zero() {
    Pack<E> r;
#pragma unroll
    for (int e = 0; e < E; ++e) r.x[e] = 0.0f;
    return r;
}

// z for parameters j0 .. j0+E-1 (j0 a multiple of E) at master step k.  The Philox block of
// floor(j0/4) is computed by every thread that needs a part of it.
template <int E>
__device__ __forceinline__ Pack<E> noise_pack(uint32_t seed_lo, uint32_t seed_hi, uint64_t j0, uint64_t k) {
    const uint64_t q = j0 >> 2;
    uint32_t x[4];
    philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), (uint32_t)k, (uint32_t)(k >> 32), seed_lo, seed_hi, x);
    Pack<E> z;
    if constexpr (E == 4) {
        box_muller_pair(x[0], x[1], z.x[0], z.x[1]);
        box_muller_pair(x[2], x[3], z.x[2], z.x[3]);
    } else {
        const bool upper = ((j0 >> 1) & 1) != 0;
        float zc, zs;
        box_muller_pair(upper ? x[2] : x[0], upper ? x[3] : x[1], zc, zs);
        if constexpr (E == 2) {
            z.x[0] = zc;
            z.x[1] = zs;
        } else {
            z.x[0] = (j0 & 1) ? zs : zc;
        }
    }
    return z;
}

}  // namespace
}  // namespace ga

#endif
