// gfx950 kernels of the Gap-Aware master update.
//
//   apply_kernel        one arrival, gradient from HBM (Alg. 2-5 + Alg. 14 fused)
//   family_apply_kernel the same for the DANA (Alg. 6-8) and Adam (Alg. 9-11) masters
//   layer_*_kernel      layer-wise / global Gap (Eq. 4, Def. 1): reduce, per-layer Gap, update
//   persistent_kernel   a chunk of arrivals per launch; every thread owns four
//                       parameters for the whole chunk and generates the
//                       quadratic-plus-noise gradients itself
//   quadratic_gradient_kernel / noise_fill_kernel   the gradient source alone
//   diag_kernel + diag_final_kernel                  Gap statistics (App. C.8)
//
// The whole path is elementwise (Sec. 4.3: every parameter is penalised
// independently), so it is bound by HBM traffic or plain vector ALU work; there
// is no contraction and therefore no MFMA.
//
// Floating point: every operation is a separately rounded IEEE float
// operation in the order given in include/ga.h.  This file must be compiled
// with -ffp-contract=off; '/' and sqrtf are correctly rounded (hipcc default).

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
// that arrays touched at every arrival (theta, and v when both fit) stay in it.
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
            r.x = p[0]; r.y = p[1]; r.z = p[2]; r.w = p[3];
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
            r.x = bf16_bits_to_float(p[0]); r.y = bf16_bits_to_float(p[1]);
            r.z = bf16_bits_to_float(p[2]); r.w = bf16_bits_to_float(p[3]);
        }
    }
    return r;
}

template <int DT>
__device__ __forceinline__ float load_g1(const void* __restrict__ g, uint64_t j) {
    if constexpr (DT == GA_F32) return static_cast<const float*>(g)[j];
    else return bf16_bits_to_float(static_cast<const uint16_t*>(g)[j]);
}

// ---------------------------------------------------------------------------
// Fused update of one arrival.  Each thread owns U groups of four consecutive
// parameters, 256 groups apart, so that every wavefront issues 1 KiB
// contiguous 128-bit loads and stores per array.  All loads of a thread are
// issued before the first dependent operation.
// ---------------------------------------------------------------------------
template <int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED, bool STREAM_V, int U>
__global__ __launch_bounds__(kBlock) void apply_kernel(float* __restrict__ theta, float* __restrict__ v,
                                                       float* __restrict__ m, float* __restrict__ snap,
                                                       const void* __restrict__ g, uint64_t N, StepConst c) {
    constexpr bool GAP = is_gap(MODE);
    const uint64_t n4 = N >> 2;
    const uint64_t base = (uint64_t)blockIdx.x * (kBlock * U) + threadIdx.x;

    f32x4 th[U], vv[U], mm[U], ss[U], gg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock;
        mm[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        ss[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (q < n4) {
            th[u] = load4<false>(theta, q);
            vv[u] = load4<STREAM_V>(v, q);
            if constexpr (KEEP_M) mm[u] = load4<true>(m, q);
            if constexpr (GAP) ss[u] = load4<true>(snap, q);
            gg[u] = load_g4<DT, ALIGNED>(g, q);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock;
        if (q < n4) {
            update4<MODE, KEEP_M>(th[u], vv[u], mm[u], ss[u], gg[u], c);
            store4<false>(theta, q, th[u]);
            store4<STREAM_V>(v, q, vv[u]);
            if constexpr (KEEP_M) store4<true>(m, q, mm[u]);
            if constexpr (SNAP) store4<true>(snap, q, th[u]);
        }
    }

    // ragged tail: the last N % 4 parameters, one per thread of block 0
    if (blockIdx.x == 0 && threadIdx.x < (N & 3)) {
        const uint64_t j = 4 * n4 + threadIdx.x;
        float t1 = theta[j], v1 = v[j], m1 = 0.0f, s1 = 0.0f;
        if constexpr (KEEP_M) m1 = m[j];
        if constexpr (GAP) s1 = snap[j];
        update_one<MODE, KEEP_M>(t1, v1, m1, s1, load_g1<DT>(g, j), c);
        theta[j] = t1;
        v[j] = v1;
        if constexpr (KEEP_M) m[j] = m1;
        if constexpr (SNAP) snap[j] = t1;
    }
}

// ---------------------------------------------------------------------------
// Fused update of one arrival for the DANA and ADAM families: the same launch
// shape as apply_kernel with one more state array.  x: vsum | m1 (touched at
// every arrival, kept in the memory-side cache when it fits); y: the arriving
// worker's v_i (streamed) | v2.
// ---------------------------------------------------------------------------
template <int FAMILY, int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED, bool STREAM_X, int U>
__global__ __launch_bounds__(kBlock) void family_apply_kernel(float* __restrict__ theta, float* __restrict__ x,
                                                              float* __restrict__ y, float* __restrict__ m,
                                                              float* __restrict__ snap,
                                                              const void* __restrict__ g, uint64_t N, StepConst c) {
    constexpr bool GAP = is_gap(MODE);
    const uint64_t n4 = N >> 2;
    const uint64_t base = (uint64_t)blockIdx.x * (kBlock * U) + threadIdx.x;

    f32x4 th[U], xx[U], yy[U], mm[U], ss[U], gg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock;
        mm[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        ss[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (q < n4) {
            th[u] = load4<false>(theta, q);
            xx[u] = load4<STREAM_X>(x, q);
            yy[u] = load4<true>(y, q);
            if constexpr (KEEP_M) mm[u] = load4<true>(m, q);
            if constexpr (GAP) ss[u] = load4<true>(snap, q);
            gg[u] = load_g4<DT, ALIGNED>(g, q);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = base + (uint64_t)u * kBlock;
        if (q < n4) {
            f32x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float t1 = th[u][e], x1 = xx[u][e], y1 = yy[u][e], m1 = mm[u][e];
                if constexpr (FAMILY == GA_FAMILY_DANA) out[e] = dana_one<MODE, KEEP_M>(t1, x1, y1, m1, ss[u][e], gg[u][e], c);
                else out[e] = adam_one<MODE, KEEP_M>(t1, x1, y1, m1, ss[u][e], gg[u][e], c);
                th[u][e] = t1; xx[u][e] = x1; yy[u][e] = y1; mm[u][e] = m1;
            }
            store4<false>(theta, q, th[u]);
            store4<STREAM_X>(x, q, xx[u]);
            store4<true>(y, q, yy[u]);
            if constexpr (KEEP_M) store4<true>(m, q, mm[u]);
            if constexpr (SNAP) store4<true>(snap, q, out);
        }
    }

    if (blockIdx.x == 0 && threadIdx.x < (N & 3)) {
        const uint64_t j = 4 * n4 + threadIdx.x;
        float t1 = theta[j], x1 = x[j], y1 = y[j], m1 = 0.0f, s1 = 0.0f, out;
        if constexpr (KEEP_M) m1 = m[j];
        if constexpr (GAP) s1 = snap[j];
        if constexpr (FAMILY == GA_FAMILY_DANA) out = dana_one<MODE, KEEP_M>(t1, x1, y1, m1, s1, load_g1<DT>(g, j), c);
        else out = adam_one<MODE, KEEP_M>(t1, x1, y1, m1, s1, load_g1<DT>(g, j), c);
        theta[j] = t1;
        x[j] = x1;
        y[j] = y1;
        if constexpr (KEEP_M) m[j] = m1;
        if constexpr (SNAP) snap[j] = out;
    }
}

// ---------------------------------------------------------------------------
// Layer-wise and global Gap (Eq. 4, Def. 1).  Three launches per arrival:
//   layer_partial_kernel   one block per chunk of a layer: sum (theta-snap)^2 and sum m in double
//   layer_gap_kernel       one block per layer adds its chunk partials in a fixed order and forms G_p
//   layer_apply_kernel     one block per chunk: the momentum update with ghat = g / G_p
// A chunk never crosses a layer boundary; boundaries are arbitrary, so a chunk has a scalar
// head and tail around its 16-byte aligned body.  Every sum has a fixed order.
// ---------------------------------------------------------------------------
constexpr int kLayerU = 4;   // 128-bit groups in flight per thread in the chunk kernels

struct ChunkRange {
    uint64_t start, end;   // parameters [start, end)
    uint64_t a0, a1;       // aligned body [a0, a1), multiples of 4
};

__device__ __forceinline__ ChunkRange chunk_range(const LayerChunk& ch) {
    ChunkRange r;
    r.start = ch.start;
    r.end = ch.start + ch.len;
    r.a0 = (r.start + 3) & ~(uint64_t)3;
    if (r.a0 > r.end) r.a0 = r.end;
    r.a1 = r.end & ~(uint64_t)3;
    if (r.a1 < r.a0) r.a1 = r.a0;
    return r;
}

__global__ __launch_bounds__(kBlock) void layer_partial_kernel(const float* __restrict__ theta,
                                                               const float* __restrict__ m,
                                                               const float* __restrict__ snap,
                                                               const LayerChunk* __restrict__ chunks,
                                                               LayerPartial* __restrict__ partials) {
    const ChunkRange r = chunk_range(chunks[blockIdx.x]);
    double d2 = 0.0, ms = 0.0;
    auto one = [&](float th, float s, float mm) {
        const float diff = th - s;
        d2 += (double)diff * (double)diff;
        ms += (double)mm;
    };
    for (uint64_t j = r.start + threadIdx.x; j < r.a0; j += kBlock) one(theta[j], snap[j], m[j]);
    const uint64_t q_end = r.a1 >> 2;
    for (uint64_t q0 = (r.a0 >> 2) + threadIdx.x; q0 < q_end; q0 += (uint64_t)kLayerU * kBlock) {
        f32x4 th[kLayerU], sv[kLayerU], mm[kLayerU];
#pragma unroll
        for (int u = 0; u < kLayerU; ++u) {
            const uint64_t q = q0 + (uint64_t)u * kBlock;
            if (q < q_end) {
                th[u] = load4<false>(theta, q);
                sv[u] = load4<true>(snap, q);
                mm[u] = load4<true>(m, q);
            }
        }
#pragma unroll
        for (int u = 0; u < kLayerU; ++u) {
            if (q0 + (uint64_t)u * kBlock < q_end) {
                one(th[u].x, sv[u].x, mm[u].x); one(th[u].y, sv[u].y, mm[u].y);
                one(th[u].z, sv[u].z, mm[u].z); one(th[u].w, sv[u].w, mm[u].w);
            }
        }
    }
    for (uint64_t j = r.a1 + threadIdx.x; j < r.end; j += kBlock) one(theta[j], snap[j], m[j]);

    __shared__ double part[2][kBlock / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        d2 += __shfl_xor(d2, off, 64);
        ms += __shfl_xor(ms, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        part[0][threadIdx.x >> 6] = d2;
        part[1][threadIdx.x >> 6] = ms;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        LayerPartial out = {part[0][0], part[1][0]};
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) {
            out.dist2 += part[0][w];
            out.msum += part[1][w];
        }
        partials[blockIdx.x] = out;
    }
}

template <bool HINGE>
__global__ __launch_bounds__(kBlock) void layer_gap_kernel(const LayerPartial* __restrict__ partials,
                                                           const LayerSpan* __restrict__ spans, float inv_bc_prev,
                                                           float eta_max, float eps, float* __restrict__ gaps) {
    // one block per layer: strided partial sums, 64-lane butterfly, then the waves in order
    const LayerSpan sp = spans[blockIdx.x];
    double d2 = 0.0, ms = 0.0;
    for (uint32_t i = threadIdx.x; i < sp.n_chunks; i += kBlock) {
        d2 += partials[sp.first_chunk + i].dist2;
        ms += partials[sp.first_chunk + i].msum;
    }
    __shared__ double part[2][kBlock / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        d2 += __shfl_xor(d2, off, 64);
        ms += __shfl_xor(ms, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        part[0][threadIdx.x >> 6] = d2;
        part[1][threadIdx.x >> 6] = ms;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    d2 = part[0][0];
    ms = part[1][0];
#pragma unroll
    for (int w = 1; w < kBlock / 64; ++w) {
        d2 += part[0][w];
        ms += part[1][w];
    }
    const float delta = (float)sqrt(d2);
    const float mhat = (float)ms * inv_bc_prev;
    const float root = sqrtf(mhat);
    const float sum = root + eps;
    const float C = eta_max * sum;
    const float graw = delta / C;
    gaps[blockIdx.x] = HINGE ? fmaxf(1.0f, graw) : 1.0f + graw;
}

template <bool NAG>
__device__ __forceinline__ void layer_update_one(float& th, float& v, float& m, float g, float G, const StepConst& c) {
    const float ghat = g / G;
    const float gv = c.gamma * v;
    const float vn = gv + ghat;
    float dir = vn;
    if constexpr (NAG) {
        const float look = c.gamma * vn;
        dir = ghat + look;
    }
    const float step = c.lr * dir;
    th = th - step;
    v = vn;
    m = second_moment(m, dir, c);
}

template <int DT, bool ALIGNED, bool STREAM_V, bool NAG>
__global__ __launch_bounds__(kBlock) void layer_apply_kernel(float* __restrict__ theta, float* __restrict__ v,
                                                             float* __restrict__ m, float* __restrict__ snap,
                                                             const void* __restrict__ g,
                                                             const LayerChunk* __restrict__ chunks,
                                                             const float* __restrict__ gaps, StepConst c) {
    const LayerChunk ch = chunks[blockIdx.x];
    const ChunkRange r = chunk_range(ch);
    const float G = gaps[ch.layer];
    auto scalar = [&](uint64_t j) {
        float t1 = theta[j], v1 = v[j], m1 = m[j];
        layer_update_one<NAG>(t1, v1, m1, load_g1<DT>(g, j), G, c);
        theta[j] = t1; v[j] = v1; m[j] = m1; snap[j] = t1;
    };
    for (uint64_t j = r.start + threadIdx.x; j < r.a0; j += kBlock) scalar(j);
    constexpr int U = 2;
    const uint64_t q_end = r.a1 >> 2;
    for (uint64_t q0 = (r.a0 >> 2) + threadIdx.x; q0 < q_end; q0 += (uint64_t)U * kBlock) {
        f32x4 th[U], vv[U], mm[U], gg[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t q = q0 + (uint64_t)u * kBlock;
            if (q < q_end) {
                th[u] = load4<false>(theta, q);
                vv[u] = load4<STREAM_V>(v, q);
                mm[u] = load4<true>(m, q);
                gg[u] = load_g4<DT, ALIGNED>(g, q);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t q = q0 + (uint64_t)u * kBlock;
            if (q < q_end) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float t1 = th[u][e], v1 = vv[u][e], m1 = mm[u][e];
                    layer_update_one<NAG>(t1, v1, m1, gg[u][e], G, c);
                    th[u][e] = t1; vv[u][e] = v1; mm[u][e] = m1;
                }
                store4<false>(theta, q, th[u]);
                store4<STREAM_V>(v, q, vv[u]);
                store4<true>(m, q, mm[u]);
                store4<true>(snap, q, th[u]);
            }
        }
    }
    for (uint64_t j = r.a1 + threadIdx.x; j < r.end; j += kBlock) scalar(j);
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

__global__ __launch_bounds__(kBlock) void noise_fill_kernel(uint32_t seed_lo, uint32_t seed_hi, uint64_t k,
                                                            uint64_t j0, uint64_t n, float* __restrict__ out) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint64_t j = j0 + i;
    const f32x4 z = noise4(seed_lo, seed_hi, j >> 2, k);
    const uint32_t lane = (uint32_t)(j & 3);
    out[i] = lane == 0 ? z.x : lane == 1 ? z.y : lane == 2 ? z.z : z.w;
}

__global__ __launch_bounds__(kBlock) void box_muller_raw_kernel(const uint32_t* __restrict__ xa,
                                                                const uint32_t* __restrict__ xb, uint64_t n,
                                                                float* __restrict__ zc, float* __restrict__ zs) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    float c, s;
    box_muller_pair(xa[i], xb[i], c, s);
    zc[i] = c;
    zs[i] = s;
}

__global__ __launch_bounds__(kBlock) void quadratic_gradient_kernel(const float* __restrict__ snap,
                                                                    const float* __restrict__ a,
                                                                    const float* __restrict__ ts, uint64_t N,
                                                                    uint64_t k, RunConst rc,
                                                                    float* __restrict__ g_out) {
    const uint64_t q = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t j0 = 4 * q;
    if (j0 >= N) return;
    const f32x4 z = noise4(rc.seed_lo, rc.seed_hi, q, k);
    if (j0 + 3 < N) {
        const f32x4 s = reinterpret_cast<const f32x4*>(snap)[q];
        const f32x4 a4 = reinterpret_cast<const f32x4*>(a)[q];
        const f32x4 t4 = reinterpret_cast<const f32x4*>(ts)[q];
        f32x4 g;
        g.x = quadratic_g(s.x, a4.x, t4.x, rc.sigma, z.x);
        g.y = quadratic_g(s.y, a4.y, t4.y, rc.sigma, z.y);
        g.z = quadratic_g(s.z, a4.z, t4.z, rc.sigma, z.z);
        g.w = quadratic_g(s.w, a4.w, t4.w, rc.sigma, z.w);
        reinterpret_cast<f32x4*>(g_out)[q] = g;
    } else {
        const float zz[4] = {z.x, z.y, z.z, z.w};
        for (int e = 0; e < 4 && j0 + e < N; ++e)
            g_out[j0 + e] = quadratic_g(snap[j0 + e], a[j0 + e], ts[j0 + e], rc.sigma, zz[e]);
    }
}

// ---------------------------------------------------------------------------
// Persistent multi-arrival kernel.  Thread = one group of four parameters.
// theta, v, m, a, theta* stay in registers for the whole chunk; per arrival
// the thread reads and rewrites only its 16 bytes of the arriving worker's
// snapshot (DANA: and of that worker's momentum; Adam keeps m1 and v2 in
// registers too).  No thread ever needs another thread's data, so there is no
// grid-wide or block-wide synchronisation.  The snapshot of the next arrival
// is requested before the arithmetic of the current one.
// ---------------------------------------------------------------------------
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

// ---------------------------------------------------------------------------
// Gap statistics: per-thread accumulation, wavefront (64 lanes) butterfly,
// one partial per block, then a single block adds the partials in a fixed
// order so that the result does not depend on scheduling.
// ---------------------------------------------------------------------------
struct DiagAcc {
    double sum;
    uint32_t gt1, gt0, bad;
};

__device__ __forceinline__ void diag_one(DiagAcc& acc, float th, float s, float m, float inv_bc, float eta_max,
                                         float eps) {
    const float diff = th - s;
    const float delta = fabsf(diff);
    const float mhat = m * inv_bc;
    const float root = sqrtf(mhat);
    const float sum = root + eps;
    const float C = eta_max * sum;
    const float graw = delta / C;
    if (!isfinite(graw)) {
        acc.bad += 1;
    } else {
        acc.sum += (double)graw;
        acc.gt1 += (graw > 1.0f);
        acc.gt0 += (graw > 0.0f);
    }
}

__device__ __forceinline__ DiagPartial block_reduce(double sum, unsigned long long gt1, unsigned long long gt0,
                                                    unsigned long long bad) {
    __shared__ DiagPartial wave_part[kBlock / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        sum += __shfl_xor(sum, off, 64);
        gt1 += __shfl_xor(gt1, off, 64);
        gt0 += __shfl_xor(gt0, off, 64);
        bad += __shfl_xor(bad, off, 64);
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        wave_part[wave].sum_graw = sum;
        wave_part[wave].n_gt1 = gt1;
        wave_part[wave].n_gt0 = gt0;
        wave_part[wave].n_bad = bad;
    }
    __syncthreads();
    DiagPartial r = wave_part[0];
#pragma unroll
    for (int w = 1; w < kBlock / 64; ++w) {
        r.sum_graw += wave_part[w].sum_graw;
        r.n_gt1 += wave_part[w].n_gt1;
        r.n_gt0 += wave_part[w].n_gt0;
        r.n_bad += wave_part[w].n_bad;
    }
    return r;
}

__global__ __launch_bounds__(kBlock) void diag_kernel(const float* __restrict__ theta, const float* __restrict__ m,
                                                      const float* __restrict__ snap, uint64_t N, float inv_bc,
                                                      float eta_max, float eps,
                                                      DiagPartial* __restrict__ partials) {
    const uint64_t n4 = N >> 2;
    DiagAcc acc = {0.0, 0u, 0u, 0u};
    for (uint64_t q = (uint64_t)blockIdx.x * kBlock + threadIdx.x; q < n4; q += (uint64_t)gridDim.x * kBlock) {
        const f32x4 th = reinterpret_cast<const f32x4*>(theta)[q];
        const f32x4 s = reinterpret_cast<const f32x4*>(snap)[q];
        const f32x4 mm = reinterpret_cast<const f32x4*>(m)[q];
        diag_one(acc, th.x, s.x, mm.x, inv_bc, eta_max, eps);
        diag_one(acc, th.y, s.y, mm.y, inv_bc, eta_max, eps);
        diag_one(acc, th.z, s.z, mm.z, inv_bc, eta_max, eps);
        diag_one(acc, th.w, s.w, mm.w, inv_bc, eta_max, eps);
    }
    if (blockIdx.x == 0 && threadIdx.x < (N & 3)) {
        const uint64_t j = 4 * n4 + threadIdx.x;
        diag_one(acc, theta[j], snap[j], m[j], inv_bc, eta_max, eps);
    }
    const DiagPartial r = block_reduce(acc.sum, acc.gt1, acc.gt0, acc.bad);
    if (threadIdx.x == 0) partials[blockIdx.x] = r;
}

__global__ __launch_bounds__(kBlock) void diag_final_kernel(const DiagPartial* __restrict__ partials,
                                                            uint32_t n_partials, DiagPartial* __restrict__ total) {
    double sum = 0.0;
    unsigned long long gt1 = 0, gt0 = 0, bad = 0;
    for (uint32_t i = threadIdx.x; i < n_partials; i += kBlock) {
        sum += partials[i].sum_graw;
        gt1 += partials[i].n_gt1;
        gt0 += partials[i].n_gt0;
        bad += partials[i].n_bad;
    }
    const DiagPartial r = block_reduce(sum, gt1, gt0, bad);
    if (threadIdx.x == 0) *total = r;
}

// ---------------------------------------------------------------------------
// Fills.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void fill_kernel(float* __restrict__ dst, uint64_t n, float value) {
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock)
        dst[i] = value;
}

__global__ __launch_bounds__(kBlock) void broadcast_rows_kernel(float* __restrict__ dst, uint64_t stride,
                                                                uint32_t rows, const float* __restrict__ src,
                                                                uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) {
        const float x = src[i];
        for (uint32_t r = 0; r < rows; ++r) dst[(uint64_t)r * stride + i] = x;
    }
}

uint32_t blocks_for(uint64_t items, uint64_t per_block, uint32_t cap) {
    const uint64_t b = (items + per_block - 1) / per_block;
    return (uint32_t)(b < 1 ? 1 : (b > cap ? cap : b));
}

// ---------------------------------------------------------------------------
// Dispatch of the apply kernel over (mode, dtype, keep_m, aligned).
// ---------------------------------------------------------------------------
constexpr int kApplyU = 2;
// below this many parameters the persistent kernel gives each thread 2 instead of 4 of them
#ifndef GA_PERSIST_WIDE_MIN_N
#define GA_PERSIST_WIDE_MIN_N (1ull << 21)
#endif
constexpr uint64_t kPersistWideMinN = GA_PERSIST_WIDE_MIN_N;

// theta and v together must fit the memory-side cache with room to spare for v to be kept in it
constexpr uint64_t kKeepVMaxN = (uint64_t)208 * 1024 * 1024 / 8;

template <int MODE, int DT, bool KEEP_M, bool SNAP, bool ALIGNED>
hipError_t launch_apply_t(const StatePtrs& st, float* snap, const void* g, uint64_t N, const StepConst& c,
                          hipStream_t stream) {
    const uint64_t n4 = N >> 2;
    const uint64_t per_block = (uint64_t)kBlock * kApplyU;
    const uint64_t blocks = (n4 + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid(blocks == 0 ? 1u : (uint32_t)blocks), block(kBlock);
    if (N <= kKeepVMaxN)
        hipLaunchKernelGGL((apply_kernel<MODE, DT, KEEP_M, SNAP, ALIGNED, false, kApplyU>), grid, block, 0, stream,
                           st.theta, st.v, st.m, snap, g, N, c);
    else
        hipLaunchKernelGGL((apply_kernel<MODE, DT, KEEP_M, SNAP, ALIGNED, true, kApplyU>), grid, block, 0, stream,
                           st.theta, st.v, st.m, snap, g, N, c);
    return hipGetLastError();
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
                           const StepConst& c, hipStream_t stream) {
    const uint64_t n4 = N >> 2;
    const uint64_t per_block = (uint64_t)kBlock * kFamilyU;
    const uint64_t blocks = (n4 + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid(blocks == 0 ? 1u : (uint32_t)blocks), block(kBlock);
    if (N <= kKeepVMaxN)
        hipLaunchKernelGGL((family_apply_kernel<FAMILY, MODE, DT, KEEP_M, SNAP, ALIGNED, false, kFamilyU>), grid, block,
                           0, stream, theta, x, y, m, snap, g, N, c);
    else
        hipLaunchKernelGGL((family_apply_kernel<FAMILY, MODE, DT, KEEP_M, SNAP, ALIGNED, true, kFamilyU>), grid, block,
                           0, stream, theta, x, y, m, snap, g, N, c);
    return hipGetLastError();
}

template <int FAMILY, int MODE, bool KEEP_M, bool SNAP>
hipError_t launch_family_m(float* theta, float* x, float* y, float* m, float* snap, const void* g, int dt,
                           uint64_t N, const StepConst& c, hipStream_t stream) {
    const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
    if (dt == GA_F32) {
        if ((addr & 15u) == 0)
            return launch_family_t<FAMILY, MODE, GA_F32, KEEP_M, SNAP, true>(theta, x, y, m, snap, g, N, c, stream);
        return launch_family_t<FAMILY, MODE, GA_F32, KEEP_M, SNAP, false>(theta, x, y, m, snap, g, N, c, stream);
    }
    if ((addr & 7u) == 0)
        return launch_family_t<FAMILY, MODE, GA_BF16, KEEP_M, SNAP, true>(theta, x, y, m, snap, g, N, c, stream);
    return launch_family_t<FAMILY, MODE, GA_BF16, KEEP_M, SNAP, false>(theta, x, y, m, snap, g, N, c, stream);
}

template <int FAMILY>
hipError_t launch_family(float* theta, float* x, float* y, float* m, float* snap, const void* g, int dt, uint64_t N,
                         int mode, bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream) {
#define GA_FAM(MODE, KEEP, SNAP) launch_family_m<FAMILY, MODE, KEEP, SNAP>(theta, x, y, m, snap, g, dt, N, c, stream)
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
                                         write_snap, c, stream);
}

hipError_t launch_apply_adam(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype, int mode,
                             bool keep_m, bool write_snap, const StepConst& c, hipStream_t stream) {
    return launch_family<GA_FAMILY_ADAM>(st.theta, st.v, st.v2, st.m, st.snaps + (uint64_t)worker * st.stride, g,
                                         grad_dtype, N, mode, keep_m, write_snap, c, stream);
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

hipError_t launch_apply_layerwise(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype,
                                  int mode, bool nesterov, const LayerTables& lt, const StepConst& c,
                                  hipStream_t stream) {
    if (lt.n_chunks == 0 || lt.n_layers == 0) return hipErrorInvalidValue;
    float* snap = st.snaps + (uint64_t)worker * st.stride;
    const dim3 block(kBlock), grid(lt.n_chunks), lgrid(lt.n_layers);
    hipLaunchKernelGGL(layer_partial_kernel, grid, block, 0, stream, st.theta, st.m, snap, lt.chunks, lt.partials);
    if (mode == GA_MODE_GA_HINGE)
        hipLaunchKernelGGL(layer_gap_kernel<true>, lgrid, block, 0, stream, lt.partials, lt.spans, c.inv_bc_prev,
                           c.eta_max, c.eps, lt.gaps);
    else
        hipLaunchKernelGGL(layer_gap_kernel<false>, lgrid, block, 0, stream, lt.partials, lt.spans, c.inv_bc_prev,
                           c.eta_max, c.eps, lt.gaps);
    const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
    const bool stream_v = N > kKeepVMaxN;
#define GA_LAYER_APPLY(DT, AL, SV)                                                                                  \
    do {                                                                                                            \
        if (nesterov)                                                                                               \
            hipLaunchKernelGGL((layer_apply_kernel<DT, AL, SV, true>), grid, block, 0, stream, st.theta, st.v, st.m, \
                               snap, g, lt.chunks, lt.gaps, c);                                                     \
        else                                                                                                        \
            hipLaunchKernelGGL((layer_apply_kernel<DT, AL, SV, false>), grid, block, 0, stream, st.theta, st.v,     \
                               st.m, snap, g, lt.chunks, lt.gaps, c);                                               \
    } while (0)
    if (grad_dtype == GA_F32) {
        if ((addr & 15u) == 0) { if (stream_v) GA_LAYER_APPLY(GA_F32, true, true); else GA_LAYER_APPLY(GA_F32, true, false); }
        else { if (stream_v) GA_LAYER_APPLY(GA_F32, false, true); else GA_LAYER_APPLY(GA_F32, false, false); }
    } else {
        if ((addr & 7u) == 0) { if (stream_v) GA_LAYER_APPLY(GA_BF16, true, true); else GA_LAYER_APPLY(GA_BF16, true, false); }
        else { if (stream_v) GA_LAYER_APPLY(GA_BF16, false, true); else GA_LAYER_APPLY(GA_BF16, false, false); }
    }
#undef GA_LAYER_APPLY
    return hipGetLastError();
}

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

hipError_t launch_quadratic_gradient(const StatePtrs& st, uint64_t N, uint32_t worker, const float* a,
                                     const float* theta_star, uint64_t k, const RunConst& rc, float* g_out,
                                     hipStream_t stream) {
    const uint64_t groups = (N + 3) >> 2;
    const uint64_t blocks = (groups + kBlock - 1) / kBlock;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quadratic_gradient_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, stream,
                       st.snaps + (uint64_t)worker * st.stride, a, theta_star, N, k, rc, g_out);
    return hipGetLastError();
}

hipError_t launch_diagnostics(const StatePtrs& st, uint64_t N, uint32_t worker, float inv_bc, float eta_max,
                              float eps, DiagPartial* dev_partials, hipStream_t stream) {
    const uint32_t grid = blocks_for(N >> 2, (uint64_t)kBlock * 4, kDiagMaxBlocks);
    hipLaunchKernelGGL(diag_kernel, dim3(grid), dim3(kBlock), 0, stream, st.theta, st.m,
                       st.snaps + (uint64_t)worker * st.stride, N, inv_bc, eta_max, eps, dev_partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(diag_final_kernel, dim3(1), dim3(kBlock), 0, stream, dev_partials, grid,
                       dev_partials + kDiagMaxBlocks);
    return hipGetLastError();
}

hipError_t launch_box_muller_raw(const uint32_t* xa, const uint32_t* xb, uint64_t n, float* zc, float* zs,
                                 hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(box_muller_raw_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, xa, xb, n, zc, zs);
    return hipGetLastError();
}

hipError_t launch_noise_fill(uint64_t seed, uint64_t k, uint64_t j0, uint64_t n, float* out, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(noise_fill_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, (uint32_t)seed,
                       (uint32_t)(seed >> 32), k, j0, n, out);
    return hipGetLastError();
}

hipError_t launch_fill(float* dst, uint64_t n, float value, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_kernel, dim3(blocks_for(n, kBlock * 8, 65536)), dim3(kBlock), 0, stream, dst, n, value);
    return hipGetLastError();
}

hipError_t launch_broadcast_rows(float* dst, uint64_t stride, uint32_t rows, const float* src, uint64_t n,
                                 hipStream_t stream) {
    if (n == 0 || rows == 0) return hipSuccess;
    hipLaunchKernelGGL(broadcast_rows_kernel, dim3(blocks_for(n, kBlock * 4, 65536)), dim3(kBlock), 0, stream, dst,
                       stride, rows, src, n);
    return hipGetLastError();
}

}  // namespace ga
