// libga, gfx950: layer-wise and global Gap (Eq. 4, Def. 1): reduce, per-layer Gap, update.

#include "ga_device.h"

namespace ga {
namespace {

// ---------------------------------------------------------------------------
// Layer-wise and global Gap (Eq. 4, Def. 1).  Three launches per arrival:
//   layer_partial_kernel   one block per chunk of a layer: sum (theta-snap)^2 and sum m in double
//   layer_gap_kernel       one block per layer adds its chunk partials in a fixed order and forms G_p
//   layer_apply_kernel     one block per chunk: the momentum update with ghat = g / G_p
// A chunk never crosses a layer boundary; boundaries are arbitrary, so a chunk has a scalar
// head and tail around its 16-byte aligned body.  Every sum has a fixed order.
//
// When the caller already knows which worker arrives next, layer_apply_kernel<LOOK = true> also
// forms that arrival's chunk sums from the values it holds (the new theta and m) and the next
// worker's snapshot, so the separate reduction pass is not launched for it.  Both kernels give a
// thread the same elements in the same order and reduce the block the same way: the sums are
// the same bits either way.
// ---------------------------------------------------------------------------
constexpr int kLayerU = 4;   // 128-bit groups in flight per thread in the chunk kernels

__device__ __forceinline__ void gap_terms(double& d2, double& ms, float th, float s, float mm) {
    const float diff = th - s;
    d2 += (double)diff * (double)diff;
    ms += (double)mm;
}

// Wave butterfly, then the waves of the block in order; thread 0 stores the chunk's sums.
__device__ __forceinline__ void store_chunk_partial(double d2, double ms, LayerPartial* __restrict__ out) {
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
        LayerPartial p = {part[0][0], part[1][0]};
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) {
            p.dist2 += part[0][w];
            p.msum += part[1][w];
        }
        *out = p;
    }
}

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

// The 128-bit body of a chunk of the reduction pass; NT_TH: theta is read with the non-temporal hint.
template <bool NT_TH>
__device__ __forceinline__ void partial_body(const float* __restrict__ theta, const float* __restrict__ m,
                                             const float* __restrict__ snap, const ChunkRange& r, double& d2,
                                             double& ms) {
    const uint64_t q_end = r.a1 >> 2;
    for (uint64_t q0 = (r.a0 >> 2) + threadIdx.x; q0 < q_end; q0 += (uint64_t)kLayerU * kBlock) {
        f32x4 th[kLayerU], sv[kLayerU], mm[kLayerU];
#pragma unroll
        for (int u = 0; u < kLayerU; ++u) {
            const uint64_t q = q0 + (uint64_t)u * kBlock;
            if (q < q_end) {
                const uint64_t qs = state_index<4>(q);   // theta and m are tiled (ga_internal.h); a chunk may cross tiles
                th[u] = load4<NT_TH>(theta, qs);
                sv[u] = load4<true>(snap, q);
                mm[u] = load4<true>(m, qs);
            }
        }
#pragma unroll
        for (int u = 0; u < kLayerU; ++u) {
            if (q0 + (uint64_t)u * kBlock < q_end) {
                gap_terms(d2, ms, th[u].x, sv[u].x, mm[u].x); gap_terms(d2, ms, th[u].y, sv[u].y, mm[u].y);
                gap_terms(d2, ms, th[u].z, sv[u].z, mm[u].z); gap_terms(d2, ms, th[u].w, sv[u].w, mm[u].w);
            }
        }
    }
}

// keep_theta: parameters [0, keep_theta) of theta are read without the hint (the part the update keeps in the
// memory-side cache, see ga_device.h)
__global__ __launch_bounds__(kBlock) void layer_partial_kernel(const float* __restrict__ theta,
                                                               const float* __restrict__ m,
                                                               const float* __restrict__ snap,
                                                               const LayerChunk* __restrict__ chunks,
                                                               LayerPartial* __restrict__ partials,
                                                               uint64_t keep_theta) {
    const ChunkRange r = chunk_range(chunks[blockIdx.x]);
    double d2 = 0.0, ms = 0.0;
    auto scalar = [&](uint64_t j) {
        const uint64_t js = state_index<1>(j);
        gap_terms(d2, ms, theta[js], snap[j], m[js]);
    };
    for (uint64_t j = r.start + threadIdx.x; j < r.a0; j += kBlock) scalar(j);
    if (r.end <= keep_theta) GA_HINT_PATH("theta kept", partial_body<false>(theta, m, snap, r, d2, ms));
    else GA_HINT_PATH("all streamed", partial_body<true>(theta, m, snap, r, d2, ms));
    for (uint64_t j = r.a1 + threadIdx.x; j < r.end; j += kBlock) scalar(j);
    store_chunk_partial(d2, ms, partials + blockIdx.x);
}

template <bool HINGE>
__global__ __launch_bounds__(kBlock) void layer_gap_kernel(const LayerPartial* __restrict__ partials,
                                                           const LayerSpan* __restrict__ spans, float inv_bc_prev,
                                                           float eta_max, float eps, float* __restrict__ gaps) {
    // one block per layer: strided partial sums, 64-lane butterfly, then the waves in order
    const LayerSpan sp = spans[blockIdx.x];
    double d2 = 0.0, ms = 0.0;
    constexpr int B = 8;   // loads in flight per thread; the additions keep their order
    for (uint32_t i0 = threadIdx.x; i0 < sp.n_chunks; i0 += B * kBlock) {
        LayerPartial p[B];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const uint32_t i = i0 + b * kBlock;
            p[b] = i < sp.n_chunks ? partials[sp.first_chunk + i] : LayerPartial{0.0, 0.0};
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            if (i0 + b * kBlock < sp.n_chunks) {
                d2 += p[b].dist2;
                ms += p[b].msum;
            }
        }
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

// The 128-bit body of a chunk of the update pass.  NT_TH / NT_V: theta / v carry the non-temporal hint.
template <int DT, bool ALIGNED, bool NAG, bool LOOK, bool NT_TH, bool NT_V>
__device__ __forceinline__ void apply_body(float* __restrict__ theta, float* __restrict__ v, float* __restrict__ m,
                                           float* __restrict__ snap, const void* __restrict__ g,
                                           const ChunkRange& r, float G, const StepConst& c,
                                           const float* __restrict__ next_snap, double& d2, double& ms) {
    constexpr int U = 2;
    const uint64_t q_end = r.a1 >> 2;
    for (uint64_t q0 = (r.a0 >> 2) + threadIdx.x; q0 < q_end; q0 += (uint64_t)U * kBlock) {
        f32x4 th[U], vv[U], mm[U], gg[U], nx[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t q = q0 + (uint64_t)u * kBlock;
            if (q < q_end) {
                const uint64_t qs = state_index<4>(q);   // theta, v, m are tiled; a chunk may cross tiles
                th[u] = load4<NT_TH>(theta, qs);
                vv[u] = load4<NT_V>(v, qs);
                mm[u] = load4<true>(m, qs);
                gg[u] = load_g4<DT, ALIGNED>(g, q);
                if constexpr (LOOK)
                    if (next_snap) nx[u] = load4<true>(next_snap, q);
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
                    if constexpr (LOOK) gap_terms(d2, ms, t1, next_snap ? nx[u][e] : t1, m1);
                    th[u][e] = t1; vv[u][e] = v1; mm[u][e] = m1;
                }
                const uint64_t qs = state_index<4>(q);
                store4<NT_TH>(theta, qs, th[u]);
                store4<NT_V>(v, qs, vv[u]);
                store4<true>(m, qs, mm[u]);
                store4<true>(snap, q, th[u]);
            }
        }
    }
}

// LOOK: also leave the chunk sums of the arrival that follows.  next_snap is the next worker's
// snapshot, or null when the same worker arrives again (its snapshot is the theta written here:
// the distance is zero).  keep_theta >= keep_v: the leading parameters whose theta / v stay in the
// memory-side cache (accessed without the hint), as in the parameter-wise kernel.
template <int DT, bool ALIGNED, bool NAG, bool LOOK>
__global__ __launch_bounds__(kBlock) void layer_apply_kernel(float* __restrict__ theta, float* __restrict__ v,
                                                             float* __restrict__ m, float* __restrict__ snap,
                                                             const void* __restrict__ g,
                                                             const LayerChunk* __restrict__ chunks,
                                                             const float* __restrict__ gaps, StepConst c,
                                                             const float* __restrict__ next_snap,
                                                             LayerPartial* __restrict__ partials,
                                                             uint64_t keep_theta, uint64_t keep_v) {
    const LayerChunk ch = chunks[blockIdx.x];
    const ChunkRange r = chunk_range(ch);
    const float G = gaps[ch.layer];
    double d2 = 0.0, ms = 0.0;
    auto scalar = [&](uint64_t j) {
        const uint64_t js = state_index<1>(j);
        float t1 = theta[js], v1 = v[js], m1 = m[js];
        layer_update_one<NAG>(t1, v1, m1, load_g1<DT>(g, j), G, c);
        if constexpr (LOOK) gap_terms(d2, ms, t1, next_snap ? next_snap[j] : t1, m1);
        theta[js] = t1; v[js] = v1; m[js] = m1; snap[j] = t1;
    };
    for (uint64_t j = r.start + threadIdx.x; j < r.a0; j += kBlock) scalar(j);
#define GA_LAYER_BODY(NT_TH, NT_V) \
    apply_body<DT, ALIGNED, NAG, LOOK, NT_TH, NT_V>(theta, v, m, snap, g, r, G, c, next_snap, d2, ms)
    if (r.end > keep_theta) GA_HINT_PATH("all streamed", GA_LAYER_BODY(true, true));
    else if (r.end > keep_v) GA_HINT_PATH("theta kept", GA_LAYER_BODY(false, true));
    else GA_HINT_PATH("theta and v kept", GA_LAYER_BODY(false, false));
#undef GA_LAYER_BODY
    for (uint64_t j = r.a1 + threadIdx.x; j < r.end; j += kBlock) scalar(j);
    if constexpr (LOOK) store_chunk_partial(d2, ms, partials + blockIdx.x);
}

}  // namespace

hipError_t launch_apply_layerwise(const StatePtrs& st, uint64_t N, uint32_t worker, const void* g, int grad_dtype,
                                  int mode, bool nesterov, const LayerTables& lt, const StepConst& c,
                                  bool sums_ready, int64_t next_worker, hipStream_t stream) {
    if (lt.n_chunks == 0 || lt.n_layers == 0) return hipErrorInvalidValue;
    float* snap = st.snaps + (uint64_t)worker * st.stride;
    const dim3 block(kBlock), grid(lt.n_chunks), lgrid(lt.n_layers);
    // leading parameters whose theta, then v, stay in the memory-side cache
    const uint64_t budget = st.resident_bytes / sizeof(float);
    const uint64_t keep_theta = N < budget ? N : budget;
    const uint64_t keep_v = N < budget - keep_theta ? N : budget - keep_theta;
    if (!sums_ready)
        hipLaunchKernelGGL(layer_partial_kernel, grid, block, 0, stream, st.theta, st.m, snap, lt.chunks, lt.partials,
                           keep_theta);
    if (mode == GA_MODE_GA_HINGE)
        hipLaunchKernelGGL(layer_gap_kernel<true>, lgrid, block, 0, stream, lt.partials, lt.spans, c.inv_bc_prev,
                           c.eta_max, c.eps, lt.gaps);
    else
        hipLaunchKernelGGL(layer_gap_kernel<false>, lgrid, block, 0, stream, lt.partials, lt.spans, c.inv_bc_prev,
                           c.eta_max, c.eps, lt.gaps);
    const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
    const bool look = next_worker >= 0;
    const float* next_snap =
        (look && (uint32_t)next_worker != worker) ? st.snaps + (uint64_t)next_worker * st.stride : nullptr;
#define GA_LAYER_APPLY3(DT, AL, NG, LK)                                                                         \
    hipLaunchKernelGGL((layer_apply_kernel<DT, AL, NG, LK>), grid, block, 0, stream, st.theta, st.v, st.m, snap, \
                       g, lt.chunks, lt.gaps, c, next_snap, lt.partials, keep_theta, keep_v)
#define GA_LAYER_APPLY(DT, AL)                                                                                  \
    do {                                                                                                        \
        if (nesterov) { if (look) GA_LAYER_APPLY3(DT, AL, true, true); else GA_LAYER_APPLY3(DT, AL, true, false); } \
        else { if (look) GA_LAYER_APPLY3(DT, AL, false, true); else GA_LAYER_APPLY3(DT, AL, false, false); }    \
    } while (0)
    if (grad_dtype == GA_F32) {
        if ((addr & 15u) == 0) GA_LAYER_APPLY(GA_F32, true);
        else GA_LAYER_APPLY(GA_F32, false);
    } else {
        if ((addr & 7u) == 0) GA_LAYER_APPLY(GA_BF16, true);
        else GA_LAYER_APPLY(GA_BF16, false);
    }
#undef GA_LAYER_APPLY
#undef GA_LAYER_APPLY3
    return hipGetLastError();
}

}  // namespace ga
