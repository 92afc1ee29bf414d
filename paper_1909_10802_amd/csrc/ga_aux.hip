// libga, gfx950: the gradient source alone (quadratic_gradient_kernel, noise_fill_kernel,
// box_muller_raw_kernel), Gap statistics (diag_kernel + diag_final_kernel, App. C.8) and fills.

#include <mutex>

#include "ga_device.h"

namespace ga {
namespace {

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

// SROWS: snapshot_rows of the master's family (ga_internal.h).
template <int SROWS>
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
        const f32x4 s = reinterpret_cast<const f32x4*>(snap)[row_index<4, SROWS>(q)];
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
            g_out[j0 + e] = quadratic_g(snap[row_index<1, SROWS>(j0 + e)], a[j0 + e], ts[j0 + e], rc.sigma, zz[e]);
    }
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

// One block's groups [q0, q1): thread t takes q0 + t, q0 + t + kBlock, ..., two in flight, accumulated in that order.
// NT_TH: theta is read with the non-temporal hint.
// ROWS: theta and m are tiled state arrays of a master with that many arrays per tile (ga_internal.h); 0: plain
// arrays of the caller.
template <bool NT_TH, int ROWS, int SROWS>
__device__ __forceinline__ void diag_span(DiagAcc& acc, const float* __restrict__ theta, const float* __restrict__ m,
                                          const float* __restrict__ snap, uint64_t q0, uint64_t q1, float inv_bc,
                                          float eta_max, float eps) {
    constexpr int U = 2;
    for (uint64_t q = q0 + threadIdx.x; q < q1; q += (uint64_t)U * kBlock) {
        f32x4 th[U], s[U], mm[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t qu = q + (uint64_t)u * kBlock;
            if (qu < q1) {
                const uint64_t qs = ROWS ? state_index<4, ROWS ? ROWS : 3>(qu) : qu;
                th[u] = load4<NT_TH>(theta, qs);
                s[u] = load4<true>(snap, row_index<4, SROWS>(qu));
                mm[u] = load4<true>(m, qs);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (q + (uint64_t)u * kBlock < q1) {
                diag_one(acc, th[u].x, s[u].x, mm[u].x, inv_bc, eta_max, eps);
                diag_one(acc, th[u].y, s[u].y, mm[u].y, inv_bc, eta_max, eps);
                diag_one(acc, th[u].z, s[u].z, mm[u].z, inv_bc, eta_max, eps);
                diag_one(acc, th[u].w, s[u].w, mm[u].w, inv_bc, eta_max, eps);
            }
        }
    }
}

// Block b reads the contiguous groups [b * per_block, (b + 1) * per_block) of the three arrays (a grid-stride walk
// over the same data is a quarter slower at 10^8 parameters).  keep_q: a block whose groups all lie below keep_q
// reads theta without the hint (the part the update kernels keep in the memory-side cache); reading the rest of
// theta without it would push that part out.
template <int ROWS, int SROWS>
__global__ __launch_bounds__(kBlock) void diag_kernel(const float* __restrict__ theta, const float* __restrict__ m,
                                                      const float* __restrict__ snap, uint64_t N, float inv_bc,
                                                      float eta_max, float eps, uint64_t per_block, uint64_t keep_q,
                                                      DiagPartial* __restrict__ partials) {
    const uint64_t n4 = N >> 2;
    DiagAcc acc = {0.0, 0u, 0u, 0u};
    const uint64_t q0 = (uint64_t)blockIdx.x * per_block;
    const uint64_t q1 = q0 + per_block < n4 ? q0 + per_block : n4;
    if (q1 <= keep_q) GA_HINT_PATH("theta kept", diag_span<false, ROWS, SROWS>(acc, theta, m, snap, q0, q1, inv_bc, eta_max, eps));
    else GA_HINT_PATH("all streamed", diag_span<true, ROWS, SROWS>(acc, theta, m, snap, q0, q1, inv_bc, eta_max, eps));
    if (blockIdx.x == 0 && threadIdx.x < (N & 3)) {
        const uint64_t j = 4 * n4 + threadIdx.x, js = ROWS ? state_index<1, ROWS ? ROWS : 3>(j) : j;
        diag_one(acc, theta[js], snap[row_index<1, SROWS>(j)], m[js], inv_bc, eta_max, eps);
    }
    const DiagPartial r = block_reduce(acc.sum, acc.gt1, acc.gt0, acc.bad);
    if (threadIdx.x == 0) partials[blockIdx.x] = r;
}

// Launch shape of diag_kernel: at most kDiagMaxBlocks blocks (all resident at once on 256 compute units), each with a
// whole number of block-wide steps.
struct DiagShape {
    uint32_t grid;
    uint64_t per_block;
};
inline DiagShape diag_shape(uint64_t N) {
    const uint64_t n4 = N >> 2;
    DiagShape d;
    d.grid = blocks_for(n4, (uint64_t)kBlock * 4, kDiagMaxBlocks);
    d.per_block = ((n4 + d.grid - 1) / d.grid + kBlock - 1) / kBlock * kBlock;
    if (d.per_block == 0) d.per_block = kBlock;
    return d;
}

// All partials added by one block in a fixed order; every thread returns the total.
__device__ __forceinline__ DiagPartial add_partials(const DiagPartial* __restrict__ partials, uint32_t n_partials) {
    double sum = 0.0;
    unsigned long long gt1 = 0, gt0 = 0, bad = 0;
    constexpr uint32_t U = 4;   // loads in flight per thread
    for (uint32_t i = threadIdx.x; i < n_partials; i += U * kBlock) {
        DiagPartial p[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
            if (i + u * kBlock < n_partials) p[u] = partials[i + u * kBlock];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (i + u * kBlock < n_partials) {
                sum += p[u].sum_graw;
                gt1 += p[u].n_gt1;
                gt0 += p[u].n_gt0;
                bad += p[u].n_bad;
            }
        }
    }
    return block_reduce(sum, gt1, gt0, bad);
}

__global__ __launch_bounds__(kBlock) void diag_final_kernel(const DiagPartial* __restrict__ partials,
                                                            uint32_t n_partials, DiagPartial* __restrict__ total) {
    const DiagPartial r = add_partials(partials, n_partials);
    if (threadIdx.x == 0) *total = r;
}

// The same total turned into the report on the device (the divisions are IEEE double divisions, as on the host).
__global__ __launch_bounds__(kBlock) void diag_report_kernel(const DiagPartial* __restrict__ partials,
                                                             uint32_t n_partials, uint64_t N,
                                                             ga_diag* __restrict__ out) {
    const DiagPartial r = add_partials(partials, n_partials);
    if (threadIdx.x == 0) {
        const double n = (double)N;
        out->mean_graw = r.sum_graw / n;
        out->frac_gt1 = (double)r.n_gt1 / n;
        out->frac_gt0 = (double)r.n_gt0 / n;
        out->n_nonfinite = r.n_bad;
    }
}

// Reduction partials for callers that bring no workspace and cannot allocate one: one copy of this array per
// GPU, held until the process ends, shared by every such call on that GPU.  In host code `scratch` is only a
// handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) DiagPartial scratch[kDiagMaxBlocks];
static_assert(sizeof(DiagPartial) * kDiagMaxBlocks == GA_STATIC_SCRATCH_BYTES, "documented size of the static scratch array");

constexpr int kMaxDevices = 64;
DiagPartial* scratch_of_device[kMaxDevices];   // device address of `scratch` on each GPU, resolved on first use
std::mutex scratch_lock;

// ---------------------------------------------------------------------------
// Fills.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void fill_kernel(float* __restrict__ dst, uint64_t n, float value) {
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock)
        dst[i] = value;
}

// One tiled state array (theta, v or m of a master; ga_internal.h) copied to or from a plain array of n floats.
template <bool TO_STATE, int ROWS>
__global__ __launch_bounds__(kBlock) void state_copy_kernel(float* __restrict__ state, float* __restrict__ plain, uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) {
        if constexpr (TO_STATE) state[state_index<1, ROWS>(i)] = plain[i];
        else plain[i] = state[state_index<1, ROWS>(i)];
    }
}

template <int SROWS>
__global__ __launch_bounds__(kBlock) void broadcast_rows_kernel(float* __restrict__ dst, uint64_t stride,
                                                                uint32_t rows, const float* __restrict__ src,
                                                                uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) {
        const float x = src[i];
        const uint64_t ir = row_index<1, SROWS>(i);
        for (uint32_t r = 0; r < rows; ++r) dst[(uint64_t)r * stride + ir] = x;
    }
}

}  // namespace

hipError_t launch_quadratic_gradient(const StatePtrs& st, uint64_t N, uint32_t worker, const float* a,
                                     const float* theta_star, uint64_t k, const RunConst& rc, float* g_out,
                                     hipStream_t stream) {
    const uint64_t groups = (N + 3) >> 2;
    const uint64_t blocks = (groups + kBlock - 1) / kBlock;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (st.snap_rows == 2)
        hipLaunchKernelGGL(quadratic_gradient_kernel<2>, dim3((uint32_t)blocks), dim3(kBlock), 0, stream,
                           st.snaps + (uint64_t)worker * st.stride, a, theta_star, N, k, rc, g_out);
    else
        hipLaunchKernelGGL(quadratic_gradient_kernel<1>, dim3((uint32_t)blocks), dim3(kBlock), 0, stream,
                           st.snaps + (uint64_t)worker * st.stride, a, theta_star, N, k, rc, g_out);
    return hipGetLastError();
}

hipError_t launch_diagnostics(const StatePtrs& st, uint64_t N, uint32_t worker, float inv_bc, float eta_max,
                              float eps, DiagPartial* dev_partials, ga_diag* dev_report, hipStream_t stream) {
    const DiagShape shape = diag_shape(N);
    const uint32_t grid = shape.grid;
#define GA_DIAG(ROWS, SROWS)                                                                                       \
    hipLaunchKernelGGL((diag_kernel<ROWS, SROWS>), dim3(grid), dim3(kBlock), 0, stream, st.theta, st.m,             \
                       st.snaps + (uint64_t)worker * st.stride, N, inv_bc, eta_max, eps, shape.per_block,           \
                       st.resident_bytes / sizeof(f32x4), dev_partials)
    if (st.rows == 4) GA_DIAG(4, 1);
    else if (st.snap_rows == 2) GA_DIAG(3, 2);
    else GA_DIAG(3, 1);
#undef GA_DIAG
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (dev_report)
        hipLaunchKernelGGL(diag_report_kernel, dim3(1), dim3(kBlock), 0, stream, dev_partials, grid, N, dev_report);
    else
        hipLaunchKernelGGL(diag_final_kernel, dim3(1), dim3(kBlock), 0, stream, dev_partials, grid,
                           dev_partials + kDiagMaxBlocks);
    return hipGetLastError();
}

hipError_t static_scratch_address(DiagPartial** out) {
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_of_device[device]) {
        DiagPartial* p = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_of_device[device] = p;
    }
    *out = scratch_of_device[device];
    return hipSuccess;
}

hipError_t launch_diagnostics_static(const float* theta, const float* snap, const float* m, uint64_t N, float inv_bc,
                                     float eta_max, float eps, ga_diag* dev_report, hipStream_t stream) {
    DiagPartial* partials = nullptr;
    hipError_t e = static_scratch_address(&partials);
    if (e != hipSuccess) return e;
    // every partial that the report kernel reads is written by this launch first: nothing has to start at zero
    const DiagShape shape = diag_shape(N);
    const uint32_t grid = shape.grid;
    hipLaunchKernelGGL((diag_kernel<0, 1>), dim3(grid), dim3(kBlock), 0, stream, theta, m, snap, N, inv_bc, eta_max, eps,
                       shape.per_block, kResidentBytes / sizeof(f32x4), partials);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(diag_report_kernel, dim3(1), dim3(kBlock), 0, stream, partials, grid, N, dev_report);
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

hipError_t launch_broadcast_rows(float* dst, uint64_t stride, uint32_t rows, int snap_rows, const float* src, uint64_t n,
                                 hipStream_t stream) {
    if (n == 0 || rows == 0) return hipSuccess;
    const dim3 grid(blocks_for(n, kBlock * 4, 65536)), block(kBlock);
    if (snap_rows == 2) hipLaunchKernelGGL(broadcast_rows_kernel<2>, grid, block, 0, stream, dst, stride, rows, src, n);
    else hipLaunchKernelGGL(broadcast_rows_kernel<1>, grid, block, 0, stream, dst, stride, rows, src, n);
    return hipGetLastError();
}

hipError_t launch_state_get(const float* state, int rows, float* dst, uint64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const dim3 grid(blocks_for(n, kBlock * 8, 65536)), block(kBlock);
    if (rows == 4) hipLaunchKernelGGL((state_copy_kernel<false, 4>), grid, block, 0, stream, const_cast<float*>(state), dst, n);
    else if (rows == 2) hipLaunchKernelGGL((state_copy_kernel<false, 2>), grid, block, 0, stream, const_cast<float*>(state), dst, n);
    else if (rows == 3) hipLaunchKernelGGL((state_copy_kernel<false, 3>), grid, block, 0, stream, const_cast<float*>(state), dst, n);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_state_put(float* state, int rows, const float* src, uint64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const dim3 grid(blocks_for(n, kBlock * 8, 65536)), block(kBlock);
    if (rows == 4) hipLaunchKernelGGL((state_copy_kernel<true, 4>), grid, block, 0, stream, state, const_cast<float*>(src), n);
    else if (rows == 2) hipLaunchKernelGGL((state_copy_kernel<true, 2>), grid, block, 0, stream, state, const_cast<float*>(src), n);
    else if (rows == 3) hipLaunchKernelGGL((state_copy_kernel<true, 3>), grid, block, 0, stream, state, const_cast<float*>(src), n);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ga
