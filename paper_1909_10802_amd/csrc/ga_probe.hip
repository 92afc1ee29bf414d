// libga, gfx950: measurement aids behind `bench.py --ceiling`.  They run none of the method's arithmetic; they
// measure what this part delivers for the access pattern and the instruction mix of the kernels, so that the
// roofline fractions quoted for those kernels can be re-derived on any machine:
//   stream_probe_kernel   R arrays read and W arrays written at once, 128-bit accesses with the non-temporal hint
//                         (the first KEEP read and written arrays without it: data held in the memory-side cache;
//                         TILED: the first three as the tile-interleaved state arrays of a master),
//                         the launch shape of the fused update (one group of four per thread)
//   valu_probe_kernel     8 independent instructions of one kind per loop iteration

#include <utility>

#include "ga_device.h"

namespace ga {
namespace {

constexpr int kProbeMaxStreams = 6;
struct ProbePtrs {
    const float* r[kProbeMaxStreams];
    float* w[kProbeMaxStreams];
};

// Streams I = 0 .. of one group: the first KEEP without the hint.  The choice is made per instantiation (a fold over
// the stream indices): a run-time or loop-carried choice between two accesses that differ only in the hint is merged
// by the optimiser, which drops the hint.
// TILED: the first three arrays are the three tile-interleaved state arrays of a master (ga_internal.h): group q of
// each is at state_index<4>(q) from its pointer.
template <int KEEP, bool TILED, int... I>
__device__ __forceinline__ f32x4 probe_load(const ProbePtrs& p, uint64_t q, uint64_t qs, std::integer_sequence<int, I...>) {
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    ((acc += load4<(I >= KEEP)>(p.r[I], (TILED && I < 3) ? qs : q)), ...);
    return acc;
}
template <int KEEP, bool TILED, int... I>
__device__ __forceinline__ void probe_store(const ProbePtrs& p, uint64_t q, uint64_t qs, const f32x4& acc,
                                            std::integer_sequence<int, I...>) {
    ((store4<(I >= KEEP)>(p.w[I], (TILED && I < 3) ? qs : q, acc + (float)I)), ...);
}

// An output may be the input of the same index (an update in place): a thread loads its group before it stores it.
template <int R, int W, int KEEP, bool TILED>
__global__ __launch_bounds__(kBlock) void stream_probe_kernel(ProbePtrs p, uint64_t n4) {
    const uint64_t q = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (q >= n4) return;
    const uint64_t qs = state_index<4>(q);
    const f32x4 acc = probe_load<KEEP, TILED>(p, q, qs, std::make_integer_sequence<int, R>{});
    probe_store<KEEP, TILED>(p, q, qs, acc, std::make_integer_sequence<int, W>{});
    if constexpr (W == 0)
        if (acc.x == 12345.678f) const_cast<float*>(p.r[0])[0] = acc.y;   // keeps the loads alive; never true for the probe's data
}

#define GA_PROBE_KERNEL(NAME, INSTR)                                                                               \
    __global__ __launch_bounds__(kBlock) void NAME(uint32_t* out, uint32_t iterations, uint32_t seed) {            \
        uint32_t a0 = threadIdx.x + seed, a1 = a0 * 3 + 1, a2 = a0 * 5 + 2, a3 = a0 * 7 + 3;                       \
        uint32_t a4 = a0 * 11 + 4, a5 = a0 * 13 + 5, a6 = a0 * 17 + 6, a7 = a0 * 19 + 7;                           \
        const uint32_t b = seed | 0x3f800001u;                                                                     \
        for (uint32_t i = 0; i < iterations; ++i)                                                                  \
            asm volatile(INSTR(0) INSTR(1) INSTR(2) INSTR(3) INSTR(4) INSTR(5) INSTR(6) INSTR(7)                   \
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)          \
                         : "v"(b)                                                                                  \
                         : "vcc");                                                                                 \
        if ((a0 ^ a1 ^ a2 ^ a3 ^ a4 ^ a5 ^ a6 ^ a7) == 0x12345678u) out[0] = a0;                                   \
    }
#define GA_I_FMA(n) "v_fma_f32 %" #n ", %" #n ", %8, %" #n "\n"
#define GA_I_XOR(n) "v_xor_b32 %" #n ", %" #n ", %8\n"
#define GA_I_MULHI(n) "v_mul_hi_u32 %" #n ", %" #n ", %8\n"
#define GA_I_RCP(n) "v_rcp_f32 %" #n ", %" #n "\n"
#define GA_I_SQRT(n) "v_sqrt_f32 %" #n ", %" #n "\n"
#define GA_I_DIVSCALE(n) "v_div_scale_f32 %" #n ", vcc, %" #n ", %8, %" #n "\n"
#define GA_I_DIVFMAS(n) "v_div_fmas_f32 %" #n ", %" #n ", %8, %" #n "\n"
#define GA_I_DIVFIXUP(n) "v_div_fixup_f32 %" #n ", %" #n ", %8, %" #n "\n"
GA_PROBE_KERNEL(valu_fma_kernel, GA_I_FMA)
GA_PROBE_KERNEL(valu_xor_kernel, GA_I_XOR)
GA_PROBE_KERNEL(valu_mulhi_kernel, GA_I_MULHI)
GA_PROBE_KERNEL(valu_rcp_kernel, GA_I_RCP)
GA_PROBE_KERNEL(valu_sqrt_kernel, GA_I_SQRT)
GA_PROBE_KERNEL(valu_divscale_kernel, GA_I_DIVSCALE)
GA_PROBE_KERNEL(valu_divfmas_kernel, GA_I_DIVFMAS)
GA_PROBE_KERNEL(valu_divfixup_kernel, GA_I_DIVFIXUP)

// 32 x 32 -> 64-bit multiply-add (Philox): one instruction gives the high and the low word
__global__ __launch_bounds__(kBlock) void valu_mad64_kernel(uint32_t* out, uint32_t iterations, uint32_t seed) {
    uint64_t a0 = threadIdx.x + seed, a1 = a0 * 3 + 1, a2 = a0 * 5 + 2, a3 = a0 * 7 + 3;
    const uint32_t b = seed | 0x3f800001u;
    for (uint32_t i = 0; i < iterations; ++i)
        asm volatile("v_mad_u64_u32 %0, vcc, %4, %4, %0\nv_mad_u64_u32 %1, vcc, %4, %4, %1\n"
                     "v_mad_u64_u32 %2, vcc, %4, %4, %2\nv_mad_u64_u32 %3, vcc, %4, %4, %3\n"
                     "v_mad_u64_u32 %0, vcc, %4, %4, %0\nv_mad_u64_u32 %1, vcc, %4, %4, %1\n"
                     "v_mad_u64_u32 %2, vcc, %4, %4, %2\nv_mad_u64_u32 %3, vcc, %4, %4, %3\n"
                     : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3)
                     : "v"(b)
                     : "vcc");
    if ((a0 ^ a1 ^ a2 ^ a3) == 0x12345678ull) out[0] = (uint32_t)a0;
}

template <int R, int KEEP, bool TILED>
hipError_t launch_streams_w(const ProbePtrs& p, uint32_t n_write, uint64_t n4, dim3 grid, hipStream_t stream) {
    switch (n_write) {
        case 0: hipLaunchKernelGGL((stream_probe_kernel<R, 0, KEEP, TILED>), grid, dim3(kBlock), 0, stream, p, n4); break;
        case 1: hipLaunchKernelGGL((stream_probe_kernel<R, 1, KEEP, TILED>), grid, dim3(kBlock), 0, stream, p, n4); break;
        case 2: hipLaunchKernelGGL((stream_probe_kernel<R, 2, KEEP, TILED>), grid, dim3(kBlock), 0, stream, p, n4); break;
        case 4: hipLaunchKernelGGL((stream_probe_kernel<R, 4, KEEP, TILED>), grid, dim3(kBlock), 0, stream, p, n4); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int KEEP, bool TILED>
hipError_t launch_streams_r(const ProbePtrs& p, uint32_t n_read, uint32_t n_write, uint64_t n4, dim3 grid,
                            hipStream_t stream) {
    switch (n_read) {
        case 0: return launch_streams_w<0, KEEP, TILED>(p, n_write, n4, grid, stream);
        case 1: return launch_streams_w<1, KEEP, TILED>(p, n_write, n4, grid, stream);
        case 2: return launch_streams_w<2, KEEP, TILED>(p, n_write, n4, grid, stream);
        case 4: return launch_streams_w<4, KEEP, TILED>(p, n_write, n4, grid, stream);
        case 5: return launch_streams_w<5, KEEP, TILED>(p, n_write, n4, grid, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_probe_streams(uint32_t n_read, uint32_t n_write, uint32_t n_resident, bool tiled, uint64_t n,
                                const float* const* reads, float* const* writes, hipStream_t stream) {
    if (n_read > (uint32_t)kProbeMaxStreams || n_write > (uint32_t)kProbeMaxStreams || n_read + n_write == 0)
        return hipErrorInvalidValue;
    ProbePtrs p = {};
    for (uint32_t i = 0; i < n_read; ++i) p.r[i] = reads[i];
    for (uint32_t i = 0; i < n_write; ++i) p.w[i] = writes[i];
    const uint64_t n4 = n >> 2;
    const uint64_t blocks = (n4 + kBlock - 1) / kBlock;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)blocks);
    switch (n_resident * 2 + (tiled ? 1 : 0)) {
        case 0: return launch_streams_r<0, false>(p, n_read, n_write, n4, grid, stream);
        case 1: return launch_streams_r<0, true>(p, n_read, n_write, n4, grid, stream);
        case 2: return launch_streams_r<1, false>(p, n_read, n_write, n4, grid, stream);
        case 3: return launch_streams_r<1, true>(p, n_read, n_write, n4, grid, stream);
        case 4: return launch_streams_r<2, false>(p, n_read, n_write, n4, grid, stream);
        case 5: return launch_streams_r<2, true>(p, n_read, n_write, n4, grid, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_probe_valu(int op, uint32_t blocks, uint32_t iterations, uint32_t* dev_out, hipStream_t stream) {
    if (blocks == 0) return hipErrorInvalidValue;
    const dim3 grid(blocks), block(kBlock);
#define GA_PROBE_LAUNCH(K) hipLaunchKernelGGL(K, grid, block, 0, stream, dev_out, iterations, 1u)
    switch (op) {
        case GA_PROBE_FMA: GA_PROBE_LAUNCH(valu_fma_kernel); break;
        case GA_PROBE_XOR: GA_PROBE_LAUNCH(valu_xor_kernel); break;
        case GA_PROBE_MUL_HI: GA_PROBE_LAUNCH(valu_mulhi_kernel); break;
        case GA_PROBE_MAD_U64: GA_PROBE_LAUNCH(valu_mad64_kernel); break;
        case GA_PROBE_RCP: GA_PROBE_LAUNCH(valu_rcp_kernel); break;
        case GA_PROBE_SQRT: GA_PROBE_LAUNCH(valu_sqrt_kernel); break;
        case GA_PROBE_DIV_SCALE: GA_PROBE_LAUNCH(valu_divscale_kernel); break;
        case GA_PROBE_DIV_FMAS: GA_PROBE_LAUNCH(valu_divfmas_kernel); break;
        case GA_PROBE_DIV_FIXUP: GA_PROBE_LAUNCH(valu_divfixup_kernel); break;
        default: return hipErrorInvalidValue;
    }
#undef GA_PROBE_LAUNCH
    return hipGetLastError();
}

}  // namespace ga
