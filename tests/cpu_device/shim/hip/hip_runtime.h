// Test scaffolding (CPU only).  Found in place of the HIP device header when the library's kernel sources are
// compiled as ordinary C++ for the host: every kernel then runs on the CPU, one fiber per GPU thread, block after
// block, under AddressSanitizer and UndefinedBehaviorSanitizer, so that indexing and launch shapes are checked for
// every access and the results can be compared with the oracle without a GPU.  Nothing here is used by the product.
#ifndef GA_TEST_CPU_DEVICE_HIP_RUNTIME_H
#define GA_TEST_CPU_DEVICE_HIP_RUNTIME_H

#include <hip/hip_runtime_api.h>   // the real API header: types, error codes, host function declarations

#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>

// the API header brings host-side meanings of the device keywords; here a kernel is an ordinary function
#undef __global__
#undef __device__
#undef __host__
#undef __forceinline__
#undef __launch_bounds__
#undef __shared__
#undef __align__
#undef HIP_SYMBOL
#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __launch_bounds__(...)
#define __shared__ static   // one copy for the block that is running: blocks run one after another
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) x   // the API header's C++ overload of hipGetSymbolAddress takes the variable itself

// the cache-hint paths need no markers here (and an x86 assembler would not take them)
#define GA_HINT_PATH(name, ...) \
    do {                        \
        __VA_ARGS__;            \
    } while (0)

// the hardware's approximate reciprocal and square root: any value within 1 ulp serves the callers' corrections
#define __builtin_amdgcn_rcpf(x) (1.0f / (x))
#define __builtin_amdgcn_sqrtf(x) (::sqrtf(x))

using std::isfinite;

namespace cpu_device {
struct Index {
    uint32_t x, y, z;
};
void launch(dim3 grid, dim3 block, const std::function<void()>& thread_body);
void sync_block();
uint64_t shuffle_xor_bits(uint64_t bits, int lane_mask);
}  // namespace cpu_device

extern cpu_device::Index threadIdx, blockIdx;
extern dim3 blockDim, gridDim;

#undef hipLaunchKernelGGL
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
    ((void)(stream), ::cpu_device::launch(dim3(grid), dim3(block), [=]() { kernel(__VA_ARGS__); }))

inline void __syncthreads() { cpu_device::sync_block(); }

template <typename T>
inline T __shfl_xor(T value, int lane_mask, int width = 64) {
    static_assert(sizeof(T) <= 8, "shuffle of at most 64 bits");
    (void)width;
    uint64_t bits = 0;
    std::memcpy(&bits, &value, sizeof(T));
    bits = cpu_device::shuffle_xor_bits(bits, lane_mask);
    T out;
    std::memcpy(&out, &bits, sizeof(T));
    return out;
}

inline uint32_t __float_as_uint(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    return u;
}
inline float __uint_as_float(uint32_t u) {
    float x;
    std::memcpy(&x, &u, 4);
    return x;
}

#endif
