// Test scaffolding (CPU only): stand-ins for the HIP runtime calls that the library's host code makes.  "Device"
// memory is host memory, a copy is a memmove, streams and events are formalities: everything completes at once.
#include <hip/hip_runtime_api.h>

#include <cstdlib>
#include <cstring>

extern "C" {
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind, hipStream_t) {
    std::memmove(dst, src, bytes);
    return hipSuccess;
}
hipError_t hipHostMalloc(void** p, size_t bytes, unsigned int) {
    *p = std::malloc(bytes);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipHostFree(void* p) {
    std::free(p);
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) {
    *e = reinterpret_cast<hipEvent_t>(std::malloc(1));
    return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t e) {
    std::free(e);
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "fake device"; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipGetDevice(int* device) {
    *device = 0;
    return hipSuccess;
}
hipError_t hipGetSymbolAddress(void** p, const void* symbol) {
    *p = const_cast<void*>(symbol);
    return hipSuccess;
}
}
