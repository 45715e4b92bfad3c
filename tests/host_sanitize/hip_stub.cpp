// Stand-in for the HIP runtime, for a host-only build of the library under AddressSanitizer and
// UndefinedBehaviorSanitizer (CPU only).  "Device" and pinned memory are ordinary heap blocks of
// exactly the requested size, so that every table the planner fills and every copy it enqueues is
// checked against the size it allocated; copies and fills happen at once; kernel launches do
// nothing (the result block a launch would have written stays zero: "no error, empty message");
// events and streams are inert.  One device.
#include <hip/hip_runtime_api.h>

#include <cstdlib>
#include <cstring>

static long g_launches = 0;
static long g_live_blocks = 0;
static long g_fail_alloc_at = -1;      // the n-th allocation from now fails (tests the clean-up path)

extern "C" long stub_launches() { return g_launches; }
extern "C" long stub_live_blocks() { return g_live_blocks; }
extern "C" void stub_fail_allocation(long nth) { g_fail_alloc_at = nth; }

static hipError_t stub_alloc(void** p, size_t bytes) {
    if (!p) return hipErrorInvalidValue;
    if (g_fail_alloc_at >= 0 && g_fail_alloc_at-- == 0) { *p = nullptr; return hipErrorOutOfMemory; }
    *p = std::calloc(bytes ? bytes : 1, 1);          // (zero-filled: a result block no kernel wrote reads "no error")
    if (!*p) return hipErrorOutOfMemory;
    ++g_live_blocks;
    return hipSuccess;
}
static hipError_t stub_free(void* p) {
    if (p) { std::free(p); --g_live_blocks; }
    return hipSuccess;
}

extern "C" {

hipError_t hipGetDeviceCount(int* n) { *n = 1; return hipSuccess; }
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipSetDevice(int d) { return d == 0 ? hipSuccess : hipErrorInvalidDevice; }
hipError_t hipGetLastError(void) { return hipSuccess; }

hipError_t hipMalloc(void** p, size_t bytes) { return stub_alloc(p, bytes); }
hipError_t hipFree(void* p) { return stub_free(p); }
hipError_t hipHostMalloc(void** p, size_t bytes, unsigned int) { return stub_alloc(p, bytes); }
hipError_t hipHostFree(void* p) { return stub_free(p); }
hipError_t hipHostGetDevicePointer(void** dev, void* host, unsigned int) { *dev = host; return hipSuccess; }

hipError_t hipMemcpy(void* dst, const void* src, size_t bytes, hipMemcpyKind) { if (bytes) std::memcpy(dst, src, bytes); return hipSuccess; }
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind, hipStream_t) {
    if (bytes) std::memcpy(dst, src, bytes);
    return hipSuccess;
}
hipError_t hipMemset(void* dst, int value, size_t bytes) { if (bytes) std::memset(dst, value, bytes); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }

hipError_t hipEventCreate(hipEvent_t* e) { return stub_alloc(reinterpret_cast<void**>(e), 8); }
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { return stub_alloc(reinterpret_cast<void**>(e), 8); }
hipError_t hipEventDestroy(hipEvent_t e) { return stub_free(e); }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }

hipError_t hipLaunchKernel(const void*, dim3 grid, dim3 block, void**, size_t, hipStream_t) {
    if (grid.x == 0 || grid.y == 0 || grid.z == 0 || block.x == 0 || block.x * block.y * block.z > 1024) return hipErrorInvalidConfiguration;
    ++g_launches;
    return hipSuccess;
}
hipError_t hipExtLaunchKernel(const void* f, dim3 grid, dim3 block, void** args, size_t shmem, hipStream_t s, hipEvent_t,
                              hipEvent_t, int) {
    return hipLaunchKernel(f, grid, block, args, shmem, s);
}
// the host-side shadow of a device variable has the variable's size: it serves as its storage
hipError_t hipGetSymbolAddress(void** p, const void* symbol) { *p = const_cast<void*>(symbol); return hipSuccess; }

// what the compiler-generated registration code calls
void** __hipRegisterFatBinary(const void*) { static void* handle = nullptr; return &handle; }
void __hipUnregisterFatBinary(void**) {}
void __hipRegisterFunction(void**, const void*, char*, const char*, unsigned, void*, void*, void*, void*, int*) {}
void __hipRegisterVar(void**, void*, char*, char*, int, size_t, int, int) {}
static dim3 g_grid, g_block;
static size_t g_shmem;
static hipStream_t g_stream;
hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shmem, hipStream_t s) {
    g_grid = grid; g_block = block; g_shmem = shmem; g_stream = s;
    return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3* grid, dim3* block, size_t* shmem, hipStream_t* s) {
    *grid = g_grid; *block = g_block; *shmem = g_shmem; *s = g_stream;
    return hipSuccess;
}

}  // extern "C"
