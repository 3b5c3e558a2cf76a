// A stand-in for the HIP runtime that lets the C-ABI layer (csrc/ddef_api.hip) be compiled with a
// plain host compiler and run on a CPU under AddressSanitizer / UBSan: "device" memory is host
// memory, copies are memcpy (so a wrong size on the host side is an ASan report), kernel launches
// run nothing but are checked (non-empty grid and block) and logged with their pointer arguments,
// and allocations, streams and events can be made to fail on request.  Test infrastructure only:
// nothing here computes anything of the method.
#ifndef DDEF_TESTS_FAKE_HIP_RUNTIME_H
#define DDEF_TESTS_FAKE_HIP_RUNTIME_H

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

#define __global__
#define __device__
#define __host__
#define __align__(n) __attribute__((aligned(n)))
#define __launch_bounds__(...)
#define HIP_SYMBOL(x) (&(x))

enum hipError_t { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2, hipErrorInvalidConfiguration = 9,
                  hipErrorUnknown = 999 };
enum hipMemcpyKind { hipMemcpyHostToHost = 0, hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2,
                     hipMemcpyDeviceToDevice = 3 };
enum hipStreamCaptureMode { hipStreamCaptureModeGlobal = 0, hipStreamCaptureModeThreadLocal = 1 };
enum hipDeviceAttribute_t { hipDeviceAttributeMultiprocessorCount = 63 };
constexpr unsigned hipStreamNonBlocking = 1, hipEventDisableTiming = 2;

struct fake_hip_stream { int id; };
struct fake_hip_event { int id; };
struct fake_hip_graph { int nodes; };
typedef fake_hip_stream* hipStream_t;
typedef fake_hip_event* hipEvent_t;
typedef fake_hip_graph* hipGraph_t;
typedef fake_hip_graph* hipGraphExec_t;

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct uint2 { unsigned x, y; };
inline uint2 make_uint2(unsigned x, unsigned y) { return uint2{x, y}; }

struct hipDeviceProp_t {
    int multiProcessorCount = 4, warpSize = 64, clockRate = 1000000, memoryClockRate = 1000000, memoryBusWidth = 64;
    size_t maxSharedMemoryPerMultiProcessor = 65536, totalGlobalMem = (size_t)1 << 30;
    char gcnArchName[256] = "host-build";
};

namespace fake_hip {

struct Launch {
    std::string kernel;
    dim3 grid, block;
    hipStream_t stream;
    std::vector<const void*> pointers;      // the pointer arguments in order (others are skipped)
};

struct State {
    std::vector<Launch> launches;
    long fail_malloc_in = -1;               // >= 0: the (n+1)-th hipMalloc from now fails with out-of-memory
    long fail_stream_in = -1, fail_event_in = -1;
    long mallocs = 0, frees = 0, live = 0;
    hipError_t last = hipSuccess;
    int capturing = 0;
};
inline State& state() { static State s; return s; }

inline bool countdown(long& c) {
    if (c < 0) return false;
    if (c == 0) { c = -1; return true; }
    --c;
    return false;
}
inline hipError_t note(hipError_t e) { if (e != hipSuccess) state().last = e; return e; }

template <class T>
inline void collect(std::vector<const void*>& out, const T& v) {
    if constexpr (std::is_pointer<T>::value) out.push_back((const void*)v);
    else if constexpr (std::is_null_pointer<T>::value) out.push_back(nullptr);
}

template <class... Args>
inline void launch(const char* kernel, dim3 grid, dim3 block, hipStream_t stream, const Args&... args) {
    Launch l{kernel, grid, block, stream, {}};
    (collect(l.pointers, args), ...);
    if (grid.x == 0 || grid.y == 0 || grid.z == 0 || block.x == 0 || block.x * block.y * block.z > 1024u ||
        grid.y > 65535u || grid.z > 65535u)
        note(hipErrorInvalidConfiguration);
    state().launches.push_back(l);
}

}  // namespace fake_hip

#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
    fake_hip::launch(#kernel, (grid), (block), (stream), __VA_ARGS__)

inline hipError_t hipGetLastError() { hipError_t e = fake_hip::state().last; fake_hip::state().last = hipSuccess; return e; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipSetDevice(int d) { return d == 0 ? hipSuccess : fake_hip::note(hipErrorInvalidValue); }
inline hipError_t hipGetDeviceProperties(hipDeviceProp_t* p, int) { *p = hipDeviceProp_t(); return hipSuccess; }
inline hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) { *v = 4; return hipSuccess; }
inline hipError_t hipDeviceSynchronize() { return hipSuccess; }

inline hipError_t hipMalloc(void** p, size_t bytes) {
    fake_hip::State& s = fake_hip::state();
    *p = nullptr;
    if (fake_hip::countdown(s.fail_malloc_in)) return fake_hip::note(hipErrorOutOfMemory);
    *p = std::calloc(bytes ? bytes : 1, 1);  // zeroed: no kernel ever writes it here, and the host reads some of it back
    if (!*p) return fake_hip::note(hipErrorOutOfMemory);
    s.mallocs += 1; s.live += 1;
    return hipSuccess;
}
inline hipError_t hipFree(void* p) {
    if (p) { std::free(p); fake_hip::state().frees += 1; fake_hip::state().live -= 1; }
    return hipSuccess;
}
inline hipError_t hipMemset(void* p, int v, size_t bytes) { std::memset(p, v, bytes); return hipSuccess; }
inline hipError_t hipMemsetAsync(void* p, int v, size_t bytes, hipStream_t) { std::memset(p, v, bytes); return hipSuccess; }
inline hipError_t hipMemcpy(void* dst, const void* src, size_t bytes, hipMemcpyKind) {
    std::memmove(dst, src, bytes);
    return hipSuccess;
}
inline hipError_t hipMemcpy2D(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height,
                              hipMemcpyKind) {
    for (size_t r = 0; r < height; ++r) std::memmove((char*)dst + r * dpitch, (const char*)src + r * spitch, width);
    return hipSuccess;
}
template <class T>
inline hipError_t hipGetSymbolAddress(void** out, T* symbol) { *out = (void*)symbol; return hipSuccess; }

inline hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) {
    *s = nullptr;
    if (fake_hip::countdown(fake_hip::state().fail_stream_in)) return fake_hip::note(hipErrorUnknown);
    *s = new fake_hip_stream{1};
    return hipSuccess;
}
inline hipError_t hipStreamDestroy(hipStream_t s) { delete s; return hipSuccess; }
inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t e, unsigned) { return e ? hipSuccess : fake_hip::note(hipErrorInvalidValue); }
inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) {
    *e = nullptr;
    if (fake_hip::countdown(fake_hip::state().fail_event_in)) return fake_hip::note(hipErrorUnknown);
    *e = new fake_hip_event{1};
    return hipSuccess;
}
inline hipError_t hipEventCreate(hipEvent_t* e) { return hipEventCreateWithFlags(e, 0); }
inline hipError_t hipEventDestroy(hipEvent_t e) { delete e; return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t e, hipStream_t) { return e ? hipSuccess : fake_hip::note(hipErrorInvalidValue); }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.001f; return hipSuccess; }

inline hipError_t hipStreamBeginCapture(hipStream_t, hipStreamCaptureMode) { fake_hip::state().capturing = 1; return hipSuccess; }
inline hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t* g) {
    fake_hip::state().capturing = 0;
    *g = new fake_hip_graph{1};
    return hipSuccess;
}
inline hipError_t hipGraphInstantiate(hipGraphExec_t* e, hipGraph_t, void*, void*, size_t) { *e = new fake_hip_graph{2}; return hipSuccess; }
inline hipError_t hipGraphDestroy(hipGraph_t g) { delete g; return hipSuccess; }
inline hipError_t hipGraphExecDestroy(hipGraphExec_t g) { delete g; return hipSuccess; }
inline hipError_t hipGraphLaunch(hipGraphExec_t, hipStream_t) { return hipSuccess; }

#endif
