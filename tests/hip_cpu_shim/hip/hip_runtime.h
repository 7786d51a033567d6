// A stand-in for <hip/hip_runtime.h> that lets the library's kernel sources be compiled for the
// HOST and run there under AddressSanitizer / UBSan.  TEST INFRASTRUCTURE ONLY: it exists so that
// index arithmetic of the kernels and launchers (global memory, LDS, grids) can be bounds-checked
// on a CPU; the product never uses it.
//
// Model: the lanes of a workgroup are real threads (one per lane, kept for a whole launch) that
// walk the workgroups in order and meet only where the kernel synchronises (__syncthreads, lane
// shuffles); device memory is host heap (so every hipMalloc'd buffer has sanitizer red zones);
// dynamic LDS and a kernel's static __shared__ array are fresh heap blocks per workgroup; streams
// and events do nothing (a launch returns when all its workgroups are done).
#pragma once

#include <atomic>
#include <condition_variable>
#include <cstddef>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))

struct dim3 {
    unsigned x = 1, y = 1, z = 1;
    dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {}
};
struct shim_uint3 {
    unsigned x, y, z;
};
extern thread_local shim_uint3 threadIdx, blockIdx;
extern thread_local dim3 blockDim, gridDim;

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2 };
typedef struct shim_stream *hipStream_t;
typedef struct shim_event *hipEvent_t;
enum hipStreamCaptureStatus { hipStreamCaptureStatusNone = 0, hipStreamCaptureStatusActive = 1 };
enum { hipEventDisableTiming = 2 };
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 };
enum hipDeviceAttribute_t { hipDeviceAttributeMultiprocessorCount = 1 };

namespace shim {
extern thread_local unsigned char *dyn_smem;          // dynamic LDS of the running workgroup
extern int compute_units;                               // what the device attribute query answers
extern int blocks_per_cu;                               // what the occupancy query answers
extern size_t max_dynamic_lds;                          // launches asking for more are refused
extern std::atomic<long> launches;
void barrier_wait();                                    // __syncthreads()
void *block_static(size_t bytes);                       // the running workgroup's static __shared__ array
uint32_t shuffle_xor(uint32_t v, int mask);             // all lanes of the workgroup call it together
void launch(dim3 grid, dim3 block, size_t lds, const std::function<void()> &body);
}  // namespace shim

inline void __syncthreads() { shim::barrier_wait(); }
inline int __shfl_xor(int v, int mask, int /*width*/) { return (int)shim::shuffle_xor((uint32_t)v, mask); }
inline uint32_t __float_as_uint(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float __uint_as_float(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

hipError_t hipMalloc(void **p, size_t bytes);
hipError_t hipFree(void *p);
hipError_t hipMemcpy(void *dst, const void *src, size_t bytes, hipMemcpyKind);
hipError_t hipGetDevice(int *dev);
hipError_t hipSetDevice(int dev);
hipError_t hipGetLastError();
hipError_t hipDeviceGetAttribute(int *out, hipDeviceAttribute_t, int dev);
hipError_t hipEventCreateWithFlags(hipEvent_t *ev, unsigned flags);
hipError_t hipEventDestroy(hipEvent_t ev);
hipError_t hipEventRecord(hipEvent_t ev, hipStream_t st);
hipError_t hipStreamWaitEvent(hipStream_t st, hipEvent_t ev, unsigned flags);
hipError_t hipStreamIsCapturing(hipStream_t st, hipStreamCaptureStatus *out);
hipError_t hipGetSymbolAddress(void **out, const void *symbol);
template <class K>
hipError_t hipOccupancyMaxActiveBlocksPerMultiprocessor(int *out, K, int /*block*/, size_t lds)
{
    if (lds > shim::max_dynamic_lds) return hipErrorInvalidValue;
    *out = shim::blocks_per_cu;
    return hipSuccess;
}
