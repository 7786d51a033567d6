// Shared by the kernel translation units: algebras, packs, launch helpers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "ccdc.h"
#include "plan.hpp"

namespace ccdc {

// ----------------------------------------------------------------- algebras
struct SumF32 {
    using elem = float;
    static __device__ __forceinline__ elem zero() { return 0.0f; }
    static __device__ __forceinline__ elem add(elem a, elem b) { return a + b; }
    static __device__ __forceinline__ elem sub(elem a, elem b) { return a - b; }
};
struct XorU32 {
    using elem = uint32_t;
    static __device__ __forceinline__ elem zero() { return 0u; }
    static __device__ __forceinline__ elem add(elem a, elem b) { return a ^ b; }
    static __device__ __forceinline__ elem sub(elem a, elem b) { return a ^ b; }
};

// VEC consecutive elements moved by one load/store.
template <class E, int VEC>
struct alignas(sizeof(E) * VEC) Pack {
    E v[VEC];
};

template <class A, int VEC>
struct Ops {
    using P = Pack<typename A::elem, VEC>;
    static __device__ __forceinline__ P zero()
    {
        P z;
#pragma unroll
        for (int i = 0; i < VEC; i++) z.v[i] = A::zero();
        return z;
    }
    static __device__ __forceinline__ P add(P a, P b)
    {
#pragma unroll
        for (int i = 0; i < VEC; i++) a.v[i] = A::add(a.v[i], b.v[i]);
        return a;
    }
    static __device__ __forceinline__ P sub(P a, P b)
    {
#pragma unroll
        for (int i = 0; i < VEC; i++) a.v[i] = A::sub(a.v[i], b.v[i]);
        return a;
    }
};

constexpr int kBlock = 256;

__device__ __forceinline__ int label_rank(int a, int b) { return a - (a > b ? 1 : 0); }

template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_reduce_final(const typename A::elem *__restrict__ part,
                                                         typename A::elem *__restrict__ Phi, int split,
                                                         int64_t chunk_packs, uint32_t items)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const P *src = reinterpret_cast<const P *>(part) + idx;
    P acc = src[0];
    for (int s = 1; s < split; s++) acc = O::add(acc, src[(int64_t)s * chunk_packs]);
    reinterpret_cast<P *>(Phi)[idx] = acc;
}

// ------------------------------------------------------------ host helpers
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline uint32_t cdiv(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

inline int ready(const ccdc_plan_t *p)
{
    if (!p) return CCDC_EINVAL;
    if (!p->bound || !p->uploaded) return CCDC_ESTATE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return CCDC_EHIP;
    if (dev != p->device) return CCDC_ESTATE;
    return CCDC_OK;
}

// Pack width for this call: 4 when the value length and every pointer allow it.
template <class... Ptr>
int pick_vec(const ccdc_plan_t *p, int *vec, Ptr... ptrs)
{
    const void *list[] = {ptrs...};
    bool a16 = true;
    for (const void *q : list) {
        if (!q) return CCDC_EINVAL;
        if (!aligned(q, 4)) return CCDC_EINVAL;
        a16 = a16 && aligned(q, 16);
    }
    *vec = (p->T % 4 == 0 && a16) ? 4 : 1;
    return CCDC_OK;
}

inline int launched()
{
    return hipGetLastError() == hipSuccess ? CCDC_OK : CCDC_EHIP;
}

}  // namespace ccdc
