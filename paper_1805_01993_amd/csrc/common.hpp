// Shared by the kernel translation units: algebras, packs, launch helpers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "ccdc.h"
#include "plan.hpp"

namespace ccdc {

// ----------------------------------------------------------------- algebras
// add: pre-combining and the final reduction.  code / uncode: forming a coded
// packet and cancelling side information from it.
struct SumF32 {                       // real numbers throughout
    using elem = float;
    static __device__ __forceinline__ elem zero() { return 0.0f; }
    static __device__ __forceinline__ elem add(elem a, elem b) { return a + b; }
    static __device__ __forceinline__ elem code(elem a, elem b) { return a + b; }
    static __device__ __forceinline__ elem uncode(elem a, elem b) { return a - b; }
};
struct XorU32 {                       // the field F_{2^T} throughout
    using elem = uint32_t;
    static __device__ __forceinline__ elem zero() { return 0u; }
    static __device__ __forceinline__ elem add(elem a, elem b) { return a ^ b; }
    static __device__ __forceinline__ elem code(elem a, elem b) { return a ^ b; }
    static __device__ __forceinline__ elem uncode(elem a, elem b) { return a ^ b; }
};
struct HybF32 {                       // numbers are summed, packets are XOR-coded bit patterns (Sec. II)
    using elem = float;
    static __device__ __forceinline__ elem zero() { return 0.0f; }    // all-zero bits: also the XOR identity
    static __device__ __forceinline__ elem add(elem a, elem b) { return a + b; }
    static __device__ __forceinline__ elem code(elem a, elem b)
    {
        return __uint_as_float(__float_as_uint(a) ^ __float_as_uint(b));
    }
    static __device__ __forceinline__ elem uncode(elem a, elem b) { return code(a, b); }
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
    static __device__ __forceinline__ P code(P a, P b)
    {
#pragma unroll
        for (int i = 0; i < VEC; i++) a.v[i] = A::code(a.v[i], b.v[i]);
        return a;
    }
    static __device__ __forceinline__ P uncode(P a, P b)
    {
#pragma unroll
        for (int i = 0; i < VEC; i++) a.v[i] = A::uncode(a.v[i], b.v[i]);
        return a;
    }
    static __device__ __forceinline__ P select(bool c, P a, P b)
    {
#pragma unroll
        for (int i = 0; i < VEC; i++) a.v[i] = c ? a.v[i] : b.v[i];
        return a;
    }
};

// Streaming accesses: data that is read or written exactly once is marked
// non-temporal so that it does not displace anything worth keeping in cache.
#ifndef CCDC_STREAMING_HINTS
#define CCDC_STREAMING_HINTS 1
#endif
template <int VEC>
struct Bits {
    typedef uint32_t type __attribute__((ext_vector_type(VEC)));
};
template <>
struct Bits<1> {
    typedef uint32_t type;
};
template <class P>
__device__ __forceinline__ P load_stream(const void *p)
{
#if CCDC_STREAMING_HINTS
    using B = typename Bits<sizeof(P) / 4>::type;
    const B b = __builtin_nontemporal_load(reinterpret_cast<const B *>(p));
    P out;
    __builtin_memcpy(&out, &b, sizeof(P));
    return out;
#else
    return *reinterpret_cast<const P *>(p);
#endif
}
template <class P>
__device__ __forceinline__ void store_stream(void *p, const P &v)
{
#if CCDC_STREAMING_HINTS
    using B = typename Bits<sizeof(P) / 4>::type;
    B b;
    __builtin_memcpy(&b, &v, sizeof(P));
    __builtin_nontemporal_store(b, reinterpret_cast<B *>(p));
#else
    *reinterpret_cast<P *>(p) = v;
#endif
}

constexpr int kBlock = 256;

__device__ __forceinline__ int label_rank(int a, int b) { return a - (a > b ? 1 : 0); }

// Phi = sum over chunks of the per-chunk outputs part[split][chunk_packs].
// A workgroup owns kBlock/G consecutive packs; its G thread groups each add
// every G-th chunk (g, g+G, ...), then the G group sums are added in group
// order.  The order is fixed by (split, G), so results repeat run to run.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_reduce_final(const typename A::elem *__restrict__ part,
                                                         typename A::elem *__restrict__ Phi, int split,
                                                         int64_t chunk_packs, uint32_t items, int G)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    __shared__ P sums[kBlock];
    const int per_block = kBlock / G;                    // packs of this workgroup
    const int e = threadIdx.x % per_block, g = threadIdx.x / per_block;
    const uint32_t idx = blockIdx.x * per_block + e;
    P acc = O::zero();
    if (idx < items) {
        const P *src = reinterpret_cast<const P *>(part) + idx;
#pragma unroll 4
        for (int s = g; s < split; s += G) acc = O::add(acc, src[(int64_t)s * chunk_packs]);
    }
    sums[threadIdx.x] = acc;
    __syncthreads();
    if (g == 0 && idx < items) {
        for (int k = 1; k < G; k++) acc = O::add(acc, sums[k * per_block + e]);
        reinterpret_cast<P *>(Phi)[idx] = acc;
    }
}

// Launch geometry of k_reduce_final: more thread groups when there are few packs.
inline int reduce_final_groups(int64_t items, int split)
{
    int G = 1;
    while (G < 16 && G * 2 <= split && items * G < (1 << 18)) G *= 2;
    return G;
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
