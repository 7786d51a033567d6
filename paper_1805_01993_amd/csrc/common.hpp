// Shared by the kernel translation units: algebras, packs, launch helpers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "ccdc.h"
#include "plan.hpp"

namespace ccdc {

// ----------------------------------------------------------------- algebras
// elem: what V, Vbar, X, D and Phi hold.  acc: what sums are carried in.
// widen / add / narrow: pre-combining and the final reduction (a sum is
// narrowed once, when it is stored as an elem).  code / uncode: forming a coded
// packet and cancelling side information from it.  fixed_order: the bits of a
// pre-combined packet are part of the result (they are XOR-coded), so every
// kernel adds a batch's files in ascending order.
struct SumF32 {                       // real numbers throughout
    using elem = float;
    using acc = float;
    static constexpr bool fixed_order = false;
    static __device__ __forceinline__ elem zero() { return 0.0f; }
    static __device__ __forceinline__ acc azero() { return 0.0f; }
    static __device__ __forceinline__ acc widen(elem a) { return a; }
    static __device__ __forceinline__ elem narrow(acc a) { return a; }
    static __device__ __forceinline__ acc add(acc a, acc b) { return a + b; }
    static __device__ __forceinline__ elem code(elem a, elem b) { return a + b; }
    static __device__ __forceinline__ elem uncode(elem a, elem b) { return a - b; }
    static __device__ __forceinline__ elem gradient(elem theta, elem data) { return theta - data; }
};
struct XorU32 {                       // the field F_{2^T} throughout
    using elem = uint32_t;
    using acc = uint32_t;
    static constexpr bool fixed_order = false;
    static __device__ __forceinline__ elem zero() { return 0u; }
    static __device__ __forceinline__ acc azero() { return 0u; }
    static __device__ __forceinline__ acc widen(elem a) { return a; }
    static __device__ __forceinline__ elem narrow(acc a) { return a; }
    static __device__ __forceinline__ acc add(acc a, acc b) { return a ^ b; }
    static __device__ __forceinline__ elem code(elem a, elem b) { return a ^ b; }
    static __device__ __forceinline__ elem uncode(elem a, elem b) { return a ^ b; }
    static __device__ __forceinline__ elem gradient(elem theta, elem data) { return theta ^ data; }   // - is XOR in F_{2^T}
};
struct HybF32 {                       // numbers are summed, packets are XOR-coded bit patterns (Sec. II)
    using elem = float;
    using acc = float;
    static constexpr bool fixed_order = true;
    static __device__ __forceinline__ elem zero() { return 0.0f; }    // all-zero bits: also the XOR identity
    static __device__ __forceinline__ acc azero() { return 0.0f; }
    static __device__ __forceinline__ acc widen(elem a) { return a; }
    static __device__ __forceinline__ elem narrow(acc a) { return a; }
    static __device__ __forceinline__ acc add(acc a, acc b) { return a + b; }
    static __device__ __forceinline__ elem code(elem a, elem b)
    {
        return __uint_as_float(__float_as_uint(a) ^ __float_as_uint(b));
    }
    static __device__ __forceinline__ elem uncode(elem a, elem b) { return code(a, b); }
    static __device__ __forceinline__ elem gradient(elem theta, elem data) { return theta - data; }
};
// The same hybrid for 16-bit floating-point payloads: elements are bit patterns
// of bfloat16 (BF) or IEEE binary16 numbers, sums are carried in fp32 and
// rounded once, to nearest even, when stored.  A batch of one file is not a sum:
// its packet is the file's values as they are, pattern for pattern (every kernel
// copies in that case), so signalling or signed NaN patterns in the input pass
// through the coding untouched.
template <bool BF>
struct Hyb16 {
    using elem = uint16_t;
    using acc = float;
    static constexpr bool fixed_order = true;
    static __device__ __forceinline__ elem zero() { return 0; }
    static __device__ __forceinline__ acc azero() { return 0.0f; }
    static __device__ __forceinline__ acc widen(elem a)
    {
        if constexpr (BF) {
            return __uint_as_float((uint32_t)a << 16);
        } else {
            _Float16 h;
            __builtin_memcpy(&h, &a, 2);
            return (float)h;
        }
    }
    // A sum that is not a number is stored as the format's quiet NaN with a clear sign and
    // payload (0x7FC0 / 0x7E00), whatever NaN the additions produced.
    static __device__ __forceinline__ elem narrow(acc a)
    {
        if constexpr (BF) {
            if (a != a) return (elem)0x7FC0u;
            // keep the upper 16 bits; round up when the dropped half is above the midpoint, or
            // on it with an odd kept part (the increment may carry into the exponent, up to infinity)
            const uint32_t b = __float_as_uint(a);
            const uint32_t kept = b >> 16, dropped = b & 0xFFFFu;
            return (elem)(kept + ((dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u))) ? 1u : 0u));
        } else {
            if (a != a) return (elem)0x7E00u;
            const _Float16 h = (_Float16)a;              // the hardware conversion rounds to nearest even
            elem out;
            __builtin_memcpy(&out, &h, 2);
            return out;
        }
    }
    static __device__ __forceinline__ acc add(acc a, acc b) { return a + b; }
    static __device__ __forceinline__ elem code(elem a, elem b) { return (elem)(a ^ b); }
    static __device__ __forceinline__ elem uncode(elem a, elem b) { return (elem)(a ^ b); }
    // the difference of the two values in fp32 (one rounding), rounded once more to the format
    static __device__ __forceinline__ elem gradient(elem theta, elem data) { return narrow(widen(theta) - widen(data)); }
};
using HybBF16 = Hyb16<true>;
using HybF16 = Hyb16<false>;

// VEC consecutive elements moved by one load/store.
template <class E, int VEC>
struct alignas(sizeof(E) * VEC) Pack {
    E v[VEC];
};

template <class A, int VEC>
struct Ops {
    using P = Pack<typename A::elem, VEC>;       // as stored
    using Q = Pack<typename A::acc, VEC>;        // as summed
    static __device__ __forceinline__ P zero()
    {
        P z;
#pragma unroll
        for (int i = 0; i < VEC; i++) z.v[i] = A::zero();
        return z;
    }
    static __device__ __forceinline__ Q azero()
    {
        Q z;
#pragma unroll
        for (int i = 0; i < VEC; i++) z.v[i] = A::azero();
        return z;
    }
    static __device__ __forceinline__ Q widen(P a)
    {
        Q q;
#pragma unroll
        for (int i = 0; i < VEC; i++) q.v[i] = A::widen(a.v[i]);
        return q;
    }
    static __device__ __forceinline__ P narrow(Q a)
    {
        P p;
#pragma unroll
        for (int i = 0; i < VEC; i++) p.v[i] = A::narrow(a.v[i]);
        return p;
    }
    static __device__ __forceinline__ Q add(Q a, Q b)
    {
#pragma unroll
        for (int i = 0; i < VEC; i++) a.v[i] = A::add(a.v[i], b.v[i]);
        return a;
    }
    static __device__ __forceinline__ Q accum(Q a, P b) { return add(a, widen(b)); }
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
    static __device__ __forceinline__ P gradient(P theta, P data)
    {
#pragma unroll
        for (int i = 0; i < VEC; i++) theta.v[i] = A::gradient(theta.v[i], data.v[i]);
        return theta;
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
template <int BYTES>
struct Bits {                                       // 8 or 16 bytes: a vector of 32-bit words
    typedef uint32_t type __attribute__((ext_vector_type(BYTES / 4)));
};
template <>
struct Bits<4> {
    typedef uint32_t type;
};
template <>
struct Bits<2> {
    typedef uint16_t type;
};
template <class P>
__device__ __forceinline__ P load_stream(const void *p)
{
#if CCDC_STREAMING_HINTS
    using B = typename Bits<sizeof(P)>::type;
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
    using B = typename Bits<sizeof(P)>::type;
    B b;
    __builtin_memcpy(&b, &v, sizeof(P));
    __builtin_nontemporal_store(b, reinterpret_cast<B *>(p));
#else
    *reinterpret_cast<P *>(p) = v;
#endif
}

constexpr int kBlock = 256;
// Work items (and workgroups) of one launch are numbered in 32 bits.  ccdc_plan_bind checks the
// counts for the widest packs a shape allows; a call that has to fall back to narrower packs
// (pointers not aligned for the wide ones) has more items and checks again for itself.
constexpr uint64_t kMaxLaunchItems = 2147483647ull;
inline bool fits_launch(uint64_t items) { return items <= kMaxLaunchItems; }

// Which segment of packet b carries sender a's label: the rank of a among the members other than b.
__device__ __forceinline__ int segment_rank(int a, int b) { return a - (a > b ? 1 : 0); }

// Phi = sum over chunks of the per-chunk outputs part[split][chunk_packs].
// A workgroup owns kBlock/G consecutive packs; its G thread groups each add
// every G-th chunk (g, g+G, ...), then the G group sums are added in group
// order.  The order is fixed by (split, G), so results repeat run to run.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_reduce_final(const typename A::acc *__restrict__ part,
                                                         typename A::elem *__restrict__ Phi, int split,
                                                         int64_t chunk_packs, uint32_t items, int G)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    using Q = typename O::Q;
    __shared__ Q sums[kBlock];
    const int per_block = kBlock / G;                    // packs of this workgroup
    const int e = threadIdx.x % per_block, g = threadIdx.x / per_block;
    const uint32_t idx = blockIdx.x * per_block + e;
    Q acc = O::azero();
    if (idx < items) {
        const Q *src = reinterpret_cast<const Q *>(part) + idx;
#pragma unroll 4
        for (int s = g; s < split; s += G) acc = O::add(acc, src[(int64_t)s * chunk_packs]);
    }
    sums[threadIdx.x] = acc;
    __syncthreads();
    if (g == 0 && idx < items) {
        for (int k = 1; k < G; k++) acc = O::add(acc, sums[k * per_block + e]);
        reinterpret_cast<P *>(Phi)[idx] = O::narrow(acc);
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

inline int elem_bytes(int mode) { return (mode == CCDC_BF16_SUM_XOR || mode == CCDC_F16_SUM_XOR) ? 2 : 4; }

// Pack width (elements) for this call: 16 bytes when the value length, the
// segment length and every pointer allow it; for 2-byte elements else 8 bytes;
// else one element.
template <class... Ptr>
int pick_vec(const ccdc_plan_t *p, int *vec, Ptr... ptrs)
{
    const void *list[] = {ptrs...};
    const size_t eb = (size_t)elem_bytes(p->mode);
    bool a16 = true, a8 = true;
    for (const void *q : list) {
        if (!q) return CCDC_EINVAL;
        if (!aligned(q, eb)) return CCDC_EINVAL;
        a16 = a16 && aligned(q, 16);
        a8 = a8 && aligned(q, 8);
    }
    if (eb == 4) {
        *vec = (p->T % 4 == 0 && a16) ? 4 : 1;
    } else {
        if (p->T % 8 == 0 && p->ell % 8 == 0 && a16) *vec = 8;
        else if (p->T % 4 == 0 && a8) *vec = 4;
        else *vec = 1;
    }
    return CCDC_OK;
}

inline int launched()
{
    return hipGetLastError() == hipSuccess ? CCDC_OK : CCDC_EHIP;
}

// The plan's workspace holds partial sums between the two kernels of one call.
// Calls that use it are put in order also when they come on different streams:
// the plan remembers the stream of the last such call, and a call that arrives
// on another stream first records the plan's event at the tail of that earlier
// stream and makes its own stream wait for it (so it waits for everything the
// earlier stream had been given, the earlier call included).  Calls that stay
// on one stream, the usual case, add no event and no wait.  Host threads take
// turns through the plan's mutex.  A stream under graph capture is left alone
// and forgotten (an event recorded outside a capture cannot be waited for
// inside one): whoever replays the graph keeps it apart from other users of
// the plan.  The earlier stream must still exist when the later call comes.
class WorkspaceOrder {
public:
    WorkspaceOrder(const ccdc_plan_t *p, hipStream_t st, bool uses_workspace)
        : p_(p), st_(st), on_(uses_workspace && p->ws_event != nullptr)
    {
        if (!on_) return;
        p_->ws_mutex.lock();
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st_, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
            (void)hipGetLastError();
            p_->ws_mutex.unlock();
            on_ = false;
            return;
        }
        if (p_->ws_used && p_->ws_stream != (void *)st_) {
            hipEvent_t ev = (hipEvent_t)p_->ws_event;
            hipStream_t earlier = (hipStream_t)p_->ws_stream;
            hipStreamCaptureStatus es = hipStreamCaptureStatusNone;       // nothing is recorded into someone's capture
            if (hipStreamIsCapturing(earlier, &es) != hipSuccess || es != hipStreamCaptureStatusNone ||
                hipEventRecord(ev, earlier) != hipSuccess || hipStreamWaitEvent(st_, ev, 0) != hipSuccess)
                (void)hipGetLastError();
        }
    }
    ~WorkspaceOrder()
    {
        if (!on_) return;
        p_->ws_used = true;
        p_->ws_stream = (void *)st_;
        p_->ws_mutex.unlock();
    }
    WorkspaceOrder(const WorkspaceOrder &) = delete;
    WorkspaceOrder &operator=(const WorkspaceOrder &) = delete;

private:
    const ccdc_plan_t *p_;
    hipStream_t st_;
    bool on_;
};

}  // namespace ccdc

// Dispatch on (payload mode, pack width): evaluates CALL with the algebra as type A and the
// pack width as constant VEC, inside a function that has `using namespace ccdc`.
#define CCDC_DISPATCH(p, vec, CALL)                                   \
    do {                                                              \
        if ((p)->mode == CCDC_F32_SUM) {                              \
            using A = SumF32;                                         \
            if ((vec) == 4) { constexpr int VEC = 4; return CALL; }   \
            constexpr int VEC = 1;                                    \
            return CALL;                                              \
        } else if ((p)->mode == CCDC_F32_SUM_XOR) {                   \
            using A = HybF32;                                         \
            if ((vec) == 4) { constexpr int VEC = 4; return CALL; }   \
            constexpr int VEC = 1;                                    \
            return CALL;                                              \
        } else if ((p)->mode == CCDC_BF16_SUM_XOR) {                  \
            using A = HybBF16;                                        \
            if ((vec) == 8) { constexpr int VEC = 8; return CALL; }   \
            if ((vec) == 4) { constexpr int VEC = 4; return CALL; }   \
            constexpr int VEC = 1;                                    \
            return CALL;                                              \
        } else if ((p)->mode == CCDC_F16_SUM_XOR) {                   \
            using A = HybF16;                                         \
            if ((vec) == 8) { constexpr int VEC = 8; return CALL; }   \
            if ((vec) == 4) { constexpr int VEC = 4; return CALL; }   \
            constexpr int VEC = 1;                                    \
            return CALL;                                              \
        } else {                                                      \
            using A = XorU32;                                         \
            if ((vec) == 4) { constexpr int VEC = 4; return CALL; }   \
            constexpr int VEC = 1;                                    \
            return CALL;                                              \
        }                                                             \
    } while (0)
