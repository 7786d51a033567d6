// What one node does in the shuffle (Sec. IV-B), from nothing but the files it
// stores and the coded packets it receives: the node-local form of the path.
// Run for every node it is the emulation in which no result is shared between
// nodes: each of the r nodes that store a batch pre-combines it for itself,
// as a real cluster would.
#include "common.hpp"

namespace {
using namespace ccdc;

// Pack `pos` of the packet pre-combined for a round member from the batch that
// starts at element offset `src` of V (files ascending, narrowed once).
template <class A, int VEC>
__device__ __forceinline__ typename Ops<A, VEC>::P combined_pack(const typename A::elem *__restrict__ V, int64_t src,
                                                                 uint32_t pos, int m, int64_t file_stride)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const typename A::elem *s = V + src + (int64_t)pos * VEC;
    const P first = load_stream<P>(s);
    if (m == 1) return first;                         // a one-file batch is sent as it is
    typename O::Q acc = O::widen(first);
    for (int f = 1; f < m; f++) acc = O::accum(acc, load_stream<P>(s + f * file_stride));
    return O::narrow(acc);
}

// ------------------------------------------------------- a sender's packets
// Coded-packet equation of Sec. IV-B for the packets listed in `rows` (those one
// node sends; null = every packet).  One work item = one pack of X[u][a]: the
// sender pre-combines, for each other member b, the segment of b's packet that
// carries the sender's label; it stores all those batches.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_node_encode(const typename A::elem *__restrict__ V,
                                                        typename A::elem *__restrict__ X,
                                                        const int64_t *__restrict__ src_off,
                                                        const int32_t *__restrict__ rows, int r1, uint32_t Lv,
                                                        uint32_t Wv, int m, int64_t file_stride, uint32_t items)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const uint32_t j = idx / Lv, x = idx - j * Lv;
    const uint32_t i = rows ? (uint32_t)rows[j] : j;
    const uint32_t u = i / r1;
    const int a = (int)(i - u * r1);
    const int64_t *src = src_off + (size_t)u * r1;
    P coded = O::zero();
    for (int b = 0; b < r1; b++) {
        if (b == a) continue;
        const uint32_t pos = segment_rank(a, b) * Lv + x;
        if (pos < Wv) coded = O::code(coded, combined_pack<A, VEC>(V, src[b], pos, m, file_stride));
    }
    store_stream(reinterpret_cast<P *>(X) + (size_t)i * Lv + x, coded);
}

// --------------------------------------------- a receiver's decoding + output
// Decoding and final reduction of Sec. IV-B for the output blocks o_first,
// o_first + o_step, ... (one node's block in every job, or all blocks).  The
// row list of a block is ccdc_reduce's: the files the node stores, then the
// packets it receives.  A received packet is not read from a buffer: pack e of
// it lies in segment rho, carried by the sender whose label that segment has, and
// is recovered here as that sender's coded pack minus the packs of the other
// members' packets in it, which the receiver pre-combines from its own files.
// The list is cut into `split` chunks as in ccdc_reduce.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_node_decode_reduce(
    const typename A::elem *__restrict__ V, const typename A::elem *__restrict__ X, typename A::elem *__restrict__ out,
    typename A::acc *__restrict__ part, const int64_t *__restrict__ red_ptr, const int64_t *__restrict__ red_row,
    const int64_t *__restrict__ red_out, const int64_t *__restrict__ src_off, int r1, uint32_t Lv, uint32_t Wv,
    int64_t W, int m, int64_t file_stride, uint32_t tiles, int split, int64_t chunk_stride, uint32_t o_first,
    uint32_t o_step)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t tile = blockIdx.x % tiles;
    const uint32_t oc = blockIdx.x / tiles;
    const uint32_t oi = oc / split;
    const int s = (int)(oc - oi * split);
    const uint32_t o = o_first + oi * o_step;
    const uint32_t e = tile * kBlock + threadIdx.x;
    if (e >= Wv) return;
    const uint32_t rho = e / Lv, x = e - rho * Lv;
    const int64_t first = red_ptr[o], n = red_ptr[o + 1] - first;
    const int64_t lo = first + n * s / split, hi = first + n * (s + 1) / split;
    typename O::Q acc = O::azero();
    for (int64_t i = lo; i < hi; i++) {
        const int64_t row = red_row[i];
        if (!(row & 1)) {                                    // a file the node stores
            acc = O::accum(acc, load_stream<P>(reinterpret_cast<const P *>(V + (row >> 1)) + e));
            continue;
        }
        const int64_t pk = (row >> 1) / W;                   // packet u*(r+1)+b meant for this node
        const uint32_t u = (uint32_t)(pk / r1);
        const int b = (int)(pk - (int64_t)u * r1);
        const int a = (int)rho < b ? (int)rho : (int)rho + 1;
        const int64_t *src = src_off + (size_t)u * r1;
        P d = load_stream<P>(reinterpret_cast<const P *>(X) + ((size_t)u * r1 + a) * Lv + x);
        for (int b2 = 0; b2 < r1; b2++) {
            if (b2 == a || b2 == b) continue;
            const uint32_t pos = segment_rank(a, b2) * Lv + x;
            if (pos < Wv) d = O::uncode(d, combined_pack<A, VEC>(V, src[b2], pos, m, file_stride));
        }
        acc = O::accum(acc, d);
    }
    if (split > 1) reinterpret_cast<typename O::Q *>(part + (int64_t)s * chunk_stride + red_out[o])[e] = acc;
    else reinterpret_cast<P *>(out + red_out[o])[e] = O::narrow(acc);
}

// Adds the chunk sums of the selected output blocks in chunk order.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_node_final(const typename A::acc *__restrict__ part,
                                                       typename A::elem *__restrict__ Phi,
                                                       const int64_t *__restrict__ red_out, uint32_t Wv, int split,
                                                       int64_t chunk_stride, uint32_t o_first, uint32_t o_step,
                                                       uint32_t items)
{
    using O = Ops<A, VEC>;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const uint32_t oi = idx / Wv, e = idx - oi * Wv;
    const int64_t base = red_out[o_first + oi * o_step];
    typename O::Q acc = O::azero();
    for (int s = 0; s < split; s++)
        acc = O::add(acc, reinterpret_cast<const typename O::Q *>(part + (int64_t)s * chunk_stride + base)[e]);
    reinterpret_cast<typename O::P *>(Phi + base)[e] = O::narrow(acc);
}

template <class A, int VEC>
int run_node_encode(const ccdc_plan_t *p, int node, const void *V, void *X, hipStream_t st)
{
    using E = typename A::elem;
    const uint32_t Wv = (uint32_t)(p->W / VEC), Lv = (uint32_t)(p->ell / VEC);
    const int64_t rows = node < 0 ? p->nrows : p->rows_per_node;
    const uint64_t items = (uint64_t)rows * Lv;
    if (items == 0) return CCDC_OK;
    if (!fits_launch(items)) return CCDC_ESIZE;
    const int32_t *list = node < 0 ? nullptr : p->d_node_rows + (size_t)node * p->rows_per_node;
    k_node_encode<A, VEC><<<cdiv(items, kBlock), kBlock, 0, st>>>((const E *)V, (E *)X, p->d_src_off, list, p->r + 1,
                                                                   Lv, Wv, p->m, (int64_t)p->Q * p->T,
                                                                   (uint32_t)items);
    return launched();
}

template <class A, int VEC>
int run_node_decode_reduce(const ccdc_plan_t *p, int node, const void *V, const void *X, void *Phi, hipStream_t st)
{
    using E = typename A::elem;
    using Acc = typename A::acc;
    const uint32_t Wv = (uint32_t)(p->W / VEC), Lv = (uint32_t)(p->ell / VEC);
    const uint32_t tiles = cdiv(Wv, kBlock);
    const int split = p->red_split;
    const uint32_t count = node < 0 ? (uint32_t)p->nout : (uint32_t)p->J;
    const uint32_t o_first = node < 0 ? 0u : (uint32_t)node, o_step = node < 0 ? 1u : (uint32_t)p->K;
    const int64_t chunk_stride = (int64_t)p->J * p->Q * p->T;
    const uint64_t blocks = (uint64_t)count * split * tiles;
    if (!fits_launch(blocks) || !fits_launch((uint64_t)count * Wv)) return CCDC_ESIZE;
    WorkspaceOrder order(p, st, split > 1);
    k_node_decode_reduce<A, VEC><<<(uint32_t)blocks, kBlock, 0, st>>>(
        (const E *)V, (const E *)X, (E *)Phi, (Acc *)p->d_workspace, p->d_red_ptr, p->d_red_row, p->d_red_out,
        p->d_src_off, p->r + 1, Lv, Wv, p->W, p->m, (int64_t)p->Q * p->T, tiles, split, chunk_stride, o_first, o_step);
    int rc = launched();
    if (rc != CCDC_OK || split == 1) return rc;
    const uint64_t items = (uint64_t)count * Wv;
    k_node_final<A, VEC><<<cdiv(items, kBlock), kBlock, 0, st>>>((const Acc *)p->d_workspace, (E *)Phi, p->d_red_out, Wv,
                                                                  split, chunk_stride, o_first, o_step, (uint32_t)items);
    return launched();
}

int node_ready(const ccdc_plan_t *plan, int node)
{
    const int rc = ready(plan);
    if (rc != CCDC_OK) return rc;
    if (plan->compression) return CCDC_ESTATE;       // nothing is coded in that scheme
    if (node < -1 || node >= plan->K) return CCDC_EINVAL;
    return CCDC_OK;
}

}  // namespace

extern "C" {

int ccdc_node_encode(const ccdc_plan_t *plan, int node, const void *V, void *X, void *stream)
{
    int rc = node_ready(plan, node), vec = 1;
    if (rc != CCDC_OK) return rc;
    if ((rc = pick_vec(plan, &vec, V, (const void *)X)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_node_encode<A, VEC>(plan, node, V, X, st)));
}

int ccdc_node_decode_reduce(const ccdc_plan_t *plan, int node, const void *V, const void *X, void *Phi, void *stream)
{
    int rc = node_ready(plan, node), vec = 1;
    if (rc != CCDC_OK) return rc;
    if ((rc = pick_vec(plan, &vec, V, X, (const void *)Phi)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_node_decode_reduce<A, VEC>(plan, node, V, X, Phi, st)));
}

}  // extern "C"
