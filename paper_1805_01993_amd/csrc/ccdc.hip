// HIP kernels (gfx950) and the C entry points of libccdc.
//
// Everything here is a streaming, bandwidth-bound elementwise pass: every
// work item moves one pack (16 bytes when the value length allows it, else 8
// bytes or one element) per operand, consecutive lanes touch consecutive packs of the same
// row, and there is no reuse across work items, so no LDS tiling and no MFMA.
#include <new>

#include "common.hpp"

namespace {
using namespace ccdc;

// ------------------------------------------------------------------ combine
// Sec. IV-B pre-combining.  One work item = one pack of one packet Vbar[u][b]:
// it adds the same pack of the files of the served batch (m of them, or
// row_files[row] when batches differ in size).
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_combine(const typename A::elem *__restrict__ V,
                                                    typename A::elem *__restrict__ Vbar,
                                                    const int64_t *__restrict__ src_off,
                                                    const int32_t *__restrict__ row_files, uint32_t Wv, int m,
                                                    int64_t file_stride, uint32_t items)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const uint32_t row = idx / Wv, e = idx - row * Wv;
    const typename A::elem *src = V + src_off[row] + (int64_t)e * VEC;
    const int files = row_files ? row_files[row] : m;
    const P first = load_stream<P>(src);
    if (files == 1) {                                 // not a sum: the packet is the file's values as they are
        reinterpret_cast<P *>(Vbar)[idx] = first;
        return;
    }
    typename O::Q acc = O::widen(first);
    for (int f = 1; f < files; f++) acc = O::accum(acc, load_stream<P>(src + f * file_stride));
    reinterpret_cast<P *>(Vbar)[idx] = O::narrow(acc);
}

// Pre-combining for short packets and long batches (few packs per packet, many
// files to add): one wavefront per packet.  The 64 lanes are cut into SEG-lane
// segments, SEG = packs of the packet rounded up to a power of two; segment g
// adds files g, g+G, g+2G, ... (G = 64/SEG) of the batch, each lane one pack, and
// the G segment sums are then added across the wavefront by a butterfly of lane
// exchanges.  The order of additions is fixed by (m, SEG), not by timing; it
// differs from k_combine's file order, so the algebras whose packets are coded
// bit patterns (fixed_order) do not use it.
template <class A, int VEC>
__global__ __launch_bounds__(64) void k_combine_wave(const typename A::elem *__restrict__ V,
                                                     typename A::elem *__restrict__ Vbar,
                                                     const int64_t *__restrict__ src_off, uint32_t Wv, int seg,
                                                     int m, int64_t file_stride, uint32_t rows)
{
    using E = typename A::elem;
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t row = blockIdx.x;
    if (row >= rows) return;
    const int lane = threadIdx.x;
    const int e = lane % seg, g = lane / seg, G = 64 / seg;
    const E *src = V + src_off[row] + (int64_t)e * VEC;
    typename O::Q acc = O::azero();
    if ((uint32_t)e < Wv)
        for (int f = g; f < m; f += G) acc = O::accum(acc, load_stream<P>(src + f * file_stride));
    // segmented butterfly: after the step with distance d, lane l holds the sum of
    // the segments whose index differs from its own only in the bits below d/seg
    for (int d = seg; d < 64; d <<= 1) {
        typename O::Q other;
#pragma unroll
        for (int i = 0; i < VEC; i++) {
            uint32_t bits;
            __builtin_memcpy(&bits, &acc.v[i], 4);
            bits = (uint32_t)__shfl_xor((int)bits, d, 64);
            __builtin_memcpy(&other.v[i], &bits, 4);
        }
        // lower segment first on both sides so that every lane adds in the same order
        acc = (lane & d) ? O::add(other, acc) : O::add(acc, other);
    }
    if (g == 0 && (uint32_t)e < Wv) reinterpret_cast<P *>(Vbar)[(size_t)row * Wv + e] = O::narrow(acc);
}

// ------------------------------------------------------------------- encode
// Sec. IV-B coded packet.  One work item = one pack of X[u][a]: the sum over
// the other members b of segment segment_rank(a,b) of Vbar[u][b] at the same
// in-segment position; positions past the end of a short segment add nothing.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_encode(const typename A::elem *__restrict__ Vbar,
                                                   typename A::elem *__restrict__ X, int r1, uint32_t Lv,
                                                   uint32_t Wv, uint32_t items)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const uint32_t ua = idx / Lv, x = idx - ua * Lv;
    const uint32_t u = ua / r1;
    const int a = (int)(ua - u * r1);
    const P *rows = reinterpret_cast<const P *>(Vbar) + (size_t)u * r1 * Wv;
    P acc = O::zero();
    for (int b = 0; b < r1; b++) {
        if (b == a) continue;
        const uint32_t pos = segment_rank(a, b) * Lv + x;
        if (pos < Wv) acc = O::code(acc, rows[(size_t)b * Wv + pos]);
    }
    reinterpret_cast<P *>(X)[idx] = acc;
}

// ------------------------------------------------------------------- decode
// Sec. IV-B decoding.  One work item = one pack of D[u][b].  The pack lies in
// segment rho of the packet meant for b, which was carried by the sender a
// whose label that segment has; from X[u][a] the receiver removes the packs
// of the other packets in it (b' not in {a,b}), all of which it stores.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_decode(const typename A::elem *__restrict__ X,
                                                   const typename A::elem *__restrict__ Vbar,
                                                   typename A::elem *__restrict__ D, int r1, uint32_t Lv,
                                                   uint32_t Wv, uint32_t items)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const uint32_t ub = idx / Wv, e = idx - ub * Wv;
    const uint32_t u = ub / r1;
    const int b = (int)(ub - u * r1);
    const int rho = (int)(e / Lv);
    const uint32_t x = e - rho * Lv;
    const int a = rho < b ? rho : rho + 1;
    const P *rows = reinterpret_cast<const P *>(Vbar) + (size_t)u * r1 * Wv;
    P acc = reinterpret_cast<const P *>(X)[((size_t)u * r1 + a) * Lv + x];
    for (int b2 = 0; b2 < r1; b2++) {
        if (b2 == a || b2 == b) continue;
        const uint32_t pos = segment_rank(a, b2) * Lv + x;
        if (pos < Wv) acc = O::uncode(acc, rows[(size_t)b2 * Wv + pos]);
    }
    reinterpret_cast<P *>(D)[idx] = acc;
}

// ----------------------------------------------- combine + encode + decode
// One work item = (round u, sender a, in-segment pack x).  It pre-combines the
// r packs sender a's packet is made of straight from V (each read once),
// writes the coded pack, and produces for each of the r receivers the decoded
// pack of its own packet by removing the other r-1 from the coded pack.
// R1 = r+1 at compile time keeps the r combined packs in registers; R1 = 0 is
// the any-r fallback that re-reads them (cache hits) instead.
template <class A, int VEC, int R1>
__global__ __launch_bounds__(kBlock) void k_shuffle_fused(const typename A::elem *__restrict__ V,
                                                          typename A::elem *__restrict__ X,
                                                          typename A::elem *__restrict__ D,
                                                          const int64_t *__restrict__ src_off, int r1_rt,
                                                          uint32_t Lv, uint32_t Wv, int m, int64_t file_stride,
                                                          uint32_t items)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const int r1 = R1 > 0 ? R1 : r1_rt;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const uint32_t ua = idx / Lv, x = idx - ua * Lv;
    const uint32_t u = ua / r1;
    const int a = (int)(ua - u * r1);
    const int64_t *src = src_off + (size_t)u * r1;

    auto combined = [&](int b) -> P {       // pack of Vbar[u][b] that sender a carries
        const uint32_t pos = segment_rank(a, b) * Lv + x;
        if (pos >= Wv) return O::zero();
        const typename A::elem *s = V + src[b] + (int64_t)pos * VEC;
        const P first = load_stream<P>(s);
        if (m == 1) return first;                     // a one-file batch is sent as it is
        typename O::Q acc = O::widen(first);
        for (int f = 1; f < m; f++) acc = O::accum(acc, load_stream<P>(s + f * file_stride));
        return O::narrow(acc);
    };

    P *Drows = reinterpret_cast<P *>(D) + (size_t)u * r1 * Wv;
    if constexpr (R1 > 0) {
        P v[R1];
#pragma unroll
        for (int b = 0; b < R1; b++)
            if (b != a) v[b] = combined(b);
        P coded = O::zero();
#pragma unroll
        for (int b = 0; b < R1; b++)
            if (b != a) coded = O::code(coded, v[b]);
        store_stream(reinterpret_cast<P *>(X) + idx, coded);
#pragma unroll
        for (int b = 0; b < R1; b++) {
            if (b == a) continue;
            const uint32_t pos = segment_rank(a, b) * Lv + x;
            if (pos >= Wv) continue;
            P acc = coded;
#pragma unroll
            for (int b2 = 0; b2 < R1; b2++)
                if (b2 != a && b2 != b) acc = O::uncode(acc, v[b2]);
            store_stream(Drows + (size_t)b * Wv + pos, acc);
        }
    } else {
        P coded = O::zero();
        for (int b = 0; b < r1; b++)
            if (b != a) coded = O::code(coded, combined(b));
        store_stream(reinterpret_cast<P *>(X) + idx, coded);
        for (int b = 0; b < r1; b++) {
            if (b == a) continue;
            const uint32_t pos = segment_rank(a, b) * Lv + x;
            if (pos >= Wv) continue;
            P acc = coded;
            for (int b2 = 0; b2 < r1; b2++)
                if (b2 != a && b2 != b) acc = O::uncode(acc, combined(b2));
            store_stream(Drows + (size_t)b * Wv + pos, acc);
        }
    }
}

// ------------------------------------------------------------------- reduce
// Sec. IV-B final reduction as a gather-sum of rows: output block o (one node's
// c functions of one job) is the sum of a list of W-long rows, some in V (files
// the node stores), some in D (packets it decoded).  The list is cut into
// `split` chunks; work item = (o, chunk, pack).  With split > 1 the chunk sums
// go, not yet narrowed, to the workspace and k_reduce_final adds them in chunk order.
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_reduce_rows(const typename A::elem *__restrict__ V,
                                                        const typename A::elem *__restrict__ D,
                                                        typename A::elem *__restrict__ out,
                                                        typename A::acc *__restrict__ part,
                                                        const int64_t *__restrict__ red_ptr,
                                                        const int64_t *__restrict__ red_row,
                                                        const int64_t *__restrict__ red_out, uint32_t Wv,
                                                        uint32_t tiles, int split, int64_t chunk_stride)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t tile = blockIdx.x % tiles;
    const uint32_t oc = blockIdx.x / tiles;
    const uint32_t o = oc / split;
    const int s = (int)(oc - o * split);
    const uint32_t e = tile * kBlock + threadIdx.x;
    if (e >= Wv) return;
    const int64_t first = red_ptr[o], n = red_ptr[o + 1] - first;
    const int64_t lo = first + n * s / split, hi = first + n * (s + 1) / split;
    typename O::Q acc = O::azero();
#pragma unroll 4
    for (int64_t i = lo; i < hi; i++) {
        const int64_t row = red_row[i];
        const typename A::elem *base = (row & 1) ? D : V;
        acc = O::accum(acc, load_stream<P>(reinterpret_cast<const P *>(base + (row >> 1)) + e));
    }
    if (split > 1) reinterpret_cast<typename O::Q *>(part + (int64_t)s * chunk_stride + red_out[o])[e] = acc;
    else reinterpret_cast<P *>(out + red_out[o])[e] = O::narrow(acc);
}

void release_device(ccdc_plan_t *p)
{
    if (!p) return;
    if (p->uploaded || p->d_src_off || p->d_red_ptr || p->d_red_row || p->d_red_out || p->d_loc_row || p->d_member ||
        p->d_row_files || p->d_node_rows || p->d_workspace || p->ws_event) {
        int cur = -1;
        const bool sw = hipGetDevice(&cur) == hipSuccess && p->device >= 0 && cur != p->device &&
                        hipSetDevice(p->device) == hipSuccess;
        (void)hipFree(p->d_src_off);
        (void)hipFree(p->d_red_ptr);
        (void)hipFree(p->d_red_row);
        (void)hipFree(p->d_red_out);
        (void)hipFree(p->d_loc_row);
        (void)hipFree(p->d_member);
        (void)hipFree(p->d_row_files);
        (void)hipFree(p->d_node_rows);
        (void)hipFree(p->d_workspace);
        if (p->ws_event) (void)hipEventDestroy((hipEvent_t)p->ws_event);
        if (sw) (void)hipSetDevice(cur);
    }
    p->d_src_off = p->d_red_ptr = p->d_red_row = p->d_red_out = p->d_loc_row = nullptr;
    p->d_member = nullptr;
    p->d_row_files = nullptr;
    p->d_node_rows = nullptr;
    p->d_workspace = nullptr;
    p->pipe_chunks[0] = p->pipe_chunks[1] = p->pipe_chunks[2] = 0;
    p->ws_event = nullptr;
    p->ws_stream = nullptr;
    p->ws_used = false;
    p->uploaded = false;
    p->device = -1;
}

template <class T>
int to_device(const std::vector<T> &h, T **d)
{
    const size_t bytes = (h.empty() ? 1 : h.size()) * sizeof(T);
    if (hipMalloc((void **)d, bytes) != hipSuccess) {
        *d = nullptr;
        (void)hipGetLastError();
        return CCDC_ENOMEM;
    }
    if (!h.empty() && hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess)
        return CCDC_EHIP;
    return CCDC_OK;
}

// ---- typed launchers: A = algebra, VEC = pack width
template <class A, int VEC>
int run_combine(const ccdc_plan_t *p, const void *V, void *Vbar, hipStream_t st)
{
    using E = typename A::elem;
    const uint32_t Wv = (uint32_t)(p->W / VEC);
    const uint64_t items = (uint64_t)p->nrows * Wv;
    if (items == 0) return CCDC_OK;
    if (!fits_launch(items)) return CCDC_ESIZE;
    // short packets, long batches: a wavefront per packet with a cross-lane reduction
#ifndef CCDC_COMBINE_WAVE_MIN_FILES
#define CCDC_COMBINE_WAVE_MIN_FILES 8
#endif
    if constexpr (!A::fixed_order) {
        if (Wv <= 16 && p->m >= CCDC_COMBINE_WAVE_MIN_FILES && !p->d_row_files) {
            int seg = 1;
            while ((uint32_t)seg < Wv) seg <<= 1;
            const uint32_t rows = (uint32_t)p->nrows;
            k_combine_wave<A, VEC><<<rows, 64, 0, st>>>((const E *)V, (E *)Vbar, p->d_src_off, Wv, seg, p->m,
                                                        (int64_t)p->Q * p->T, rows);
            return launched();
        }
    }
    k_combine<A, VEC><<<cdiv(items, kBlock), kBlock, 0, st>>>((const E *)V, (E *)Vbar, p->d_src_off, p->d_row_files,
                                                               Wv, p->m, (int64_t)p->Q * p->T, (uint32_t)items);
    return launched();
}

template <class A, int VEC>
int run_encode(const ccdc_plan_t *p, const void *Vbar, void *X, hipStream_t st)
{
    using E = typename A::elem;
    const uint32_t Wv = (uint32_t)(p->W / VEC), Lv = (uint32_t)(p->ell / VEC);
    const uint64_t items = (uint64_t)p->nround * (p->r + 1) * Lv;
    if (!fits_launch(items)) return CCDC_ESIZE;
    k_encode<A, VEC><<<cdiv(items, kBlock), kBlock, 0, st>>>((const E *)Vbar, (E *)X, p->r + 1, Lv, Wv,
                                                              (uint32_t)items);
    return launched();
}

template <class A, int VEC>
int run_decode(const ccdc_plan_t *p, const void *X, const void *Vbar, void *D, hipStream_t st)
{
    using E = typename A::elem;
    const uint32_t Wv = (uint32_t)(p->W / VEC), Lv = (uint32_t)(p->ell / VEC);
    const uint64_t items = (uint64_t)p->nround * (p->r + 1) * Wv;
    if (!fits_launch(items)) return CCDC_ESIZE;
    k_decode<A, VEC><<<cdiv(items, kBlock), kBlock, 0, st>>>((const E *)X, (const E *)Vbar, (E *)D, p->r + 1, Lv,
                                                              Wv, (uint32_t)items);
    return launched();
}

template <class A, int VEC, int R1>
void launch_shuffle(const ccdc_plan_t *p, const void *V, void *X, void *D, hipStream_t st)
{
    using E = typename A::elem;
    const uint32_t Wv = (uint32_t)(p->W / VEC), Lv = (uint32_t)(p->ell / VEC);
    const uint64_t items = (uint64_t)p->nround * (p->r + 1) * Lv;
    k_shuffle_fused<A, VEC, R1><<<cdiv(items, kBlock), kBlock, 0, st>>>(
        (const E *)V, (E *)X, (E *)D, p->d_src_off, p->r + 1, Lv, Wv, p->m, (int64_t)p->Q * p->T, (uint32_t)items);
}

template <class A, int VEC>
int run_shuffle(const ccdc_plan_t *p, const void *V, void *X, void *D, hipStream_t st)
{
    if (!fits_launch((uint64_t)p->nround * (p->r + 1) * (uint64_t)(p->ell / VEC))) return CCDC_ESIZE;
    switch (p->r + 1) {
    case 2: launch_shuffle<A, VEC, 2>(p, V, X, D, st); break;
    case 3: launch_shuffle<A, VEC, 3>(p, V, X, D, st); break;
    case 4: launch_shuffle<A, VEC, 4>(p, V, X, D, st); break;
    case 5: launch_shuffle<A, VEC, 5>(p, V, X, D, st); break;
    case 6: launch_shuffle<A, VEC, 6>(p, V, X, D, st); break;
    case 7: launch_shuffle<A, VEC, 7>(p, V, X, D, st); break;
    case 8: launch_shuffle<A, VEC, 8>(p, V, X, D, st); break;
    default: launch_shuffle<A, VEC, 0>(p, V, X, D, st); break;
    }
    return launched();
}

template <class A, int VEC>
int run_reduce(const ccdc_plan_t *p, const void *V, const void *D, void *Phi, hipStream_t st)
{
    using E = typename A::elem;
    const uint32_t Wv = (uint32_t)(p->W / VEC);
    const uint32_t tiles = cdiv(Wv, kBlock);
    const int split = p->red_split;
    const uint64_t blocks = (uint64_t)p->nout * split * tiles;
    const int64_t chunk_stride = (int64_t)p->J * p->Q * p->T;
    if (!fits_launch(blocks) || !fits_launch((uint64_t)chunk_stride / VEC)) return CCDC_ESIZE;
    using Acc = typename A::acc;
    WorkspaceOrder order(p, st, split > 1);
    k_reduce_rows<A, VEC><<<(uint32_t)blocks, kBlock, 0, st>>>((const E *)V, (const E *)D, (E *)Phi,
                                                                (Acc *)p->d_workspace, p->d_red_ptr, p->d_red_row,
                                                                p->d_red_out, Wv, tiles, split, chunk_stride);
    int rc = launched();
    if (rc != CCDC_OK || split == 1) return rc;
    const uint64_t items = (uint64_t)chunk_stride / VEC;
    const int G = reduce_final_groups((int64_t)items, split);
    k_reduce_final<A, VEC><<<cdiv(items, kBlock / G), kBlock, 0, st>>>((const Acc *)p->d_workspace, (E *)Phi, split,
                                                                        chunk_stride / VEC, (uint32_t)items, G);
    return launched();
}

}  // namespace

// ------------------------------------------------------------ entry points
extern "C" {

int ccdc_plan(int K, int r, int Q, int N, ccdc_plan_t **out) { return ccdc::build_plan(K, r, Q, N, false, 1, out); }

int ccdc_plan_jobs(int K, int r, int Q, int N, ccdc_plan_t **out) { return ccdc::build_plan(K, r, Q, N, true, 1, out); }

int ccdc_plan_jobs_repeated(int K, int r, int Q, int N, int gamma, ccdc_plan_t **out)
{
    return ccdc::build_plan(K, r, Q, N, true, gamma, out);
}

int ccdc_plan_compression(int K, int r, int Q, int N, ccdc_plan_t **out)
{
    return ccdc::build_compression_plan(K, r, Q, N, out);
}

void ccdc_plan_destroy(ccdc_plan_t *plan)
{
    if (!plan) return;
    release_device(plan);
    delete plan;
}

int ccdc_plan_bind(ccdc_plan_t *plan, int64_t T, int mode)
{
    if (!plan) return CCDC_EINVAL;
    const int rc = ccdc::bind_plan(plan, T, mode);
    if (rc == CCDC_OK) release_device(plan);     // tables of an earlier binding are stale
    return rc;
}

int ccdc_plan_upload(ccdc_plan_t *plan)
{
    if (!plan) return CCDC_EINVAL;
    if (!plan->bound) return CCDC_ESTATE;
    release_device(plan);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return CCDC_EHIP;
    }
    plan->device = dev;
    int rc = to_device(plan->src_off, &plan->d_src_off);
    if (rc == CCDC_OK) rc = to_device(plan->red_ptr, &plan->d_red_ptr);
    if (rc == CCDC_OK) rc = to_device(plan->red_row, &plan->d_red_row);
    if (rc == CCDC_OK) rc = to_device(plan->red_out, &plan->d_red_out);
    if (rc == CCDC_OK) rc = to_device(plan->loc_row, &plan->d_loc_row);
    if (rc == CCDC_OK) rc = to_device(plan->round_member, &plan->d_member);
    if (rc == CCDC_OK && !plan->row_files.empty()) rc = to_device(plan->row_files, &plan->d_row_files);
    if (rc == CCDC_OK && !plan->node_rows.empty()) rc = to_device(plan->node_rows, &plan->d_node_rows);
    if (rc == CCDC_OK && plan->workspace_bytes > 0 &&
        hipMalloc(&plan->d_workspace, plan->workspace_bytes) != hipSuccess) {
        plan->d_workspace = nullptr;
        (void)hipGetLastError();
        rc = CCDC_ENOMEM;
    }
    if (rc == CCDC_OK && plan->workspace_bytes > 0) {
        hipEvent_t ev = nullptr;
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
            (void)hipGetLastError();
            rc = CCDC_EHIP;
        }
        plan->ws_event = ev;
    }
    if (rc != CCDC_OK) {
        release_device(plan);
        return rc;
    }
    ccdc::pipeline_prepare(plan);                 // launch geometry of the one-pass kernel on this device
    (void)ccdc::scratch_address(nullptr);         // set-up for ccdc_pipeline_fused_noalloc, which reports a failure itself
    plan->uploaded = true;
    return CCDC_OK;
}

int ccdc_plan_query(const ccdc_plan_t *p, int what, void *out, size_t out_bytes)
{
    if (!p || !out) return CCDC_EINVAL;
    auto scalar = [&](int64_t v) {
        if (out_bytes < sizeof(int64_t)) return (int)CCDC_EINVAL;
        *static_cast<int64_t *>(out) = v;
        return (int)CCDC_OK;
    };
    auto table = [&](const void *src, size_t bytes) {
        if (out_bytes < bytes) return (int)CCDC_EINVAL;
        if (bytes) __builtin_memcpy(out, src, bytes);
        return (int)CCDC_OK;
    };
    const int64_t r1 = p->r + 1;
    switch (what) {
    case CCDC_Q_K: return scalar(p->K);
    case CCDC_Q_R: return scalar(p->r);
    case CCDC_Q_Q: return scalar(p->Q);
    case CCDC_Q_N: return scalar(p->N);
    case CCDC_Q_J: return scalar(p->J);
    case CCDC_Q_C: return scalar(p->c);
    case CCDC_Q_M: return scalar(p->m);
    case CCDC_Q_NBATCH: return scalar(p->nbatch);
    case CCDC_Q_NROUND: return scalar(p->nround);
    case CCDC_Q_NROWS: return scalar(p->nrows);
    case CCDC_Q_SCHEME: return scalar(p->compression ? 2 : (p->paper_jobs ? 1 : 0));
    case CCDC_Q_BATCH_FIRST: return table(p->batch_first.data(), p->batch_first.size() * 4);
    case CCDC_Q_NODE_BATCH: return table(p->node_batch.data(), p->node_batch.size() * 4);
    case CCDC_Q_PACKET_RECV: return table(p->pkt_recv.data(), p->pkt_recv.size() * 4);
    case CCDC_Q_PACKET_BATCH: return table(p->pkt_batch.data(), p->pkt_batch.size() * 4);
    case CCDC_Q_PACKET_SEND: return table(p->pkt_send.data(), p->pkt_send.size() * 4);
    case CCDC_Q_ROWS_PER_NODE: return scalar(p->rows_per_node);
    case CCDC_Q_NODE_ROWS: return table(p->node_rows.data(), p->node_rows.size() * 4);
    case CCDC_Q_FILE_NODES:
        return p->compression ? (int)CCDC_ESTATE : table(p->file_nodes.data(), p->file_nodes.size() * 4);
    case CCDC_Q_FILES_PER_NODE: return p->compression ? (int)CCDC_ESTATE : scalar(p->files_per_node);
    case CCDC_Q_NODE_FILES:
        return p->compression ? (int)CCDC_ESTATE : table(p->node_files.data(), p->node_files.size() * 4);
    case CCDC_Q_BATCH_JOB: return table(p->batch_job.data(), p->batch_job.size() * 4);
    case CCDC_Q_BATCH_FILE0: return table(p->batch_file0.data(), p->batch_file0.size() * 4);
    case CCDC_Q_BATCH_LABEL: return table(p->batch_label.data(), p->batch_label.size() * 4);
    case CCDC_Q_ROUND_MEMBER: return table(p->round_member.data(), p->round_member.size() * 4);
    case CCDC_Q_ROUND_BATCH: return table(p->round_batch.data(), p->round_batch.size() * 4);
    default: break;
    }
    if (!p->bound) {
        switch (what) {
        case CCDC_Q_T: case CCDC_Q_MODE: case CCDC_Q_W: case CCDC_Q_SEG_LEN: case CCDC_Q_SCHEDULED_ELEMS:
        case CCDC_Q_CLOSED_FORM_NUM: case CCDC_Q_CLOSED_FORM_DEN: case CCDC_Q_V_ELEMS: case CCDC_Q_VBAR_ELEMS:
        case CCDC_Q_X_ELEMS: case CCDC_Q_D_ELEMS: case CCDC_Q_PHI_ELEMS: case CCDC_Q_WORKSPACE_BYTES:
        case CCDC_Q_PACKET_LEN:
            return CCDC_ESTATE;
        default:
            return CCDC_EINVAL;
        }
    }
    switch (what) {
    case CCDC_Q_T: return scalar(p->T);
    case CCDC_Q_MODE: return scalar(p->mode);
    case CCDC_Q_W: return scalar(p->W);
    case CCDC_Q_SEG_LEN: return scalar(p->ell);
    case CCDC_Q_SCHEDULED_ELEMS: return scalar(p->scheduled);
    case CCDC_Q_CLOSED_FORM_NUM: return scalar(p->compression ? p->nrows * p->W : p->nround * r1 * p->W);
    case CCDC_Q_CLOSED_FORM_DEN: return scalar(p->compression ? 1 : p->r);
    case CCDC_Q_V_ELEMS: return scalar((int64_t)p->J * p->N * p->Q * p->T);
    case CCDC_Q_VBAR_ELEMS: return scalar(p->nrows * p->W);
    case CCDC_Q_X_ELEMS: return scalar(p->compression ? 0 : p->nrows * p->ell);
    case CCDC_Q_D_ELEMS: return scalar(p->nrows * p->W);
    case CCDC_Q_PHI_ELEMS: return scalar((int64_t)p->J * p->Q * p->T);
    case CCDC_Q_WORKSPACE_BYTES: return scalar((int64_t)p->workspace_bytes);
    case CCDC_Q_PACKET_LEN: return table(p->packet_len.data(), p->packet_len.size() * 8);
    default: return CCDC_EINVAL;
    }
}

const char *ccdc_strerror(int status)
{
    switch (status) {
    case CCDC_OK: return "ok";
    case CCDC_EINVAL: return "invalid argument";
    case CCDC_ENOMEM: return "out of memory";
    case CCDC_EHIP: return "HIP runtime error";
    case CCDC_ESIZE: return "size exceeds what the library indexes";
    case CCDC_ESTATE: return "plan is not bound/uploaded, or its device is not current";
    default: return "unknown status";
    }
}

int ccdc_combine(const ccdc_plan_t *plan, const void *V, void *Vbar, void *stream)
{
    int rc = ready(plan), vec = 1;
    if (rc != CCDC_OK) return rc;
    if ((rc = pick_vec(plan, &vec, V, (const void *)Vbar)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_combine<A, VEC>(plan, V, Vbar, st)));
}

int ccdc_encode(const ccdc_plan_t *plan, const void *Vbar, void *X, void *stream)
{
    int rc = ready(plan), vec = 1;
    if (rc != CCDC_OK) return rc;
    if (plan->compression) return CCDC_ESTATE;       // nothing is coded in that scheme
    if ((rc = pick_vec(plan, &vec, Vbar, (const void *)X)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_encode<A, VEC>(plan, Vbar, X, st)));
}

int ccdc_decode(const ccdc_plan_t *plan, const void *X, const void *Vbar, void *D, void *stream)
{
    int rc = ready(plan), vec = 1;
    if (rc != CCDC_OK) return rc;
    if (plan->compression) return CCDC_ESTATE;       // nothing is coded in that scheme
    if ((rc = pick_vec(plan, &vec, X, Vbar, (const void *)D)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_decode<A, VEC>(plan, X, Vbar, D, st)));
}

int ccdc_reduce(const ccdc_plan_t *plan, const void *V, const void *D, void *Phi, void *stream)
{
    int rc = ready(plan), vec = 1;
    if (rc != CCDC_OK) return rc;
    if ((rc = pick_vec(plan, &vec, V, D, (const void *)Phi)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_reduce<A, VEC>(plan, V, D, Phi, st)));
}

int ccdc_shuffle_fused(const ccdc_plan_t *plan, const void *V, void *X, void *D, void *stream)
{
    int rc = ready(plan), vec = 1;
    if (rc != CCDC_OK) return rc;
    if (plan->compression) return CCDC_ESTATE;       // nothing is coded in that scheme
    if ((rc = pick_vec(plan, &vec, V, (const void *)X, (const void *)D)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_shuffle<A, VEC>(plan, V, X, D, st)));
}

}  // extern "C"
