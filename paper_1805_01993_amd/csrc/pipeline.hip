// One-pass pipeline kernel (combine + encode + decode + reduce) and its entry point.
#include <type_traits>

#include "common.hpp"

namespace {
using namespace ccdc;

// ------------------------------------------------- whole path in one pass
// combine + encode + decode + reduce for a single-job plan.  A workgroup is one
// wavefront; lane = in-segment pack x; the workgroup walks a chunk of rounds.
// For a round it reads the r packs of each of the r+1 packets that sit at
// x (every needed element of V once), forms each sender's coded pack (written
// to X), decodes it for each receiver exactly as k_decode does, and adds the
// decoded pack to the receiver's running output.  Those running outputs (K nodes
// x r segments per lane) live in LDS, one private slot per lane: no atomics, no
// barriers, and since only the owning lane touches a slot the summation order is
// program order.  (LDS float atomics were measured several times slower than
// this read-add-write of the round's slots.)
// The files a node stores itself are added from V the same way.  With more than
// one chunk the per-chunk outputs go to the workspace and k_reduce_final adds
// them in chunk order.  Running outputs and chunk outputs are sums in the making
// (the algebra's acc type); they are narrowed to elements once, when Phi is written.
//
// LDS capacity, not registers, bounds how many wavefronts fit on a compute
// unit, so the loads of the next PF rounds are kept in flight in registers
// while the current round is decoded.  The round loop is branch-free so that
// the hardware load counter can be waited on partially: a short or empty last
// segment (RAGGED) is read at a clamped position and replaced by zeros.
// MULTI (a batch has more than one file) adds the file loop and gives up the
// prefetch.
#ifndef CCDC_PIPE_PREFETCH_REGS
#define CCDC_PIPE_PREFETCH_REGS 160               // registers a lane may spend on rounds in flight
#endif
#ifndef CCDC_PIPE_PREFETCH_MAX
#define CCDC_PIPE_PREFETCH_MAX 8
#endif
#ifndef CCDC_PIPE_VMCNT_BUDGET
#define CCDC_PIPE_VMCNT_BUDGET 56                 // outstanding loads+stores; the counter has 6 bits
#endif
template <int VEC, int R1>
constexpr int prefetch_depth()
{
    constexpr int by_regs = CCDC_PIPE_PREFETCH_REGS / (VEC * R1 * (R1 - 1));
    constexpr int by_cnt = CCDC_PIPE_VMCNT_BUDGET / (R1 * (R1 - 1) + R1);
    constexpr int d = by_regs < by_cnt ? by_regs : by_cnt;
    return d < 1 ? 1 : (d > CCDC_PIPE_PREFETCH_MAX ? CCDC_PIPE_PREFETCH_MAX : d);
}

template <class A, int VEC, int R1, bool MULTI, bool RAGGED>
__global__ __launch_bounds__(ccdc::kPipeLanes) void k_pipeline(
    const typename A::elem *__restrict__ V, typename A::elem *__restrict__ X, typename A::elem *__restrict__ Phi,
    typename A::acc *__restrict__ part, const int64_t *__restrict__ src_off, const int32_t *__restrict__ member, const int64_t *__restrict__ loc_row,
    int K, uint32_t Lv, uint32_t Wv, int m, int64_t file_stride, uint32_t R, uint32_t tiles, uint32_t chunks,
    uint32_t n_loc, int64_t chunk_stride)
{
    using E = typename A::elem;
    using O = Ops<A, VEC>;
    using P = typename O::P;
    using Q = typename O::Q;
    constexpr int r = R1 - 1;
    constexpr int LANES = ccdc::kPipeLanes;
    constexpr int PF = MULTI ? 1 : prefetch_depth<VEC, R1>();
    constexpr int PFL = PF * R1;                     // own-file rows in flight (r packs each)
    extern __shared__ __align__(16) unsigned char smem[];
    Q *acc = reinterpret_cast<Q *>(smem) + threadIdx.x;      // slot i of this lane: acc[i * LANES]

    // Workgroups are handed to the 8 XCDs round-robin.  When the rounds are cut
    // into chunks, renumber them so that each XCD gets a contiguous range of
    // (chunk, tile) pairs: the tiles of one chunk (adjacent pieces of the same
    // rows, the same table entries) then run next to each other in time behind one
    // L2.  With a single chunk the hardware order is kept: all XCDs then sweep the
    // same window of every row together (measured: 2 % either way).
    constexpr uint32_t XCDS = 8;
    const uint32_t nb = gridDim.x, q = nb / XCDS, rem = nb % XCDS;
    const uint32_t xcd = blockIdx.x % XCDS, j = blockIdx.x / XCDS;
    const uint32_t logical =
        chunks > 1 ? (xcd < rem ? xcd * (q + 1) : rem * (q + 1) + (xcd - rem) * q) + j : blockIdx.x;
    const uint32_t tile = logical % tiles, chunk = logical / tiles;
    const uint32_t x = tile * LANES + threadIdx.x;
    if (x >= Lv) return;

    bool valid[r];                    // does segment rho reach position x (short / empty tail)
    uint32_t offb[r];                 // byte offset of pack x of segment rho inside a packet
#pragma unroll
    for (int rho = 0; rho < r; rho++) {
        const uint32_t pos = rho * Lv + x;
        valid[rho] = !RAGGED || pos < Wv;
        offb[rho] = (valid[rho] ? pos : Wv - 1) * (uint32_t)(VEC * sizeof(E));
    }
    auto pack_at = [](const E *row, uint32_t byte_off) -> P {
        return load_stream<P>(reinterpret_cast<const char *>(row) + byte_off);
    };
    for (int i = 0; i < K * r; i++) acc[i * LANES] = O::azero();

    struct Row {                      // one round's table entries (wave-uniform)
        int64_t src[R1];              // element offset in V of packet b's first file
        int node[R1];                 // s_b
    };
    struct Stage {
        P w[R1][r];                   // w[b][rho]: pack x of segment rho of Vbar[u][b]
        int node[R1];
    };
    auto fetch_row = [&](uint32_t u, Row &t) {
        const int64_t *src = src_off + (size_t)u * R1;
        const int32_t *mem = member + (size_t)u * R1;
#pragma unroll
        for (int b = 0; b < R1; b++) {
            t.src[b] = src[b];
            t.node[b] = mem[b];
        }
    };
    auto issue = [&](const Row &t, Stage &s) {
#pragma unroll
        for (int b = 0; b < R1; b++) {
            s.node[b] = t.node[b];
            const E *row = V + t.src[b];
#pragma unroll
            for (int rho = 0; rho < r; rho++) {
                P v = pack_at(row, offb[rho]);
                if constexpr (MULTI) {
                    Q sum = O::widen(v);
                    for (int f = 1; f < m; f++) sum = O::accum(sum, pack_at(row + f * file_stride, offb[rho]));
                    v = O::narrow(sum);
                }
                if constexpr (RAGGED) v = O::select(valid[rho], v, O::zero());
                s.w[b][rho] = v;
            }
        }
    };
    // Decode one round and add the r(r+1) decoded packs to their owners' outputs.
    // The r(r+1) slots of a round are distinct (receiver b, segment rank(a,b)), so
    // they are read together, updated, and written together: one LDS wait a round.
    auto consume = [&](uint32_t u, const Stage &s) {
        Q cur[R1][r];                 // cur[b][rho]: running output of node s_b, segment rho
#pragma unroll
        for (int b = 0; b < R1; b++)
#pragma unroll
            for (int rho = 0; rho < r; rho++) cur[b][rho] = acc[(s.node[b] * r + rho) * LANES];
#pragma unroll
        for (int a = 0; a < R1; a++) {
            P coded = O::zero();
#pragma unroll
            for (int b = 0; b < R1; b++)
                if (b != a) coded = O::code(coded, s.w[b][a - (a > b ? 1 : 0)]);
            store_stream(reinterpret_cast<P *>(X) + ((size_t)u * R1 + a) * Lv + x, coded);
#pragma unroll
            for (int b = 0; b < R1; b++) {
                if (b == a) continue;
                const int rho = a - (a > b ? 1 : 0);
                P d = coded;
#pragma unroll
                for (int b2 = 0; b2 < R1; b2++)
                    if (b2 != a && b2 != b) d = O::uncode(d, s.w[b2][a - (a > b2 ? 1 : 0)]);
                // a slot past a short segment collects zeros and is never written out
                cur[b][rho] = O::accum(cur[b][rho], d);
            }
        }
#pragma unroll
        for (int b = 0; b < R1; b++)
#pragma unroll
            for (int rho = 0; rho < r; rho++) acc[(s.node[b] * r + rho) * LANES] = cur[b][rho];
    };

    const uint32_t u0 = (uint32_t)((uint64_t)R * chunk / chunks);
    const uint32_t u1 = (uint32_t)((uint64_t)R * (chunk + 1) / chunks);
    const uint32_t n = u1 - u0;
    if (n > 0) {
        Stage st[PF];
#pragma unroll
        for (int s = 0; s < PF; s++) {
            Row t;
            fetch_row(u0 + ((uint32_t)s < n ? s : n - 1), t);
            issue(t, st[s]);
        }
        // Full groups of PF rounds with no branch inside (a branch makes the
        // compiler drain every outstanding load); the remainder is handled after
        // the loop.  Past the end the last round is read again (never consumed).
        // The table row is requested before decoding so that it arrives meanwhile.
        const uint32_t full = n / PF;
        for (uint32_t g = 0; g < full; g++) {
#pragma unroll
            for (int s = 0; s < PF; s++) {
                const uint32_t i = g * PF + s, nxt = i + PF;
                Row t;
                fetch_row(u0 + (nxt < n ? nxt : n - 1), t);
                consume(u0 + i, st[s]);
                issue(t, st[s]);
            }
        }
#pragma unroll
        for (int s = 0; s < PF; s++)
            if (full * PF + s < n) consume(u0 + full * PF + s, st[s]);
    }

    // the files each node stores itself; a table entry is (element offset << 12) | node
    struct Own {
        P w[r];
        int k;
    };
    auto issue_own = [&](int64_t e, Own &s) {
        s.k = (int)(e & 4095);
        const E *row = V + (e >> 12);
#pragma unroll
        for (int rho = 0; rho < r; rho++) {
            P t = pack_at(row, offb[rho]);
            if constexpr (RAGGED) t = O::select(valid[rho], t, O::zero());
            s.w[rho] = t;
        }
    };
    auto consume_own = [&](const Own &s) {
        Q cur[r];
#pragma unroll
        for (int rho = 0; rho < r; rho++) cur[rho] = acc[(s.k * r + rho) * LANES];
#pragma unroll
        for (int rho = 0; rho < r; rho++) acc[(s.k * r + rho) * LANES] = O::accum(cur[rho], s.w[rho]);
    };
    const uint32_t i0 = (uint32_t)((uint64_t)n_loc * chunk / chunks);
    const uint32_t i1 = (uint32_t)((uint64_t)n_loc * (chunk + 1) / chunks);
    const uint32_t nl = i1 - i0;
    if (nl > 0) {
        Own ow[PFL];
#pragma unroll
        for (int s = 0; s < PFL; s++) issue_own(loc_row[i0 + ((uint32_t)s < nl ? s : nl - 1)], ow[s]);
        const uint32_t full = nl / PFL;
        for (uint32_t g = 0; g < full; g++) {
#pragma unroll
            for (int s = 0; s < PFL; s++) {
                const uint32_t nxt = g * PFL + s + PFL;
                const int64_t e = loc_row[i0 + (nxt < nl ? nxt : nl - 1)];
                consume_own(ow[s]);
                issue_own(e, ow[s]);
            }
        }
#pragma unroll
        for (int s = 0; s < PFL; s++)
            if (full * PFL + s < nl) consume_own(ow[s]);
    }

    // write the chunk's outputs: the only chunk straight to Phi, else to its slice of the workspace
    const int64_t W = (int64_t)Wv * VEC;
    typename A::acc *dst = part + (int64_t)chunk * chunk_stride;
    for (int k = 0; k < K; k++) {
#pragma unroll
        for (int rho = 0; rho < r; rho++) {
            if (!valid[rho]) continue;
            const int64_t pos = k * W + (int64_t)(offb[rho] / sizeof(E));        // element index in [K][W]
            const Q v = acc[(k * r + rho) * LANES];
            if (chunks == 1) *reinterpret_cast<P *>(Phi + pos) = O::narrow(v);
            else *reinterpret_cast<Q *>(dst + pos) = v;
        }
    }
}

// Every k_pipeline<A, VEC, R1, *, *> has this signature.
template <class A>
using PipeKernel = void (*)(const typename A::elem *, typename A::elem *, typename A::elem *, typename A::acc *,
                            const int64_t *, const int32_t *, const int64_t *, int, uint32_t, uint32_t, int, int64_t,
                            uint32_t, uint32_t, uint32_t, uint32_t, int64_t);

// The instantiation a plan runs: MULTI when a batch has several files, RAGGED
// when the last segment is short or empty.  Null for an r the kernel is not
// unrolled for.
template <class A, int VEC>
PipeKernel<A> pipeline_kernel(const ccdc_plan_t *p)
{
    const bool ragged = p->ell * p->r != p->W;
    auto of = [&](auto r1) -> PipeKernel<A> {
        constexpr int R1 = decltype(r1)::value;
        if (p->m > 1) return k_pipeline<A, VEC, R1, true, true>;
        if (ragged) return k_pipeline<A, VEC, R1, false, true>;
        return k_pipeline<A, VEC, R1, false, false>;
    };
    switch (p->r + 1) {
    case 2: return of(std::integral_constant<int, 2>());
    case 3: return of(std::integral_constant<int, 3>());
    case 4: return of(std::integral_constant<int, 4>());
    case 5: return of(std::integral_constant<int, 5>());
    case 6: return of(std::integral_constant<int, 6>());
    default: return nullptr;
    }
}

template <int VEC>
size_t pipeline_lds(const ccdc_plan_t *p)
{
    return (size_t)p->K * p->r * ccdc::kPipeLanes * VEC * sizeof(float);     // every algebra sums in 4 bytes
}

template <int VEC>
uint32_t pipeline_tiles(const ccdc_plan_t *p)
{
    return cdiv((uint64_t)(p->ell / VEC), ccdc::kPipeLanes);
}

// Round chunks for a launch with VEC-element packs: when there are fewer column
// tiles than wavefront slots on the device, the rounds are cut so that the grid
// is one resident wave of equally loaded workgroups (bounded by the workspace).
template <class A, int VEC>
int chunks_for(const ccdc_plan_t *p)
{
    PipeKernel<A> kernel = pipeline_kernel<A, VEC>(p);
    if (!kernel || p->ell % VEC != 0 || p->T % VEC != 0) return 1;
    int per_cu = 0, cus = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, ccdc::kPipeLanes, pipeline_lds<VEC>(p)) !=
            hipSuccess ||
        per_cu < 1 || cus < 1) {
        (void)hipGetLastError();
        return 1;
    }
    int64_t chunks = (int64_t)per_cu * cus / pipeline_tiles<VEC>(p);
    if (chunks < 1) chunks = 1;
    if (chunks > p->pipe_max_chunks) chunks = p->pipe_max_chunks;
    return (int)chunks;
}

template <class A>
void prepare(ccdc_plan_t *p)
{
    p->pipe_chunks[0] = chunks_for<A, 1>(p);
    p->pipe_chunks[1] = p->pipe_vec >= 2 ? chunks_for<A, 2>(p) : 1;
    p->pipe_chunks[2] = p->pipe_vec >= 4 ? chunks_for<A, 4>(p) : 1;
}

// One launch of the pass with `chunks` round chunks; partial outputs of the
// chunks go to `part` (chunks * K * W sums) and k_reduce_final adds them.
template <class A, int VEC>
int run_pipeline(const ccdc_plan_t *p, const void *V, void *X, void *Phi, void *part, int chunks, bool wide_final,
                 hipStream_t st)
{
    using E = typename A::elem;
    using Acc = typename A::acc;
    PipeKernel<A> kernel = pipeline_kernel<A, VEC>(p);
    if (!kernel) return CCDC_ESIZE;
    const uint32_t Wv = (uint32_t)(p->W / VEC), Lv = (uint32_t)(p->ell / VEC);
    const uint32_t tiles = pipeline_tiles<VEC>(p);
    if (!fits_launch((uint64_t)tiles * (uint64_t)chunks) || !fits_launch((uint64_t)p->K * (uint64_t)p->W)) return CCDC_ESIZE;
    kernel<<<tiles * (uint32_t)chunks, ccdc::kPipeLanes, pipeline_lds<VEC>(p), st>>>(
        (const E *)V, (E *)X, (E *)Phi, (Acc *)part, p->d_src_off, p->d_member, p->d_loc_row, p->K, Lv, Wv, p->m,
        (int64_t)p->Q * p->T, (uint32_t)p->nround, tiles, (uint32_t)chunks, (uint32_t)(p->K * p->pipe_local_rows),
        (int64_t)p->K * p->W);
    int rc = launched();
    if (rc != CCDC_OK || chunks == 1) return rc;
    const int64_t n = (int64_t)p->K * p->W;
    if (wide_final) {
        const int G = reduce_final_groups(n / 4, chunks);
        k_reduce_final<A, 4><<<cdiv(n / 4, kBlock / G), kBlock, 0, st>>>((const Acc *)part, (E *)Phi, chunks, n / 4,
                                                                          (uint32_t)(n / 4), G);
    } else {
        const int G = reduce_final_groups(n, chunks);
        k_reduce_final<A, 1><<<cdiv(n, kBlock / G), kBlock, 0, st>>>((const Acc *)part, (E *)Phi, chunks, n,
                                                                      (uint32_t)n, G);
    }
    return launched();
}

}  // namespace

namespace ccdc {

// ccdc_pipeline_fused: checks, pack width, dispatch on the algebra.  The partial
// outputs of round chunks go to the plan's workspace, or, when the caller brings
// a buffer (own_part, of own_part_bytes bytes), to that one; a launch whose
// chunks do not fit a brought buffer is refused.
int pipeline_entry(const ccdc_plan_t *plan, const void *V, void *X, void *Phi, void *stream, void *own_part,
                   size_t own_part_bytes)
{
    int rc = ready(plan), vec_any = 1;
    if (rc != CCDC_OK) return rc;
    if (plan->compression) return CCDC_ESTATE;       // nothing is coded in that scheme
    if (!plan->pipe_ok) return CCDC_ESIZE;
    if ((rc = pick_vec(plan, &vec_any, V, (const void *)X, (const void *)Phi)) != CCDC_OK) return rc;
    // widest pack allowed by the plan's LDS budget (the running outputs take 4 bytes
    // an element in every mode) and by the pointers
    const size_t eb = (size_t)elem_bytes(plan->mode);
    int vec = plan->pipe_vec;
    while (vec > 1 && !(aligned(V, eb * vec) && aligned(X, eb * vec) && aligned(Phi, eb * vec))) vec /= 2;
    const bool wide_final = vec_any >= 4;            // Phi can be written four elements at a time
    const int chunks = plan->pipe_chunks[vec == 4 ? 2 : (vec == 2 ? 1 : 0)];
    if (chunks < 1) return CCDC_ESTATE;
    void *part = plan->d_workspace;
    if (own_part) {
        if (chunks > 1 && (uint64_t)chunks * (uint64_t)plan->K * (uint64_t)plan->W * 4u > (uint64_t)own_part_bytes)
            return CCDC_ESIZE;
        part = own_part;
    }
    hipStream_t st = (hipStream_t)stream;
    WorkspaceOrder order(plan, st, !own_part && chunks > 1);
    if (plan->mode == CCDC_F32_SUM) {
        if (vec == 4) return run_pipeline<SumF32, 4>(plan, V, X, Phi, part, chunks, wide_final, st);
        if (vec == 2) return run_pipeline<SumF32, 2>(plan, V, X, Phi, part, chunks, wide_final, st);
        return run_pipeline<SumF32, 1>(plan, V, X, Phi, part, chunks, wide_final, st);
    }
    if (plan->mode == CCDC_F32_SUM_XOR) {
        if (vec == 4) return run_pipeline<HybF32, 4>(plan, V, X, Phi, part, chunks, wide_final, st);
        if (vec == 2) return run_pipeline<HybF32, 2>(plan, V, X, Phi, part, chunks, wide_final, st);
        return run_pipeline<HybF32, 1>(plan, V, X, Phi, part, chunks, wide_final, st);
    }
    if (plan->mode == CCDC_BF16_SUM_XOR) {
        if (vec == 4) return run_pipeline<HybBF16, 4>(plan, V, X, Phi, part, chunks, wide_final, st);
        if (vec == 2) return run_pipeline<HybBF16, 2>(plan, V, X, Phi, part, chunks, wide_final, st);
        return run_pipeline<HybBF16, 1>(plan, V, X, Phi, part, chunks, wide_final, st);
    }
    if (plan->mode == CCDC_F16_SUM_XOR) {
        if (vec == 4) return run_pipeline<HybF16, 4>(plan, V, X, Phi, part, chunks, wide_final, st);
        if (vec == 2) return run_pipeline<HybF16, 2>(plan, V, X, Phi, part, chunks, wide_final, st);
        return run_pipeline<HybF16, 1>(plan, V, X, Phi, part, chunks, wide_final, st);
    }
    if (vec == 4) return run_pipeline<XorU32, 4>(plan, V, X, Phi, part, chunks, wide_final, st);
    if (vec == 2) return run_pipeline<XorU32, 2>(plan, V, X, Phi, part, chunks, wide_final, st);
    return run_pipeline<XorU32, 1>(plan, V, X, Phi, part, chunks, wide_final, st);
}

void pipeline_prepare(ccdc_plan_t *p)
{
    p->pipe_chunks[0] = p->pipe_chunks[1] = p->pipe_chunks[2] = 1;
    if (!p->pipe_ok) return;
    switch (p->mode) {
    case CCDC_F32_SUM: prepare<SumF32>(p); break;
    case CCDC_F32_SUM_XOR: prepare<HybF32>(p); break;
    case CCDC_BF16_SUM_XOR: prepare<HybBF16>(p); break;
    case CCDC_F16_SUM_XOR: prepare<HybF16>(p); break;
    default: prepare<XorU32>(p); break;
    }
}

}  // namespace ccdc

extern "C" {

int ccdc_pipeline_fused(const ccdc_plan_t *plan, const void *V, void *X, void *Phi, void *stream)
{
    return ccdc::pipeline_entry(plan, V, X, Phi, stream, nullptr, 0);
}

}  // extern "C"
