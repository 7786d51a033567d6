// One-pass pipeline kernel (combine + encode + decode + reduce) and its entry point.
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
// x r segments per lane) live in LDS, one private slot per lane, so there are no
// atomics and no barriers and the summation order is fixed.  The files a node
// stores itself are added from V the same way.  With more than one chunk the
// per-chunk outputs go to the workspace and k_reduce_final adds them in order.
//
// LDS capacity, not registers, bounds how many wavefronts fit on a compute
// unit, so the loads of the next PF rounds are kept in flight in registers
// while the current round is decoded (PF = 1 and a file loop when a batch has
// more than one file).
template <int VEC, int R1>
constexpr int prefetch_depth()
{
    constexpr int regs = VEC * R1 * (R1 - 1);      // registers one round's packs take
    constexpr int d = 160 / regs;
    return d < 1 ? 1 : (d > 8 ? 8 : d);
}

template <class A, int VEC, int R1, bool MULTI>
__global__ __launch_bounds__(ccdc::kPipeLanes) void k_pipeline(
    const typename A::elem *__restrict__ V, typename A::elem *__restrict__ X, typename A::elem *__restrict__ out,
    const int64_t *__restrict__ src_off, const int32_t *__restrict__ member, const int64_t *__restrict__ loc_row,
    int K, uint32_t Lv, uint32_t Wv, int m, int64_t file_stride, uint32_t R, uint32_t tiles, uint32_t chunks,
    uint32_t n_loc, uint32_t loc_rows, int64_t chunk_stride)
{
    using E = typename A::elem;
    using O = Ops<A, VEC>;
    using P = typename O::P;
    constexpr int r = R1 - 1;
    constexpr int LANES = ccdc::kPipeLanes;
    constexpr int PF = MULTI ? 1 : prefetch_depth<VEC, R1>();
    constexpr int PFL = PF * R1;                     // own-file rows in flight (r packs each)
    extern __shared__ __align__(16) unsigned char smem[];
    P *acc = reinterpret_cast<P *>(smem) + threadIdx.x;      // slot i of this lane: acc[i * LANES]

    const uint32_t tile = blockIdx.x % tiles, chunk = blockIdx.x / tiles;
    const uint32_t x = tile * LANES + threadIdx.x;
    if (x >= Lv) return;

    bool valid[r];                    // does segment rho reach position x (short / empty tail)
#pragma unroll
    for (int rho = 0; rho < r; rho++) valid[rho] = rho * Lv + x < Wv;

    for (int i = 0; i < K * r; i++) acc[i * LANES] = O::zero();

    struct Stage {
        P w[R1][r];                   // w[b][rho]: pack x of segment rho of Vbar[u][b]
        int node[R1];                 // s_b
    };
    auto issue = [&](uint32_t u, Stage &s) {
        const int64_t *src = src_off + (size_t)u * R1;
        const int32_t *mem = member + (size_t)u * R1;
#pragma unroll
        for (int b = 0; b < R1; b++) s.node[b] = mem[b];
#pragma unroll
        for (int b = 0; b < R1; b++) {
            const E *p0 = V + src[b] + (int64_t)x * VEC;
#pragma unroll
            for (int rho = 0; rho < r; rho++) {
                if (valid[rho]) {
                    const E *q = p0 + (int64_t)rho * Lv * VEC;
                    P t = *reinterpret_cast<const P *>(q);
                    if constexpr (MULTI)
                        for (int f = 1; f < m; f++) t = O::add(t, *reinterpret_cast<const P *>(q + f * file_stride));
                    s.w[b][rho] = t;
                } else {
                    s.w[b][rho] = O::zero();
                }
            }
        }
    };
    auto consume = [&](uint32_t u, const Stage &s) {
#pragma unroll
        for (int a = 0; a < R1; a++) {
            P coded = O::zero();
#pragma unroll
            for (int b = 0; b < R1; b++)
                if (b != a) coded = O::add(coded, s.w[b][a - (a > b ? 1 : 0)]);
            reinterpret_cast<P *>(X)[((size_t)u * R1 + a) * Lv + x] = coded;
#pragma unroll
            for (int b = 0; b < R1; b++) {
                if (b == a) continue;
                const int rho = a - (a > b ? 1 : 0);
                if (!valid[rho]) continue;
                P d = coded;
#pragma unroll
                for (int b2 = 0; b2 < R1; b2++)
                    if (b2 != a && b2 != b) d = O::sub(d, s.w[b2][a - (a > b2 ? 1 : 0)]);
                P *slot = acc + (s.node[b] * r + rho) * LANES;
                *slot = O::add(*slot, d);
            }
        }
    };

    const uint32_t u0 = (uint32_t)((uint64_t)R * chunk / chunks);
    const uint32_t u1 = (uint32_t)((uint64_t)R * (chunk + 1) / chunks);
    const uint32_t n = u1 - u0;
    if (n > 0) {
        Stage st[PF];
#pragma unroll
        for (int s = 0; s < PF; s++) issue(u0 + ((uint32_t)s < n ? s : n - 1), st[s]);
        for (uint32_t base = 0; base < n; base += PF) {
#pragma unroll
            for (int s = 0; s < PF; s++) {
                const uint32_t i = base + s;
                if (i < n) consume(u0 + i, st[s]);
                // keep PF rounds in flight; past the end the last round is read again
                const uint32_t nxt = i + PF;
                issue(u0 + (nxt < n ? nxt : n - 1), st[s]);
            }
        }
    }

    // the files each node stores itself
    struct Own {
        P w[r];
        uint32_t k;
    };
    auto issue_own = [&](uint32_t i, Own &s) {
        s.k = i / loc_rows;
        const E *row = V + loc_row[i] + (int64_t)x * VEC;
#pragma unroll
        for (int rho = 0; rho < r; rho++)
            s.w[rho] = valid[rho] ? *reinterpret_cast<const P *>(row + (int64_t)rho * Lv * VEC) : O::zero();
    };
    auto consume_own = [&](const Own &s) {
#pragma unroll
        for (int rho = 0; rho < r; rho++) {
            if (!valid[rho]) continue;
            P *slot = acc + (s.k * r + rho) * LANES;
            *slot = O::add(*slot, s.w[rho]);
        }
    };
    const uint32_t i0 = (uint32_t)((uint64_t)n_loc * chunk / chunks);
    const uint32_t i1 = (uint32_t)((uint64_t)n_loc * (chunk + 1) / chunks);
    const uint32_t nl = i1 - i0;
    if (nl > 0) {
        Own ow[PFL];
#pragma unroll
        for (int s = 0; s < PFL; s++) issue_own(i0 + ((uint32_t)s < nl ? s : nl - 1), ow[s]);
        for (uint32_t base = 0; base < nl; base += PFL) {
#pragma unroll
            for (int s = 0; s < PFL; s++) {
                const uint32_t i = base + s;
                if (i < nl) consume_own(ow[s]);
                const uint32_t nxt = i + PFL;
                issue_own(i0 + (nxt < nl ? nxt : nl - 1), ow[s]);
            }
        }
    }

    E *dst = out + (int64_t)chunk * chunk_stride + (int64_t)x * VEC;
    const int64_t W = (int64_t)Wv * VEC;
    for (int k = 0; k < K; k++) {
#pragma unroll
        for (int rho = 0; rho < r; rho++)
            if (valid[rho]) *reinterpret_cast<P *>(dst + k * W + (int64_t)rho * Lv * VEC) = acc[(k * r + rho) * LANES];
    }
}

// Round chunks for this launch: when there are fewer column tiles than
// wavefront slots on the device, cut the rounds so that the grid is one
// resident wave of equally loaded workgroups (bounded by the workspace).
template <class KernelT>
int chunks_for(const ccdc_plan_t *p, KernelT kernel, uint32_t tiles, size_t lds)
{
    int per_cu = 0, cus = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, ccdc::kPipeLanes, lds) != hipSuccess ||
        per_cu < 1 || cus < 1) {
        (void)hipGetLastError();
        return 1;
    }
    const int64_t slots = (int64_t)per_cu * cus;
    int64_t chunks = slots / tiles;
    if (chunks < 1) chunks = 1;
    if (chunks > p->pipe_max_chunks) chunks = p->pipe_max_chunks;
    return (int)chunks;
}

template <class A, int VEC, int R1>
int launch_pipeline(const ccdc_plan_t *p, const void *V, void *X, void *Phi, hipStream_t st, int *chunks_out)
{
    using E = typename A::elem;
    const uint32_t Wv = (uint32_t)(p->W / VEC), Lv = (uint32_t)(p->ell / VEC);
    const uint32_t tiles = cdiv(Lv, ccdc::kPipeLanes);
    const size_t lds = (size_t)p->K * p->r * ccdc::kPipeLanes * VEC * sizeof(E);
    auto go = [&](auto kernel) {
        const int chunks = chunks_for(p, kernel, tiles, lds);
        void *out = chunks > 1 ? p->d_workspace : Phi;
        kernel<<<tiles * (uint32_t)chunks, ccdc::kPipeLanes, lds, st>>>(
            (const E *)V, (E *)X, (E *)out, p->d_src_off, p->d_member, p->d_loc_row, p->K, Lv, Wv, p->m,
            (int64_t)p->Q * p->T, (uint32_t)p->nround, tiles, (uint32_t)chunks,
            (uint32_t)(p->K * p->pipe_local_rows), (uint32_t)p->pipe_local_rows, (int64_t)p->K * p->W);
        *chunks_out = chunks;
    };
    if (p->m > 1) go(k_pipeline<A, VEC, R1, true>);
    else go(k_pipeline<A, VEC, R1, false>);
    return launched();
}

template <class A, int VEC>
int run_pipeline(const ccdc_plan_t *p, const void *V, void *X, void *Phi, bool wide_final, hipStream_t st)
{
    using E = typename A::elem;
    int chunks = 1, rc;
    switch (p->r + 1) {
    case 2: rc = launch_pipeline<A, VEC, 2>(p, V, X, Phi, st, &chunks); break;
    case 3: rc = launch_pipeline<A, VEC, 3>(p, V, X, Phi, st, &chunks); break;
    case 4: rc = launch_pipeline<A, VEC, 4>(p, V, X, Phi, st, &chunks); break;
    case 5: rc = launch_pipeline<A, VEC, 5>(p, V, X, Phi, st, &chunks); break;
    case 6: rc = launch_pipeline<A, VEC, 6>(p, V, X, Phi, st, &chunks); break;
    default: return CCDC_ESIZE;
    }
    if (rc != CCDC_OK || chunks == 1) return rc;
    const int64_t n = (int64_t)p->K * p->W;
    if (wide_final) {
        k_reduce_final<A, 4><<<cdiv(n / 4, kBlock), kBlock, 0, st>>>((const E *)p->d_workspace, (E *)Phi, chunks, n / 4,
                                                                      (uint32_t)(n / 4));
    } else {
        k_reduce_final<A, 1><<<cdiv(n, kBlock), kBlock, 0, st>>>((const E *)p->d_workspace, (E *)Phi, chunks, n,
                                                                  (uint32_t)n);
    }
    return launched();
}

}  // namespace

extern "C" {

int ccdc_pipeline_fused(const ccdc_plan_t *plan, const void *V, void *X, void *Phi, void *stream)
{
    int rc = ready(plan), vec4 = 1;
    if (rc != CCDC_OK) return rc;
    if (!plan->pipe_ok) return CCDC_ESIZE;
    if ((rc = pick_vec(plan, &vec4, V, (const void *)X, (const void *)Phi)) != CCDC_OK) return rc;
    // widest pack allowed by the plan's LDS budget and by the pointers
    int vec = plan->pipe_vec;
    while (vec > 1 && !(aligned(V, 4 * vec) && aligned(X, 4 * vec) && aligned(Phi, 4 * vec))) vec /= 2;
    const bool wide_final = vec4 == 4;
    hipStream_t st = (hipStream_t)stream;
    if (plan->mode == CCDC_F32_SUM) {
        if (vec == 4) return run_pipeline<SumF32, 4>(plan, V, X, Phi, wide_final, st);
        if (vec == 2) return run_pipeline<SumF32, 2>(plan, V, X, Phi, wide_final, st);
        return run_pipeline<SumF32, 1>(plan, V, X, Phi, wide_final, st);
    }
    if (vec == 4) return run_pipeline<XorU32, 4>(plan, V, X, Phi, wide_final, st);
    if (vec == 2) return run_pipeline<XorU32, 2>(plan, V, X, Phi, wide_final, st);
    return run_pipeline<XorU32, 1>(plan, V, X, Phi, wide_final, st);
}

}  // extern "C"
