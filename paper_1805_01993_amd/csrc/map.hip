// A stand-in for the Map phase (Sec. III): every file w_n of a job is mapped into the Q
// intermediate values v_{q,n} = g_q(w_n).  The paper leaves g_q free; the stand-in is the
// gradient step its motivation (distributed gradient descent, Sec. I) is about, for the
// quadratic model whose minimiser is the mean of the data: a file is a data vector of Q*T
// numbers, the job has a model theta of Q*T numbers, and
//     v_{q,n}[t] = d/dtheta (1/2 |theta - w_n|^2) at chunk q  =  theta[q][t] - w_n[q][t]
// (XOR in the field F_{2^T}).  Summed over the files by the shuffle path, the outputs are
// the chunks of the full gradient N*theta - sum_n w_n.  One streaming pass: a work item
// makes one pack of V from one pack of a file and one pack of theta (which every file of
// the job re-reads, so it stays in cache).
#include "common.hpp"

namespace {
using namespace ccdc;

template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_map(const typename A::elem *files,      // may be V itself
                                                const typename A::elem *__restrict__ theta,
                                                typename A::elem *V, uint64_t job_packs, uint64_t model_packs,
                                                uint64_t items)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint64_t idx = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= items) return;
    const uint64_t job = idx / job_packs, e = (idx - job * job_packs) % model_packs;
    const P data = load_stream<P>(reinterpret_cast<const P *>(files) + idx);
    const P model = reinterpret_cast<const P *>(theta)[job * model_packs + e];
    store_stream(reinterpret_cast<P *>(V) + idx, O::gradient(model, data));
}

template <class A, int VEC>
int run_map(const ccdc_plan_t *p, const void *files, const void *theta, void *V, hipStream_t st)
{
    using E = typename A::elem;
    const uint64_t model_packs = (uint64_t)p->Q * p->T / VEC, job_packs = (uint64_t)p->N * model_packs;
    const uint64_t items = (uint64_t)p->J * job_packs;
    if (!fits_launch((items + kBlock - 1) / kBlock)) return CCDC_ESIZE;
    k_map<A, VEC><<<(uint32_t)((items + kBlock - 1) / kBlock), kBlock, 0, st>>>((const E *)files, (const E *)theta, (E *)V,
                                                                                 job_packs, model_packs, items);
    return launched();
}

}  // namespace

extern "C" int ccdc_map(const ccdc_plan_t *plan, const void *files, const void *theta, void *V, void *stream)
{
    int rc = ready(plan), vec = 1;
    if (rc != CCDC_OK) return rc;
    if ((rc = pick_vec(plan, &vec, files, theta, (const void *)V)) != CCDC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    CCDC_DISPATCH(plan, vec, (run_map<A, VEC>(plan, files, theta, V, st)));
}
