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

// A workgroup covers kBlock consecutive packs (a tile) of ONE file (row), so that the file
// and job indices are wave-uniform and no work item divides.  Workgroups are ordered
// (group of kMapGroup tiles, file, tile in the group): the piece of theta a group covers
// (1 MiB) is used by every file before the next piece is touched, so it is fetched from
// HBM once and re-read from cache, while every file is still read in runs of 1 MiB.
constexpr uint32_t kMapGroup = 256;
template <class A, int VEC>
__global__ __launch_bounds__(kBlock) void k_map(const typename A::elem *files,      // may be V itself
                                                const typename A::elem *__restrict__ theta,
                                                typename A::elem *V, uint32_t model_packs, uint32_t tiles,
                                                uint32_t rows, uint32_t files_per_job)
{
    using O = Ops<A, VEC>;
    using P = typename O::P;
    const uint32_t per_group = rows * kMapGroup;
    const uint32_t group = blockIdx.x / per_group, in_group = blockIdx.x - group * per_group;
    const uint32_t row = in_group / kMapGroup, tile = group * kMapGroup + (in_group - row * kMapGroup);
    if (tile >= tiles) return;                        // the last group may be short
    const uint32_t e = tile * kBlock + threadIdx.x;
    if (e >= model_packs) return;
    const uint32_t job = row / files_per_job;
    const size_t at = (size_t)row * model_packs + e;
    const P data = load_stream<P>(reinterpret_cast<const P *>(files) + at);
    const P model = reinterpret_cast<const P *>(theta)[(size_t)job * model_packs + e];
    store_stream(reinterpret_cast<P *>(V) + at, O::gradient(model, data));
}

template <class A, int VEC>
int run_map(const ccdc_plan_t *p, const void *files, const void *theta, void *V, hipStream_t st)
{
    using E = typename A::elem;
    const uint64_t model_packs = (uint64_t)p->Q * p->T / VEC, rows = (uint64_t)p->J * p->N;
    if (!fits_launch(model_packs)) return CCDC_ESIZE;
    const uint64_t tiles = (model_packs + kBlock - 1) / kBlock, groups = (tiles + kMapGroup - 1) / kMapGroup;
    if (!fits_launch(rows * groups * kMapGroup)) return CCDC_ESIZE;
    k_map<A, VEC><<<(uint32_t)(rows * groups * kMapGroup), kBlock, 0, st>>>(
        (const E *)files, (const E *)theta, (E *)V, (uint32_t)model_packs, (uint32_t)tiles, (uint32_t)rows, (uint32_t)p->N);
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
