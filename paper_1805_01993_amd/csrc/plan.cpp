// Host side of the plan: file placement (Sec. IV-A), round schedule (Sec. IV-B),
// segment split and the index tables the kernels consume.  Subsets are handled
// through their lexicographic rank (combinatorial number system), no subset
// table is ever materialised.
#include "plan.hpp"

#include <algorithm>
#include <limits>
#include <new>

namespace ccdc {
namespace {

constexpr int64_t kMaxTable = 2147483647LL;          // int32 indexable
constexpr int64_t kMaxElems = 1LL << 40;             // per buffer
constexpr int64_t kMaxItems = 2147483647LL;          // work items of one launch

// Pascal's triangle with saturation, C[n][k] for 0 <= k <= n <= nmax.
struct Binom {
    int nmax;
    std::vector<int64_t> tab;
    explicit Binom(int n) : nmax(n), tab((size_t)(n + 1) * (n + 1), 0) {
        const int64_t cap = std::numeric_limits<int64_t>::max() / 2;
        for (int i = 0; i <= n; i++) {
            at(i, 0) = 1;
            for (int k = 1; k <= i; k++) at(i, k) = std::min(cap, at(i - 1, k - 1) + (k <= i - 1 ? at(i - 1, k) : 0));
        }
    }
    int64_t &at(int n, int k) { return tab[(size_t)n * (nmax + 1) + k]; }
    int64_t operator()(int n, int k) const {
        if (n < 0 || k < 0 || k > n) return 0;
        return tab[(size_t)n * (nmax + 1) + k];
    }
};

// Number of k-subsets of {0..n-1} that precede the ascending subset s in
// lexicographic order.
int64_t lex_rank(const Binom &C, int n, int k, const int *s)
{
    int64_t rank = 0;
    int lo = 0;
    for (int i = 0; i < k; i++) {
        // subsets that agree on s[0..i-1] and have a smaller element at position i
        for (int v = lo; v < s[i]; v++) rank += C(n - 1 - v, k - 1 - i);
        lo = s[i] + 1;
    }
    return rank;
}

// Inverse of lex_rank.
void lex_unrank(const Binom &C, int n, int k, int64_t rank, int *s)
{
    int v = 0;
    for (int i = 0; i < k; i++) {
        while (C(n - 1 - v, k - 1 - i) <= rank) {
            rank -= C(n - 1 - v, k - 1 - i);
            v++;
        }
        s[i] = v++;
    }
}

}  // namespace

int build_plan(int K, int r, int Q, int N, bool paper_jobs, int gamma, ccdc_plan_t **out)
{
    if (!out) return CCDC_EINVAL;
    *out = nullptr;
    if (gamma < 1 || (gamma > 1 && !paper_jobs)) return CCDC_EINVAL;
    // Sec. III network model (K | Q, K <= N) and Theorem 1 (mu*K in 1..K-1)
    if (K < 2 || r < 1 || r > K - 1 || Q < 1 || N < 1 || Q % K != 0 || K > N) return CCDC_EINVAL;
    if (K > 4096) return CCDC_ESIZE;

    const Binom C(K);
    const int r1 = r + 1;
    const int64_t nlabel = C(K, r), G = C(K, r1);
    if (nlabel > kMaxTable || G > kMaxTable) return CCDC_ESIZE;
    const int64_t per_job = paper_jobs ? r1 : nlabel;
    if (N % per_job != 0) return CCDC_EINVAL;                 // Sec. IV-A: even batches
    const int64_t nround = paper_jobs ? G * (K - r) : G;
    const int64_t nbatch = paper_jobs ? G * r1 : nlabel;
    if (nround * r1 > kMaxTable / gamma || nbatch * r > kMaxTable / gamma || G > kMaxTable / gamma) return CCDC_ESIZE;

    ccdc_plan_t *p = new (std::nothrow) ccdc_plan_t;
    if (!p) return CCDC_ENOMEM;
    try {
        p->K = K; p->r = r; p->Q = Q; p->N = N;
        p->c = Q / K;
        p->m = (int)(N / per_job);
        p->paper_jobs = paper_jobs;
        p->J = paper_jobs ? (int)G : 1;
        p->nbatch = nbatch;
        p->nround = nround;
        p->nrows = nround * r1;
        p->batch_job.resize((size_t)nbatch);
        p->batch_file0.resize((size_t)nbatch);
        p->batch_label.resize((size_t)nbatch * r);
        p->round_member.resize((size_t)nround * r1);
        p->round_batch.resize((size_t)nround * r1);

        std::vector<int> S(r1 + 1), P(r1 + 1);
        if (!paper_jobs) {
            // One job over the whole cluster: batch p <-> p-th r-subset.
            for (int64_t b = 0; b < nbatch; b++) {
                lex_unrank(C, K, r, b, P.data());
                p->batch_job[b] = 0;
                p->batch_file0[b] = (int32_t)(b * p->m);
                std::copy(P.begin(), P.begin() + r, p->batch_label.begin() + b * r);
            }
            // Round u <-> u-th (r+1)-subset; member b is served the batch whose
            // label is the subset without s_b.
            for (int64_t u = 0; u < nround; u++) {
                lex_unrank(C, K, r1, u, S.data());
                for (int b = 0; b < r1; b++) {
                    p->round_member[u * r1 + b] = S[b];
                    int w = 0;
                    for (int i = 0; i < r1; i++)
                        if (i != b) P[w++] = S[i];
                    p->round_batch[u * r1 + b] = (int32_t)lex_rank(C, K, r, P.data());
                }
            }
        } else {
            // Job j lives on the j-th (r+1)-subset K_j.  Its r+1 batches are its
            // r-subsets in lexicographic order: local batch q drops position r-q.
            for (int64_t j = 0; j < G; j++) {
                lex_unrank(C, K, r1, j, S.data());
                for (int q = 0; q < r1; q++) {
                    const int64_t bt = j * r1 + q;
                    p->batch_job[bt] = (int32_t)j;
                    p->batch_file0[bt] = q * p->m;
                    int w = 0;
                    for (int i = 0; i < r1; i++)
                        if (i != r - q) p->batch_label[bt * r + w++] = S[i];
                }
            }
            int64_t u = 0;
            for (int64_t j = 0; j < G; j++) {
                lex_unrank(C, K, r1, j, S.data());
                // stage 1: job j inside K_j
                for (int b = 0; b < r1; b++) {
                    p->round_member[u * r1 + b] = S[b];
                    p->round_batch[u * r1 + b] = (int32_t)(j * r1 + (r - b));
                }
                u++;
                // stage 2: one round per outside node i.  Member s_b is served the
                // batch labelled K_j \ {s_b} of the job living on K_j \ {s_b} + {i}.
                int next_member = 0;
                for (int i = 0; i < K; i++) {
                    if (next_member < r1 && S[next_member] == i) { next_member++; continue; }
                    for (int b = 0; b < r1; b++) {
                        int w = 0, pos = -1;
                        for (int t = 0; t < r1; t++) {
                            if (t == b) continue;
                            if (pos < 0 && S[t] > i) { pos = w; P[w++] = i; }
                            P[w++] = S[t];
                        }
                        if (pos < 0) { pos = w; P[w++] = i; }
                        const int64_t jb = lex_rank(C, K, r1, P.data());
                        p->round_member[u * r1 + b] = S[b];
                        p->round_batch[u * r1 + b] = (int32_t)(jb * r1 + (r - pos));
                    }
                    u++;
                }
            }
        }
        // J = gamma * C(K, r+1) jobs (Sec. IV): the same placement and the same rounds
        // again for every further block of C(K, r+1) jobs
        if (gamma > 1) {
            const int64_t nb1 = p->nbatch, nr1 = p->nround;
            const int J1 = p->J;
            p->J = J1 * gamma;
            p->nbatch = nb1 * gamma;
            p->nround = nr1 * gamma;
            p->nrows = p->nround * r1;
            p->batch_job.resize((size_t)p->nbatch);
            p->batch_file0.resize((size_t)p->nbatch);
            p->batch_label.resize((size_t)p->nbatch * r);
            p->round_member.resize((size_t)p->nround * r1);
            p->round_batch.resize((size_t)p->nround * r1);
            for (int g = 1; g < gamma; g++) {
                for (int64_t b = 0; b < nb1; b++) {
                    p->batch_job[g * nb1 + b] = p->batch_job[b] + g * J1;
                    p->batch_file0[g * nb1 + b] = p->batch_file0[b];
                    for (int s = 0; s < r; s++) p->batch_label[(g * nb1 + b) * r + s] = p->batch_label[b * r + s];
                }
                for (int64_t i = 0; i < nr1 * r1; i++) {
                    p->round_member[g * nr1 * r1 + i] = p->round_member[i];
                    p->round_batch[g * nr1 * r1 + i] = p->round_batch[i] + (int32_t)(g * nb1);
                }
            }
        }
        // packets each node sends: by symmetry nrows / K of them (C(K-1,r) rounds, times K-r for the J-job schedule)
        p->rows_per_node = p->nrows / K;
        p->node_rows.assign((size_t)p->nrows, 0);
        std::vector<int64_t> fill((size_t)K, 0);
        for (int64_t i = 0; i < p->nrows; i++) {
            const int k = p->round_member[i];
            if (fill[k] < p->rows_per_node) p->node_rows[(size_t)k * p->rows_per_node + fill[k]] = (int32_t)i;
            fill[k]++;
        }
        for (int k = 0; k < K; k++)
            if (fill[k] != p->rows_per_node) {
                delete p;
                return CCDC_EINVAL;
            }
        // placement seen from the files and from the nodes (Sec. IV-A): file -> the label of its
        // batch; node -> every file of every batch whose label holds it
        const int64_t nfiles = (int64_t)p->J * N;
        if (nfiles * r > kMaxTable) {
            delete p;
            return CCDC_ESIZE;
        }
        p->file_nodes.assign((size_t)nfiles * r, -1);
        std::vector<std::vector<int32_t>> held((size_t)K);
        for (int64_t bt = 0; bt < p->nbatch; bt++)
            for (int f = 0; f < p->m; f++) {
                const int64_t file = (int64_t)p->batch_job[bt] * N + p->batch_file0[bt] + f;
                for (int s = 0; s < r; s++) {
                    p->file_nodes[(size_t)file * r + s] = p->batch_label[bt * r + s];
                    held[p->batch_label[bt * r + s]].push_back((int32_t)file);
                }
            }
        p->files_per_node = nfiles * r / K;
        p->node_files.clear();
        for (int k = 0; k < K; k++) {
            if ((int64_t)held[k].size() != p->files_per_node) {     // symmetric placement: |M_k| = mu*J*N
                delete p;
                return CCDC_EINVAL;
            }
            std::sort(held[k].begin(), held[k].end());
            p->node_files.insert(p->node_files.end(), held[k].begin(), held[k].end());
        }
    } catch (const std::bad_alloc &) {
        delete p;
        return CCDC_ENOMEM;
    }
    *out = p;
    return CCDC_OK;
}

// Compression-only comparison scheme (appendix of the paper): no coding.  With
// mu = r/K (taken as 1/2 when larger) the files are cut into nb = ceil(1/mu)
// consecutive batches of mu*N files (the last takes the rest), node k stores
// batch k mod nb, and for every node k and batch t it does not store, the next
// node after k (cyclically) that stores B_t pre-combines and sends one packet.
int build_compression_plan(int K, int r, int Q, int N, ccdc_plan_t **out)
{
    if (!out) return CCDC_EINVAL;
    *out = nullptr;
    if (K < 2 || r < 1 || r > K - 1 || Q < 1 || N < 1 || Q % K != 0 || K > N) return CCDC_EINVAL;
    if (K > 4096) return CCDC_ESIZE;
    int64_t num = r, den = K;
    if (2 * r > K) { num = 1; den = 2; }                   // more than half the files does not help here
    if (((int64_t)N * num) % den != 0) return CCDC_EINVAL;  // mu*N files per batch
    const int64_t per = (int64_t)N * num / den;
    const int nb = (int)((den + num - 1) / num);
    ccdc_plan_t *p = new (std::nothrow) ccdc_plan_t;
    if (!p) return CCDC_ENOMEM;
    try {
        p->K = K; p->r = r; p->Q = Q; p->N = N;
        p->c = Q / K;
        p->m = (int)per;
        p->compression = true;
        p->J = 1;
        p->nbatch = nb;
        p->nround = K;                                     // one group of packets per receiver
        p->nrows = (int64_t)K * (nb - 1);
        p->batch_first.resize((size_t)nb + 1);
        for (int t = 0; t < nb; t++) p->batch_first[t] = (int32_t)(t * per);
        p->batch_first[nb] = N;
        p->batch_job.assign((size_t)nb, 0);
        p->batch_file0.assign(p->batch_first.begin(), p->batch_first.end() - 1);
        p->node_batch.resize((size_t)K);
        for (int k = 0; k < K; k++) p->node_batch[k] = k % nb;
        for (int k = 0; k < K; k++)
            for (int t = 0; t < nb; t++) {
                if (t == p->node_batch[k]) continue;
                int sender = -1;
                for (int d = 1; d < K && sender < 0; d++)
                    if (p->node_batch[(k + d) % K] == t) sender = (k + d) % K;
                p->pkt_recv.push_back(k);
                p->pkt_batch.push_back(t);
                p->pkt_send.push_back(sender);
                p->row_files.push_back(p->batch_first[t + 1] - p->batch_first[t]);
            }
    } catch (const std::bad_alloc &) {
        delete p;
        return CCDC_ENOMEM;
    }
    *out = p;
    return CCDC_OK;
}

namespace {

// ccdc_plan_bind for the compression-only scheme: the packet is sent whole (no
// segments), so ell = W, and every packet is both what is transmitted and what
// the receiver adds.
int bind_compression(ccdc_plan_t *p, int64_t T, int mode)
{
    if (mode != CCDC_F32_SUM && mode != CCDC_U32_XOR) return CCDC_EINVAL;   // nothing is coded: no hybrid of it
    if (T > kMaxElems / p->c) return CCDC_ESIZE;
    const int64_t W = (int64_t)p->c * T;
    const int vec = (T % 4 == 0) ? 4 : 1;
    if ((double)p->N * p->Q * (double)T > (double)kMaxElems || (double)p->nrows * (double)W > (double)kMaxElems)
        return CCDC_ESIZE;
    if ((double)std::max<int64_t>(p->nrows, p->K) * (double)((W + vec - 1) / vec) > (double)kMaxItems) return CCDC_ESIZE;
    try {
        std::vector<int64_t> src((size_t)p->nrows);
        for (int64_t i = 0; i < p->nrows; i++)
            src[i] = ((int64_t)p->batch_first[p->pkt_batch[i]] * p->Q + (int64_t)p->pkt_recv[i] * p->c) * T;
        // reduce lists: own batch from V, then the received packets in order
        const int64_t nout = p->K;
        std::vector<int64_t> ptr((size_t)nout + 1, 0), rows, outs((size_t)nout);
        int64_t min_rows = std::numeric_limits<int64_t>::max();
        for (int k = 0; k < p->K; k++) {
            const int j = p->node_batch[k];
            for (int n = p->batch_first[j]; n < p->batch_first[j + 1]; n++)
                rows.push_back((((int64_t)n * p->Q + (int64_t)k * p->c) * T) << 1);
            for (int64_t i = 0; i < p->nrows; i++)
                if (p->pkt_recv[i] == k) rows.push_back(((i * W) << 1) | 1);
            ptr[k + 1] = (int64_t)rows.size();
            outs[k] = (int64_t)k * W;
            min_rows = std::min(min_rows, ptr[k + 1] - ptr[k]);
        }
        const int64_t items = nout * ((W + vec - 1) / vec);
        int64_t split = 1;
        if (items < (1 << 18)) split = std::min<int64_t>({(int64_t)256, std::max<int64_t>(1, min_rows), ((1 << 19) + items - 1) / items});
        p->T = T; p->W = W; p->ell = W; p->mode = mode;
        p->packet_len.assign(1, W);
        p->scheduled = p->nrows * W;
        p->src_off.swap(src);
        p->red_ptr.swap(ptr);
        p->red_row.swap(rows);
        p->red_out.swap(outs);
        p->nout = nout;
        p->red_split = (int)split;
        p->workspace_bytes = split > 1 ? (size_t)split * (size_t)p->Q * (size_t)T * 4 : 0;
        p->pipe_ok = false;
        p->loc_row.clear();
        p->bound = true;
    } catch (const std::bad_alloc &) {
        return CCDC_ENOMEM;
    }
    return CCDC_OK;
}

}  // namespace

int bind_plan(ccdc_plan_t *p, int64_t T, int mode)
{
    if (!p || T < 1 || mode < CCDC_F32_SUM || mode > CCDC_F16_SUM_XOR) return CCDC_EINVAL;
    if (p->compression) return bind_compression(p, T, mode);
    const int r = p->r, r1 = r + 1;
    if (T > kMaxElems / p->c) return CCDC_ESIZE;
    const int64_t W = (int64_t)p->c * T;

    // Split of a packet into r segments (Sec. IV-B): exact when 4r | W, else
    // ceil(W/r) rounded up to a multiple of 4 elements with a short/empty tail.
    int64_t ell;
    if (W % (4 * (int64_t)r) == 0) {
        ell = W / r;
    } else {
        ell = (W + r - 1) / r;
        ell = (ell + 3) / 4 * 4;
    }

    // size limits of buffers and of one launch
    const double v_elems = (double)p->J * p->N * p->Q * (double)T;
    const double rows = (double)p->nround * r1;
    if (v_elems > (double)kMaxElems || rows * (double)W > (double)kMaxElems) return CCDC_ESIZE;
    const int vec = (T % 4 == 0) ? 4 : 1;
    if (rows * (double)((W + vec - 1) / vec) > (double)kMaxItems) return CCDC_ESIZE;

    try {
        // true length of what sender a transmits: the longest segment it carries
        std::vector<int64_t> plen(r1, 0);
        int64_t per_round = 0;
        for (int a = 0; a < r1; a++) {
            for (int b = 0; b < r1; b++) {
                if (b == a) continue;
                const int64_t lo = label_rank(a, b) * ell;
                const int64_t cnt = lo >= W ? 0 : std::min(ell, W - lo);
                plen[a] = std::max(plen[a], cnt);
            }
            per_round += plen[a];
        }

        // where each round's r+1 packets are combined from
        std::vector<int64_t> src((size_t)p->nround * r1);
        for (int64_t i = 0; i < p->nround * r1; i++) {
            const int32_t bt = p->round_batch[i];
            const int64_t file = (int64_t)p->batch_job[bt] * p->N + p->batch_file0[bt];
            src[i] = (file * p->Q + (int64_t)p->round_member[i] * p->c) * T;
        }

        // Row lists of the final reduction: for output block (job, node) first the
        // files the node stores itself (batch order), then what it decoded (round order).
        const int64_t nout = (int64_t)p->J * p->K;
        std::vector<int64_t> cnt((size_t)nout + 1, 0);
        for (int64_t bt = 0; bt < p->nbatch; bt++)
            for (int s = 0; s < r; s++)
                cnt[(int64_t)p->batch_job[bt] * p->K + p->batch_label[bt * r + s] + 1] += p->m;
        for (int64_t i = 0; i < p->nround * r1; i++)
            cnt[(int64_t)p->batch_job[p->round_batch[i]] * p->K + p->round_member[i] + 1] += 1;
        for (int64_t o = 0; o < nout; o++) cnt[o + 1] += cnt[o];
        std::vector<int64_t> rows_tab((size_t)cnt[nout]);
        std::vector<int64_t> fill(cnt.begin(), cnt.end() - 1);
        for (int64_t bt = 0; bt < p->nbatch; bt++)
            for (int s = 0; s < r; s++) {
                const int k = p->batch_label[bt * r + s];
                const int64_t o = (int64_t)p->batch_job[bt] * p->K + k;
                for (int f = 0; f < p->m; f++) {
                    const int64_t file = (int64_t)p->batch_job[bt] * p->N + p->batch_file0[bt] + f;
                    rows_tab[fill[o]++] = ((file * p->Q + (int64_t)k * p->c) * T) << 1;
                }
            }
        for (int64_t i = 0; i < p->nround * r1; i++) {
            const int64_t o = (int64_t)p->batch_job[p->round_batch[i]] * p->K + p->round_member[i];
            rows_tab[fill[o]++] = ((i * W) << 1) | 1;
        }
        std::vector<int64_t> outs((size_t)nout);
        int64_t min_rows = std::numeric_limits<int64_t>::max();
        for (int64_t o = 0; o < nout; o++) {
            outs[o] = ((o / p->K) * p->Q + (o % p->K) * (int64_t)p->c) * T;
            min_rows = std::min(min_rows, cnt[o + 1] - cnt[o]);
        }

        // Few, long outputs (small T, many rounds) would leave the chip idle: cut
        // each row list into red_split chunks summed by different workgroups and
        // added up, in chunk order, by a second pass.
        const int64_t items = nout * ((W + vec - 1) / vec);
        int64_t split = 1;
        if (items < (1 << 18)) split = std::min<int64_t>({(int64_t)256, std::max<int64_t>(1, min_rows), ((1 << 19) + items - 1) / items});
        if (items * split > kMaxItems) return CCDC_ESIZE;

        // One-pass pipeline: single job, unrolled r, accumulators of K nodes x r
        // segments per lane must fit in LDS.  The widest pack that still leaves
        // several wavefronts per compute unit is preferred.
        bool pipe_ok = !p->paper_jobs && r1 <= kPipeMaxR1 && W < (1LL << 29) &&   // 32-bit byte offsets in a packet
                       (int64_t)p->K * r * 4 * kPipeLanes <= kPipeMaxLds;
        int pipe_vec = 1;
        int64_t pipe_cap = 1, local_rows = 0;
        std::vector<int64_t> loc;
        if (pipe_ok) {
            // Small inputs are bound by how many wavefronts share the rounds: four-element
            // packs only while six of them fit on a compute unit.  Large inputs are bound
            // by the memory system, which is served better by wide accesses from three
            // wavefronts than by narrow ones from six (both measured).
            const bool large = v_elems * 4.0 >= (double)kPipeLargeInput;
            const int64_t lds4 = large ? kPipeGoodLdsHalf : kPipeGoodLds;
            if (T % 4 == 0 && (int64_t)p->K * r * 16 * kPipeLanes <= lds4) pipe_vec = 4;
            else if (T % 2 == 0 && (int64_t)p->K * r * 8 * kPipeLanes <= kPipeGoodLdsHalf) pipe_vec = 2;
            // chunk partials are written and read once more: keep them under ~1/4 of |V|
            const double v = (double)p->N * p->Q * (double)T, kw = (double)p->K * (double)W;
            pipe_cap = std::max<int64_t>(1, std::min<int64_t>({(int64_t)1024, p->nround, (int64_t)(0.125 * v / kw)}));
            // rows of V each node adds from its own files: the V entries of its
            // reduce list (the same count for every node of a single job)
            for (int64_t i = cnt[0]; i < cnt[1]; i++) local_rows += !(rows_tab[i] & 1);
            loc.resize((size_t)p->K * local_rows);
            for (int k = 0; k < p->K; k++) {
                int64_t w = 0;
                for (int64_t i = cnt[k]; i < cnt[k + 1]; i++)
                    if (!(rows_tab[i] & 1)) {
                        // entry = (element offset << 12) | node; K <= 4096, offsets < 2^40
                        if (w < local_rows) loc[(size_t)k * local_rows + w] = ((rows_tab[i] >> 1) << 12) | k;
                        w++;
                    }
                if (w != local_rows) pipe_ok = false;
            }
        }

        p->T = T; p->W = W; p->ell = ell; p->mode = mode;
        p->pipe_ok = pipe_ok;
        p->pipe_vec = pipe_vec;
        p->pipe_max_chunks = (int)pipe_cap;
        p->pipe_local_rows = pipe_ok ? local_rows : 0;
        p->loc_row.swap(loc);
        p->packet_len.swap(plen);
        p->scheduled = per_round * p->nround;
        p->src_off.swap(src);
        p->red_ptr.swap(cnt);
        p->red_row.swap(rows_tab);
        p->red_out.swap(outs);
        p->nout = nout;
        p->red_split = (int)split;
        p->workspace_bytes = split > 1 ? (size_t)split * (size_t)p->J * p->Q * (size_t)T * 4 : 0;
        if (pipe_ok && pipe_cap > 1)
            p->workspace_bytes = std::max(p->workspace_bytes, (size_t)pipe_cap * (size_t)p->K * (size_t)W * 4);
        p->bound = true;
    } catch (const std::bad_alloc &) {
        return CCDC_ENOMEM;
    }
    return CCDC_OK;
}

}  // namespace ccdc
