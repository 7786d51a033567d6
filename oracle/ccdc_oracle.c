/*
 * Oracle for the compressed CDC shuffle: placement, round schedule and byte
 * counts.  The stage arithmetic lives in ccdc_oracle_stages.inc.
 * Test infrastructure only (see ccdc_oracle.h): plain, single-threaded,
 * unoptimised on purpose, and independent of the GPU library.
 */
#include "ccdc_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

int64_t orc_binom(int n, int k)
{
    if (n < 0 || k < 0 || k > n) return -1;
    if (k > n - k) k = n - k;
    int64_t v = 1;
    for (int i = 1; i <= k; i++) {
        /* v = v * (n-k+i) / i stays integral at every step */
        const int64_t f = n - k + i;
        if (v > INT64_MAX / f) return -1;
        v = v * f / i;
    }
    return v;
}

/* Advance the ascending k-subset s of {0..n-1} to its lexicographic successor.
 * Returns 0 when s was the last one. */
static int next_subset(int *s, int k, int n)
{
    int i = k - 1;
    while (i >= 0 && s[i] == n - k + i) i--;
    if (i < 0) return 0;
    s[i]++;
    for (int j = i + 1; j < k; j++) s[j] = s[j - 1] + 1;
    return 1;
}

/* All k-subsets of {0..n-1}, ascending inside, lexicographic across: [count][k]. */
static int *all_subsets(int n, int k, int64_t count)
{
    int *out = (int *)malloc(sizeof(int) * (size_t)count * (size_t)k);
    int *s = (int *)malloc(sizeof(int) * (size_t)k);
    if (!out || !s) { free(out); free(s); return NULL; }
    for (int i = 0; i < k; i++) s[i] = i;
    int64_t idx = 0;
    do {
        memcpy(out + idx * k, s, sizeof(int) * (size_t)k);
        idx++;
    } while (next_subset(s, k, n));
    free(s);
    return (idx == count) ? out : (free(out), (int *)NULL);
}

static int cmp_width;   /* single-threaded program: comparator width for bsearch */
static int cmp_subset(const void *a, const void *b)
{
    const int *x = (const int *)a, *y = (const int *)b;
    for (int i = 0; i < cmp_width; i++)
        if (x[i] != y[i]) return x[i] < y[i] ? -1 : 1;
    return 0;
}

/* Position of subset s in the lexicographically sorted table. */
static int64_t find_subset(const int *table, int64_t count, int k, const int *s)
{
    cmp_width = k;
    const int *hit = (const int *)bsearch(s, table, (size_t)count, sizeof(int) * (size_t)k, cmp_subset);
    return hit ? (hit - table) / k : -1;
}

/* dst = src without its element at position skip. */
static void drop_member(const int *src, int len, int skip, int *dst)
{
    for (int i = 0, j = 0; i < len; i++)
        if (i != skip) dst[j++] = src[i];
}

static int is_permutation(const int *order, int64_t len)
{
    char *seen = (char *)calloc((size_t)len, 1);
    if (!seen) return 0;
    int ok = 1;
    for (int64_t i = 0; i < len && ok; i++) {
        if (order[i] < 0 || order[i] >= len || seen[order[i]]) ok = 0;
        else seen[order[i]] = 1;
    }
    free(seen);
    return ok;
}

void orc_plan_free(orc_plan *p)
{
    if (!p) return;
    free(p->batch_job); free(p->batch_file0); free(p->batch_label);
    free(p->round_member); free(p->round_batch);
    free(p);
}

orc_plan *orc_plan_build(int K, int r, int Q, int N, int schedule, const int *batch_order, int order_sets)
{
    /* Sec. III, network model: K | Q, K <= N; Theorem 1: mu*K in {1..K-1}. */
    if (K < 2 || r < 1 || r > K - 1 || Q < 1 || N < 1 || Q % K != 0 || K > N) return NULL;
    if (schedule != ORC_SINGLE_JOB && schedule != ORC_PAPER_JOBS) return NULL;
    const int r1 = r + 1;
    const int64_t n_lab = orc_binom(K, r);     /* r-subsets: batch labels */
    const int64_t G = orc_binom(K, r1);        /* (r+1)-subsets: shuffle subsets */
    if (n_lab < 0 || G < 0 || n_lab > INT32_MAX || G > INT32_MAX) return NULL;

    const int64_t per_job = (schedule == ORC_SINGLE_JOB) ? n_lab : r1;
    if (N % per_job != 0) return NULL;
    const int64_t n_jobs = (schedule == ORC_SINGLE_JOB) ? 1 : G;
    if (batch_order) {
        if (order_sets != 1 && order_sets != n_jobs) return NULL;
        for (int s = 0; s < order_sets; s++)
            if (!is_permutation(batch_order + s * per_job, per_job)) return NULL;
    }

    orc_plan *p = (orc_plan *)calloc(1, sizeof(orc_plan));
    int *labels = all_subsets(K, r, n_lab);
    int *groups = all_subsets(K, r1, G);
    int *tmp = (int *)malloc(sizeof(int) * (size_t)(r1 + 1));
    if (!p || !labels || !groups || !tmp) goto fail;

    p->K = K; p->r = r; p->Q = Q; p->N = N; p->c = Q / K;
    p->m = (int)(N / per_job);
    if (schedule == ORC_SINGLE_JOB) {
        p->J = 1; p->n_batch = n_lab; p->n_round = G;
    } else {
        if (G * (int64_t)(K - r) > INT32_MAX) goto fail;
        p->J = (int)G; p->n_batch = G * r1; p->n_round = G * (K - r);
    }
    p->batch_job = (int *)malloc(sizeof(int) * (size_t)p->n_batch);
    p->batch_file0 = (int *)malloc(sizeof(int) * (size_t)p->n_batch);
    p->batch_label = (int *)malloc(sizeof(int) * (size_t)p->n_batch * (size_t)r);
    p->round_member = (int *)malloc(sizeof(int) * (size_t)p->n_round * (size_t)r1);
    p->round_batch = (int *)malloc(sizeof(int) * (size_t)p->n_round * (size_t)r1);
    if (!p->batch_job || !p->batch_file0 || !p->batch_label || !p->round_member || !p->round_batch) goto fail;

    if (schedule == ORC_SINGLE_JOB) {
        /* Placement of Sec. IV-A with the whole cluster in the role of K_j: the
         * files are cut into one batch per r-subset P, batch P is stored on the
         * nodes of P. */
        for (int64_t pr = 0; pr < n_lab; pr++) {
            p->batch_job[pr] = 0;
            p->batch_file0[pr] = (batch_order ? batch_order[pr] : (int)pr) * p->m;
            memcpy(p->batch_label + pr * r, labels + pr * r, sizeof(int) * (size_t)r);
        }
        /* One stage-1 round (Sec. IV-B) in every (r+1)-subset S: member s_b is
         * served the batch labelled S minus s_b. */
        for (int64_t u = 0; u < G; u++) {
            const int *S = groups + u * r1;
            memcpy(p->round_member + u * r1, S, sizeof(int) * (size_t)r1);
            for (int b = 0; b < r1; b++) {
                drop_member(S, r1, b, tmp);
                const int64_t bt = find_subset(labels, n_lab, r, tmp);
                if (bt < 0) goto fail;
                p->round_batch[u * r1 + b] = (int)bt;
            }
        }
    } else {
        /* Sec. IV-A: job j is placed on the j-th (r+1)-subset K_j; its files are
         * cut into r+1 batches labelled by the r-subsets of K_j (taken here in
         * lexicographic order, i.e. dropping s_r first, s_0 last). */
        for (int64_t j = 0; j < G; j++) {
            const int *Kj = groups + j * r1;
            for (int pr = 0; pr < r1; pr++) {
                const int64_t bt = j * r1 + pr;
                p->batch_job[bt] = (int)j;
                const int *order = batch_order ? batch_order + (order_sets == 1 ? 0 : j * r1) : NULL;
                p->batch_file0[bt] = (order ? order[pr] : pr) * p->m;
                drop_member(Kj, r1, r - pr, p->batch_label + bt * r);
            }
        }
        int64_t u = 0;
        for (int64_t j = 0; j < G; j++) {
            const int *Kj = groups + j * r1;
            /* Stage 1 (Sec. IV-B): job j inside its own subset. */
            memcpy(p->round_member + u * r1, Kj, sizeof(int) * (size_t)r1);
            for (int b = 0; b < r1; b++)
                p->round_batch[u * r1 + b] = (int)(j * r1 + (r - b));   /* label K_j minus s_b */
            u++;
            /* Stage 2 (Sec. IV-B): for every node i outside K_j, member s_b is
             * served the batch labelled K_j minus s_b of the job that lives on
             * {i} union K_j minus s_b. */
            for (int i = 0; i < K; i++) {
                int inside = 0;
                for (int b = 0; b < r1; b++) inside |= (Kj[b] == i);
                if (inside) continue;
                memcpy(p->round_member + u * r1, Kj, sizeof(int) * (size_t)r1);
                for (int b = 0; b < r1; b++) {
                    /* tmp = sorted({i} union K_j minus s_b); pos = where i landed */
                    drop_member(Kj, r1, b, tmp);
                    int pos = r;
                    while (pos > 0 && tmp[pos - 1] > i) { tmp[pos] = tmp[pos - 1]; pos--; }
                    tmp[pos] = i;
                    const int64_t jb = find_subset(groups, G, r1, tmp);
                    if (jb < 0) goto fail;
                    /* in job jb the wanted label is its subset minus i, i.e. the
                     * batch that drops position pos */
                    p->round_batch[u * r1 + b] = (int)(jb * r1 + (r - pos));
                }
                u++;
            }
        }
        if (u != p->n_round) goto fail;
    }
    free(labels); free(groups); free(tmp);
    return p;
fail:
    free(labels); free(groups); free(tmp);
    orc_plan_free(p);
    return NULL;
}

/* Copy of a plan that keeps all batches but only the listed rounds (in the
 * given order); lets a test run the stages on a sample of a large schedule. */
orc_plan *orc_plan_select_rounds(const orc_plan *src, const int64_t *rounds, int64_t n)
{
    if (!src || n < 0 || (n > 0 && !rounds)) return NULL;
    const int r = src->r, r1 = src->r + 1;
    for (int64_t i = 0; i < n; i++)
        if (rounds[i] < 0 || rounds[i] >= src->n_round) return NULL;
    orc_plan *p = (orc_plan *)calloc(1, sizeof(orc_plan));
    if (!p) return NULL;
    *p = *src;
    p->n_round = n;
    const size_t nb = (size_t)src->n_batch, nr = (size_t)(n > 0 ? n : 1);
    p->batch_job = (int *)malloc(sizeof(int) * nb);
    p->batch_file0 = (int *)malloc(sizeof(int) * nb);
    p->batch_label = (int *)malloc(sizeof(int) * nb * (size_t)r);
    p->round_member = (int *)malloc(sizeof(int) * nr * (size_t)r1);
    p->round_batch = (int *)malloc(sizeof(int) * nr * (size_t)r1);
    if (!p->batch_job || !p->batch_file0 || !p->batch_label || !p->round_member || !p->round_batch) {
        orc_plan_free(p);
        return NULL;
    }
    memcpy(p->batch_job, src->batch_job, sizeof(int) * nb);
    memcpy(p->batch_file0, src->batch_file0, sizeof(int) * nb);
    memcpy(p->batch_label, src->batch_label, sizeof(int) * nb * (size_t)r);
    for (int64_t i = 0; i < n; i++) {
        memcpy(p->round_member + i * r1, src->round_member + rounds[i] * r1, sizeof(int) * (size_t)r1);
        memcpy(p->round_batch + i * r1, src->round_batch + rounds[i] * r1, sizeof(int) * (size_t)r1);
    }
    return p;
}

/* Sec. IV: with J = gamma * C(K, r+1) jobs the scheme works on C(K, r+1) jobs at
 * a time and repeats the same operations gamma times.  Repetition g takes jobs
 * g*J1 .. g*J1+J1-1 (J1 = jobs of the plan given) with the same placement and
 * the same rounds. */
orc_plan *orc_plan_repeat(const orc_plan *src, int gamma)
{
    if (!src || gamma < 1) return NULL;
    const int r = src->r, r1 = src->r + 1;
    if ((int64_t)src->J * gamma > INT32_MAX || src->n_batch * gamma > INT32_MAX || src->n_round * gamma > INT32_MAX)
        return NULL;
    orc_plan *p = (orc_plan *)calloc(1, sizeof(orc_plan));
    if (!p) return NULL;
    *p = *src;
    p->J = src->J * gamma;
    p->n_batch = src->n_batch * gamma;
    p->n_round = src->n_round * gamma;
    const size_t nb = (size_t)p->n_batch, nr = (size_t)p->n_round;
    p->batch_job = (int *)malloc(sizeof(int) * nb);
    p->batch_file0 = (int *)malloc(sizeof(int) * nb);
    p->batch_label = (int *)malloc(sizeof(int) * nb * (size_t)r);
    p->round_member = (int *)malloc(sizeof(int) * nr * (size_t)r1);
    p->round_batch = (int *)malloc(sizeof(int) * nr * (size_t)r1);
    if (!p->batch_job || !p->batch_file0 || !p->batch_label || !p->round_member || !p->round_batch) {
        orc_plan_free(p);
        return NULL;
    }
    for (int g = 0; g < gamma; g++) {
        for (int64_t b = 0; b < src->n_batch; b++) {
            const int64_t bt = g * src->n_batch + b;
            p->batch_job[bt] = g * src->J + src->batch_job[b];
            p->batch_file0[bt] = src->batch_file0[b];
            for (int s = 0; s < r; s++) p->batch_label[bt * r + s] = src->batch_label[b * r + s];
        }
        for (int64_t u = 0; u < src->n_round; u++)
            for (int b = 0; b < r1; b++) {
                const int64_t i = (g * src->n_round + u) * r1 + b;
                p->round_member[i] = src->round_member[u * r1 + b];
                p->round_batch[i] = (int)(g * src->n_batch + src->round_batch[u * r1 + b]);
            }
    }
    return p;
}

/* Sec. IV-B says the packet is split evenly into r segments and silently
 * assumes r | W.  Reading used here: if 4r | W the split is exact; otherwise
 * ell = ceil(W/r) rounded up to a multiple of 4 elements, segment rho covers
 * [rho*ell, min(W,(rho+1)*ell)) and the last segments may be short or empty. */
int64_t orc_segment_len(int64_t W, int r)
{
    const int64_t A = 4;
    if (W % (r * A) == 0) return W / r;
    const int64_t q = (W + r - 1) / r;
    return (q + A - 1) / A * A;
}

int64_t orc_segment_count(int64_t W, int r, int rho)
{
    const int64_t ell = orc_segment_len(W, r);
    const int64_t lo = rho * ell;
    if (lo >= W) return 0;
    const int64_t hi = (lo + ell < W) ? lo + ell : W;
    return hi - lo;
}

int orc_label_rank(int a, int b)
{
    return a > b ? a - 1 : a;
}

int64_t orc_packet_len(int64_t W, int r, int a)
{
    int64_t len = 0;
    for (int b = 0; b <= r; b++) {
        if (b == a) continue;
        const int64_t n = orc_segment_count(W, r, orc_label_rank(a, b));
        if (n > len) len = n;
    }
    return len;
}

int64_t orc_scheduled_elems(const orc_plan *p, int64_t T)
{
    const int64_t W = (int64_t)p->c * T;
    int64_t per_round = 0;
    for (int a = 0; a <= p->r; a++) per_round += orc_packet_len(W, p->r, a);
    return per_round * p->n_round;
}

#define CAT2(a, b) a##b
#define CAT(a, b) CAT2(a, b)

#define FN(name) CAT(name, _f64)
#define TIN float
#define TEL double
#define ZERO 0.0
#define ADD(a, b) ((a) + (b))
#define SUB(a, b) ((a) - (b))
#include "ccdc_oracle_stages.inc"
#undef FN
#undef TIN
#undef TEL
#undef ZERO
#undef ADD
#undef SUB

#define FN(name) CAT(name, _u32)
#define TIN uint32_t
#define TEL uint32_t
#define ZERO 0u
#define ADD(a, b) ((a) ^ (b))
#define SUB(a, b) ((a) ^ (b))
#include "ccdc_oracle_stages.inc"

/*
 * Third algebra, "h32": the scheme as Sec. II narrates it for real-valued data.
 * Pre-combining sums the intermediate values as numbers (fp32, files in
 * ascending order, one rounding per addition); coding and decoding take the
 * bit-wise XOR of the 32-bit patterns of the combined packets, so a receiver
 * gets back exactly the bits of the packet meant for it; the final reduction
 * adds numbers again (fp64 here).  Vbar and D hold fp32 values, X holds bit
 * patterns.  Written out on its own because the three artefacts differ in
 * type; the loops are those of ccdc_oracle_stages.inc.
 */
static uint32_t f32_bits(float v) { uint32_t b; memcpy(&b, &v, 4); return b; }
static float bits_f32(uint32_t b) { float v; memcpy(&v, &b, 4); return v; }

void orc_combine_h32(const orc_plan *p, int64_t T, const float *V, float *Vbar)
{
    const int r1 = p->r + 1;
    const int64_t W = (int64_t)p->c * T;
    for (int64_t u = 0; u < p->n_round; u++)
        for (int b = 0; b < r1; b++) {
            const int target = p->round_member[u * r1 + b];
            const int bt = p->round_batch[u * r1 + b];
            const int job = p->batch_job[bt], f0 = p->batch_file0[bt];
            for (int64_t e = 0; e < W; e++) {
                volatile float acc = 0.0f;              /* volatile: one fp32 rounding per step */
                for (int n = f0; n < f0 + p->m; n++) {
                    const int64_t file = (int64_t)job * p->N + n;
                    const float v = V[(file * p->Q + (int64_t)target * p->c) * T + e];
                    acc = (n == f0) ? v : acc + v;
                }
                Vbar[(u * r1 + b) * W + e] = acc;
            }
        }
}

void orc_encode_h32(const orc_plan *p, int64_t T, const float *Vbar, uint32_t *X)
{
    const int r = p->r, r1 = p->r + 1;
    const int64_t W = (int64_t)p->c * T;
    const int64_t ell = orc_segment_len(W, r);
    for (int64_t u = 0; u < p->n_round; u++)
        for (int a = 0; a < r1; a++)
            for (int64_t x = 0; x < ell; x++) {
                uint32_t acc = 0;
                for (int b = 0; b < r1; b++) {
                    if (b == a) continue;
                    const int rho = orc_label_rank(a, b);
                    if (x < orc_segment_count(W, r, rho)) acc ^= f32_bits(Vbar[(u * r1 + b) * W + rho * ell + x]);
                }
                X[(u * r1 + a) * ell + x] = acc;
            }
}

void orc_decode_h32(const orc_plan *p, int64_t T, const uint32_t *X, const float *Vbar, float *D)
{
    const int r = p->r, r1 = p->r + 1;
    const int64_t W = (int64_t)p->c * T;
    const int64_t ell = orc_segment_len(W, r);
    for (int64_t u = 0; u < p->n_round; u++)
        for (int b = 0; b < r1; b++)
            for (int a = 0; a < r1; a++) {
                if (a == b) continue;
                const int rho = orc_label_rank(a, b);
                const int64_t cnt = orc_segment_count(W, r, rho);
                for (int64_t x = 0; x < cnt; x++) {
                    uint32_t acc = X[(u * r1 + a) * ell + x];
                    for (int b2 = 0; b2 < r1; b2++) {
                        if (b2 == a || b2 == b) continue;
                        const int rho2 = orc_label_rank(a, b2);
                        if (x < orc_segment_count(W, r, rho2))
                            acc ^= f32_bits(Vbar[(u * r1 + b2) * W + rho2 * ell + x]);
                    }
                    D[(u * r1 + b) * W + rho * ell + x] = bits_f32(acc);
                }
            }
}

void orc_reduce_h32(const orc_plan *p, int64_t T, const float *V, const float *D, double *Phi)
{
    const int r = p->r, r1 = p->r + 1;
    const int64_t W = (int64_t)p->c * T;
    for (int64_t i = 0; i < (int64_t)p->J * p->Q * T; i++) Phi[i] = 0.0;
    for (int64_t bt = 0; bt < p->n_batch; bt++) {
        const int job = p->batch_job[bt];
        for (int s = 0; s < r; s++) {
            const int k = p->batch_label[bt * r + s];
            double *out = Phi + ((int64_t)job * p->Q + (int64_t)k * p->c) * T;
            for (int n = p->batch_file0[bt]; n < p->batch_file0[bt] + p->m; n++) {
                const int64_t file = (int64_t)job * p->N + n;
                const float *mine = V + (file * p->Q + (int64_t)k * p->c) * T;
                for (int64_t e = 0; e < W; e++) out[e] += (double)mine[e];
            }
        }
    }
    for (int64_t u = 0; u < p->n_round; u++)
        for (int b = 0; b < r1; b++) {
            const int k = p->round_member[u * r1 + b];
            const int job = p->batch_job[p->round_batch[u * r1 + b]];
            double *out = Phi + ((int64_t)job * p->Q + (int64_t)k * p->c) * T;
            const float *got = D + (u * r1 + b) * W;
            for (int64_t e = 0; e < W; e++) out[e] += (double)got[e];
        }
}

/* ------------------------------------------------------------------------
 * Compression-only comparison scheme (appendix of the paper).
 */
void orc_cplan_free(orc_cplan *p)
{
    if (!p) return;
    free(p->batch_first); free(p->node_batch); free(p->pkt_recv); free(p->pkt_batch); free(p->pkt_send);
    free(p);
}

orc_cplan *orc_cplan_build(int K, int r, int Q, int N)
{
    if (K < 2 || r < 1 || r > K - 1 || Q < 1 || N < 1 || Q % K != 0 || K > N) return NULL;
    /* mu = r/K; storage beyond one half of the files is not used by this scheme */
    int num = r, den = K;
    if (2 * r > K) { num = 1; den = 2; }
    if (((int64_t)N * num) % den != 0) return NULL;          /* mu*N files per batch */
    const int per = (int)((int64_t)N * num / den);
    const int nb = (den + num - 1) / num;                    /* ceil(1/mu) */
    orc_cplan *p = (orc_cplan *)calloc(1, sizeof(orc_cplan));
    if (!p) return NULL;
    p->K = K; p->r = r; p->Q = Q; p->N = N; p->c = Q / K; p->nb = nb;
    p->n_packet = (int64_t)K * (nb - 1);
    p->batch_first = (int *)malloc(sizeof(int) * (size_t)(nb + 1));
    p->node_batch = (int *)malloc(sizeof(int) * (size_t)K);
    p->pkt_recv = (int *)malloc(sizeof(int) * (size_t)(p->n_packet > 0 ? p->n_packet : 1));
    p->pkt_batch = (int *)malloc(sizeof(int) * (size_t)(p->n_packet > 0 ? p->n_packet : 1));
    p->pkt_send = (int *)malloc(sizeof(int) * (size_t)(p->n_packet > 0 ? p->n_packet : 1));
    if (!p->batch_first || !p->node_batch || !p->pkt_recv || !p->pkt_batch || !p->pkt_send) {
        orc_cplan_free(p);
        return NULL;
    }
    for (int t = 0; t < nb; t++) p->batch_first[t] = t * per;    /* the last batch takes the rest */
    p->batch_first[nb] = N;
    for (int k = 0; k < K; k++) p->node_batch[k] = k % nb;
    int64_t i = 0;
    for (int k = 0; k < K; k++)
        for (int t = 0; t < nb; t++) {
            if (t == p->node_batch[k]) continue;
            int sender = -1;                                     /* next node after k that stores B_t */
            for (int d = 1; d < K && sender < 0; d++)
                if (p->node_batch[(k + d) % K] == t) sender = (k + d) % K;
            if (sender < 0) { orc_cplan_free(p); return NULL; }
            p->pkt_recv[i] = k; p->pkt_batch[i] = t; p->pkt_send[i] = sender;
            i++;
        }
    return p;
}

int64_t orc_cplan_scheduled_elems(const orc_cplan *p, int64_t T)
{
    return p->n_packet * (int64_t)p->c * T;
}

#undef FN
#undef TIN
#undef TEL
#undef ZERO
#undef ADD
#undef SUB
#define FN(name) CAT(name, _f64)
#define TIN float
#define TEL double
#define ZERO 0.0
#define ADD(a, b) ((a) + (b))
#include "ccdc_oracle_compression.inc"
#undef FN
#undef TIN
#undef TEL
#undef ZERO
#undef ADD
#define FN(name) CAT(name, _u32)
#define TIN uint32_t
#define TEL uint32_t
#define ZERO 0u
#define ADD(a, b) ((a) ^ (b))
#include "ccdc_oracle_compression.inc"

/* ------------------------------------------------------------------------
 * Hybrid scheme for 16-bit floating-point payloads.
 */
#include "ccdc_oracle_h16.inc"

/* ---------------------------------------------------------------- Map stand-in
 * Sec. III, Map phase: v_{q,n} = g_q(w_n) for every file.  Here g is the gradient of
 * 1/2 |theta - w_n|^2, chunk q of it: theta_q - w_{n,q}. */
void orc_map_f32(int J, int N, int Q, int64_t T, const float *files, const float *theta, float *V)
{
    for (int j = 0; j < J; j++)
        for (int n = 0; n < N; n++)
            for (int q = 0; q < Q; q++)
                for (int64_t t = 0; t < T; t++) {
                    const int64_t at = (((int64_t)j * N + n) * Q + q) * T + t;
                    volatile float d = theta[((int64_t)j * Q + q) * T + t] - files[at];
                    V[at] = d;
                }
}

void orc_map_u32(int J, int N, int Q, int64_t T, const uint32_t *files, const uint32_t *theta, uint32_t *V)
{
    for (int j = 0; j < J; j++)
        for (int n = 0; n < N; n++)
            for (int q = 0; q < Q; q++)
                for (int64_t t = 0; t < T; t++) {
                    const int64_t at = (((int64_t)j * N + n) * Q + q) * T + t;
                    V[at] = theta[((int64_t)j * Q + q) * T + t] ^ files[at];
                }
}

void orc_map_h16(int J, int N, int Q, int64_t T, int fmt, const uint16_t *files, const uint16_t *theta, uint16_t *V)
{
    for (int j = 0; j < J; j++)
        for (int n = 0; n < N; n++)
            for (int q = 0; q < Q; q++)
                for (int64_t t = 0; t < T; t++) {
                    const int64_t at = (((int64_t)j * N + n) * Q + q) * T + t;
                    volatile float d = h16_widen(theta[((int64_t)j * Q + q) * T + t], fmt) - h16_widen(files[at], fmt);
                    V[at] = h16_narrow(d, fmt);
                }
}
