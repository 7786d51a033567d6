/*
 * Reference ("oracle") implementation of the compressed coded distributed
 * computing shuffle: pre-combine, split + encode, decode, final reduction.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, single-threaded, deliberately
 * slow CPU program whose only job is to be checkable against the paper by
 * eye.  It shares no code with the GPU library, and the GPU library must
 * never call it.  Only tests, the smoke check and the CPU-baseline leg of
 * the benchmark may use it.
 *
 * Notation (paper, Sec. III and Sec. IV):
 *   K nodes, r = mu*K (replication), Q functions per job, c = Q/K functions
 *   reduced per node, N files per job, J jobs, T elements per intermediate
 *   value, W = c*T elements in one concatenated pre-combined packet.
 *   Node ids, file ids, function ids and job ids are 0-based here.
 *
 * Memory layout (all row-major, all owned by the caller):
 *   V   [J][N][Q][T]      intermediate values v_{q,n} of every job, file-major:
 *                         the Q values mapped from one file are contiguous, so
 *                         the c values meant for one node are one run of W.
 *   Vbar[R][r+1][W]       pre-combined packet of round u for member b.
 *   X   [R][r+1][ell]     coded packet of round u sent by member a (stride
 *                         ell = segment length; unused tail holds the zero).
 *   D   [R][r+1][W]       what member b decodes in round u.
 *   Phi [J][Q][T]         the reduced outputs.
 *
 * Two algebras: "f64" = real numbers (inputs are fp32, every artefact and all
 * arithmetic is fp64, + to code and - to decode); "u32" = the paper's own
 * field F_{2^T} seen as T-bit strings in 32-bit words (+ and - are both XOR).
 *
 * A "round" is one run of the five shuffle steps of Sec. IV-B inside one
 * subset of r+1 nodes: r+1 packets are pre-combined (one per member, from
 * the batch stored on the other r members), every member sends one coded
 * packet, every member decodes one packet.
 */
#ifndef CCDC_ORACLE_H
#define CCDC_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct orc_plan {
    int K, r, Q, N;      /* per job */
    int J;               /* number of jobs */
    int c;               /* Q / K */
    int m;               /* files per batch */
    int64_t n_batch;     /* batches over all jobs */
    int64_t n_round;     /* rounds (R) */
    int *batch_job;      /* [n_batch]     job the batch belongs to */
    int *batch_file0;    /* [n_batch]     first file of the batch (index inside its job) */
    int *batch_label;    /* [n_batch][r]  the r nodes that store the batch, ascending */
    int *round_member;   /* [n_round][r+1] the nodes s_0 < ... < s_r of the round */
    int *round_batch;    /* [n_round][r+1] batch combined for member b: its label is
                            {s_0..s_r} minus s_b */
} orc_plan;

enum { ORC_SINGLE_JOB = 0, ORC_PAPER_JOBS = 1 };

/* Binomial coefficient; -1 on overflow of int64 or bad arguments. */
int64_t orc_binom(int n, int k);

/*
 * Build placement and round schedule.
 *   ORC_SINGLE_JOB: one job whose N files are spread one batch per r-subset
 *     of all K nodes; one round per (r+1)-subset (stage 1 of Sec. IV-B applied
 *     to every subset).  Needs C(K,r) | N.
 *   ORC_PAPER_JOBS: the scheme exactly as in Sec. IV: J = C(K,r+1) jobs, job j
 *     lives on the j-th (r+1)-subset, r+1 batches per job, and every subset
 *     runs stage 1 plus one stage-2 round per outside node.  Needs (r+1) | N.
 * batch_order (may be NULL = identity): permutation of the batch ranks that
 *   says which block of m consecutive files the p-th subset label gets; the
 *   paper leaves this labelling free and its examples use a non-identity one.
 *   One permutation has length C(K,r) for ORC_SINGLE_JOB, r+1 for
 *   ORC_PAPER_JOBS.  order_sets says how many permutations follow each other
 *   in batch_order: 1 (shared by all jobs) or J (one per job).
 * Returns NULL on invalid parameters (K<2, r<1, r>K-1, K does not divide Q,
 * K>N, batch count does not divide N, overflow).
 */
orc_plan *orc_plan_build(int K, int r, int Q, int N, int schedule, const int *batch_order, int order_sets);
void orc_plan_free(orc_plan *p);
/* Same batches, only the listed rounds (for sampling a large schedule); NULL on bad index. */
orc_plan *orc_plan_select_rounds(const orc_plan *src, const int64_t *rounds, int64_t n);
/* J = gamma * (jobs of src): the same placement and rounds repeated gamma times on
 * consecutive blocks of jobs (Sec. IV: with gamma times as many jobs the scheme is run gamma times over). */
orc_plan *orc_plan_repeat(const orc_plan *src, int gamma);

/* Segment length ell for a packet of W elements cut into r segments. */
int64_t orc_segment_len(int64_t W, int r);
/* Number of elements in segment rho (0 if it starts past the end). */
int64_t orc_segment_count(int64_t W, int r, int rho);
/* Index, inside S minus s_b, of member a (a != b): the segment of packet b
 * that carries sender a's label. */
int orc_label_rank(int a, int b);
/* Elements put on the wire by the whole schedule for value length T. */
int64_t orc_scheduled_elems(const orc_plan *p, int64_t T);
/* Elements actually sent by member a in one round. */
int64_t orc_packet_len(int64_t W, int r, int a);

/* The four stages, real-number algebra (fp32 in, fp64 everywhere else). */
void orc_combine_f64(const orc_plan *p, int64_t T, const float *V, double *Vbar);
void orc_encode_f64 (const orc_plan *p, int64_t T, const double *Vbar, double *X);
void orc_decode_f64 (const orc_plan *p, int64_t T, const double *X, const double *Vbar, double *D);
void orc_reduce_f64 (const orc_plan *p, int64_t T, const float *V, const double *D, double *Phi);
void orc_direct_f64 (const orc_plan *p, int64_t T, const float *V, double *Phi);   /* eq. (1) */

/* The four stages, XOR algebra on 32-bit words. */
void orc_combine_u32(const orc_plan *p, int64_t T, const uint32_t *V, uint32_t *Vbar);
void orc_encode_u32 (const orc_plan *p, int64_t T, const uint32_t *Vbar, uint32_t *X);
void orc_decode_u32 (const orc_plan *p, int64_t T, const uint32_t *X, const uint32_t *Vbar, uint32_t *D);
void orc_reduce_u32 (const orc_plan *p, int64_t T, const uint32_t *V, const uint32_t *D, uint32_t *Phi);
void orc_direct_u32 (const orc_plan *p, int64_t T, const uint32_t *V, uint32_t *Phi);  /* eq. (1) */

/* The four stages, "h32" algebra: numbers are summed (fp32 when pre-combining,
 * files ascending, one rounding per addition; fp64 in the final reduction) and
 * packets are coded by XOR of their 32-bit patterns, as Sec. II narrates it.
 * Vbar and D are fp32 values, X are bit patterns; D equals Vbar bit for bit. */
void orc_combine_h32(const orc_plan *p, int64_t T, const float *V, float *Vbar);
void orc_encode_h32 (const orc_plan *p, int64_t T, const float *Vbar, uint32_t *X);
void orc_decode_h32 (const orc_plan *p, int64_t T, const uint32_t *X, const float *Vbar, float *D);
void orc_reduce_h32 (const orc_plan *p, int64_t T, const float *V, const float *D, double *Phi);

/*
 * Comparison scheme "compression only" (appendix of the paper): one job, no
 * coding.  With mu = r/K (taken as 1/2 when larger: more storage does not help
 * this scheme) the files are cut into nb = ceil(1/mu) consecutive batches, the
 * first nb-1 of mu*N files, the last of the rest; node k stores batch k mod nb.
 * For every node k and every batch t it does not store, one node that stores
 * B_t (the next one after k, cyclically) pre-combines the c values k reduces
 * and sends that packet to k.  P[n_packet][W] holds the packets, receiver-major,
 * batches ascending; Phi[Q][T].
 */
typedef struct orc_cplan {
    int K, r, Q, N, c;
    int nb;              /* batches */
    int *batch_first;    /* [nb+1] file ranges */
    int *node_batch;     /* [K] batch stored by node k */
    int64_t n_packet;    /* K * (nb-1) */
    int *pkt_recv;       /* [n_packet] receiving node */
    int *pkt_batch;      /* [n_packet] batch the packet pre-combines */
    int *pkt_send;       /* [n_packet] node that sends it (stores pkt_batch) */
} orc_cplan;

/* NULL on invalid parameters (as orc_plan_build, and mu*N must be whole). */
orc_cplan *orc_cplan_build(int K, int r, int Q, int N);
void orc_cplan_free(orc_cplan *p);
int64_t orc_cplan_scheduled_elems(const orc_cplan *p, int64_t T);
void orc_ccombine_f64(const orc_cplan *p, int64_t T, const float *V, double *P);
void orc_creduce_f64 (const orc_cplan *p, int64_t T, const float *V, const double *P, double *Phi);
void orc_ccombine_u32(const orc_cplan *p, int64_t T, const uint32_t *V, uint32_t *P);
void orc_creduce_u32 (const orc_cplan *p, int64_t T, const uint32_t *V, const uint32_t *P, uint32_t *Phi);

/* The four stages, "h16" algebra: the hybrid scheme for 16-bit floating-point
 * payloads (fmt 0 = bfloat16, 1 = IEEE binary16), every artefact a 16-bit
 * pattern.  Pre-combining adds in fp32 (files ascending) and rounds the sum
 * once to the format, to nearest even; packets are coded by XOR of their
 * patterns; the final reduction is exact fp64 arithmetic on the 16-bit values
 * and is not rounded.  D equals Vbar bit for bit. */
void orc_h16_widen (const uint16_t *in, float *out, int64_t n, int fmt);      /* exact */
void orc_h16_narrow(const float *in, uint16_t *out, int64_t n, int fmt);      /* nearest, ties to even */
void orc_combine_h16(const orc_plan *p, int64_t T, int fmt, const uint16_t *V, uint16_t *Vbar);
void orc_encode_h16 (const orc_plan *p, int64_t T, const uint16_t *Vbar, uint16_t *X);
void orc_decode_h16 (const orc_plan *p, int64_t T, const uint16_t *X, const uint16_t *Vbar, uint16_t *D);
void orc_reduce_h16 (const orc_plan *p, int64_t T, int fmt, const uint16_t *V, const uint16_t *D, double *Phi);
void orc_direct_h16 (const orc_plan *p, int64_t T, int fmt, const uint16_t *V, double *Phi);   /* eq. (1) */

/*
 * Stand-in for the Map phase (Sec. III): a file is a data vector of Q*T elements, a job has
 * a model theta of Q*T elements, and the intermediate values are the chunks of the gradient
 * of 1/2 |theta - w_n|^2:  V[j][n][q][t] = theta[j][q][t] - files[j][n][q][t].
 * f32: one fp32 subtraction (the values ARE fp32: they are the inputs of the stages);
 * u32: XOR; h16: the fp32 difference of the two exact values, rounded once to the format.
 */
void orc_map_f32(int J, int N, int Q, int64_t T, const float *files, const float *theta, float *V);
void orc_map_u32(int J, int N, int Q, int64_t T, const uint32_t *files, const uint32_t *theta, uint32_t *V);
void orc_map_h16(int J, int N, int Q, int64_t T, int fmt, const uint16_t *files, const uint16_t *theta, uint16_t *V);

#ifdef __cplusplus
}
#endif
#endif
