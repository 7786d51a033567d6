/*
 * libccdc: the shuffle-stage packet pipeline of compressed coded distributed
 * computing (pre-combine -> split + encode -> decode -> final reduction) for
 * AMD CDNA4 (gfx950), with all K nodes of the cluster emulated on one GPU.
 *
 * Model and notation (paper, Sec. III and Sec. IV): K nodes, each file stored
 * on r = mu*K nodes, Q output functions per job (K | Q, node k reduces the
 * c = Q/K functions k*c .. k*c+c-1), N files per job, J jobs, intermediate
 * values v_{q,n} of T elements.  W = c*T is the length of one concatenated
 * pre-combined packet.  A "round" is one run of the shuffle steps of Sec. IV-B
 * inside one subset S = {s_0 < ... < s_r} of r+1 nodes: member b is served the
 * batch stored on the other r members.  All ids are 0-based.
 *
 * Buffers (row-major, 4-byte elements, DEVICE memory owned by the caller,
 * 16-byte aligned for the vector path; sizes come from ccdc_plan_query):
 *   V    [J][N][Q][T]     intermediate values, file-major
 *   Vbar [R][r+1][W]      pre-combined packet of round u for member b
 *   X    [R][r+1][ell]    coded packet of round u sent by member a; ell is
 *                         the segment length, words past a sender's true
 *                         packet length hold the zero of the algebra
 *   D    [R][r+1][W]      packet decoded by member b in round u
 *   Phi  [J][Q][T]        reduced outputs
 * Subsets (batch labels and rounds) are numbered in lexicographic order.
 * Sec. IV-B cuts a packet into r segments of equal length; when r does not
 * divide W that is read as: ell = W/r if 4r | W, else ceil(W/r) rounded up to a multiple of
 * 4; segment rho = [rho*ell, min(W,(rho+1)*ell)), the tail may be short/empty.
 *
 * Payload modes: CCDC_F32_SUM (fp32, real + to combine/encode/reduce, real -
 * to decode), CCDC_U32_XOR (uint32 words of the paper's field F_{2^T},
 * + and - are both XOR; bit-exact), CCDC_F32_SUM_XOR (fp32 values summed,
 * packets XOR-coded as bit patterns; decoding is bit-exact) and the same hybrid
 * for 2-byte elements, CCDC_BF16_SUM_XOR / CCDC_F16_SUM_XOR.  Every buffer of a
 * call holds elements of the bound mode's size (4 or 2 bytes) and must be
 * aligned to it; wider alignment (16 bytes) selects the wide kernels.
 *
 * Every function returns CCDC_OK (0) or a negative ccdc_status; nothing is
 * written to an output on error and the library never aborts or throws.
 * Stage calls only enqueue kernels on `stream` (a hipStream_t passed as
 * void*, NULL = the default stream) and allocate nothing; execution errors
 * surface at the caller's next synchronisation.  The calls that keep partial
 * sums in the plan's workspace (ccdc_reduce, ccdc_pipeline_fused,
 * ccdc_node_decode_reduce) are put in order by the library when they come on
 * different streams or host threads: the later call's stream waits for what the
 * earlier call's stream had been given (keep that stream alive until then).  A
 * stream under graph capture is not ordered this way; replay such a graph apart
 * from other work on the same plan.
 */
#ifndef CCDC_H
#define CCDC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ccdc_plan_s ccdc_plan_t;   /* opaque, owned by the library */

enum ccdc_status {
    CCDC_OK = 0,
    CCDC_EINVAL = -1,    /* bad parameter, null pointer, misaligned or unknown enum */
    CCDC_ENOMEM = -2,    /* host or device allocation failed */
    CCDC_EHIP = -3,      /* a HIP runtime call failed (no device, bad launch) */
    CCDC_ESIZE = -4,     /* a count exceeds what tables/kernels index (see ccdc_plan_bind) */
    CCDC_ESTATE = -5     /* plan not bound / not uploaded / wrong device for this call */
};

enum ccdc_mode {
    CCDC_F32_SUM = 0,       /* fp32: + to combine, encode, reduce; - to decode */
    CCDC_U32_XOR = 1,       /* uint32 words of F_{2^T}: XOR everywhere, bit-exact */
    CCDC_F32_SUM_XOR = 2,   /* fp32 values summed when pre-combining (files ascending) and in the
                               final reduction, packets coded and decoded by XOR of their 32-bit
                               patterns, as Sec. II narrates the scheme: X holds bit patterns and
                               D equals Vbar bit for bit */
    CCDC_BF16_SUM_XOR = 3,  /* the same hybrid on bfloat16 bit patterns (2-byte elements): sums are
                               carried in fp32 and rounded once, to nearest even, when a packet or an
                               output is stored; X holds XORs of 16-bit patterns */
    CCDC_F16_SUM_XOR = 4    /* the same on IEEE binary16 bit patterns */
};

/* Items for ccdc_plan_query.  Scalars are written as one int64_t; tables as
 * arrays of the stated type and shape. */
enum ccdc_query {
    CCDC_Q_K = 0, CCDC_Q_R, CCDC_Q_Q, CCDC_Q_N, CCDC_Q_J, CCDC_Q_C, CCDC_Q_M,
    CCDC_Q_NBATCH,           /* batches over all jobs */
    CCDC_Q_NROUND,           /* rounds R (K for ccdc_plan_compression) */
    CCDC_Q_T, CCDC_Q_MODE, CCDC_Q_W,                 /* need a bound plan from here on */
    CCDC_Q_SEG_LEN,          /* ell */
    CCDC_Q_SCHEDULED_ELEMS,  /* elements all coded packets really carry */
    CCDC_Q_CLOSED_FORM_NUM,  /* R*(r+1)*c*T  (Sec. IV-B: r+1 packets of c*T/r per round) */
    CCDC_Q_CLOSED_FORM_DEN,  /* r */
    CCDC_Q_V_ELEMS, CCDC_Q_VBAR_ELEMS, CCDC_Q_X_ELEMS, CCDC_Q_D_ELEMS, CCDC_Q_PHI_ELEMS,
    CCDC_Q_WORKSPACE_BYTES,  /* device bytes ccdc_plan_upload allocates besides tables */
    CCDC_Q_PACKET_LEN = 64,  /* int64_t[r+1]      true packet length of sender a        */
    CCDC_Q_BATCH_JOB,        /* int32_t[NBATCH]    job of the batch                     */
    CCDC_Q_BATCH_FILE0,      /* int32_t[NBATCH]    first file (index inside its job)    */
    CCDC_Q_BATCH_LABEL,      /* int32_t[NBATCH][r] nodes storing the batch, ascending   */
    CCDC_Q_ROUND_MEMBER,     /* int32_t[R][r+1]    nodes of the round, ascending        */
    CCDC_Q_ROUND_BATCH,      /* int32_t[R][r+1]    batch served to member b             */
    CCDC_Q_NROWS = 128,      /* packets = rows of Vbar and D: R*(r+1), or K*(nb-1) uncoded      */
    CCDC_Q_SCHEME,           /* 0 ccdc_plan, 1 ccdc_plan_jobs, 2 ccdc_plan_compression          */
    CCDC_Q_BATCH_FIRST,      /* int32_t[NBATCH+1]  file ranges of the batches   (compression)   */
    CCDC_Q_NODE_BATCH,       /* int32_t[K]         batch stored by node k       (compression)   */
    CCDC_Q_PACKET_RECV,      /* int32_t[NROWS]     receiver of packet i         (compression)   */
    CCDC_Q_PACKET_BATCH,     /* int32_t[NROWS]     batch packet i pre-combines  (compression)   */
    CCDC_Q_PACKET_SEND,      /* int32_t[NROWS]     node that sends packet i     (compression)   */
    CCDC_Q_ROWS_PER_NODE,    /* packets every node sends: NROWS / K                   (coded plans)   */
    CCDC_Q_NODE_ROWS,        /* int32_t[K][ROWS_PER_NODE] packets u*(r+1)+a node k sends, ascending   */
    /* File placement of Sec. IV-A (coded plans; CCDC_ESTATE for ccdc_plan_compression, whose
     * placement is BATCH_FIRST + NODE_BATCH).  A file is numbered job*N + n. */
    CCDC_Q_FILE_NODES,       /* int32_t[J*N][r]    the r nodes that store the file, ascending         */
    CCDC_Q_FILES_PER_NODE,   /* |M_k|: files every node stores, r*J*N/K (= mu*J*N, Sec. IV-A)         */
    CCDC_Q_NODE_FILES        /* int32_t[K][FILES_PER_NODE] the set M_k: files node k stores, ascending */
};

/*
 * Placement and schedule, host only (no GPU needed).
 * ccdc_plan: ONE job; its N files are cut into C(K,r) batches, batch p (files
 *   [p*m,(p+1)*m), m = N/C(K,r)) is stored on the p-th r-subset of the K nodes
 *   (placement of Sec. IV-A with the whole cluster as the job's subset), and
 *   every (r+1)-subset runs one stage-1 round of Sec. IV-B.  R = C(K,r+1).
 * ccdc_plan_jobs: the scheme as Sec. IV states it: J = C(K,r+1) jobs, job j on
 *   the j-th (r+1)-subset in r+1 batches (m = N/(r+1)); each subset runs its
 *   stage-1 round, then one stage-2 round per outside node in ascending order.
 *   R = C(K,r+1)*(K-r).  Its load is Theorem 1's.
 * Errors: CCDC_EINVAL for K<2, r<1, r>K-1 (Theorem 1: mu*K in 1..K-1), Q<1,
 *   K not dividing Q or K>N (Sec. III network model), batch count not dividing
 *   N (Sec. IV-A), null out; CCDC_ESIZE if a table would pass 2^31-1 entries.
 * The plan is owned by the library; release it with ccdc_plan_destroy.
 */
int ccdc_plan(int K, int r, int Q, int N, ccdc_plan_t **out);
int ccdc_plan_jobs(int K, int r, int Q, int N, ccdc_plan_t **out);
/* J = gamma*C(K,r+1) jobs (Sec. IV): the scheme of ccdc_plan_jobs repeated on gamma consecutive
 * blocks of C(K,r+1) jobs, same placement and rounds in each; R and the tables grow gamma-fold.
 * CCDC_EINVAL for gamma < 1. */
int ccdc_plan_jobs_repeated(int K, int r, int Q, int N, int gamma, ccdc_plan_t **out);

/*
 * The comparison scheme that only pre-combines (appendix of the paper), one job,
 * nothing coded: with mu = r/K (taken as 1/2 when larger) the files are cut into
 * nb = ceil(1/mu) consecutive batches of mu*N files (the last takes the rest),
 * node k stores batch k mod nb, and for every node k and every batch t it does
 * not store, the next node after k (cyclically) that stores B_t pre-combines the
 * values of k's c functions and sends that packet.  Vbar = D = [K*(nb-1)][W]
 * (receiver-major, batches ascending) are the packets; there is no X.  Only
 * ccdc_combine and ccdc_reduce (called with D = Vbar) apply; the coding entry
 * points return CCDC_ESTATE.  Its load is ceil(1/mu)-1 (mu < 1/2) or 1 (Sec. III).
 * Errors as ccdc_plan, with "batch count divides N" replaced by "mu*N is whole".
 */
int ccdc_plan_compression(int K, int r, int Q, int N, ccdc_plan_t **out);
void ccdc_plan_destroy(ccdc_plan_t *plan);   /* frees host and device parts; NULL is fine */

/*
 * Fix the value length T (elements) and the payload mode: computes W, the
 * segment split (Sec. IV-B) and the traffic the schedule puts on the wire.
 * Host only.  May be called again; that drops any device tables.
 * Errors: CCDC_EINVAL (T<1, unknown mode, a hybrid mode on a plan of
 * ccdc_plan_compression, which codes nothing), CCDC_ESIZE when a buffer would
 * hold more than 2^40 elements or a kernel's work-item count would pass 2^31-1.
 */
int ccdc_plan_bind(ccdc_plan_t *plan, int64_t T, int mode);

/*
 * Copy the index tables to the CURRENT HIP device and allocate the reduction
 * workspace there (the only device allocations the library ever makes).
 * Needs a bound plan.  CCDC_EHIP / CCDC_ENOMEM on failure; the host side of
 * the plan stays valid.
 */
int ccdc_plan_upload(ccdc_plan_t *plan);

/* Read a scalar or copy a table (host memory).  CCDC_EINVAL on unknown item,
 * null pointer or out_bytes smaller than the item; CCDC_ESTATE if the item
 * needs ccdc_plan_bind first. */
int ccdc_plan_query(const ccdc_plan_t *plan, int what, void *out, size_t out_bytes);

const char *ccdc_strerror(int status);

/*
 * A stand-in for the Map phase (Sec. III: node k maps every file it stores into the Q
 * intermediate values v_{q,n} = g_q(w_n); the paper leaves g_q free).  A file is a data
 * vector of Q*T elements, files = [J][N][Q][T] like V; every job has a model
 * theta = [J][Q][T]; the map is the gradient of 1/2 |theta - w_n|^2 chunk by chunk,
 *     V[j][n][q][t] = theta[j][q][t] - files[j][n][q][t]
 * (XOR in CCDC_U32_XOR; in the 16-bit modes the fp32 difference rounded once to the
 * format).  The shuffle path then sums it over the files: Phi = N*theta - sum_n w_n.
 * Every file is mapped once per call (the r nodes that store it would compute the same
 * values).  V may be the files buffer itself (the values replace the files in place) or
 * a separate one; theta must not overlap V.  Device pointers, errors and alignment rules
 * as for the stage calls below; any coded or uncoded plan.
 */
int ccdc_map(const ccdc_plan_t *plan, const void *files, const void *theta, void *V, void *stream);

/*
 * The four stages.  All pointers are device pointers; see the buffer table
 * above for shapes.  Each needs an uploaded plan (CCDC_ESTATE otherwise) and
 * the plan's device to be current.  The caller owns every buffer and keeps it
 * alive until the stream has run the call; inputs are only read, outputs are
 * written in full (no accumulation into what they held).  CCDC_EINVAL for a
 * null pointer or one not aligned to the element size; pointers aligned to 16
 * bytes (with T a multiple of 4, or of 8 for 2-byte elements) take the wide
 * kernels, others the one-element kernels with the same results.  A call that
 * falls back to narrower packs has up to 8 times as many work items as
 * ccdc_plan_bind checked for: it answers CCDC_ESIZE, before anything is
 * launched, when one of its launches would pass 2^31-1 of them.
 */

/* Pre-combining (Sec. IV-B): Vbar[u][b][e] = sum over the m files n of the
 * batch served to member b of V[job][n][s_b*c*T + e]. */
int ccdc_combine(const ccdc_plan_t *plan, const void *V, void *Vbar, void *stream);

/* Split and encode (Sec. IV-B, coded-packet equation): sender a adds, over the
 * other members b, the segment of Vbar[u][b] that carries a's label, i.e.
 * segment rank(a,b) = a - [a>b]:  X[u][a][x] = sum_{b!=a} Vbar[u][b][rank*ell+x]. */
int ccdc_encode(const ccdc_plan_t *plan, const void *Vbar, void *X, void *stream);

/* Decode (Sec. IV-B): receiver b removes from X[u][a] the segments of the
 * packets Vbar[u][b'], b' not in {a,b}, which it can compute itself because it
 * stores their batches:  D[u][b][rank(a,b)*ell+x] = X[u][a][x] - sum Vbar[u][b'][rank(a,b')*ell+x].
 * Row Vbar[u][b] (the packet being recovered) is never read for receiver b. */
int ccdc_decode(const ccdc_plan_t *plan, const void *X, const void *Vbar, void *D, void *stream);

/* Final reduction (Sec. IV-B, last paragraphs): Phi[job][k*c*T+e] = sum of V over
 * the files node k stores itself (batch order) + sum of D[u][b] over the rounds
 * in which k was member b (round order).  Uses the plan's workspace when the
 * sum is split. */
int ccdc_reduce(const ccdc_plan_t *plan, const void *V, const void *D, void *Phi, void *stream);

/* The three shuffle steps of Sec. IV-B (pre-combining, the coded-packet equation,
 * the decoding paragraph) in one pass: every needed element of V is read once, X
 * and D are written; Vbar is never materialised.  A coded pack is decoded for each
 * of its r receivers as in ccdc_decode, from the packs of the OTHER packets in it.
 * Results equal the three separate calls (bit-exact in XOR mode; same operation
 * order in fp32). */
int ccdc_shuffle_fused(const ccdc_plan_t *plan, const void *V, void *X, void *D, void *stream);

/* The whole path of Sec. IV-B in one pass for single-job plans (ccdc_plan):
 * pre-combining, the coded-packet equation, the decoding paragraph and the final
 * reduction of its last paragraphs; every element of V is read once, X and Phi are written,
 * neither Vbar nor D is materialised.  Each coded pack is decoded for each
 * receiver as in ccdc_decode (coded pack minus the receiver's side information)
 * and added to that receiver's output, together with the files it stores itself.
 * X equals ccdc_encode's bit for bit; Phi is bit-exact in XOR mode and, in fp32,
 * a fixed summation order different from ccdc_reduce's.  Uses the plan's
 * workspace.  CCDC_ESIZE for plans of ccdc_plan_jobs, for r > 5 and for
 * K*r > 256 (the per-lane outputs of all nodes must fit in 64 KB of LDS):
 * use ccdc_shuffle_fused + ccdc_reduce there. */
int ccdc_pipeline_fused(const ccdc_plan_t *plan, const void *V, void *X, void *Phi, void *stream);

/* ccdc_pipeline_fused for callers that cannot have device memory allocated for
 * them: code recorded into a HIP graph, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same X bit for bit and the same Phi (same
 * chunks, same summation order) as ccdc_pipeline_fused, but the partial outputs
 * of the round chunks go to a fixed 64 MiB array in device memory that the
 * library holds on every GPU it runs on, instead of the plan's workspace; the
 * call itself allocates and frees nothing.  CCDC_ESIZE when the plan's chunks
 * need more than 64 MiB (chunks * K * W * 4 bytes; a launch with a single chunk
 * needs none and is never refused for its size); other errors as
 * ccdc_pipeline_fused.  All calls on one GPU share the array: two of them that
 * overlap in time (different streams, different plans) race; keep them on one
 * stream or order them yourself. */
int ccdc_pipeline_fused_noalloc(const ccdc_plan_t *plan, const void *V, void *X, void *Phi, void *stream);

/*
 * The node-local form of the path: what ONE node of the cluster does in the
 * shuffle, from nothing but the files it stores and the coded packets it
 * receives (Sec. IV-B, the steps every member of a subset takes: pre-combine, split, code, multicast;
 * then decode with locally computed side information and reduce).  V and X are
 * the same arrays as above, but node k's calls read only the files k stores
 * (its batches, Sec. IV-A) and the packets sent to k, so X plays the network.
 * node = -1 runs every node in one launch: the emulation in which no result is
 * shared between nodes (each of the r nodes storing a batch pre-combines it
 * for itself).
 *
 * ccdc_node_encode writes the packets X[u][a] the node sends (rounds u it is
 *   member a of); they equal ccdc_encode's bit for bit.
 * ccdc_node_decode_reduce writes the node's c outputs of every job,
 *   Phi[job][node*c*T ...]: its own files plus, for every round it is in, the
 *   packet it decodes from the other members' coded packets; the decoded packet
 *   is never stored.  Same row order as ccdc_reduce; uses the plan's workspace
 *   when the sum is split (chunk sums are added in chunk order).
 * Call ccdc_node_encode for all senders of a round before a receiver decodes it.
 * Errors as the stage calls; CCDC_EINVAL for node outside -1..K-1, CCDC_ESTATE
 * for plans of ccdc_plan_compression.
 */
int ccdc_node_encode(const ccdc_plan_t *plan, int node, const void *V, void *X, void *stream);
int ccdc_node_decode_reduce(const ccdc_plan_t *plan, int node, const void *V, const void *X, void *Phi, void *stream);

#ifdef __cplusplus
}
#endif
#endif
