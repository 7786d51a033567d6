// Internal layout of a plan: host combinatorics, the bound segment schedule and
// the handles of the device tables.  Not part of the public interface.
#pragma once

#include <cstddef>
#include <cstdint>
#include <mutex>
#include <vector>

#include "ccdc.h"

struct ccdc_plan_s {
    // problem (Sec. III): per job
    int K = 0, r = 0, Q = 0, N = 0;
    int J = 1;            // jobs
    int c = 0;            // Q / K functions per node
    int m = 0;            // files per batch
    bool paper_jobs = false;
    bool compression = false;           // uncoded comparison scheme (appendix): combine + reduce only
    int64_t nbatch = 0, nround = 0;
    int64_t nrows = 0;                  // packets: rows of Vbar and of D (nround*(r+1) for coded plans)

    // compression-only scheme: consecutive batches, node k stores batch k mod nbatch,
    // one uncoded packet per (receiver, batch it does not store)
    std::vector<int32_t> batch_first;   // [nbatch+1]
    std::vector<int32_t> node_batch;    // [K]
    std::vector<int32_t> pkt_recv, pkt_batch, pkt_send;   // [nrows]
    std::vector<int32_t> row_files;     // [nrows] files added into each packet (batches differ in size)

    // placement (Sec. IV-A) and rounds (Sec. IV-B)
    std::vector<int32_t> batch_job;     // [nbatch]
    std::vector<int32_t> batch_file0;   // [nbatch]
    std::vector<int32_t> batch_label;   // [nbatch][r]
    std::vector<int32_t> round_member;  // [nround][r+1]
    std::vector<int32_t> round_batch;   // [nround][r+1]
    std::vector<int32_t> node_rows;     // [K][rows_per_node] packets (u*(r+1)+a) that node k sends, ascending
    int64_t rows_per_node = 0;          // nrows / K: every node is in the same number of rounds
    std::vector<int32_t> file_nodes;    // [J*N][r] nodes storing file job*N+n, ascending (Sec. IV-A)
    std::vector<int32_t> node_files;    // [K][files_per_node] the sets M_k, ascending
    int64_t files_per_node = 0;         // r*J*N/K

    // fixed by ccdc_plan_bind
    bool bound = false;
    int64_t T = 0, W = 0, ell = 0;
    int mode = 0;
    std::vector<int64_t> packet_len;    // [r+1]
    int64_t scheduled = 0;              // elements on the wire

    // tables the kernels read (host copies)
    std::vector<int64_t> src_off;       // [nround][r+1] element offset in V of the served
                                        //   batch's first file, at the target's functions
    std::vector<int64_t> red_ptr;       // [nout+1] row-list bounds of each (job, node) output
    std::vector<int64_t> red_row;       // rows: (element offset << 1) | (1 = in D, 0 = in V)
    std::vector<int64_t> red_out;       // [nout] element offset of the output block in Phi
    int64_t nout = 0;                   // J * K output blocks of W elements
    int red_split = 1;                  // the row list of an output is summed in this many chunks
    size_t workspace_bytes = 0;

    // whole path in one pass (single-job plans): the partial outputs of all K
    // nodes are accumulated in LDS, one private slot per (node, segment, lane)
    bool pipe_ok = false;               // shape supported by ccdc_pipeline_fused
    int pipe_vec = 1;                   // widest pack the LDS budget allows
    int pipe_max_chunks = 1;            // upper bound on round chunks (sizes the workspace)
    int64_t pipe_local_rows = 0;        // rows of V every node adds from its own files
    std::vector<int64_t> loc_row;       // [K][pipe_local_rows] element offsets in V

    // device side, set by ccdc_plan_upload
    bool uploaded = false;
    int device = -1;
    int64_t *d_src_off = nullptr, *d_red_ptr = nullptr, *d_red_row = nullptr, *d_red_out = nullptr;
    int64_t *d_loc_row = nullptr;
    int32_t *d_member = nullptr;
    int32_t *d_row_files = nullptr;     // null when every packet adds m files
    int32_t *d_node_rows = nullptr;
    void *d_workspace = nullptr;

    // round chunks of the one-pass kernel on this device for packs of 1, 2 and 4
    // elements (index log2 of the width), from an occupancy query at upload time
    int pipe_chunks[3] = {0, 0, 0};

    // Order of the calls that use the workspace, across streams: the last such call
    // recorded ws_event (a hipEvent_t made by ccdc_plan_upload) on ws_stream.
    mutable std::mutex ws_mutex;
    mutable void *ws_event = nullptr;
    mutable void *ws_stream = nullptr;
    mutable bool ws_used = false;
};

namespace ccdc {

// Host-side construction; both return a ccdc_status.
int build_plan(int K, int r, int Q, int N, bool paper_jobs, int gamma, ccdc_plan_t **out);
int build_compression_plan(int K, int r, int Q, int N, ccdc_plan_t **out);
int bind_plan(ccdc_plan_t *p, int64_t T, int mode);

// Limits of the one-pass pipeline kernel.
constexpr int kPipeLanes = 64;                 // one wavefront per workgroup
constexpr int kPipeMaxLds = 64 * 1024;         // bytes of LDS one workgroup may take
// LDS a wavefront may take for its running outputs before a narrower pack is
// preferred (measured): four-element packs only while >= 6 wavefronts fit on a
// compute unit, unless the input is large, then down to 3 wavefronts like
// two-element packs (narrow accesses cost more than the lost occupancy).
#ifndef CCDC_PIPE_GOOD_LDS
#define CCDC_PIPE_GOOD_LDS (26 * 1024)
#endif
#ifndef CCDC_PIPE_GOOD_LDS_HALF
#define CCDC_PIPE_GOOD_LDS_HALF (50 * 1024)
#endif
constexpr int kPipeGoodLds = CCDC_PIPE_GOOD_LDS;
constexpr int kPipeGoodLdsHalf = CCDC_PIPE_GOOD_LDS_HALF;
constexpr int64_t kPipeLargeInput = 256LL << 20;   // bytes of V (at 4 bytes an element) from which an input counts as large
constexpr int kPipeMaxR1 = 6;                  // r+1 the kernel is unrolled for

// One-pass pipeline (pipeline.hip): fills p->pipe_chunks for the current device.
void pipeline_prepare(ccdc_plan_t *p);
// Body of ccdc_pipeline_fused.  own_part = null: partial outputs of round chunks go
// to the plan's workspace; else to the caller's buffer of own_part_bytes bytes
// (CCDC_ESIZE when they do not fit).
int pipeline_entry(const ccdc_plan_t *plan, const void *V, void *X, void *Phi, void *stream, void *own_part,
                   size_t own_part_bytes);

// Device address of the fixed scratch array of ccdc_pipeline_fused_noalloc on the
// current device (noalloc.hip); out may be null to only look it up ahead of time.
int scratch_address(void **out);

// Rank of sender a's label among the members other than b.
inline int label_rank(int a, int b) { return a - (a > b ? 1 : 0); }

}  // namespace ccdc
