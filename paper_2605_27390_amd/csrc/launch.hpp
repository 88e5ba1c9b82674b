// Launcher interface between the C ABI layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.hpp"

namespace evospec {

// One set of slab partials as the merge kernel sees it.
struct MergeSet {
    const void* keys = nullptr;     // u64 [n_slabs][row_stride][list_len or k]
    const void* stats = nullptr;    // float2 [n_slabs][row_stride]
    int n_slabs = 0;
    int row_base = 0;               // slot of the launch's first row inside the set
    int row_stride = 64;            // draft-row slots per slab in the layout (slab-major sets)
    int list_len = 0;               // slots per list; 0 = k keys, descending.  Otherwise the slots hold
                                    // the slab's candidates as (logit bits << 32 | id) in any order,
                                    // all ones = empty
    bool row_major = false;         // true: [row][slab][slot] (large-M path), row_stride unused
};

// Where the chunks of a batched launch find their operands and leave their partials: chunk i reads
// the rows [seq[i] * seq_rows, +V_act) of the matrix and id list, and writes at byte offset
// i * chunk_bytes (a multiple of 8) from `keys` and `stats`.
struct BatchLayout {
    int seq_rows = 0;
    size_t chunk_bytes = 0;
    bool packed = false;            // the matrix is in operand-tile layout (plan.hpp), one padded matrix per sequence
};

hipError_t launch_partials_batch(const Plan& p, const void* h, const ChunkBatch& cb, const BatchLayout& bl,
                                 int d, const void* W, const int32_t* ids, int V_act, int k, void* keys,
                                 void* stats, hipStream_t stream);
// One launch merges every chunk of the batch: row r of chunk i takes slot a_slot[i] + r of the first
// set (moved by a_pass[i] * a_pass_bytes) and slot r of the second (moved by i * b_chunk_bytes), and
// writes output row m0[i] + r.  `update`, if given, is applied by extra blocks of the same launch (one
// block per row).
hipError_t launch_merge_batch(const MergeSet& a, size_t a_pass_bytes, const MergeSet& b, size_t b_chunk_bytes,
                              const ChunkBatch& cb, int k, float* out_vals, int32_t* out_ids,
                              float* out_logz, hipStream_t stream, const GatherArgs* update = nullptr);
hipError_t launch_partials(const Plan& p, const void* h, int rows, int d, const void* W,
                           const int32_t* ids, int V_act, int k, void* keys, void* stats,
                           hipStream_t stream, bool packed = false);
// Large-M path: partials of all M draft rows, row-major: keys u64 [M][ceil(V_act/128)][gemm_list_len(k)]
// in any order, stats float2 [M][ceil(V_act/128)].
hipError_t launch_gemm_partials(const void* h, int M, int d, const void* W, const int32_t* ids, int V_act,
                                int k, void* keys, void* stats, hipStream_t stream, bool packed = false);
hipError_t launch_merge(const MergeSet& a, const MergeSet& b, int k, float* out_vals, int32_t* out_ids,
                        float* out_logz, int out_row0, int nrows, hipStream_t stream,
                        const GatherArgs* update = nullptr);
hipError_t launch_gather(const void* W_lm, int V, int d, const int32_t* src_ids, const int32_t* slots,
                         int n, void* W_act, int32_t* act_ids, int V_act, hipStream_t stream,
                         bool packed = false);
// The same for at most kInlineRows rows whose ids and slots are HOST arrays: they are passed to the
// kernel by value, so the call neither uploads nor waits.
hipError_t launch_gather_inline(const void* W_lm, int V, int d, const int32_t* host_ids, const int32_t* host_slots,
                                int n, void* W_act, int32_t* act_ids, int V_act, hipStream_t stream, bool packed);
// Retained-support KL gate (K <= 256, d * 2 bytes <= 48 KB of LDS); workspace of kl_gate_workspace_bytes.
size_t kl_gate_workspace_bytes(int E, int V);
hipError_t launch_kl_gate(const float* z_target, int E, int V, const void* h_draft, int d, const void* W_lm,
                          int K, float T, int32_t* out_support, float* out_zt, float* out_zq, float* out_kl,
                          void* workspace, hipStream_t stream);
hipError_t run_validate_ids(const int32_t* ids, int n, int V, hipStream_t stream, int* bad);

// The head behind evospec_active_lmhead_topk (api.cpp): validates, plans and launches on the given
// scratch buffer; returns an evospec_status.  `update`, if given, rides on the last launch.
int head_impl(const void* h, int M, int d, const void* W_act, const int32_t* ids, int V_act, int layout, int k,
              float* out_vals, int32_t* out_ids, float* out_logz, void* workspace, size_t workspace_bytes,
              void* stream, const GatherArgs* update);
// Stores the text of a HIP error for evospec_last_hip_error() and returns EVOSPEC_HIP_ERROR.
int record_hip_error(hipError_t e);

}  // namespace evospec
