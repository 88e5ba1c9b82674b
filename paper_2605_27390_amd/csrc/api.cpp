// C ABI of the active-vocabulary LM head (declared in include/evospec.h): argument
// validation on the host, launch planning, and the sequence of kernel launches.
// Nothing here allocates device memory or waits for the GPU (evospec_validate_ids aside).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdio>
#include <cstring>

#include "evospec.h"
#include "launch.hpp"
#include "plan.hpp"

namespace {

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e) {
    std::snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", hipGetErrorName(e), hipGetErrorString(e));
    return EVOSPEC_HIP_ERROR;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Compute units of the current device (cached per device id).
int device_num_cu(int* out) {
    static std::atomic<int> cached[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev >= 0 && dev < 64 && cached[dev].load() > 0) { *out = cached[dev].load(); return EVOSPEC_OK; }
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_fail(e);
    if (n <= 0) n = 256;
    if (dev >= 0 && dev < 64) cached[dev].store(n);
    *out = n;
    return EVOSPEC_OK;
}

bool bad_layout(int layout) { return layout != EVOSPEC_ROW_MAJOR && layout != EVOSPEC_PACKED; }

int check_head_args(const void* h, int M, int d, const void* W, int V_act, int k) {
    if (M < 0 || d <= 0 || (d % 8) != 0 || V_act <= 0) return EVOSPEC_BAD_SHAPE;
    if (k < 1 || k > EVOSPEC_K_MAX || k > V_act) return EVOSPEC_BAD_K;
    if (M > 0 && (!h || !W)) return EVOSPEC_NULL_POINTER;
    if (M > 0 && (!aligned16(h) || !aligned16(W))) return EVOSPEC_MISALIGNED;
    return EVOSPEC_OK;
}

// Scratch for the shared core of the segmented head: one set of partials per 64-row pass, or
// the large-M layout from kGemmMinRows rows on.
size_t core_workspace_bytes(int M, int d, int V_core, int k) {
    if (evospec::use_gemm(M, d)) return evospec::make_gemm_plan(M, V_core, k).total_bytes;
    const size_t passes = ((size_t)M + evospec::kMTile - 1) / evospec::kMTile;
    return passes * evospec::workspace_upper_bound(V_core, k);
}

// Chunks (pieces of at most 64 rows of one sequence) whose extension partials one launch keeps.
size_t arc_chunks(int M, int S) {
    const size_t n = (size_t)S + (size_t)M / evospec::kMTile + 1;
    return n < (size_t)evospec::kMaxChunks ? n : (size_t)evospec::kMaxChunks;
}

}  // namespace

using namespace evospec;

extern "C" {

int evospec_version(void) { return EVOSPEC_VERSION; }

const char* evospec_status_string(int status) {
    switch (status) {
        case EVOSPEC_OK: return "ok";
        case EVOSPEC_NULL_POINTER: return "a required pointer is NULL";
        case EVOSPEC_BAD_SHAPE: return "bad shape (negative size, V_act <= 0, d <= 0 or d not a multiple of 8)";
        case EVOSPEC_BAD_K: return "k must satisfy 1 <= k <= min(EVOSPEC_K_MAX, active-set size)";
        case EVOSPEC_MISALIGNED: return "matrix or workspace pointer is not 16-byte aligned";
        case EVOSPEC_WORKSPACE_TOO_SMALL: return "workspace is smaller than evospec_workspace_bytes reports";
        case EVOSPEC_BAD_SEGMENTS: return "row_off must start at 0, be non-decreasing and end at M";
        case EVOSPEC_INVALID_IDS: return "ids out of range or not unique";
        case EVOSPEC_HIP_ERROR: return "HIP error (see evospec_last_hip_error)";
        case EVOSPEC_BAD_LAYOUT: return "layout must be EVOSPEC_ROW_MAJOR or EVOSPEC_PACKED";
        case EVOSPEC_STATIC_SCRATCH_EXCEEDED:
            return "shapes need more scratch than EVOSPEC_STATIC_SCRATCH_BYTES (use the workspace variant)";
        default: return "unknown status";
    }
}

const char* evospec_last_hip_error(void) { return g_hip_error; }

int evospec_matrix_bytes(int rows, int d, int layout, size_t* out_bytes) {
    if (!out_bytes) return EVOSPEC_NULL_POINTER;
    if (rows < 0 || d <= 0 || (d % 8) != 0) return EVOSPEC_BAD_SHAPE;
    if (bad_layout(layout)) return EVOSPEC_BAD_LAYOUT;
    *out_bytes = matrix_elems((size_t)rows, d, layout == EVOSPEC_PACKED) * 2;
    return EVOSPEC_OK;
}

int evospec_workspace_bytes(int M, int V_act, int d, int k, size_t* out_bytes) {
    if (!out_bytes) return EVOSPEC_NULL_POINTER;
    if (M < 0 || d <= 0 || (d % 8) != 0 || V_act <= 0) return EVOSPEC_BAD_SHAPE;
    if (k < 1 || k > EVOSPEC_K_MAX || k > V_act) return EVOSPEC_BAD_K;
    size_t need = workspace_upper_bound(V_act, k);     // passes over M reuse the same scratch
    if (use_gemm(M, d)) need = make_gemm_plan(M, V_act, k).total_bytes;     // one launch for all rows
    *out_bytes = need;
    return EVOSPEC_OK;
}

int evospec_workspace_bytes_segmented(int M, int V_core, int V_arc, int S, int d, int k, size_t* out_bytes) {
    if (!out_bytes) return EVOSPEC_NULL_POINTER;
    if (M < 0 || d <= 0 || (d % 8) != 0 || V_core < 0 || V_arc < 0 || V_core + V_arc <= 0 || S <= 0)
        return EVOSPEC_BAD_SHAPE;
    if (k < 1 || k > EVOSPEC_K_MAX || k > V_core + V_arc) return EVOSPEC_BAD_K;
    // core partials are kept for every draft row (per 64-row pass, or one large-M launch); the
    // extension scratch is reused per chunk
    size_t total = 0;
    if (V_core > 0) total += core_workspace_bytes(M, d, V_core, k);
    if (V_arc > 0) total += arc_chunks(M, S) * workspace_upper_bound(V_arc, k);
    *out_bytes = total > 0 ? total : 256;
    return EVOSPEC_OK;
}

int evospec_active_gather(const void* W_lm, int V, int d, const int32_t* src_ids, const int32_t* slots,
                          int n, void* W_act, int32_t* act_ids, int V_act, int layout, void* stream) {
    if (V <= 0 || d <= 0 || (d % 8) != 0 || V_act <= 0 || n < 0) return EVOSPEC_BAD_SHAPE;
    if (bad_layout(layout)) return EVOSPEC_BAD_LAYOUT;
    if (!slots && n > V_act) return EVOSPEC_BAD_SHAPE;
    if (n == 0) return EVOSPEC_OK;
    if (!W_lm || !src_ids || !W_act || !act_ids) return EVOSPEC_NULL_POINTER;
    if (!aligned16(W_lm) || !aligned16(W_act)) return EVOSPEC_MISALIGNED;
    hipError_t e = launch_gather(W_lm, V, d, src_ids, slots, n, W_act, act_ids, V_act,
                                 static_cast<hipStream_t>(stream), layout == EVOSPEC_PACKED);
    return e == hipSuccess ? EVOSPEC_OK : hip_fail(e);
}

int evospec_active_lmhead_partials(const void* h, int M, int d, const void* W_act, const int32_t* ids,
                                   int V_act, int layout, int k, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    int rc = check_head_args(h, M, d, W_act, V_act, k);
    if (rc) return rc;
    if (bad_layout(layout)) return EVOSPEC_BAD_LAYOUT;
    if (M == 0) return EVOSPEC_OK;
    if (M > kMTile) return EVOSPEC_BAD_SHAPE;          // the split halves handle one 64-row pass
    if (!workspace) return EVOSPEC_NULL_POINTER;
    if (!aligned16(workspace)) return EVOSPEC_MISALIGNED;
    if (workspace_bytes < workspace_upper_bound(V_act, k)) return EVOSPEC_WORKSPACE_TOO_SMALL;
    int num_cu = 0;
    rc = device_num_cu(&num_cu);
    if (rc) return rc;
    const Plan p = make_plan(M, V_act, d, k, num_cu);
    char* ws = static_cast<char*>(workspace);
    hipError_t e = launch_partials(p, h, M, d, W_act, ids, V_act, k, ws + p.keys_off, ws + p.stats_off,
                                   static_cast<hipStream_t>(stream), layout == EVOSPEC_PACKED);
    return e == hipSuccess ? EVOSPEC_OK : hip_fail(e);
}

int evospec_active_lmhead_merge(int M, int V_act, int d, int k, float* out_vals, int32_t* out_ids,
                                float* out_logz, const void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || d <= 0 || (d % 8) != 0 || V_act <= 0) return EVOSPEC_BAD_SHAPE;
    if (k < 1 || k > EVOSPEC_K_MAX || k > V_act) return EVOSPEC_BAD_K;
    if (M == 0) return EVOSPEC_OK;
    if (M > kMTile) return EVOSPEC_BAD_SHAPE;
    if (!out_vals || !out_ids || !out_logz || !workspace) return EVOSPEC_NULL_POINTER;
    if (!aligned16(workspace)) return EVOSPEC_MISALIGNED;
    if (workspace_bytes < workspace_upper_bound(V_act, k)) return EVOSPEC_WORKSPACE_TOO_SMALL;
    int num_cu = 0;
    int rc = device_num_cu(&num_cu);
    if (rc) return rc;
    const Plan p = make_plan(M, V_act, d, k, num_cu);
    const char* ws = static_cast<const char*>(workspace);
    MergeSet a{ws + p.keys_off, ws + p.stats_off, p.n_slabs, 0, kMTile};
    MergeSet none{};
    hipError_t e = launch_merge(a, none, k, out_vals, out_ids, out_logz, 0, M, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? EVOSPEC_OK : hip_fail(e);
}

}  // extern "C"

namespace evospec {
// The head, with an optional update that rides on its last merge launch.
int head_impl(const void* h, int M, int d, const void* W_act, const int32_t* ids,
              int V_act, int layout, int k, float* out_vals, int32_t* out_ids, float* out_logz,
              void* workspace, size_t workspace_bytes, void* stream, const GatherArgs* update) {
    int rc = check_head_args(h, M, d, W_act, V_act, k);
    if (rc) return rc;
    if (bad_layout(layout)) return EVOSPEC_BAD_LAYOUT;
    const bool packed = layout == EVOSPEC_PACKED;
    if (M == 0) return EVOSPEC_OK;
    if (!out_vals || !out_ids || !out_logz || !workspace) return EVOSPEC_NULL_POINTER;
    if (!aligned16(workspace)) return EVOSPEC_MISALIGNED;
    size_t need = 0;
    evospec_workspace_bytes(M, V_act, d, k, &need);
    if (workspace_bytes < need) return EVOSPEC_WORKSPACE_TOO_SMALL;
    int num_cu = 0;
    rc = device_num_cu(&num_cu);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    const uint16_t* hp = static_cast<const uint16_t*>(h);
    if (use_gemm(M, d)) {                               // bound by the contraction: all rows at once
        const GemmPlan gp = make_gemm_plan(M, V_act, k);
        hipError_t e = launch_gemm_partials(h, M, d, W_act, ids, V_act, k, ws + gp.keys_off, ws + gp.stats_off, st, packed);
        if (e != hipSuccess) return hip_fail(e);
        MergeSet a{ws + gp.keys_off, ws + gp.stats_off, gp.n_slabs, 0, M, gp.list_len, true};
        MergeSet none{};
        e = launch_merge(a, none, k, out_vals, out_ids, out_logz, 0, M, st, update);
        return e == hipSuccess ? EVOSPEC_OK : hip_fail(e);
    }
    for (int m0 = 0; m0 < M; m0 += kMTile) {            // passes of 64 draft rows share the scratch
        const int rows = (M - m0) < kMTile ? (M - m0) : kMTile;
        const Plan p = make_plan(rows, V_act, d, k, num_cu);
        hipError_t e = launch_partials(p, hp + (size_t)m0 * d, rows, d, W_act, ids, V_act, k,
                                       ws + p.keys_off, ws + p.stats_off, st, packed);
        if (e != hipSuccess) return hip_fail(e);
        MergeSet a{ws + p.keys_off, ws + p.stats_off, p.n_slabs, 0, kMTile};
        MergeSet none{};
        e = launch_merge(a, none, k, out_vals, out_ids, out_logz, m0, rows, st, m0 + kMTile >= M ? update : nullptr);
        if (e != hipSuccess) return hip_fail(e);
    }
    return EVOSPEC_OK;
}

int record_hip_error(hipError_t e) { return hip_fail(e); }
}  // namespace evospec

extern "C" {

int evospec_active_lmhead_topk(const void* h, int M, int d, const void* W_act, const int32_t* ids,
                               int V_act, int layout, int k, float* out_vals, int32_t* out_ids, float* out_logz,
                               void* workspace, size_t workspace_bytes, void* stream) {
    return head_impl(h, M, d, W_act, ids, V_act, layout, k, out_vals, out_ids, out_logz, workspace, workspace_bytes,
                     stream, nullptr);
}

int evospec_active_lmhead_topk_then_update(const void* h, int M, int d, void* W_act, int32_t* act_ids,
                                           int V_act, int layout, int k, float* out_vals, int32_t* out_ids,
                                           float* out_logz, void* workspace, size_t workspace_bytes,
                                           const void* W_lm, int V, const int32_t* src_ids, const int32_t* slots,
                                           int n, void* stream) {
    if (V <= 0 || n < 0) return EVOSPEC_BAD_SHAPE;
    if (bad_layout(layout)) return EVOSPEC_BAD_LAYOUT;
    if (!slots && n > V_act) return EVOSPEC_BAD_SHAPE;
    if (n > 0 && (!W_lm || !src_ids || !act_ids)) return EVOSPEC_NULL_POINTER;
    if (n > 0 && !aligned16(W_lm)) return EVOSPEC_MISALIGNED;
    if (M == 0 || n == 0) {                       // nothing to ride on, or nothing to carry
        int rc = head_impl(h, M, d, W_act, act_ids, V_act, layout, k, out_vals, out_ids, out_logz, workspace,
                           workspace_bytes, stream, nullptr);
        if (rc || n == 0) return rc;
        return evospec_active_gather(W_lm, V, d, src_ids, slots, n, W_act, act_ids, V_act, layout, stream);
    }
    const GatherArgs upd{W_lm, V, d / 8, src_ids, slots, n, W_act, act_ids, V_act, layout == EVOSPEC_PACKED ? 1 : 0};
    return head_impl(h, M, d, W_act, act_ids, V_act, layout, k, out_vals, out_ids, out_logz, workspace, workspace_bytes,
                     stream, &upd);
}

int evospec_active_lmhead_topk_segmented(const void* h, int M, int d, const void* W_core,
                                         const int32_t* ids_core, int V_core, const void* W_arc,
                                         const int32_t* ids_arc, int V_arc, int layout, const int32_t* row_off,
                                         int S, int k, float* out_vals, int32_t* out_ids, float* out_logz,
                                         void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || d <= 0 || (d % 8) != 0 || V_core < 0 || V_arc < 0 || V_core + V_arc <= 0 || S <= 0)
        return EVOSPEC_BAD_SHAPE;
    if (k < 1 || k > EVOSPEC_K_MAX || k > V_core + V_arc) return EVOSPEC_BAD_K;
    if (bad_layout(layout)) return EVOSPEC_BAD_LAYOUT;
    const bool packed = layout == EVOSPEC_PACKED;
    if (!row_off) return EVOSPEC_NULL_POINTER;
    if (row_off[0] != 0 || row_off[S] != M) return EVOSPEC_BAD_SEGMENTS;
    for (int s = 0; s < S; ++s)
        if (row_off[s + 1] < row_off[s]) return EVOSPEC_BAD_SEGMENTS;
    if (M == 0) return EVOSPEC_OK;
    if (!h || !out_vals || !out_ids || !out_logz || !workspace) return EVOSPEC_NULL_POINTER;
    if (V_core > 0 && !W_core) return EVOSPEC_NULL_POINTER;
    if (V_arc > 0 && (!W_arc || !ids_arc)) return EVOSPEC_NULL_POINTER;
    if (!aligned16(h) || !aligned16(W_core) || !aligned16(W_arc) || !aligned16(workspace)) return EVOSPEC_MISALIGNED;
    size_t need = 0;
    evospec_workspace_bytes_segmented(M, V_core, V_arc, S, d, k, &need);
    if (workspace_bytes < need) return EVOSPEC_WORKSPACE_TOO_SMALL;
    int num_cu = 0;
    int rc = device_num_cu(&num_cu);
    if (rc) return rc;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    const uint16_t* hp = static_cast<const uint16_t*>(h);
    const bool gemm_core = V_core > 0 && use_gemm(M, d);
    const size_t core_stride = V_core > 0 ? workspace_upper_bound(V_core, k) : 0;
    const size_t arc_stride = V_arc > 0 ? workspace_upper_bound(V_arc, k) : 0;
    char* ws_arc = ws + (V_core > 0 ? core_workspace_bytes(M, d, V_core, k) : 0);

    // shared core: every draft row against W_core, partials kept for all rows.  The 64-row
    // passes all use the plan of a full pass, so that one merge launch can address any of them.
    MergeSet core{};
    if (gemm_core) {
        const GemmPlan gp = make_gemm_plan(M, V_core, k);
        hipError_t e = launch_gemm_partials(h, M, d, W_core, ids_core, V_core, k, ws + gp.keys_off,
                                            ws + gp.stats_off, st, packed);
        if (e != hipSuccess) return hip_fail(e);
        core = MergeSet{ws + gp.keys_off, ws + gp.stats_off, gp.n_slabs, 0, M, gp.list_len, true};
    } else if (V_core > 0) {
        const Plan pc = make_plan(kMTile, V_core, d, k, num_cu);
        for (int m0 = 0, pss = 0; m0 < M; m0 += kMTile, ++pss) {
            const int rows = (M - m0) < kMTile ? (M - m0) : kMTile;
            char* w = ws + (size_t)pss * core_stride;
            hipError_t e = launch_partials(pc, hp + (size_t)m0 * d, rows, d, W_core, ids_core, V_core, k,
                                           w + pc.keys_off, w + pc.stats_off, st, packed);
            if (e != hipSuccess) return hip_fail(e);
        }
        core = MergeSet{ws + pc.keys_off, ws + pc.stats_off, pc.n_slabs, 0, kMTile};
    }

    // per sequence: its rows against its own extension, then the merge of both partial sets,
    // kMaxChunks chunks per launch.  A chunk has at most 64 rows and, with 64-row core passes,
    // never crosses a pass boundary, so its core partials sit in one pass.
    ChunkBatch cb;
    cb.n = 0;
    auto flush = [&]() -> int {
        if (cb.n == 0) return EVOSPEC_OK;
        int max_rows = 0;
        for (int i = 0; i < cb.n; ++i) max_rows = cb.rows[i] > max_rows ? cb.rows[i] : max_rows;
        MergeSet arc{};
        if (V_arc > 0) {
            const Plan pa = make_plan(max_rows, V_arc, d, k, num_cu, cb.n);
            BatchLayout bl;
            bl.seq_rows = V_arc;
            bl.chunk_bytes = arc_stride;
            bl.packed = packed;
            hipError_t e = launch_partials_batch(pa, h, cb, bl, d, W_arc, ids_arc, V_arc, k,
                                                 ws_arc + pa.keys_off, ws_arc + pa.stats_off, st);
            if (e != hipSuccess) return hip_fail(e);
            arc = MergeSet{ws_arc + pa.keys_off, ws_arc + pa.stats_off, pa.n_slabs, 0, kMTile};
        }
        hipError_t e = launch_merge_batch(core, core_stride, arc, arc_stride, cb, k, out_vals, out_ids, out_logz, st);
        if (e != hipSuccess) return hip_fail(e);
        cb.n = 0;
        return EVOSPEC_OK;
    };
    for (int s = 0; s < S; ++s) {
        int m0 = row_off[s];
        const int m_end = row_off[s + 1];
        while (m0 < m_end) {
            const int pass = m0 / kMTile;
            const int piece_end = gemm_core ? m0 + kMTile : (pass + 1) * kMTile;
            const int rows = (m_end < piece_end ? m_end : piece_end) - m0;
            const int i = cb.n++;
            cb.m0[i] = m0; cb.rows[i] = rows; cb.seq[i] = s;
            cb.a_pass[i] = gemm_core ? 0 : pass;
            cb.a_slot[i] = gemm_core ? m0 : m0 - pass * kMTile;
            if (cb.n == kMaxChunks) {
                const int rc2 = flush();
                if (rc2) return rc2;
            }
            m0 += rows;
        }
    }
    return flush();
}

int evospec_kl_gate_workspace_bytes(int E, int V, size_t* out_bytes) {
    if (!out_bytes) return EVOSPEC_NULL_POINTER;
    if (E < 0 || V <= 0) return EVOSPEC_BAD_SHAPE;
    *out_bytes = kl_gate_workspace_bytes(E > 0 ? E : 1, V);
    return EVOSPEC_OK;
}

int evospec_kl_gate(const float* z_target, int E, int V, const void* h_draft, int d, const void* W_lm,
                    int K, float T, int32_t* out_support, float* out_target_logits,
                    float* out_draft_logits, float* out_kl, void* workspace, size_t workspace_bytes,
                    void* stream) {
    if (E < 0 || V <= 0 || d <= 0 || (d % 8) != 0 || d > 24576 || !(T > 0.f)) return EVOSPEC_BAD_SHAPE;
    if (K < 1 || K > EVOSPEC_KL_K_MAX || K > V) return EVOSPEC_BAD_K;
    if (E == 0) return EVOSPEC_OK;
    if (!z_target || !h_draft || !W_lm || !out_support || !out_target_logits || !out_draft_logits || !out_kl ||
        !workspace)
        return EVOSPEC_NULL_POINTER;
    if (!aligned16(h_draft) || !aligned16(W_lm) || !aligned16(workspace)) return EVOSPEC_MISALIGNED;
    if (workspace_bytes < kl_gate_workspace_bytes(E, V)) return EVOSPEC_WORKSPACE_TOO_SMALL;
    hipError_t e = launch_kl_gate(z_target, E, V, h_draft, d, W_lm, K, T, out_support, out_target_logits,
                                  out_draft_logits, out_kl, workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? EVOSPEC_OK : hip_fail(e);
}

int evospec_validate_ids(const int32_t* ids, int n, int V, void* stream) {
    if (n < 0 || V <= 0) return EVOSPEC_BAD_SHAPE;
    if (n == 0) return EVOSPEC_OK;
    if (!ids) return EVOSPEC_NULL_POINTER;
    int bad = 0;
    hipError_t e = run_validate_ids(ids, n, V, static_cast<hipStream_t>(stream), &bad);
    if (e != hipSuccess) return hip_fail(e);
    return bad ? EVOSPEC_INVALID_IDS : EVOSPEC_OK;
}

}  // extern "C"
