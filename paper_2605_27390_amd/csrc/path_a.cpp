// One whole failure event of Path A (Algorithm 1, "Path A: Vocabulary Expansion"): exact search on
// the GPU, candidate formation and admission on the host, insertion of the admitted rows on the GPU.
// Declared in include/evospec_arc.h.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "evospec.h"
#include "evospec_arc.h"
#include "launch.hpp"

namespace {
constexpr size_t kAlign = 256;
size_t up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
constexpr int kMaxCandidates = 4096;
}  // namespace

extern "C" {

int evospec_path_a_workspace_bytes(int V, int d, int n_mips, int max_insert, size_t* out_bytes) {
    if (!out_bytes) return EVOSPEC_NULL_POINTER;
    if (max_insert < 0) return EVOSPEC_BAD_SHAPE;
    size_t head = 0;
    const int rc = evospec_workspace_bytes(1, V, d, n_mips, &head);
    if (rc) return rc;
    // head scratch | top values, ids, log-normaliser of the search | slots, ids of the update
    *out_bytes = up(head) + up((size_t)n_mips * 8 + 4) + up((size_t)max_insert * 8 + 8);
    return EVOSPEC_OK;
}

int evospec_path_a_event(evospec_arc* arc, const void* h_target, int d, const void* W_lm, int V,
                         const int32_t* target_top, int n_target, int n_mips,
                         const int64_t* row_ptr, const int32_t* col_idx, int max_successors,
                         void* W_act, int32_t* act_ids, int V_act, int layout,
                         void* workspace, size_t workspace_bytes, void* stream,
                         int32_t* out_slots, int32_t* out_ids, int* n_out) {
    // Everything is checked before the search runs and before the manager admits anything: once the
    // admission is committed, the insertion below cannot be refused any more.
    if (!arc || !n_out || !workspace || !h_target || !W_lm || !W_act || !act_ids) return EVOSPEC_NULL_POINTER;
    if (n_mips < 1 || n_mips > EVOSPEC_K_MAX) return EVOSPEC_BAD_K;
    if (n_target < 0 || (n_target > 0 && !target_top)) return n_target < 0 ? EVOSPEC_BAD_SHAPE : EVOSPEC_NULL_POINTER;
    if (max_successors < 0 || V <= 0 || d <= 0 || (d % 8) != 0 || V_act <= 0) return EVOSPEC_BAD_SHAPE;
    if (max_successors > 0 && (!row_ptr || !col_idx)) return EVOSPEC_NULL_POINTER;
    if (layout != EVOSPEC_ROW_MAJOR && layout != EVOSPEC_PACKED) return EVOSPEC_BAD_LAYOUT;
    auto misaligned = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
    if (misaligned(h_target) || misaligned(W_lm) || misaligned(W_act) || misaligned(workspace)) return EVOSPEC_MISALIGNED;
    evospec_arc_config cfg;
    int rc = evospec_arc_get_config(arc, &cfg);
    if (rc) return rc;
    // every slot the manager can hand out must exist in the compact matrix
    if ((long long)cfg.slot_base + cfg.capacity > (long long)V_act || cfg.slot_base < 0) return EVOSPEC_BAD_SHAPE;
    size_t need = 0;
    rc = evospec_path_a_workspace_bytes(V, d, n_mips, cfg.max_insert, &need);
    if (rc) return rc;
    if (workspace_bytes < need) return EVOSPEC_WORKSPACE_TOO_SMALL;
    size_t head = 0;
    evospec_workspace_bytes(1, V, d, n_mips, &head);
    char* ws = static_cast<char*>(workspace);
    float* top_vals = reinterpret_cast<float*>(ws + up(head));
    int32_t* top_ids = reinterpret_cast<int32_t*>(top_vals + n_mips);
    float* top_logz = reinterpret_cast<float*>(top_ids + n_mips);
    int32_t* upd = reinterpret_cast<int32_t*>(ws + up(head) + up((size_t)n_mips * 8 + 4));
    hipStream_t st = static_cast<hipStream_t>(stream);

    // 1. exact search over the full vocabulary (identity ids), ids to the host
    rc = evospec_active_lmhead_topk(h_target, 1, d, W_lm, nullptr, V, EVOSPEC_ROW_MAJOR, n_mips, top_vals, top_ids, top_logz,
                                    workspace, head, stream);
    if (rc) return rc;
    int32_t mips[EVOSPEC_K_MAX];
    if (hipMemcpyAsync(mips, top_ids, (size_t)n_mips * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return EVOSPEC_HIP_ERROR;
    // 2. candidates, 3. admission
    std::vector<int32_t> cand((size_t)kMaxCandidates);
    int n_cand = 0;
    rc = evospec_form_candidates(target_top, n_target, mips, n_mips, row_ptr, col_idx, V, max_successors,
                                 cand.data(), kMaxCandidates, &n_cand);
    if (rc) return rc;
    const int cap = cfg.max_insert;
    std::vector<int32_t> pairs((size_t)2 * (cap > 0 ? cap : 1), 0);
    int n_ins = 0;
    rc = evospec_arc_event(arc, cand.data(), n_cand, pairs.data(), pairs.data() + cap, &n_ins);
    if (rc) return rc;
    *n_out = n_ins;
    for (int i = 0; i < n_ins; ++i) {
        if (out_slots) out_slots[i] = pairs[i];
        if (out_ids) out_ids[i] = pairs[cap + i];
    }
    if (n_ins == 0) return EVOSPEC_OK;
    // 4. the admitted rows into the compact matrix.  A usual event (at most kInlineRows rows) hands
    //    its (slot, id) pairs to the kernel by value: no upload, nothing to wait for.  A larger one
    //    uploads both lists at once (slots in the first cap entries, ids behind them, on the host as
    //    on the device); the upload is complete when it returns (the host buffer is this call's own),
    //    whatever stream the next event uses.
    if (n_ins <= evospec::kInlineRows) {
        const hipError_t e = evospec::launch_gather_inline(W_lm, V, d, pairs.data() + cap, pairs.data(), n_ins, W_act,
                                                           act_ids, V_act, st, layout == EVOSPEC_PACKED);
        return e == hipSuccess ? EVOSPEC_OK : evospec::record_hip_error(e);
    }
    if (hipMemcpyWithStream(upd, pairs.data(), (size_t)(cap + n_ins) * 4, hipMemcpyHostToDevice, st) != hipSuccess)
        return EVOSPEC_HIP_ERROR;
    return evospec_active_gather(W_lm, V, d, upd + cap, upd, n_ins, W_act, act_ids, V_act, layout, stream);
}

}  // extern "C"
