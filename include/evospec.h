/*
 * evospec.h -- C ABI of the MI355X (gfx950) active-vocabulary LM head.
 *
 * The operation is the draft model's output projection of the EvoSpec paper,
 * Eq. 1  p = Softmax(h W_LM^T), evaluated only on the active vocabulary
 * V_t = V_static u V_dyn (Eq. 3; Algorithm 1, "construct active subspace" and
 * "draft restricted to V_t"), followed by the top-k that expands the draft tree
 * (EAGLE-2 search depth 6, 60-token budget; "Metrics and implementation details").
 *
 * Conventions for every call
 *   - extern "C", returns an evospec_status; never throws.
 *   - Pointers marked `dev` are device (HBM) addresses, `host` are host addresses.
 *     The caller owns every buffer; the library allocates no device memory and never
 *     synchronises (except evospec_validate_ids, a debug aid).
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and is ordered with other work on that stream.
 *   - bf16 matrices are row-major with contiguous rows (leading dimension == d),
 *     base pointers 16-byte aligned, d a multiple of 8 (128-bit loads).  The compact
 *     active matrix W_act may instead be kept in the packed layout below; every call
 *     that takes a W_act says which layout it is in (`layout`).
 *   - Arguments are validated on the host before the first HIP call; on an error
 *     nothing is enqueued.
 *   - M == 0 or n == 0 is a legal no-op (an update event may admit no token:
 *     App. "Additional safeguards").
 */
#ifndef EVOSPEC_H
#define EVOSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EVOSPEC_VERSION 210
#define EVOSPEC_K_MAX 64        /* largest k of the fused top-k                         */
#define EVOSPEC_M_TILE 64       /* draft rows handled by one pass over W_act            */

typedef enum evospec_status {
    EVOSPEC_OK = 0,
    EVOSPEC_NULL_POINTER = 1,       /* a required pointer is NULL                         */
    EVOSPEC_BAD_SHAPE = 2,          /* negative size, V_act <= 0, d <= 0, d % 8 != 0, ... */
    EVOSPEC_BAD_K = 3,              /* k < 1, k > EVOSPEC_K_MAX or k > active-set size    */
    EVOSPEC_MISALIGNED = 4,         /* a matrix / workspace pointer is not 16-B aligned   */
    EVOSPEC_WORKSPACE_TOO_SMALL = 5,
    EVOSPEC_BAD_SEGMENTS = 6,       /* row_off not monotone, row_off[0]!=0, row_off[S]!=M */
    EVOSPEC_INVALID_IDS = 7,        /* evospec_validate_ids only                          */
    EVOSPEC_HIP_ERROR = 8,          /* a launch failed; text via evospec_last_hip_error() */
    EVOSPEC_BAD_LAYOUT = 9,         /* layout is neither EVOSPEC_ROW_MAJOR nor EVOSPEC_PACKED */
    EVOSPEC_STATIC_SCRATCH_EXCEEDED = 10 /* evospec_active_lmhead_topk_static: the shapes need more
                                            scratch than EVOSPEC_STATIC_SCRATCH_BYTES             */
} evospec_status;

/*
 * Layouts of a compact active matrix (W_act, W_core, W_arc).  The paper does not say how the
 * restricted projection of Algorithm 1 ("draft restricted to V_t") keeps its weights; the layout
 * is this library's choice and the packed one is the fast one on MI355X (the head streams it with
 * whole-cache-line, fully coalesced loads; 0.62 against 0.53 of the HBM peak at 36,864 x 4,096).
 *   EVOSPEC_ROW_MAJOR  bf16 [rows, d], as W_lm.
 *   EVOSPEC_PACKED     rows padded to a multiple of 16, d padded to dp = a multiple of 256 (pad
 *                      elements are zero).  The 16-byte piece c (elements 8c .. 8c+7) of row r is
 *                      piece number  (r / 16) * (2 * dp) + (c / 4) * 64 + (c % 4) * 16 + (r % 16)
 *                      of the buffer: 16 rows x 32 elements form one 1 KB block in the order in
 *                      which the matrix cores take them.  Only evospec_active_gather (and the calls
 *                      that contain it) write this layout.  Rows never written hold garbage and are
 *                      never read as part of a result.
 * evospec_matrix_bytes: size of the buffer for `rows` rows in `layout` (host only, no HIP call).
 */
typedef enum evospec_layout {
    EVOSPEC_ROW_MAJOR = 0,
    EVOSPEC_PACKED = 1
} evospec_layout;
int evospec_matrix_bytes(int rows, int d, int layout, size_t *out_bytes /*host*/);

int evospec_version(void);
/* Static, never freed. */
const char *evospec_status_string(int status);
/* Text of the last HIP error seen by this thread's calls ("" if none). Static storage. */
const char *evospec_last_hip_error(void);

/*
 * Bytes of device scratch that evospec_active_lmhead_topk needs for these shapes
 * (host only, no HIP call).  The scratch holds, per slab of W_act rows and per draft
 * row, the slab's running max, sum of exponentials and k best (logit, id) pairs.
 */
int evospec_workspace_bytes(int M, int V_act, int d, int k, size_t *out_bytes /*host*/);
/* Same for the segmented call. */
int evospec_workspace_bytes_segmented(int M, int V_core, int V_arc, int S, int d, int k,
                                      size_t *out_bytes /*host*/);

/*
 * Insert rows into the compact active matrix (Eq. 3 builds V_t as a union; App.
 * "HNSW semantic retrieval": retrieved ids are inserted into the active draft
 * vocabulary; App. "ARC-based dynamic vocabulary maintenance" decides which slot).
 *   for i in [0, n):  W_act[slot_i, :] = W_lm[src_ids[i], :]   (bit-exact copy)
 *                     act_ids[slot_i]  = src_ids[i]
 *   slots == NULL means slot_i = i (full rebuild, then n <= V_act is required).
 * W_lm   dev bf16 [V, d]          src_ids dev int32 [n]     slots dev int32 [n] or NULL
 * W_act  dev bf16, V_act rows in `layout`, evospec_matrix_bytes(V_act, d, layout) bytes
 * act_ids dev int32 [V_act]
 * Preconditions not checked here (see evospec_validate_ids): 0 <= src_ids[i] < V,
 * 0 <= slots[i] < V_act, slots distinct within a call, W_act not overlapping W_lm.
 * Entries with an out-of-range id or slot are skipped by the kernel (memory safe).
 * Stream ordered: a later evospec_active_lmhead_topk on the same stream sees the update;
 * if the update is not enqueued in time the old W_act stays valid ("Retrieval latency
 * and asynchronous execution": a late result merges into a subsequent launch).
 */
int evospec_active_gather(const void *W_lm, int V, int d,
                          const int32_t *src_ids, const int32_t *slots, int n,
                          void *W_act, int32_t *act_ids, int V_act, int layout, void *stream);

/*
 * The restricted head (Eq. 1 on V_t; Algorithm 1 draft phase).  For each draft row m:
 *   z[m, i]    = sum_j h[m, j] * W_act[i, j]              i in [0, V_act)   (bf16 x bf16, fp32 accumulate)
 *   out_logz[m]= log sum_i exp(z[m, i])                   (normaliser over the active set only)
 *   out_vals[m, 0..k) = the k largest z[m, i], descending; equal logits ordered by smaller
 *                       full-vocabulary id first
 *   out_ids[m, 0..k)  = ids[i] of those entries (ids == NULL: the slot index i itself)
 * log-probability of a returned entry = out_vals - out_logz.  Logits are never written to HBM.
 * h dev bf16 [M, d]   W_act dev bf16, V_act rows in `layout`   ids dev int32 [V_act] or NULL
 * out_vals dev f32 [M, k]   out_ids dev int32 [M, k]   out_logz dev f32 [M]
 * workspace dev, 16-B aligned, at least evospec_workspace_bytes(...) bytes; contents are
 * scratch.  Two calls that share a workspace must be ordered (same stream).
 * Any M >= 0; rows are processed in passes of EVOSPEC_M_TILE.  ids must be unique
 * (Eq. 3 is a set union); duplicates are memory safe but count twice in the normaliser.
 */
int evospec_active_lmhead_topk(const void *h, int M, int d,
                               const void *W_act, const int32_t *ids, int V_act, int layout, int k,
                               float *out_vals, int32_t *out_ids, float *out_logz,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * evospec_active_lmhead_topk for callers that cannot allocate device memory or carry a workspace
 * around: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and kernels as evospec_active_lmhead_topk, except that the per-slab
 * partial results live in a fixed device array inside the library (EVOSPEC_STATIC_SCRATCH_BYTES
 * per GPU, held from the first call on that GPU until the process ends) instead of a caller
 * workspace.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine)
 * and does not synchronise; its first call on a device looks up that device's copy of the array.
 * Shapes whose evospec_workspace_bytes(M, V_act, d, k) exceeds EVOSPEC_STATIC_SCRATCH_BYTES are
 * rejected with EVOSPEC_STATIC_SCRATCH_EXCEEDED before anything is enqueued.  For M <= 128 the need
 * is 8 (k + 1) bytes per active row: the limit covers V_act <= 95,325 at k = 10 and the full
 * 151,936-row head up to k = 5; from 129 draft rows on the need also grows with M (136 bytes per
 * draft row and 128 active rows at k <= 16) and only small problems fit.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams, or different threads without ordering) race on it; order them on one stream.  Nothing in
 * the array has to start at a given value, so the contents a previous call left behind are harmless.
 */
#define EVOSPEC_STATIC_SCRATCH_BYTES (8u << 20)
int evospec_active_lmhead_topk_static(const void *h, int M, int d,
                                      const void *W_act, const int32_t *ids, int V_act, int layout, int k,
                                      float *out_vals, int32_t *out_ids, float *out_logz, void *stream);

/*
 * The two halves of evospec_active_lmhead_topk, exposed so that a caller (or a profiler)
 * can time or overlap them: _partials streams W_act once and leaves per-slab partial
 * results in the workspace; _merge reduces them into the outputs.  Calling them back to
 * back on one stream with the same arguments is exactly evospec_active_lmhead_topk.
 */
int evospec_active_lmhead_partials(const void *h, int M, int d,
                                   const void *W_act, const int32_t *ids, int V_act, int layout, int k,
                                   void *workspace, size_t workspace_bytes, void *stream);
int evospec_active_lmhead_merge(int M, int V_act, int d, int k,
                                float *out_vals, int32_t *out_ids, float *out_logz,
                                const void *workspace, size_t workspace_bytes, void *stream);

/*
 * Batched serving variant (not in the paper; several requests share the static core and
 * each carries its own dynamic buffer).  Rows [row_off[s], row_off[s+1]) of h belong to
 * sequence s and see the active set  core u arc[s]  (caller promises arc[s] is disjoint
 * from the core).  Outputs as above, normaliser over core u arc[s].
 * W_core dev bf16, V_core rows in `layout`  ids_core dev int32 [V_core] or NULL (identity)
 * W_arc  dev bf16, S matrices of V_arc rows in `layout`, back to back (each of
 *        evospec_matrix_bytes(V_arc, d, layout) bytes)       ids_arc dev int32 [S, V_arc]
 * row_off HOST int32 [S+1], row_off[0] == 0, non-decreasing, row_off[S] == M.
 */
int evospec_active_lmhead_topk_segmented(const void *h, int M, int d,
        const void *W_core, const int32_t *ids_core, int V_core,
        const void *W_arc, const int32_t *ids_arc, int V_arc, int layout,
        const int32_t *row_off, int S, int k,
        float *out_vals, int32_t *out_ids, float *out_logz,
        void *workspace, size_t workspace_bytes, void *stream);

/*
 * The head (as evospec_active_lmhead_topk, on W_act / act_ids as they are), followed by a dynamic-
 * buffer update of the same W_act / act_ids (as evospec_active_gather with these src_ids / slots / n),
 * with one launch fewer: the update's rows are written by extra workgroups of the head's last launch,
 * after everything that reads W_act has finished.  The result equals the two calls in that order.
 * Meant for the decode loop: the ids a failure event admitted (App. "Additional safeguards": at most
 * 32 per event) are applied behind the current draft step and seen by the next one (a late result
 * "merges into a subsequent launch", App. "Retrieval latency and asynchronous execution").
 */
int evospec_active_lmhead_topk_then_update(const void *h, int M, int d, void *W_act, int32_t *act_ids,
                                           int V_act, int layout, int k, float *out_vals, int32_t *out_ids, float *out_logz,
                                           void *workspace, size_t workspace_bytes,
                                           const void *W_lm, int V, const int32_t *src_ids, const int32_t *slots,
                                           int n, void *stream);

/*
 * Retained-support KL gate of Path B (Sec. "Online parameter update", Eq. 5 and the admission
 * rule; Algorithm 1, Path B).  For each of E verification events: support = the ids of the K
 * (paper: K_logit = 256; 1 <= K <= EVOSPEC_KL_K_MAX, K <= V) largest target logits, ties to the
 * smaller id, by decreasing logit; z_q[i] = h_draft . W_lm[support[i]] (Eq. 1, bf16 in, fp32
 * accumulate); p = Softmax(z_t / T), q = Softmax(z_q / T) on the support; out_kl[e] = D_KL(p || q).
 * The caller compares out_kl with the gate (paper: 0.1).
 *   z_target  dev fp32 [E, V]         h_draft  dev bf16 [E, d], 16-B aligned
 *   W_lm      dev bf16 [V, d], 16-B aligned, d % 8 == 0, d <= 24,576
 *   out_support dev int32 [E, K]; out_target_logits, out_draft_logits dev fp32 [E, K]; out_kl dev fp32 [E]
 *   workspace dev, 16-B aligned, at least evospec_kl_gate_workspace_bytes(E, V) bytes, scratch
 * T > 0.  No synchronisation; E == 0 is a no-op.
 */
#define EVOSPEC_KL_K_MAX 256
int evospec_kl_gate_workspace_bytes(int E, int V, size_t *out_bytes /*host*/);
int evospec_kl_gate(const float *z_target, int E, int V, const void *h_draft, int d, const void *W_lm,
                    int K, float T, int32_t *out_support, float *out_target_logits,
                    float *out_draft_logits, float *out_kl, void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * Debug aid: checks 0 <= ids[i] < V and that no id occurs twice (Eq. 3 is a set).
 * Launches one check kernel and waits for it (the only call that synchronises).
 * Returns EVOSPEC_OK or EVOSPEC_INVALID_IDS.  ids dev int32 [n].
 */
int evospec_validate_ids(const int32_t *ids, int n, int V, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EVOSPEC_H */
