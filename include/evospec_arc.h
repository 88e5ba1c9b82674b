/*
 * Dynamic-buffer manager of the EvoSpec active vocabulary (host only, no GPU call).
 *
 * Eq. 3 of the paper builds the active set as V_static ∪ V_dyn with |V_dyn| <= N_dyn; the
 * appendix ("ARC-based dynamic vocabulary maintenance", "Additional safeguards", hyper-parameter
 * table) maintains V_dyn with an Adaptive Replacement Cache: recent list T1, frequent list T2,
 * ghost lists B1 and B2, target p in [0, capacity].  New tokens enter T1, a second hit promotes
 * to T2, a hit in T2 refreshes it; when the buffer is full the victim comes from T1 if |T1| > p,
 * else from T2.  Safeguards: candidates are de-duplicated per event, at most `max_insert`
 * insertions per failure event, a token is evicted only after `min_residency` decoding steps,
 * p stays fixed during the first `warmup_events` events.  Paper defaults: capacity 256, p0 128,
 * ghost lists 256 each, 32 insertions, 8 steps, 50 events.
 *
 * Where the paper is silent this manager: adapts p on a ghost hit the textbook way (by
 * max(1, |other ghost| / |this ghost|), integer division) and re-admits the token at T2; skips
 * victims that are too young (the chosen list first, then the other one) and drops the
 * candidate when none is old enough; drops candidates beyond the insertion cap without touching
 * p or the ghost lists; ignores candidates of the static core and negative ids.
 *
 * An event returns the (slot, id) pairs to write, ready for evospec_active_gather: a new token
 * takes the slot its victim leaves, or the next unused slot while the buffer fills, so the used
 * slots are always slot_base .. slot_base + resident - 1.
 *
 * All pointers are host pointers owned by the caller.  Functions return an evospec status
 * (EVOSPEC_OK, EVOSPEC_NULL_POINTER, EVOSPEC_BAD_SHAPE); none of them throws or touches the GPU.
 * A manager is not thread-safe.
 */
#ifndef EVOSPEC_ARC_H
#define EVOSPEC_ARC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct evospec_arc evospec_arc;

typedef struct evospec_arc_config {
    int capacity;       /* N_dyn, >= 1                                  (paper: 256) */
    int p0;             /* initial target, 0..capacity                  (paper: 128) */
    int ghost_capacity; /* |B1| and |B2| bound, >= 0                    (paper: 256) */
    int max_insert;     /* insertions per failure event, >= 0           (paper: 32)  */
    int min_residency;  /* decoding steps before a token may be evicted (paper: 8)   */
    int warmup_events;  /* events during which p is not adapted         (paper: 50)  */
    int slot_base;      /* added to every reported slot (row of W_act where the buffer starts) */
} evospec_arc_config;

/* The paper's defaults, slot_base 0. */
void evospec_arc_default_config(evospec_arc_config *cfg);

/* core_ids[n_core] (may be NULL when n_core == 0): ids of the static core, never admitted. */
int evospec_arc_create(const evospec_arc_config *cfg, const int32_t *core_ids, int n_core, evospec_arc **out);
void evospec_arc_destroy(evospec_arc *arc);
/* The configuration the manager was created with. */
int evospec_arc_get_config(const evospec_arc *arc, evospec_arc_config *out);

/* `steps` >= 0 decoding steps have passed. */
int evospec_arc_advance(evospec_arc *arc, int steps);

/* Hits on tokens that are already resident (others are ignored): T1 -> T2, T2 -> most recent. */
int evospec_arc_touch(evospec_arc *arc, const int32_t *ids, int n);

/* One failure event with n candidate ids, in priority order.  out_slots / out_ids must hold
 * max_insert entries; *n_out receives the number of (slot, id) pairs written, in insertion order. */
int evospec_arc_event(evospec_arc *arc, const int32_t *candidates, int n,
                      int32_t *out_slots, int32_t *out_ids, int *n_out);

/* Sizes: out[0..6] = p, |T1|, |T2|, |B1|, |B2|, decoding step, events seen. */
int evospec_arc_sizes(const evospec_arc *arc, int64_t out[7]);

/* Copies list `which` (0 T1, 1 T2, 2 B1, 3 B2), least recently used first, into out[cap];
 * *n_out = its length (BAD_SHAPE if cap is too small). */
int evospec_arc_list(const evospec_arc *arc, int which, int32_t *out, int cap, int *n_out);

/* Resident tokens ordered by slot: out_slots[i], out_ids[i], i < *n_out <= capacity. */
int evospec_arc_resident(const evospec_arc *arc, int32_t *out_slots, int32_t *out_ids, int *n_out);

/*
 * Candidate formation of a failure event (Sec. "Semantic approximation", "Statistical
 * expansion"; appendix "Runtime candidate formation"): seeds = target-side top candidates, then
 * the retrieved nearest neighbours; every seed contributes its first `max_successors` (paper: 8)
 * outgoing neighbours of the co-occurrence graph, given in CSR form (row_ptr[V + 1], col_idx; a
 * row lists successors by decreasing weight); duplicates keep their first place.  Order: seeds,
 * then successors seed by seed.  out[out_cap] receives at most out_cap ids, *n_out their number.
 * Seeds and successors outside [0, V) are dropped.  row_ptr / col_idx may be NULL when
 * max_successors == 0 (no graph).  Host pointers only.
 */
int evospec_form_candidates(const int32_t *target_top, int n_target, const int32_t *mips_top, int n_mips,
                            const int64_t *row_ptr, const int32_t *col_idx, int V, int max_successors,
                            int32_t *out, int out_cap, int *n_out);

/*
 * One whole failure event of Path A (Algorithm 1, "Path A: Vocabulary Expansion") on the GPU
 * and the host, for callers that run it on a side stream:
 *   1. exact maximum-inner-product search: the n_mips (<= EVOSPEC_K_MAX) rows of W_lm with the
 *      largest inner product with the target hidden state h_target (the fused head kernel at
 *      M = 1 over the full vocabulary; the paper approximates this search with an HNSW index);
 *   2. candidate formation (above) with the host arrays target_top / row_ptr / col_idx;
 *   3. admission by the buffer manager `arc`;
 *   4. evospec_active_gather of the admitted (slot, id) pairs into W_act / act_ids.
 * h_target (bf16 [d]), W_lm (bf16 [V, d]), W_act (V_act rows in `layout`, see evospec.h), act_ids,
 * workspace are device pointers, 16-byte aligned; everything else is host memory.  The call WAITS for step 1 on `stream` (it needs the
 * ids on the host) and returns after the gather has been enqueued: up to 32 admitted pairs travel in
 * the gather's kernel arguments, more are uploaded first with a copy that is complete when it returns
 * (either way the next event may use any stream).  out_slots / out_ids
 * (host, max_insert entries each, may be NULL) receive the admitted pairs, *n_out their number.
 * workspace_bytes must be at least evospec_path_a_workspace_bytes(V, d, n_mips, max_insert).
 * All arguments, those of the final gather included (W_act, act_ids, layout, and V_act >= slot_base +
 * capacity of the manager), are checked before the search is enqueued and before the manager admits
 * anything: an argument error leaves the manager and the GPU untouched.  A HIP failure after the
 * admission (a copy or launch that fails) leaves the manager ahead of W_act: rebuild W_act from
 * evospec_arc_resident in that case.
 */
int evospec_path_a_workspace_bytes(int V, int d, int n_mips, int max_insert, size_t *out_bytes);
int evospec_path_a_event(evospec_arc *arc, const void *h_target, int d, const void *W_lm, int V,
                         const int32_t *target_top, int n_target, int n_mips,
                         const int64_t *row_ptr, const int32_t *col_idx, int max_successors,
                         void *W_act, int32_t *act_ids, int V_act, int layout,
                         void *workspace, size_t workspace_bytes, void *stream,
                         int32_t *out_slots, int32_t *out_ids, int *n_out);

#ifdef __cplusplus
}
#endif
#endif /* EVOSPEC_ARC_H */
