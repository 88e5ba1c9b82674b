/*
 * CPU oracle for the active-vocabulary LM head (test infrastructure only).
 *
 * This file is the slow, plain definition that the GPU library is checked against.
 * It is NOT part of the product: only the tests, the smoke check and the bench's
 * cpu_baseline leg may load it.  It shares no code with the HIP path.
 *
 * What it computes (EvoSpec paper):
 *   - Eq. 1 (problem formulation): p = Softmax(h W_LM^T), a dense projection of the
 *     draft hidden state onto vocabulary rows.
 *   - Algorithm 1, "construct active subspace" + "draft restricted to V_t":
 *     the projection, its softmax normaliser and the top-k used for tree expansion
 *     are taken over the active set V_t = V_static u V_dyn only (Eq. 3 gives V_t as a
 *     set union, so ids are unique and their order carries no meaning).
 *   - App. "Additional runtime details": retrieved token ids are inserted into the
 *     active draft vocabulary; here that is a row copy W_act[slot] <- W_lm[id].
 *
 * Precision: inputs are bf16 bit patterns (the paper fixes BF16 weights); every
 * arithmetic step is fp64.  Summation is a plain left-to-right loop over the hidden
 * dimension.  No blocking, fusion or reordering.
 *
 * Readings where the paper is silent (listed in the design notes as well):
 *   - normaliser runs over the active set only;
 *   - returned values are raw logits, log-prob = value - logZ;
 *   - order: logits descending, equal logits by ascending full-vocabulary id.
 *
 * Parallelism: OpenMP over vocabulary rows (independent dot products) only to
 * shorten wall time; the result does not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 -> fp64: a bf16 is the upper half of an IEEE fp32, so widening is exact. */
static double bf16_to_f64(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Row insertion into the compact active matrix (App. "Additional runtime details":
 * retrieved ids are inserted into the active vocabulary).
 *   W_act[slot_i, :] = W_lm[src_ids[i], :]   (bit copy)
 *   act_ids[slot_i]  = src_ids[i]
 * slots == NULL means slot_i = i.  Returns 0, or -1 on an out-of-range id / slot.
 */
int oracle_active_gather(const uint16_t *W_lm, int V, int d,
                         const int32_t *src_ids, const int32_t *slots, int n,
                         uint16_t *W_act, int32_t *act_ids, int V_act) {
    for (int i = 0; i < n; ++i) {
        int32_t id = src_ids[i];
        int32_t s = slots ? slots[i] : i;
        if (id < 0 || id >= V || s < 0 || s >= V_act) return -1;
        for (int j = 0; j < d; ++j) W_act[(size_t)s * d + j] = W_lm[(size_t)id * d + j];
        act_ids[s] = id;
    }
    return 0;
}

/*
 * Eq. 1 without the softmax: z[m, i] = sum_j h[m, j] * W[i, j], for every row i of W.
 * z is [M, Vn] row-major fp64.
 */
void oracle_logits(const uint16_t *h, int M, int d,
                   const uint16_t *W, int Vn, double *z) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < Vn; ++i) {
        const uint16_t *w = W + (size_t)i * d;
        for (int m = 0; m < M; ++m) {
            const uint16_t *hm = h + (size_t)m * d;
            double acc = 0.0;
            for (int j = 0; j < d; ++j) acc += bf16_to_f64(hm[j]) * bf16_to_f64(w[j]);
            z[(size_t)m * Vn + i] = acc;
        }
    }
}

/*
 * Log of the softmax denominator of Eq. 1 over the Vn entries of each row:
 *   logZ[m] = mx + log(sum_i exp(z[m,i] - mx)),  mx = max_i z[m,i].
 */
void oracle_logz(const double *z, int M, int Vn, double *logz) {
    for (int m = 0; m < M; ++m) {
        const double *zm = z + (size_t)m * Vn;
        double mx = zm[0];
        for (int i = 1; i < Vn; ++i) if (zm[i] > mx) mx = zm[i];
        double s = 0.0;
        for (int i = 0; i < Vn; ++i) s += exp(zm[i] - mx);
        logz[m] = mx + log(s);
    }
}

struct cand { double z; int32_t id; };

static int cand_cmp(const void *a, const void *b) {
    const struct cand *x = (const struct cand *)a, *y = (const struct cand *)b;
    if (x->z > y->z) return -1;
    if (x->z < y->z) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}

/*
 * Top-kk of each row of z by full sort: logits descending, ties by ascending
 * full-vocabulary id.  ids == NULL means ids[i] = i.  kk <= Vn.
 * vals [M, kk] fp64, out_ids [M, kk].
 */
int oracle_topk(const double *z, const int32_t *ids, int M, int Vn, int kk,
                double *vals, int32_t *out_ids) {
    if (kk < 0 || kk > Vn) return -1;
    struct cand *c = (struct cand *)malloc((size_t)Vn * sizeof *c);
    if (!c) return -2;
    for (int m = 0; m < M; ++m) {
        for (int i = 0; i < Vn; ++i) {
            c[i].z = z[(size_t)m * Vn + i];
            c[i].id = ids ? ids[i] : i;
        }
        qsort(c, (size_t)Vn, sizeof *c, cand_cmp);
        for (int j = 0; j < kk; ++j) {
            vals[(size_t)m * kk + j] = c[j].z;
            out_ids[(size_t)m * kk + j] = c[j].id;
        }
    }
    free(c);
    return 0;
}

/*
 * The whole restricted head for one batch of draft rows (Alg. 1 draft phase on V_t):
 * logits over the active rows, logZ over the active set, top-kk with remap to
 * full-vocabulary ids.  kk may be k+1 so that the caller sees the runner-up too.
 * z_out (optional, [M, V_act]) receives all logits.
 */
int oracle_active_lmhead_topk(const uint16_t *h, int M, int d,
                              const uint16_t *W_act, const int32_t *ids, int V_act, int kk,
                              double *vals, int32_t *out_ids, double *logz, double *z_out) {
    if (M <= 0 || d <= 0 || V_act <= 0) return -1;
    double *z = z_out ? z_out : (double *)malloc((size_t)M * V_act * sizeof(double));
    if (!z) return -2;
    oracle_logits(h, M, d, W_act, V_act, z);
    oracle_logz(z, M, V_act, logz);
    int rc = oracle_topk(z, ids, M, V_act, kk, vals, out_ids);
    if (!z_out) free(z);
    return rc;
}

/*
 * Batched serving variant: S sequences share a core active set and each adds its own
 * dynamic extension.  Rows [row_off[s], row_off[s+1]) belong to sequence s and see the
 * concatenation core || arc_s as their active set (a union, by the caller's promise that
 * arc_s is disjoint from the core).  Everything else is as above.
 */
int oracle_active_lmhead_topk_segmented(const uint16_t *h, int M, int d,
        const uint16_t *W_core, const int32_t *ids_core, int V_core,
        const uint16_t *W_arc, const int32_t *ids_arc, int V_arc,
        const int32_t *row_off, int S, int kk,
        double *vals, int32_t *out_ids, double *logz) {
    if (M <= 0 || d <= 0 || V_core < 0 || V_arc < 0 || V_core + V_arc <= 0 || S <= 0) return -1;
    if (row_off[0] != 0 || row_off[S] != M) return -3;
    const int Vn = V_core + V_arc;
    for (int s = 0; s < S; ++s) {
        int r0 = row_off[s], r1 = row_off[s + 1];
        if (r1 < r0) return -3;
        int Ms = r1 - r0;
        if (Ms == 0) continue;
        double *z = (double *)malloc((size_t)Ms * Vn * sizeof(double));
        double *zc = (double *)malloc((size_t)Ms * (V_core > 0 ? V_core : 1) * sizeof(double));
        double *za = (double *)malloc((size_t)Ms * (V_arc > 0 ? V_arc : 1) * sizeof(double));
        int32_t *ids = (int32_t *)malloc((size_t)Vn * sizeof(int32_t));
        if (!z || !zc || !za || !ids) { free(z); free(zc); free(za); free(ids); return -2; }
        const uint16_t *hs = h + (size_t)r0 * d;
        if (V_core > 0) oracle_logits(hs, Ms, d, W_core, V_core, zc);
        if (V_arc > 0) oracle_logits(hs, Ms, d, W_arc + (size_t)s * V_arc * d, V_arc, za);
        for (int m = 0; m < Ms; ++m) {
            for (int i = 0; i < V_core; ++i) z[(size_t)m * Vn + i] = zc[(size_t)m * V_core + i];
            for (int i = 0; i < V_arc; ++i) z[(size_t)m * Vn + V_core + i] = za[(size_t)m * V_arc + i];
        }
        for (int i = 0; i < V_core; ++i) ids[i] = ids_core ? ids_core[i] : i;
        for (int i = 0; i < V_arc; ++i) ids[V_core + i] = ids_arc[(size_t)s * V_arc + i];
        oracle_logz(z, Ms, Vn, logz + r0);
        int rc = oracle_topk(z, ids, Ms, Vn, kk, vals + (size_t)r0 * kk, out_ids + (size_t)r0 * kk);
        free(z); free(zc); free(za); free(ids);
        if (rc) return rc;
    }
    return 0;
}
