/* Host driver for the sanitizer build (-fsanitize=address,undefined) of the CPU oracle: every entry
 * point on small ragged shapes (single rows, k = 1 and k = all, empty segments), each buffer allocated
 * at its exact size so that any access past an end is caught.  Prints "ok". */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_active_gather(const uint16_t *W_lm, int V, int d, const int32_t *src_ids, const int32_t *slots, int n,
                         uint16_t *W_act, int32_t *act_ids, int V_act);
void oracle_logits(const uint16_t *h, int M, int d, const uint16_t *W, int Vn, double *z);
void oracle_logz(const double *z, int M, int Vn, double *logz);
int oracle_topk(const double *z, const int32_t *ids, int M, int Vn, int kk, double *vals, int32_t *out_ids);
int oracle_active_lmhead_topk(const uint16_t *h, int M, int d, const uint16_t *W_act, const int32_t *ids, int V_act, int kk,
                              double *vals, int32_t *out_ids, double *logz, double *z_out);
int oracle_active_lmhead_topk_segmented(const uint16_t *h, int M, int d, const uint16_t *W_core, const int32_t *ids_core,
                                        int V_core, const uint16_t *W_arc, const int32_t *ids_arc, int V_arc,
                                        const int32_t *row_off, int S, int kk, double *vals, int32_t *out_ids, double *logz);

static uint64_t g_state = 12345;
static uint32_t rnd(void) { g_state = g_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(g_state >> 33); }
/* a finite bf16 pattern of moderate size */
static uint16_t bf16(void) { return (uint16_t)(((rnd() & 1u) << 15) | ((120u + rnd() % 8u) << 7) | (rnd() & 127u)); }
static void *xmalloc(size_t n) { void *p = malloc(n ? n : 1); if (!p) { puts("out of memory"); exit(2); } return p; }
#define REQUIRE(c, msg) do { if (!(c)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, msg); return 1; } } while (0)

static int one_shape(int V, int d, int V_act, int M, int kk, int S) {
    uint16_t *W = xmalloc((size_t)V * d * 2), *h = xmalloc((size_t)M * d * 2), *Wa = xmalloc((size_t)V_act * d * 2);
    int32_t *ids = xmalloc((size_t)V_act * 4), *act = xmalloc((size_t)V_act * 4);
    for (size_t i = 0; i < (size_t)V * d; ++i) W[i] = bf16();
    for (size_t i = 0; i < (size_t)M * d; ++i) h[i] = bf16();
    for (int i = 0; i < V_act; ++i) ids[i] = (int32_t)(((int64_t)i * V) / V_act);       /* distinct, increasing */
    REQUIRE(oracle_active_gather(W, V, d, ids, NULL, V_act, Wa, act, V_act) == 0, "gather");
    int32_t bad_id = V, slot0 = 0;
    REQUIRE(oracle_active_gather(W, V, d, &bad_id, &slot0, 1, Wa, act, V_act) != 0, "gather accepts an id past V");
    double *z = xmalloc((size_t)M * V_act * 8), *lz = xmalloc((size_t)M * 8), *vals = xmalloc((size_t)M * kk * 8);
    int32_t *oi = xmalloc((size_t)M * kk * 4);
    oracle_logits(h, M, d, Wa, V_act, z);
    oracle_logz(z, M, V_act, lz);
    REQUIRE(oracle_topk(z, act, M, V_act, kk, vals, oi) == 0, "topk");
    REQUIRE(oracle_active_lmhead_topk(h, M, d, Wa, act, V_act, kk, vals, oi, lz, NULL) == 0, "head");
    REQUIRE(oracle_active_lmhead_topk(h, M, d, Wa, act, V_act, kk, vals, oi, lz, z) == 0, "head with logits out");
    for (int m = 0; m < M; ++m)
        for (int j = 1; j < kk; ++j) REQUIRE(vals[(size_t)m * kk + j - 1] >= vals[(size_t)m * kk + j], "descending");
    /* segmented: the first V_core rows as the shared core, the rest cut into S equal extensions;
       ragged row ranges with an empty first segment */
    const int V_arc = S > 0 ? (V_act / 2) / S : 0, V_core = V_act - V_arc * S;
    if (S > 0 && V_arc > 0 && kk <= V_core + V_arc) {
        int32_t *ro = xmalloc((size_t)(S + 1) * 4);
        ro[0] = 0; ro[1] = 0;
        for (int s = 2; s <= S; ++s) ro[s] = (int32_t)(((int64_t)(s - 1) * M) / (S - 1 > 0 ? S - 1 : 1));
        ro[S] = M;
        REQUIRE(oracle_active_lmhead_topk_segmented(h, M, d, Wa, act, V_core, Wa + (size_t)V_core * d, act + V_core, V_arc,
                                                    ro, S, kk, vals, oi, lz) == 0, "segmented");
        free(ro);
    }
    free(W); free(h); free(Wa); free(ids); free(act); free(z); free(lz); free(vals); free(oi);
    return 0;
}

int main(void) {
    const int shapes[][6] = {
        /* V, d, V_act, M, k, S */
        {64, 8, 64, 1, 1, 0}, {64, 8, 1, 3, 1, 0}, {257, 24, 100, 5, 100, 4}, {1000, 72, 333, 7, 10, 3},
        {513, 264, 129, 2, 64, 2}, {96, 16, 96, 9, 96, 1},
    };
    for (size_t i = 0; i < sizeof shapes / sizeof shapes[0]; ++i)
        if (one_shape(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4], shapes[i][5])) return 1;
    puts("ok");
    return 0;
}
