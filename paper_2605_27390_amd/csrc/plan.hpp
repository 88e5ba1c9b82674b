// Host-side launch planning for the active-vocabulary LM head (no HIP calls here).
//
// The restricted projection of Eq. 1 (EvoSpec paper) streams W_act once.  Rows of
// W_act are cut into slabs of RT = 16 * NW * RGW rows; one workgroup of NW wavefronts
// handles one slab and leaves, per draft row, a partial (max, sum-exp, k best keys)
// in the workspace.  This header decides the slab shape for a problem size and lays
// out the workspace; both halves of the head (partials, merge) derive the same plan
// from the same arguments.
#pragma once
#include <cstddef>
#include <cstdint>

namespace evospec {

constexpr int kMTile = 64;          // draft rows per pass over W_act
constexpr int kKMax = 64;           // largest supported k
constexpr int kKC = 256;            // hidden-dimension chunk staged in LDS per step
constexpr int kHStride = kKC + 8;   // LDS row stride of the h chunk (bf16 elements, +16 B pad)
constexpr int kRowsMinSlab = 64;    // smallest slab any plan uses (workspace upper bound)
constexpr int kLdsLimit = 160 * 1024;

struct SlabShape { int nw; int rgw; };
// Slab shapes that have a compiled kernel.  RT = 16 * nw * rgw.
constexpr SlabShape kShapes[] = {{4, 1}, {5, 1}, {6, 1}, {7, 1}, {8, 1}, {9, 1}, {10, 1}, {12, 1}, {8, 2}};
constexpr int kNumShapes = sizeof(kShapes) / sizeof(kShapes[0]);

struct Plan {
    int nw = 0, rgw = 0;     // wavefronts per workgroup, 16-row groups per wavefront
    int mb = 0;              // 16-row blocks of draft rows held in accumulators (1, 2 or 4)
    int rt = 0;              // slab rows
    int n_slabs = 0;
    int groups = 0;          // selection groups per draft row in the slab epilogue (>= k)
    size_t lds_bytes = 0;
    // workspace layout (bytes from the workspace base), for one pass of <= 64 draft rows
    size_t keys_off = 0, stats_off = 0, total_bytes = 0;
};

constexpr size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline int mb_for_rows(int rows) { return rows <= 16 ? 1 : (rows <= 32 ? 2 : 4); }

inline int groups_for(int rows, int k, int nthreads, int rt) {
    // number of (row, group) pairs ~ a whole number of thread rounds; at least k groups so
    // that the k-th largest group maximum bounds the slab's k-th best from below
    int rounds = (k * rows + nthreads - 1) / nthreads;
    int g = rounds * nthreads / rows;
    int cap = k > 32 ? k : 32;
    if (g > cap) g = cap;
    if (g > rt / 2) g = rt / 2;
    if (g < k) g = k;
    return g;
}

inline size_t lds_bytes_for(int nw, int rgw, int mb, int groups) {
    const int rt = 16 * nw * rgw;
    const int mrows = 16 * mb;
    size_t hs = 2ull * mrows * kHStride * 2;                               // h chunk, double buffered
    size_t sel = align_up((size_t)mrows * rt * 2, 16)                      // survivor indices (u16)
               + (size_t)mrows * groups * 8                                // group maxima (keys)
               + (size_t)mrows * groups * 4;                               // group sum-exp
    size_t u = hs > sel ? hs : sel;                                        // the two never live together
    size_t zk = (size_t)mrows * (rt + 2) * 8;                              // slab logits as sortable keys
    size_t small = align_up((size_t)rt * 4, 16) + (size_t)mrows * 4 * 4;   // ids, counters, tau, vmax
    return align_up(u, 16) + align_up(zk, 16) + small;
}

// Slab shape for V_act rows on a device with `num_cu` compute units: fewest row-rounds
// (ceil(slabs / CUs) * RT); ties go to the larger slab (fewer partials to merge).
inline Plan make_plan(int rows /*draft rows in this pass, 1..64*/, int V_act, int k, int num_cu) {
    Plan best;
    long best_cost = -1;
    const int mb = mb_for_rows(rows);
    for (int i = 0; i < kNumShapes; ++i) {
        const int nw = kShapes[i].nw, rgw = kShapes[i].rgw;
        const int rt = 16 * nw * rgw;
        const int n_slabs = (V_act + rt - 1) / rt;
        const int g = groups_for(rows, k, nw * 64, rt);
        const size_t lds = lds_bytes_for(nw, rgw, mb, g);
        if (lds > (size_t)kLdsLimit) continue;
        const long rounds = (n_slabs + num_cu - 1) / num_cu;
        const long cost = rounds * rt;
        if (best_cost < 0 || cost < best_cost || (cost == best_cost && rt > best.rt)) {
            best_cost = cost;
            best.nw = nw; best.rgw = rgw; best.mb = mb; best.rt = rt; best.n_slabs = n_slabs;
            best.groups = g; best.lds_bytes = lds;
        }
    }
    best.keys_off = 0;
    best.stats_off = align_up((size_t)best.n_slabs * kMTile * k * 8, 256);
    best.total_bytes = best.stats_off + align_up((size_t)best.n_slabs * kMTile * 8, 256);
    return best;
}

// Upper bound of Plan::total_bytes over every slab shape (independent of the device).
inline size_t workspace_upper_bound(int V_act, int k) {
    const size_t n_slabs = ((size_t)V_act + kRowsMinSlab - 1) / kRowsMinSlab;
    return align_up(n_slabs * kMTile * k * 8, 256) + align_up(n_slabs * kMTile * 8, 256);
}

}  // namespace evospec
