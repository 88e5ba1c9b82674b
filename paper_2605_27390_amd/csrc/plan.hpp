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
constexpr int kRoundRows = 37;      // fixed cost of a round of workgroups, in slab rows (see make_plan)

// Slab shapes that have a compiled kernel: X(nw, rgw, rc) with nw wavefronts per workgroup, rgw
// 16-row groups per wavefront (RT = 16 * nw * rgw rows per slab) and a W-operand ring of rc chunks
// of kKC hidden elements per lane.  (Measured on MI355X: more waves per CU beat a deeper ring per wave.)
#define EVOSPEC_SLAB_SHAPES(X) \
    X(4, 1, 2) X(5, 1, 2) X(6, 1, 2) X(7, 1, 2) X(8, 1, 2) X(9, 1, 2) X(10, 1, 2) X(12, 1, 2)
struct SlabShape { int nw; int rgw; int rc; };
#define EVOSPEC_SHAPE_ENTRY(NW_, RGW_, RC_) {NW_, RGW_, RC_},
constexpr SlabShape kShapes[] = {EVOSPEC_SLAB_SHAPES(EVOSPEC_SHAPE_ENTRY)};
#undef EVOSPEC_SHAPE_ENTRY
constexpr int kNumShapes = sizeof(kShapes) / sizeof(kShapes[0]);
constexpr bool shapes_respect_min_slab() {
    for (int i = 0; i < kNumShapes; ++i)
        if (16 * kShapes[i].nw * kShapes[i].rgw < kRowsMinSlab) return false;
    return true;
}
static_assert(shapes_respect_min_slab(), "workspace_upper_bound assumes no slab below kRowsMinSlab rows");

// A batch of independent problems handled by one launch (grid.y): chunk i is the draft rows
// [m0, m0 + rows) of h against the rows of sequence `seq` of a per-sequence matrix.  For the
// merge, a_pass / a_slot locate the chunk's rows inside the first partial set.
constexpr int kMaxChunks = 64;
struct ChunkBatch {
    int n = 0;
    int m0[kMaxChunks];
    int rows[kMaxChunks];
    int seq[kMaxChunks];
    int a_pass[kMaxChunks];
    int a_slot[kMaxChunks];
};

constexpr size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Operand-tile ("packed") layout of a compact matrix.  The slab kernel hands a wavefront 16 rows and
// feeds them to the matrix cores 32 hidden elements at a time: lane l = 16 g + n supplies the 16
// bytes (row n, elements 32 s + 8 g .. + 8) of k-step s.  The packed layout stores exactly these
// 1 KB operand blocks back to back:
//   piece (row r, 16-byte piece c = element / 8)  ->  piece index
//   (r / 16) * (16 * dp / 8) + (c / 4) * 64 + (c % 4) * 16 + (r % 16),   dp = d rounded up to kKC,
// pieces past d hold zeros, rows are padded to a multiple of 16.  A wavefront then streams one
// contiguous 16 * dp * 2 byte run with fully coalesced 1 KB loads (measured on MI355X: 61 us against
// 71 us for the same head on a row-major matrix, whose wave-loads touch 16 rows x 64 bytes).
constexpr int kPackRows = 16;
constexpr int packed_d(int d) { return (d + kKC - 1) / kKC * kKC; }
constexpr size_t packed_rows(size_t rows) { return align_up(rows, (size_t)kPackRows); }
inline size_t matrix_elems(size_t rows, int d, bool packed) {
    return packed ? packed_rows(rows) * (size_t)packed_d(d) : rows * (size_t)d;
}

// One dynamic-buffer update: n rows W_act[slots[i]] <- W_lm[src_ids[i]], act_ids[slots[i]] <- src_ids[i]
// (slots == nullptr: slot i).  Device pointers; row_vec = d / 8.  packed: layout of W_act (W_lm is
// always row-major).
struct GatherArgs {
    const void* W_lm = nullptr;
    int V = 0, row_vec = 0;
    const int32_t* src_ids = nullptr;
    const int32_t* slots = nullptr;
    int n = 0;
    void* W_act = nullptr;
    int32_t* act_ids = nullptr;
    int V_act = 0;
    int packed = 0;
};

// Rows of a small update passed to the kernel by value (see launch_gather_inline).
constexpr int kInlineRows = 32;
struct InlineRows {
    int32_t slot[kInlineRows];
    int32_t id[kInlineRows];
};

struct Plan {
    int nw = 0, rgw = 0;     // wavefronts per workgroup, 16-row groups per wavefront
    int rc = 0;              // chunks in the W-operand ring
    int mb = 0;              // 16-row blocks of draft rows held in accumulators (1, 2 or 4)
    int rt = 0;              // slab rows
    int n_slabs = 0;
    int gl = 0;              // selection group level of the slab epilogue (see group_level_for)
    size_t lds_bytes = 0;
    // workspace layout (bytes from the workspace base), for one pass of <= 64 draft rows
    size_t keys_off = 0, stats_off = 0, total_bytes = 0;
};

inline int mb_for_rows(int rows) { return rows <= 16 ? 1 : (rows <= 32 ? 2 : 4); }

// Granularity of the selection groups in the slab epilogue.  A slab's logits for one draft row
// sit 4*rgw per lane in 4*nw lanes; level 0 takes each lane as a group, level 1 pairs of lanes,
// level 2 whole wavefronts (nw groups).  The k-th largest group maximum is a lower bound of the
// slab's k-th best logit, so only entries at or above it need exact ranking.  Coarser groups cost
// less to rank and filter almost as well: take the coarsest level with at least 1.5 k groups.
inline int group_level_for(int k, int nw) {
    const int want = k + k / 2;
    if (nw >= want) return 2;
    if (2 * nw >= want) return 1;
    return 0;
}

// Row stride, in keys, of the candidate lists of the slab epilogue: two keys of padding make the rows
// start 16 bytes apart modulo the 64 LDS banks, so that accesses of the draft rows of a wavefront to
// the same list position spread over all banks (a stride of rt keys maps every row to two banks).
constexpr int list_stride(int rt) { return rt + 2; }

inline size_t lds_bytes_for(int nw, int rgw, int mb) {
    const int rt = 16 * nw * rgw;
    const int mrows = 16 * mb;
    size_t hs = 2ull * mrows * kHStride * 2;                 // h chunk, double buffered
    size_t list = (size_t)mrows * list_stride(rt) * 8;       // surviving keys per draft row
    size_t u = hs > list ? hs : list;                        // the two never live together
    size_t gm = (size_t)mrows * 4 * nw * 4;                  // group maxima
    size_t wsum = (size_t)nw * mrows * 4;                    // per-wave sum-exp
    size_t small = align_up((size_t)rt * 4, 16) + (size_t)mrows * 3 * 4;   // ids, tau, vmax, counters
    return align_up(u, 16) + gm + wsum + small;
}

// Slab shape for V_act rows of d elements on a device with `num_cu` compute units: the least
// ceil(slabs / CUs) * (RT + kRoundRows), a round of workgroups costing its rows plus a fixed part
// (first loads, epilogue: about what 37 rows of 8 KiB take to stream into one CU); ties go to the
// larger slab (fewer partials to merge).  A slab
// whose bytes are a multiple of 1 MiB is charged one eighth more: all workgroups then walk through
// memory at the same offset within a MiB and meet at the same memory channels (measured on MI355X
// at 32,256 x 4,096: 8 wavefronts = 1 MiB slabs 59 us, 9 wavefronts on fewer CUs 56 us).
inline Plan make_plan(int rows /*draft rows in this pass, 1..64*/, int V_act, int d, int k, int num_cu,
                      int replicas = 1 /*chunks that share the launch*/) {
    Plan best;
    long best_cost = -1;
    const int mb = mb_for_rows(rows);
    for (int i = 0; i < kNumShapes; ++i) {
        const int nw = kShapes[i].nw, rgw = kShapes[i].rgw;
        const int rt = 16 * nw * rgw;
        const int n_slabs = (V_act + rt - 1) / rt;
        const size_t lds = lds_bytes_for(nw, rgw, mb);
        if (lds > (size_t)kLdsLimit) continue;
        const long rounds = ((long)n_slabs * replicas + num_cu - 1) / num_cu;
        long cost = rounds * (rt + kRoundRows) * 8;
        if (((size_t)rt * (size_t)d * 2) % ((size_t)1 << 20) == 0) cost += cost / 8;
        if (best_cost < 0 || cost < best_cost || (cost == best_cost && rt > best.rt)) {
            best_cost = cost;
            best.nw = nw; best.rgw = rgw; best.rc = kShapes[i].rc; best.mb = mb; best.rt = rt; best.n_slabs = n_slabs;
            best.gl = group_level_for(k, nw); best.lds_bytes = lds;
        }
    }
    best.keys_off = 0;
    best.stats_off = align_up((size_t)best.n_slabs * kMTile * k * 8, 256);
    best.total_bytes = best.stats_off + align_up((size_t)best.n_slabs * kMTile * 8, 256);
    return best;
}

// Large-M path: 256 x 256 tiles, one partial per 128 active rows and draft row, all M rows in
// one launch.  Taken from kGemmMinRows draft rows on, where the contraction, not the stream of
// W_act, bounds the head.
constexpr int kGemmTile = 256;
constexpr int kGemmSlab = 128;
constexpr int kGemmMinRows = 129;
constexpr int kGemmKChunk = 32;       // hidden elements per MFMA step; the large-M kernel loads two chunks at
                                      // a time and needs d to be a multiple of 64
inline bool use_gemm(int M, int d) { return M >= kGemmMinRows && d % (2 * kGemmKChunk) == 0; }

// Key slots per (slab, draft row) list of the large-M path: the kernel leaves every logit that
// reaches a lower bound of the slab's k-th best, unranked; rarely more than k + a few.
inline int gemm_list_len(int k) { return k <= 16 ? 16 : (k <= 32 ? 32 : 64); }

struct GemmPlan {
    int n_slabs = 0;
    int list_len = 0;
    size_t keys_off = 0, stats_off = 0, total_bytes = 0;
};
inline GemmPlan make_gemm_plan(int M, int V_act, int k) {
    GemmPlan g;
    g.n_slabs = (V_act + kGemmSlab - 1) / kGemmSlab;
    g.list_len = gemm_list_len(k);
    g.stats_off = align_up((size_t)g.n_slabs * M * g.list_len * 8, 256);
    g.total_bytes = g.stats_off + align_up((size_t)g.n_slabs * M * 8, 256);
    return g;
}

// Upper bound of Plan::total_bytes over every slab shape (independent of the device).
inline size_t workspace_upper_bound(int V_act, int k) {
    const size_t n_slabs = ((size_t)V_act + kRowsMinSlab - 1) / kRowsMinSlab;
    return align_up(n_slabs * kMTile * k * 8, 256) + align_up(n_slabs * kMTile * 8, 256);
}

}  // namespace evospec
