// HIP kernels (gfx950 / CDNA4) for the active-vocabulary LM head of the EvoSpec paper:
// Eq. 1 (Softmax(h W_LM^T)) evaluated on the active set V_t of Eq. 3 / Algorithm 1, with the
// log-normaliser and the top-k of the draft phase fused in, plus the row insertion that
// keeps the compact matrix W_act in step with the dynamic buffer.
//
// Wavefronts are 64 wide.  The contraction uses v_mfma_f32_16x16x32_bf16 (bf16 in, fp32
// accumulate): the A operand is a 16-row group of W_act, the B operand 16 draft rows of h,
// so an accumulator register holds z[vocab row 4*(lane/16)+j][draft row lane%16].
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include <type_traits>

#include "common.hpp"
#include "plan.hpp"

namespace evospec {

// ---------------------------------------------------------------------------------------
// Row insertion  W_act[slot] <- W_lm[id], act_ids[slot] <- id  (bit copy, 16 B per lane).
// One workgroup per row.  Into a packed W_act the row's pieces go to their places in the operand
// tiles (16-byte stores 256 bytes apart) and the pieces between d and the padded row length are
// zeroed.
__device__ __forceinline__ void gather_row(const GatherArgs& g, int32_t id, int32_t s) {
    if (id < 0 || id >= g.V || s < 0 || s >= g.V_act) return;      // uniform per workgroup
    const uint4* src = static_cast<const uint4*>(g.W_lm) + (size_t)id * g.row_vec;
    const int nt = blockDim.x;
    if (g.packed) {
        const int dp_vec = packed_d(g.row_vec * 8) / 8;
        uint4* dst = static_cast<uint4*>(g.W_act) + (size_t)(s >> 4) * (kPackRows * (size_t)dp_vec) + (s & 15);
        for (int c0 = 0; c0 < dp_vec; c0 += 4 * nt) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * nt + threadIdx.x;
                v[u] = make_uint4(0u, 0u, 0u, 0u);
                if (c < g.row_vec) v[u] = src[c];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * nt + threadIdx.x;
                if (c < dp_vec) dst[(c >> 2) * 64 + (c & 3) * 16] = v[u];
            }
        }
    } else {
        uint4* dst = static_cast<uint4*>(g.W_act) + (size_t)s * g.row_vec;
        for (int c0 = 0; c0 < g.row_vec; c0 += 4 * nt) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * nt + threadIdx.x;
                if (c < g.row_vec) v[u] = src[c];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * nt + threadIdx.x;
                if (c < g.row_vec) dst[c] = v[u];
            }
        }
    }
    if (threadIdx.x == 0) g.act_ids[s] = id;
}
__device__ __forceinline__ void gather_one_row(const GatherArgs& g, int i) {
    gather_row(g, g.src_ids[i], g.slots ? g.slots[i] : i);
}

// grid-stride over the n rows of the update
__global__ void __launch_bounds__(256)
gather_rows_kernel(GatherArgs g) {
    for (int i = blockIdx.x; i < g.n; i += gridDim.x) gather_one_row(g, i);
}

// A small update whose (slot, id) pairs travel in the kernel arguments: a caller that has them on
// the host (the failure event of Path A) needs no upload and no wait for one.
__global__ void __launch_bounds__(256)
gather_rows_inline_kernel(GatherArgs g, InlineRows r) {
    gather_row(g, r.id[blockIdx.x], r.slot[blockIdx.x]);
}

// Rebuild of a row-major W_act (slot i = i): four rows per workgroup and round, so that every lane has
// eight 16-byte loads in flight, and stores that bypass the cache (the rows are not read again soon;
// measured on MI355X for 36,864 rows of 8 KB: 95 us against 119 us with one row per round and cached
// stores).
__global__ void __launch_bounds__(256)
gather_rebuild_rows_kernel(GatherArgs g) {
    constexpr int RPB = 4;
    for (int i0 = blockIdx.x * RPB; i0 < g.n; i0 += gridDim.x * RPB) {
        const uint4* src[RPB];
        bool ok[RPB];
#pragma unroll
        for (int r = 0; r < RPB; ++r) {
            const int i = i0 + r;
            const int32_t id = i < g.n ? g.src_ids[i] : -1;
            ok[r] = id >= 0 && id < g.V && i < g.V_act;                   // uniform per workgroup
            src[r] = static_cast<const uint4*>(g.W_lm) + (size_t)(ok[r] ? id : 0) * g.row_vec;
            if (ok[r] && threadIdx.x == 0) g.act_ids[i] = id;
        }
        for (int c0 = 0; c0 < g.row_vec; c0 += 512) {
            u32x4 v[RPB][2];
#pragma unroll
            for (int r = 0; r < RPB; ++r)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int c = c0 + u * 256 + threadIdx.x;
                    if (ok[r] && c < g.row_vec) v[r][u] = *(gvec_ptr)(src[r] + c);
                }
#pragma unroll
            for (int r = 0; r < RPB; ++r)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int c = c0 + u * 256 + threadIdx.x;
                    if (ok[r] && c < g.row_vec)
                        __builtin_nontemporal_store(v[r][u], reinterpret_cast<u32x4*>(g.W_act) + (size_t)(i0 + r) * g.row_vec + c);
                }
        }
    }
}

// Rebuild of a packed W_act (slot i = i): one workgroup per tile of 16 slots, whole 128-byte lines on
// both sides.  Lane 8 r + p of a wavefront reads piece 8 q + p of row r (rows 0..7 of the tile in one
// load, rows 8..15 in a second one): 8 rows x 128 bytes per load.  Piece (row, c) belongs to operand
// block c / 4 at slot (c % 4) * 16 + row, so the eight lanes that hold the same piece of rows 0..7
// write 128 contiguous bytes.  The stores bypass the cache.  (Measured for 36,864 rows of 8 KB: 99 us
// against 129 us for half-line loads with cached stores.)
__global__ void __launch_bounds__(256)
gather_tiles_kernel(GatherArgs g) {
    constexpr int UNR = 4;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r8 = lane >> 3, p = lane & 7;
    const int dp_vec = packed_d(g.row_vec * 8) / 8;
    const int npairs = dp_vec / 8;                       // line pairs per row (dp_vec is a multiple of 32)
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    for (int t = blockIdx.x; t * kPackRows < g.n; t += gridDim.x) {
        const int ia = t * kPackRows + r8, ib = ia + 8;
        const int32_t ida = ia < g.n ? g.src_ids[ia] : -1, idb = ib < g.n ? g.src_ids[ib] : -1;
        const bool oka = ida >= 0 && ida < g.V && ia < g.V_act, okb = idb >= 0 && idb < g.V && ib < g.V_act;
        const uint4* sa = static_cast<const uint4*>(g.W_lm) + (size_t)(oka ? ida : 0) * g.row_vec;
        const uint4* sb = static_cast<const uint4*>(g.W_lm) + (size_t)(okb ? idb : 0) * g.row_vec;
        u32x4* d = reinterpret_cast<u32x4*>(g.W_act) + (size_t)t * (kPackRows * (size_t)dp_vec) + (p >> 2) * 64 + (p & 3) * 16 + r8;
        for (int q0 = w; q0 < npairs; q0 += 4 * UNR) {
            u32x4 va[UNR], vb[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int c = 8 * (q0 + 4 * u) + p;      // pieces past the row's end are zero padding
                va[u] = zero4; vb[u] = zero4;
                if (oka && c < g.row_vec) va[u] = *(gvec_ptr)(sa + c);
                if (okb && c < g.row_vec) vb[u] = *(gvec_ptr)(sb + c);
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int q = q0 + 4 * u;
                if (q < npairs) {
                    if (oka) __builtin_nontemporal_store(va[u], d + (size_t)q * 128);
                    if (okb) __builtin_nontemporal_store(vb[u], d + (size_t)q * 128 + 8);
                }
            }
        }
        if (w == 0 && p == 0) {
            if (oka) g.act_ids[ia] = ida;
            if (okb) g.act_ids[ib] = idb;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Debug check of an id list: range and uniqueness (Eq. 3 is a set union).  O(n^2 / tile).
__device__ int g_validate_flag;

__global__ void __launch_bounds__(256)
validate_ids_kernel(const int32_t* __restrict__ ids, int n, int V, int* flag) {
    __shared__ int32_t tile[1024];
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int32_t mine = i < n ? ids[i] : -1;
    bool bad = i < n && (mine < 0 || mine >= V);
    for (int t0 = 0; t0 < n; t0 += 1024) {
        __syncthreads();
        for (int u = threadIdx.x; u < 1024; u += 256) tile[u] = (t0 + u < n) ? ids[t0 + u] : -2;
        __syncthreads();
        if (i < n) {
            for (int u = 0; u < 1024; ++u)
                if (tile[u] == mine && t0 + u != i) bad = true;
        }
    }
    if (bad) atomicOr(flag, 1);
}

// ---------------------------------------------------------------------------------------
// Pass 1 of the restricted head: one workgroup streams one slab of RT = 16*NW*RGW rows of
// W_act (each wave its own 16*RGW rows, loaded from HBM straight into MFMA operand layout
// with 128-bit loads), contracts it with up to 16*MB draft rows of h (K-chunks of h staged
// in LDS, double buffered, shared by all waves), and reduces the slab's logits, which stay in
// the accumulators, to
//   part_stats[slab][m] = (max_i z, sum_i exp(z - max))         over the slab's rows
//   part_keys[slab][m][0..k) = the slab's k best keys, descending (0 = none)
// Logits never leave the CU.
template <int NW, int RGW, int RC, int MB, bool FULLK, bool PACKED>
__global__ void __launch_bounds__(NW * 64)
lmhead_partials_kernel(const uint16_t* __restrict__ h_all, ChunkBatch cb, int seq_rows,
                       size_t chunk_keys, size_t chunk_stats, int d,
                       const uint16_t* __restrict__ W_all, const int32_t* __restrict__ ids_all,
                       int V_act, int k, int GL,
                       u64* __restrict__ keys_all, float2* __restrict__ stats_all) {
    // this workgroup's problem: chunk blockIdx.y of the batch (its draft rows, its sequence's
    // rows of a per-sequence matrix, its own piece of the partials)
    const int ci = blockIdx.y;
    const int rows = cb.rows[ci];
    const size_t seq_row0 = (size_t)cb.seq[ci] * seq_rows;
    const uint16_t* __restrict__ h = h_all + (size_t)cb.m0[ci] * d;
    // (a packed matrix pads every sequence's rows to whole tiles and its rows to whole chunks)
    const int dp = packed_d(d);
    const uint16_t* __restrict__ W = PACKED ? W_all + (size_t)cb.seq[ci] * packed_rows(seq_rows) * dp
                                            : W_all + seq_row0 * d;
    const int32_t* __restrict__ ids = ids_all ? ids_all + seq_row0 : nullptr;
    u64* __restrict__ part_keys = keys_all + (size_t)ci * chunk_keys;
    float2* __restrict__ part_stats = stats_all + (size_t)ci * chunk_stats;
    constexpr int NT = NW * 64;
    constexpr int RT = 16 * NW * RGW;
    constexpr int MR = 16 * MB;
    constexpr int KC = kKC;
    constexpr int KSTEPS = KC / 32;
    constexpr int HPIECES = MR * (KC / 8);
    constexpr int HP = (HPIECES + NT - 1) / NT;

    extern __shared__ __align__(16) unsigned char smem[];
    // region U: h chunks during the contraction, the survivors' keys afterwards
    uint16_t* Hs = reinterpret_cast<uint16_t*>(smem);
    u64* list = reinterpret_cast<u64*>(smem);                                 // [MR][LS]
    constexpr int LS = list_stride(RT);
    constexpr size_t hs_bytes = 2ull * MR * kHStride * 2;
    constexpr size_t list_bytes = (size_t)MR * list_stride(RT) * 8;
    constexpr size_t u_bytes = align_up(hs_bytes > list_bytes ? hs_bytes : list_bytes, 16);
    constexpr int NGS = 4 * NW;                                               // row stride of gm
    float* gm = reinterpret_cast<float*>(smem + u_bytes);                     // [MR][NGS] group maxima
    float* wsum = gm + (size_t)MR * NGS;                                      // [NW][MR] per-wave sum-exp
    int32_t* Ids = reinterpret_cast<int32_t*>(wsum + (size_t)NW * MR);        // [RT]
    float* tau = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(Ids) + align_up((size_t)RT * 4, 16));  // [MR]
    float* vmax = tau + MR;                                                   // [MR]
    int* cnt = reinterpret_cast<int*>(vmax + MR);                             // [MR]

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int row0 = blockIdx.x * RT;
    const int n_valid = min(RT, V_act - row0);

    // full-vocabulary id of slab row `tid` (RT <= NT): loaded first, parked in LDS once the operand
    // loads of the first chunks have been issued
    static_assert(RT <= NT, "one slab row per thread");
    int id_reg = 0x7fffffff;
    if (tid < RT && row0 + tid < V_act) id_reg = ids ? ids[row0 + tid] : row0 + tid;

    const uint16_t* wp[RGW];
#pragma unroll
    for (int rg = 0; rg < RGW; ++rg) {
        if constexpr (PACKED) {
            // the wavefront's tile: 1 KB operand blocks in k-step order, lane l at byte 16 l
            const int tile = min((row0 >> 4) + w * RGW + rg, (V_act - 1) >> 4);   // tail slab: a valid tile, masked later
            wp[rg] = W + (size_t)tile * kPackRows * dp + lane * 8;
        } else {
            int r = row0 + (w * RGW + rg) * 16 + n16;
            r = min(r, V_act - 1);                         // tail slab: duplicate a valid row, masked later
            wp[rg] = W + (size_t)r * d + g * 8;
        }
    }

    f32x4 acc[RGW][MB];
#pragma unroll
    for (int rg = 0; rg < RGW; ++rg)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[rg][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nchunks = (d + KC - 1) / KC;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    u32x4 hreg[HP];
    u32x4 wr[RGW][RC * KSTEPS];           // ring of W operands: k-steps of RC consecutive chunks

    // this thread's pieces (16 B each) of an h chunk: global source, LDS destination
    gvec_ptr hsrc[HP];
    int hdst[HP], hcol[HP];
#pragma unroll
    for (int p = 0; p < HP; ++p) {
        // threads beyond the last piece wrap around and re-stage an earlier piece (same bytes to
        // the same place), which keeps every load and LDS store unconditional
        const int idc = (tid + p * NT) % HPIECES;
        const int m = idc / (KC / 8), c8 = idc % (KC / 8);
        hcol[p] = c8 * 8;
        hsrc[p] = (gvec_ptr)(h + (size_t)min(m, rows - 1) * d + c8 * 8);
        hdst[p] = m * kHStride + c8 * 8;
    }
    gvec_ptr wsrc[RGW];
#pragma unroll
    for (int rg = 0; rg < RGW; ++rg) wsrc[rg] = (gvec_ptr)(wp[rg]);

    // Loads past the end of a row (only when d is not a multiple of KC) are redirected to the
    // row's last 16 bytes and replaced by zeros, so that no load is conditional.
    auto load_h = [&](int c) {
#pragma unroll
        for (int p = 0; p < HP; ++p) {
            if constexpr (FULLK) {
                hreg[p] = hsrc[p][c * (KC / 8)];
            } else {
                const int kk = c * KC + hcol[p];
                const bool in = kk < d;
                const u32x4 v = *(hsrc[p] + ((in ? kk : d - 8) - hcol[p]) / 8);
                hreg[p] = in ? v : zero4;
            }
        }
    };
    auto store_h = [&](int buf) {
#pragma unroll
        for (int p = 0; p < HP; ++p)
            *reinterpret_cast<u32x4*>(Hs + (size_t)buf * MR * kHStride + hdst[p]) = hreg[p];
    };
    // k-step s (0..7) of chunk c goes to ring slot (c % RC) * KSTEPS + s
    auto load_w_step = [&](int slot, int c, int s) {
        const int koff = c * KC + s * 32;
#pragma unroll
        for (int rg = 0; rg < RGW; ++rg) {
            if constexpr (PACKED) {
                wr[rg][slot] = wsrc[rg][(koff / 32) * 64];       // rows are padded to whole chunks
            } else if constexpr (FULLK) {
                wr[rg][slot] = wsrc[rg][koff / 8];
            } else {
                const bool in = koff + g * 8 < d;
                const u32x4 v = *(wsrc[rg] + ((in ? koff + g * 8 : d - 8) - g * 8) / 8);
                wr[rg][slot] = in ? v : zero4;
            }
        }
    };
    auto load_b = [&](bf16x8 (&b)[MB], int buf, int s) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            b[mb] = *reinterpret_cast<const bf16x8*>(Hs + ((size_t)buf * MR + mb * 16 + n16) * kHStride + s * 32 + g * 8);
    };
    auto mfma_step = [&](int slot, const bf16x8 (&b)[MB]) {
#pragma unroll
        for (int rg = 0; rg < RGW; ++rg) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, wr[rg][slot]);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                acc[rg][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b[mb], acc[rg][mb], 0, 0, 0);
        }
    };
    // One chunk (8 k-steps).  Ring part SLOT (= c % RC) holds this chunk's W operands, loaded RC
    // chunks ago; each slot is refilled with the same k-step of chunk c+RC right after the MFMAs
    // that consumed it were issued (packed matrix) or all slots at the end of the chunk (row-major
    // matrix), so up to RC*KSTEPS*RGW 16-byte loads per lane stay in flight.
    // The h chunk c+1 is fetched into registers meanwhile and published to the other LDS buffer
    // at the end.  In the steady state (chunks c+1 and c+RC exist) there is no branch in here;
    // the last chunks test for them at run time.
    auto chunk = [&](auto slot_c, int c, auto steady) {
        constexpr int SLOT = decltype(slot_c)::value;
        constexpr bool STEADY = decltype(steady)::value;
        const bool pw = STEADY || (c + RC < nchunks);
        const bool ph = STEADY || (c + 1 < nchunks);
        const int buf = c & 1;
        bf16x8 b0[MB], b1[MB];
        if (ph) load_h(c + 1);
        load_b(b0, buf, 0);
#pragma unroll
        for (int s = 0; s < KSTEPS; s += 2) {
            load_b(b1, buf, s + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(SLOT * KSTEPS + s, b0);
            if (PACKED && pw) load_w_step(SLOT * KSTEPS + s, c + RC, s);
            if (s + 2 < KSTEPS) load_b(b0, buf, s + 2);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(SLOT * KSTEPS + s + 1, b1);
            if (PACKED && pw) load_w_step(SLOT * KSTEPS + s + 1, c + RC, s + 1);
        }
        if (!PACKED && pw) {
            // row-major rows: the chunk's 8 requests go out together, so that the 512 bytes they
            // take from each row reach the memory side close in time (measured: 3.5 us of 73)
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) load_w_step(SLOT * KSTEPS + s, c + RC, s);
        }
        if (ph) store_h(buf ^ 1);
        lds_barrier();
    };
    // RC consecutive chunks starting at `base` (a multiple of RC), ring parts 0..RC-1
    auto chunk_group = [&](int base, auto steady) {
        constexpr bool STEADY = decltype(steady)::value;
#define EVOSPEC_CHUNK(I)                                                                   \
        if constexpr (I < RC) {                                                            \
            if (STEADY || base + I < nchunks) chunk(std::integral_constant<int, I>{}, base + I, steady); \
        }
        EVOSPEC_CHUNK(0) EVOSPEC_CHUNK(1) EVOSPEC_CHUNK(2) EVOSPEC_CHUNK(3)
#undef EVOSPEC_CHUNK
    };
    static_assert(RC >= 1 && RC <= 4, "ring depth");

    load_h(0);
#pragma unroll
    for (int i = 0; i < RC; ++i) {
        if (i < nchunks) {
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) load_w_step(i * KSTEPS + s, i, s);
        }
    }
    for (int i = tid; i < MR * NGS; i += NT) gm[i] = -INFINITY;      // padding of the group-maximum rows
    if (tid < RT) Ids[tid] = id_reg;
    store_h(0);
    lds_barrier();
    int c = 0;
    for (; c + 2 * RC <= nchunks; c += RC) chunk_group(c, std::true_type{});     // every prefetch target exists
    for (; c < nchunks; c += RC) chunk_group(c, std::false_type{});
    // every wave is past its last read of Hs (the loop ends on a barrier): region U is free

    // ---- slab epilogue.  The slab's logits stay in the accumulators: lane (n16, g) holds, for each
    // block mb of 16 draft rows, 4*RGW logits of draft row mb*16+n16 (slab rows 4g..4g+3 of each of
    // the wave's 16-row groups).
    if (n_valid < RT) {                                  // tail slab: rows past V_act never win
#pragma unroll
        for (int rg = 0; rg < RGW; ++rg)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((w * RGW + rg) * 16 + 4 * g + j >= n_valid) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) acc[rg][mb][j] = -INFINITY;
                }
    }
    // (1) group maxima (level GL: lane, lane pair or wave)
    const int NG = NW << (2 - GL);
    {
        const int gidx = GL == 0 ? w * 4 + g : (GL == 1 ? w * 2 + (g >> 1) : w);
        const bool owner = GL == 0 ? true : (GL == 1 ? (g & 1) == 0 : g == 0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float lm = -INFINITY;
#pragma unroll
            for (int rg = 0; rg < RGW; ++rg)
#pragma unroll
                for (int j = 0; j < 4; ++j) lm = fmaxf(lm, acc[rg][mb][j]);
            if (GL >= 1) lm = fmaxf(lm, __uint_as_float(xor_lane<16>(__float_as_uint(lm), lane)));
            if (GL >= 2) lm = fmaxf(lm, __uint_as_float(xor_lane<32>(__float_as_uint(lm), lane)));
            if (owner) gm[(mb * 16 + n16) * NGS + gidx] = lm;
        }
    }
    if (tid < MR) { cnt[tid] = 0; tau[tid] = -INFINITY; }
    __syncthreads();
    // (2) tau[m] = k-th largest group maximum (counting equal values): the group maxima are NG
    //     distinct slab entries, so at least k entries are >= tau and nothing below tau can be among
    //     the slab's k best.  (NG < k: tau stays -inf and everything is ranked.)  vmax[m] = slab
    //     maximum.  Rows of gm are padded with -inf to a multiple of 4 and read 16 bytes at a time.
    {
        const int ng4 = (NG + 3) >> 2;
        for (int p = tid; p < rows * NG; p += NT) {
            const int m = p / NG, j = p - m * NG;
            const float4* gr4 = reinterpret_cast<const float4*>(gm + m * NGS);
            const float mine = gm[m * NGS + j];
            int gt = 0, ge = 0;
            float top = -INFINITY;
            for (int i4 = 0; i4 < ng4; ++i4) {
                const float4 o = gr4[i4];
                gt += (o.x > mine) + (o.y > mine) + (o.z > mine) + (o.w > mine);
                ge += (o.x >= mine) + (o.y >= mine) + (o.z >= mine) + (o.w >= mine);
                top = fmaxf(fmaxf(top, fmaxf(o.x, o.y)), fmaxf(o.z, o.w));
            }
            if (gt < k && ge >= k) tau[m] = mine;            // equal maxima write the same value
            if (j == 0) vmax[m] = top;
        }
    }
    __syncthreads();
    // (3) sum of exponentials; entries >= tau become candidates (key = logit and full-vocabulary id).
    //     One LDS atomic per lane and draft-row block reserves room for the lane's candidates, which
    //     are then stored without branches or dependent loads.
    {
        int4 id4[RGW];
#pragma unroll
        for (int rg = 0; rg < RGW; ++rg) id4[rg] = *reinterpret_cast<const int4*>(Ids + (w * RGW + rg) * 16 + 4 * g);
        uint32_t pick[MB];
        int base[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = mb * 16 + n16;
            pick[mb] = 0;
            if (mb * 16 < rows) {                            // uniform: skip blocks of padding draft rows
                const bool live = m < rows;
                const float t = live ? tau[m] : INFINITY;
                const float vm = live ? vmax[m] : 0.f;
                float se = 0.f;
#pragma unroll
                for (int rg = 0; rg < RGW; ++rg)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float x = acc[rg][mb][j];
                        const int rl = (w * RGW + rg) * 16 + 4 * g + j;
                        se += __expf(x - vm);
                        pick[mb] |= (x >= t && rl < n_valid) ? 1u << (rg * 4 + j) : 0u;
                    }
                se += __uint_as_float(xor_lane<16>(__float_as_uint(se), lane));
                se += __uint_as_float(xor_lane<32>(__float_as_uint(se), lane));
                if (g == 0) wsum[w * MR + m] = se;
            }
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            base[mb] = pick[mb] ? atomicAdd(&cnt[mb * 16 + n16], __popc(pick[mb])) : 0;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            u64* dst = list + (size_t)(mb * 16 + n16) * LS + base[mb];
#pragma unroll
            for (int rg = 0; rg < RGW; ++rg) {
                const int idv[4] = {id4[rg].x, id4[rg].y, id4[rg].z, id4[rg].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = rg * 4 + j;
                    const u64 key = make_key(acc[rg][mb][j], idv[j]);
                    if (pick[mb] >> e & 1u) dst[__popc(pick[mb] & ((1u << e) - 1u))] = key;
                }
            }
        }
    }
    __syncthreads();
    // (4) exact order among the candidates of a draft row (NW threads per row); the k best go out.
    //     Keys are distinct because ids are, so a key's rank is the number of larger keys.
    if (tid < rows * NW) {
        const int m = tid / NW, sub = tid - m * NW;
        const int c = cnt[m];
        const u64* lst = list + (size_t)m * LS;
        u64* outk = part_keys + ((size_t)blockIdx.x * kMTile + m) * k;
        for (int q = sub; q < c; q += 2 * NW) {              // two candidates per pass share the reads of the list
            const bool two = q + NW < c;
            const u64 mine0 = lst[q], mine1 = two ? lst[q + NW] : ~0ull;
            int rank0 = 0, rank1 = 0;
            int j = 0;
            for (; j + 4 <= c; j += 4) {
                const ulonglong2 a = *reinterpret_cast<const ulonglong2*>(lst + j);
                const ulonglong2 b2 = *reinterpret_cast<const ulonglong2*>(lst + j + 2);
                rank0 += (a.x > mine0) + (a.y > mine0) + (b2.x > mine0) + (b2.y > mine0);
                rank1 += (a.x > mine1) + (a.y > mine1) + (b2.x > mine1) + (b2.y > mine1);
            }
            for (; j < c; ++j) { const u64 o = lst[j]; rank0 += o > mine0; rank1 += o > mine1; }
            if (rank0 < k) outk[rank0] = mine0;
            if (two && rank1 < k) outk[rank1] = mine1;
        }
        if (sub == 0) {
            for (int j = c; j < k; ++j) outk[j] = 0;               // slab holds fewer than k rows
            float sum = 0.f;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) sum += wsum[ww * MR + m];
            part_stats[(size_t)blockIdx.x * kMTile + m] = make_float2(vmax[m], sum);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Pass 2: one workgroup per draft row merges the slab partials:
//   logZ = M + log(sum_t s_t * exp(m_t - M)),  M = max_t m_t
//   top-k = the k largest of all slab candidates (keys are unique, so the order is total).
// Candidates come from up to two partial sets (a shared core and a per-sequence extension in the
// batched variant).  Every slab's list is sorted, so its head is its maximum: per block of 256
// lists the k-th largest head (together with the running result) bounds the answer from below,
// at most k lists reach above that bound, and only their entries are ranked exactly.

// An unranked list slot holds (logit bits << 32) | id; all ones = empty.
__device__ __forceinline__ u64 pair_key(uint32_t zbits, uint32_t id) {
    return id == 0xffffffffu ? 0ull : make_key(__uint_as_float(zbits), (int32_t)id);
}

template <int NT>
__global__ void __launch_bounds__(NT)
lmhead_merge_kernel(PartialSet A, PartialSet B, ChunkBatch cb, size_t a_pass_keys, size_t a_pass_stats,
                    size_t b_chunk_keys, size_t b_chunk_stats, int k, int pend_cap,
                    float* __restrict__ out_vals, int32_t* __restrict__ out_ids,
                    float* __restrict__ out_logz, GatherArgs upd) {
    // The blocks of grid row cb.n (present only when an update rides along) insert the rows of a
    // dynamic-buffer update into the compact matrix: the partials that this launch merges were
    // computed by an earlier launch, so nothing reads those rows any more.
    if ((int)blockIdx.y == cb.n) {
        if ((int)blockIdx.x < upd.n) gather_one_row(upd, blockIdx.x);
        return;
    }
    constexpr int NWV = NT / 64;
    __shared__ u64 run[2][kKMax];                    // running k best, descending
    __shared__ u64 cand[(NWV + 1) * kKMax];          // per-wave best heads, then the running list
    // entries that reach the bound: at most k lists of max_len entries, plus the running k
    // (dynamic LDS, sized by the launcher, so that small k leaves room for many workgroups per CU)
    extern __shared__ __align__(16) unsigned char merge_smem[];
    u64* pend = reinterpret_cast<u64*>(merge_smem);
    const int kPendCap = pend_cap;
    __shared__ const u64* qual[kKMax];             // lists whose head reaches the bound
    __shared__ int qual_len[kKMax];
    __shared__ u64 tau_s;
    __shared__ int npend, nqual;
    __shared__ float wave_m[NWV], wave_s[NWV];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // row blockIdx.x of chunk blockIdx.y: where its partials sit in the two sets
    const int chunk = blockIdx.y;
    if ((int)blockIdx.x >= cb.rows[chunk]) return;                 // uniform: the grid spans the longest chunk
    const int out_row = cb.m0[chunk] + blockIdx.x;
    A.keys += (size_t)cb.a_pass[chunk] * a_pass_keys;
    A.stats += (size_t)cb.a_pass[chunk] * a_pass_stats;
    B.keys += (size_t)chunk * b_chunk_keys;
    B.stats += (size_t)chunk * b_chunk_stats;
    const int slotA = A.row_base + cb.a_slot[chunk] + blockIdx.x, slotB = B.row_base + blockIdx.x;
    const int total = A.n_slabs + B.n_slabs;

    auto list_of = [&](int L) -> const u64* {
        return L < A.n_slabs ? A.keys + (size_t)L * A.key_slab + (size_t)slotA * A.key_row
                             : B.keys + (size_t)(L - A.n_slabs) * B.key_slab + (size_t)slotB * B.key_row;
    };
    auto len_of = [&](int L) { return L < A.n_slabs ? A.list_len : B.list_len; };
    auto sorted_of = [&](int L) { return (L < A.n_slabs ? A.sorted : B.sorted) != 0; };
    // a list's best key: its first slot if it is sorted, else the maximum over its slots (an even
    // number of (logit, id) pairs, 16-byte aligned)
    auto head_of = [&](int L) -> u64 {
        const u64* p = list_of(L);
        if (sorted_of(L)) return p[0];
        u64 hd = 0;
        const int n = len_of(L);
        for (int j0 = 0; j0 < n; j0 += 16) {            // 8 loads in flight (list lengths are 16, 32 or 64)
            u32x4 q[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) q[u] = *(gvec_ptr)(p + j0 + 2 * u);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const u64 k0 = pair_key(q[u][1], q[u][0]), k1 = pair_key(q[u][3], q[u][2]);
                hd = k0 > hd ? k0 : hd;
                hd = k1 > hd ? k1 : hd;
            }
        }
        return hd;
    };
    const int max_len = A.list_len > B.list_len ? A.list_len : B.list_len;
    // the first block's list heads are fetched together with the statistics (one memory round trip)
    const u64 head_first = tid < total ? head_of(tid) : 0;

    // ---- log-normaliser: online (max, scaled sum) per thread, fixed-shape reduction
    float mx = -INFINITY, sm = 0.f;
    for (int t = tid; t < total; t += NT) {
        const float2 st = t < A.n_slabs ? A.stats[(size_t)t * A.stat_slab + (size_t)slotA * A.stat_row]
                                        : B.stats[(size_t)(t - A.n_slabs) * B.stat_slab + (size_t)slotB * B.stat_row];
        const float nm = fmaxf(mx, st.x);
        sm = (mx == -INFINITY ? 0.f : sm * __expf(mx - nm)) + st.y * __expf(st.x - nm);
        mx = nm;
    }
    {   // wavefront: the maximum first, then one rescale per lane and a plain sum
        const float wm_ = wave_max(mx, lane);
        sm = mx == -INFINITY ? 0.f : sm * __expf(mx - wm_);
        sm = wave_sum(sm, lane);
        mx = wm_;
    }
    if (lane == 0) { wave_m[w] = mx; wave_s[w] = sm; }
    if (tid == 0) { npend = 0; nqual = 0; }
    __syncthreads();
    if (tid == 0) {
        float gm_ = wave_m[0], gs = wave_s[0];
        for (int i = 1; i < NWV; ++i) {
            const float nm = fmaxf(gm_, wave_m[i]);
            gs = (gm_ == -INFINITY ? 0.f : gs * __expf(gm_ - nm)) + (wave_m[i] == -INFINITY ? 0.f : wave_s[i] * __expf(wave_m[i] - nm));
            gm_ = nm;
        }
        out_logz[out_row] = gm_ + __logf(gs);
    }

    // ---- top-k
    int nrun = 0, cur = 0;
    u64 thr = 0;                                     // running k-th best (0 until k entries are known)
    for (int base = 0; base < total; base += NT) {
        const int L = base + tid;
        const u64* lst = L < total ? list_of(L) : nullptr;
        u64 head = base == 0 ? head_first : (lst ? head_of(L) : 0);
        if (head <= thr) head = 0;                   // cannot improve the running result
        // (1) the wave's 64 heads, sorted across the lanes; its k best go to cand
        {
            const u64 sorted = wave_sort_desc(head, lane);
            if (lane < k) cand[w * k + lane] = sorted;
        }
        if (tid < nrun) cand[NWV * k + tid] = run[cur][tid];
        __syncthreads();
        // (2) bound = k-th largest of (wave bests + running list): k real candidates are >= it
        const int ne = NWV * k + nrun;
        if (ne <= 64) {                                  // one more sort by the first wavefront
            if (w == 0) {
                const u64 c = wave_sort_desc(lane < ne ? cand[lane] : 0ull, lane);
                if (lane == k - 1) tau_s = c;
            }
        } else {
            for (int e = tid; e < ne; e += NT) {
                const u64 mine = cand[e];
                int r = 0;
                for (int j = 0; j < ne; ++j) { const u64 o = cand[j]; r += (o > mine) || (o == mine && j < e); }   // zeros tie: keep the index order
                if (r == k - 1) tau_s = mine;
            }
        }
        __syncthreads();
        // (3) lists (at most k of them) and running entries that reach the bound feed pend; the
        //     qualifying lists are read by all threads at once (one entry per thread and round)
        const u64 t = tau_s;
        // (capacity checks only matter if the caller broke the unique-id precondition)
        if (head != 0 && head >= t) { const int qi = atomicAdd(&nqual, 1); if (qi < kKMax) { qual[qi] = lst; qual_len[qi] = sorted_of(L) ? len_of(L) : -len_of(L); } }
        if (tid < nrun && run[cur][tid] >= t) pend[atomicAdd(&npend, 1)] = run[cur][tid];
        __syncthreads();
        const int nq = nqual < kKMax ? nqual : kKMax;
        for (int e = tid; e < nq * max_len; e += NT) {
            const int li = e / max_len, j = e - li * max_len;
            const int ql = qual_len[li];                // negative: (logit, id) pairs
            u64 key = j < (ql < 0 ? -ql : ql) ? qual[li][j] : 0;
            if (ql < 0) key = pair_key((uint32_t)(key >> 32), (uint32_t)key);
            if (key != 0 && key >= t) { const int pi = atomicAdd(&npend, 1); if (pi < kPendCap) pend[pi] = key; }
        }
        __syncthreads();
        // (4) exact order among pend -> new running list
        const int np = npend < kPendCap ? npend : kPendCap;
        for (int e = tid; e < np; e += NT) {
            const u64 mine = pend[e];
            int r = 0;
            for (int j = 0; j < np; ++j) r += pend[j] > mine;
            if (r < k) run[cur ^ 1][r] = mine;
        }
        __syncthreads();
        cur ^= 1;
        nrun = np < k ? np : k;
        thr = nrun == k ? run[cur][k - 1] : 0;
        if (tid == 0) { npend = 0; nqual = 0; }
        __syncthreads();
    }
    for (int j = tid; j < k; j += NT) {
        const u64 key = j < nrun ? run[cur][j] : 0;
        out_vals[(size_t)out_row * k + j] = key ? key_value(key) : -INFINITY;
        out_ids[(size_t)out_row * k + j] = key ? key_id(key) : -1;
    }
}

}  // namespace evospec

// =======================================================================================
// Host launchers (argument shapes are validated by the C ABI layer before these run).
#include "launch.hpp"

namespace evospec {

namespace {
constexpr int kMaxDevices = 64;

template <int NW, int RGW, int RC, int MB, bool FULLK, bool PACKED>
hipError_t launch_partials_k(const Plan& p, const void* h, const ChunkBatch& cb, const BatchLayout& bl, int d,
                             const void* W, const int32_t* ids, int V_act, int k, void* keys, void* stats,
                             hipStream_t stream) {
    auto kern = lmhead_partials_kernel<NW, RGW, RC, MB, FULLK, PACKED>;
    static std::atomic<bool> attr_set[kMaxDevices] = {};      // concurrent first calls may both set the (idempotent) attribute
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || !attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < kMaxDevices) attr_set[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(p.n_slabs, cb.n), dim3(NW * 64), p.lds_bytes, stream,
                       static_cast<const uint16_t*>(h), cb, bl.seq_rows, bl.chunk_bytes / 8, bl.chunk_bytes / 8, d,
                       static_cast<const uint16_t*>(W), ids,
                       V_act, k, p.gl, static_cast<u64*>(keys), static_cast<float2*>(stats));
    return hipGetLastError();
}

template <int NW, int RGW, int RC>
hipError_t launch_partials_shape(const Plan& p, const void* h, const ChunkBatch& cb, const BatchLayout& bl, int d,
                                 const void* W, const int32_t* ids, int V_act, int k, void* keys, void* stats,
                                 hipStream_t stream) {
    const bool full = d % kKC == 0;
#define EVOSPEC_ARGS p, h, cb, bl, d, W, ids, V_act, k, keys, stats, stream
#define EVOSPEC_MB(MB_)                                                                              \
    if (p.mb == MB_) {                                                                               \
        if (bl.packed)                                                                               \
            return full ? launch_partials_k<NW, RGW, RC, MB_, true, true>(EVOSPEC_ARGS)              \
                        : launch_partials_k<NW, RGW, RC, MB_, false, true>(EVOSPEC_ARGS);            \
        return full ? launch_partials_k<NW, RGW, RC, MB_, true, false>(EVOSPEC_ARGS)                 \
                    : launch_partials_k<NW, RGW, RC, MB_, false, false>(EVOSPEC_ARGS);               \
    }
    EVOSPEC_MB(1) EVOSPEC_MB(2) EVOSPEC_MB(4)
#undef EVOSPEC_MB
#undef EVOSPEC_ARGS
    return hipErrorInvalidValue;
}
}  // namespace

hipError_t launch_partials_batch(const Plan& p, const void* h, const ChunkBatch& cb, const BatchLayout& bl,
                                 int d, const void* W, const int32_t* ids, int V_act, int k, void* keys,
                                 void* stats, hipStream_t stream) {
    if (cb.n < 1 || cb.n > kMaxChunks || bl.chunk_bytes % 8 != 0) return hipErrorInvalidValue;
#define EVOSPEC_SHAPE(NW_, RGW_, RC_)                                                          \
    if (p.nw == NW_ && p.rgw == RGW_ && p.rc == RC_)                                           \
        return launch_partials_shape<NW_, RGW_, RC_>(p, h, cb, bl, d, W, ids, V_act, k, keys, stats, stream);
    EVOSPEC_SLAB_SHAPES(EVOSPEC_SHAPE)
#undef EVOSPEC_SHAPE
    return hipErrorInvalidValue;
}

hipError_t launch_partials(const Plan& p, const void* h, int rows, int d, const void* W,
                           const int32_t* ids, int V_act, int k, void* keys, void* stats,
                           hipStream_t stream, bool packed) {
    ChunkBatch cb;
    cb.n = 1; cb.m0[0] = 0; cb.rows[0] = rows; cb.seq[0] = 0; cb.a_pass[0] = 0; cb.a_slot[0] = 0;
    BatchLayout bl;
    bl.packed = packed;
    return launch_partials_batch(p, h, cb, bl, d, W, ids, V_act, k, keys, stats, stream);
}

hipError_t launch_merge_batch(const MergeSet& a, size_t a_pass_bytes, const MergeSet& b, size_t b_chunk_bytes,
                              const ChunkBatch& cb, int k, float* out_vals, int32_t* out_ids,
                              float* out_logz, hipStream_t stream, const GatherArgs* update) {
    if (cb.n < 1 || cb.n > kMaxChunks || a_pass_bytes % 8 != 0 || b_chunk_bytes % 8 != 0) return hipErrorInvalidValue;
    int max_rows = 0;
    for (int i = 0; i < cb.n; ++i) max_rows = cb.rows[i] > max_rows ? cb.rows[i] : max_rows;
    GatherArgs upd{};
    if (update && update->n > 0) upd = *update;
    if (max_rows == 0 && upd.n == 0) return hipSuccess;
    if ((a.list_len != 0 && (a.list_len < k || a.list_len > kKMax || (a.list_len & 15))) ||
        (b.list_len != 0 && (b.list_len < k || b.list_len > kKMax || (b.list_len & 15))))
        return hipErrorInvalidValue;
    auto as_set = [&](const MergeSet& m) {
        PartialSet p;
        p.keys = static_cast<const u64*>(m.keys);
        p.stats = static_cast<const float2*>(m.stats);
        p.n_slabs = m.n_slabs;
        p.row_base = m.row_base;
        p.list_len = m.list_len ? m.list_len : k;
        p.sorted = m.list_len == 0;
        if (m.row_major) {          // [row][slab][slot]: one row's lists are contiguous
            p.key_slab = (size_t)p.list_len; p.key_row = (size_t)m.n_slabs * p.list_len;
            p.stat_slab = 1; p.stat_row = (size_t)m.n_slabs;
        } else {                    // [slab][row][slot]
            p.key_slab = (size_t)m.row_stride * p.list_len; p.key_row = (size_t)p.list_len;
            p.stat_slab = (size_t)m.row_stride; p.stat_row = 1;
        }
        return p;
    };
    const PartialSet A = as_set(a), B = as_set(b);
    const int max_len = A.list_len > B.list_len ? A.list_len : B.list_len;
    const int pend_cap = k * max_len + k + 8;      // k qualifying lists in full, the running k (8-byte keys: < 34 KB)
    const int gx = max_rows > upd.n ? max_rows : upd.n;
    // enough threads to take all lists of a row in one round where possible (one list per thread and round)
    const int total = A.n_slabs + B.n_slabs;
    const dim3 grid(gx, cb.n + (upd.n > 0 ? 1 : 0));
#define EVOSPEC_MERGE(NT_)                                                                                  \
    hipLaunchKernelGGL(lmhead_merge_kernel<NT_>, grid, dim3(NT_), (size_t)pend_cap * 8, stream, A, B, cb,    \
                       a_pass_bytes / 8, a_pass_bytes / 8, b_chunk_bytes / 8, b_chunk_bytes / 8, k, pend_cap, \
                       out_vals, out_ids, out_logz, upd)
    if (total <= 256) EVOSPEC_MERGE(256);
    else if (total <= 512) EVOSPEC_MERGE(512);
    else EVOSPEC_MERGE(1024);
#undef EVOSPEC_MERGE
    return hipGetLastError();
}

hipError_t launch_merge(const MergeSet& a, const MergeSet& b, int k, float* out_vals, int32_t* out_ids,
                        float* out_logz, int out_row0, int nrows, hipStream_t stream, const GatherArgs* update) {
    ChunkBatch cb;
    cb.n = 1; cb.m0[0] = out_row0; cb.rows[0] = nrows; cb.seq[0] = 0; cb.a_pass[0] = 0; cb.a_slot[0] = 0;
    return launch_merge_batch(a, 0, b, 0, cb, k, out_vals, out_ids, out_logz, stream, update);
}

hipError_t launch_gather(const void* W_lm, int V, int d, const int32_t* src_ids, const int32_t* slots,
                         int n, void* W_act, int32_t* act_ids, int V_act, hipStream_t stream, bool packed) {
    const GatherArgs g{W_lm, V, d / 8, src_ids, slots, n, W_act, act_ids, V_act, packed ? 1 : 0};
    if (packed && !slots) {                      // rebuild: whole operand tiles per workgroup
        const int tiles = (n + kPackRows - 1) / kPackRows;
        hipLaunchKernelGGL(gather_tiles_kernel, dim3(tiles < 4096 ? tiles : 4096), dim3(256), 0, stream, g);
        return hipGetLastError();
    }
    if (!packed && !slots && n >= 1024) {        // rebuild of a row-major matrix
        hipLaunchKernelGGL(gather_rebuild_rows_kernel, dim3(4096), dim3(256), 0, stream, g);
        return hipGetLastError();
    }
    const int grid = n < 8192 ? n : 8192;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(grid), dim3(256), 0, stream, g);
    return hipGetLastError();
}

hipError_t launch_gather_inline(const void* W_lm, int V, int d, const int32_t* host_ids, const int32_t* host_slots,
                                int n, void* W_act, int32_t* act_ids, int V_act, hipStream_t stream, bool packed) {
    if (n < 0 || n > kInlineRows) return hipErrorInvalidValue;
    if (n == 0) return hipSuccess;
    const GatherArgs g{W_lm, V, d / 8, nullptr, nullptr, n, W_act, act_ids, V_act, packed ? 1 : 0};
    InlineRows r{};
    for (int i = 0; i < n; ++i) { r.slot[i] = host_slots[i]; r.id[i] = host_ids[i]; }
    hipLaunchKernelGGL(gather_rows_inline_kernel, dim3(n), dim3(256), 0, stream, g, r);
    return hipGetLastError();
}

hipError_t run_validate_ids(const int32_t* ids, int n, int V, hipStream_t stream, int* bad) {
    // one flag per device: calls from several threads take turns (the call waits for its kernel anyway)
    static std::mutex flag_mutex;
    std::lock_guard<std::mutex> lock(flag_mutex);
    int* flag = nullptr;
    hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&flag), HIP_SYMBOL(g_validate_flag));
    if (e != hipSuccess) return e;
    int zero = 0;
    e = hipMemcpyAsync(flag, &zero, sizeof(int), hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(validate_ids_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, ids, n, V, flag);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = hipMemcpyAsync(bad, flag, sizeof(int), hipMemcpyDeviceToHost, stream);
    if (e != hipSuccess) return e;
    return hipStreamSynchronize(stream);
}

}  // namespace evospec
