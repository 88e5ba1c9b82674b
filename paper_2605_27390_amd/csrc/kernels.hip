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

#include <type_traits>

#include "plan.hpp"

namespace evospec {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const u32x4 __attribute__((address_space(1))) * gvec_ptr;   // 16-byte loads from HBM

// ---------------------------------------------------------------------------------------
// (logit, id) -> one 64-bit key whose unsigned order is "larger logit first, then smaller
// full-vocabulary id".  Key 0 is reserved for "no candidate".
__device__ __forceinline__ uint32_t f32_to_ordered(float f) {
    uint32_t u = __float_as_uint(f + 0.0f);             // -0 -> +0 so that the two tie
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_f32(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ __forceinline__ u64 make_key(float z, int32_t id) {
    return ((u64)f32_to_ordered(z) << 32) | (uint32_t)(~(uint32_t)id);
}
__device__ __forceinline__ float key_value(u64 key) { return ordered_to_f32((uint32_t)(key >> 32)); }
__device__ __forceinline__ int32_t key_id(u64 key) { return (int32_t)(~(uint32_t)key); }

// Workgroup barrier that waits for this wave's LDS traffic only: global loads issued for
// the next chunk stay in flight across it (a plain __syncthreads() would drain them).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---------------------------------------------------------------------------------------
// Row insertion  W_act[slot] <- W_lm[id], act_ids[slot] <- id  (bit copy, 16 B per lane).
// One workgroup per row, grid-stride over the n rows of the update.
__global__ void __launch_bounds__(256)
gather_rows_kernel(const uint4* __restrict__ W_lm, int V, int row_vec /* d/8 */,
                   const int32_t* __restrict__ src_ids, const int32_t* __restrict__ slots, int n,
                   uint4* __restrict__ W_act, int32_t* __restrict__ act_ids, int V_act) {
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const int32_t id = src_ids[i];
        const int32_t s = slots ? slots[i] : i;
        if (id < 0 || id >= V || s < 0 || s >= V_act) continue;     // uniform per workgroup
        const uint4* src = W_lm + (size_t)id * row_vec;
        uint4* dst = W_act + (size_t)s * row_vec;
        for (int c0 = 0; c0 < row_vec; c0 += 4 * 256) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * 256 + threadIdx.x;
                if (c < row_vec) v[u] = src[c];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * 256 + threadIdx.x;
                if (c < row_vec) dst[c] = v[u];
            }
        }
        if (threadIdx.x == 0) act_ids[s] = id;
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
// in LDS, double buffered, shared by all waves), and reduces the slab's logits in LDS to
//   part_stats[slab][m] = (max_i z, sum_i exp(z - max))         over the slab's rows
//   part_keys[slab][m][0..k) = the slab's k best keys, descending (0 = none)
// Logits never leave the CU.
template <int NW, int RGW, int MB, bool FULLK>
__global__ void __launch_bounds__(NW * 64)
lmhead_partials_kernel(const uint16_t* __restrict__ h, int rows, int d,
                       const uint16_t* __restrict__ W, const int32_t* __restrict__ ids,
                       int V_act, int k, int G,
                       u64* __restrict__ part_keys, float2* __restrict__ part_stats) {
    constexpr int NT = NW * 64;
    constexpr int RT = 16 * NW * RGW;
    constexpr int MR = 16 * MB;
    constexpr int ZSTR = RT + 2;
    constexpr int KC = kKC;
    constexpr int KSTEPS = KC / 32;
    constexpr int HPIECES = MR * (KC / 8);
    constexpr int HP = (HPIECES + NT - 1) / NT;

    extern __shared__ __align__(16) unsigned char smem[];
    // region U: h chunks during the contraction, selection scratch afterwards
    uint16_t* Hs = reinterpret_cast<uint16_t*>(smem);
    uint16_t* surv = reinterpret_cast<uint16_t*>(smem);                       // [MR][RT]
    const size_t surv_bytes = align_up((size_t)MR * RT * 2, 16);
    u64* gkey = reinterpret_cast<u64*>(smem + surv_bytes);                    // [MR][G]
    float* gsum = reinterpret_cast<float*>(gkey + (size_t)MR * G);            // [MR][G]
    const size_t hs_bytes = 2ull * MR * kHStride * 2;
    const size_t sel_bytes = surv_bytes + (size_t)MR * G * 12;
    const size_t u_bytes = align_up(hs_bytes > sel_bytes ? hs_bytes : sel_bytes, 16);
    u64* Zk = reinterpret_cast<u64*>(smem + u_bytes);                         // [MR][ZSTR]
    int32_t* Ids = reinterpret_cast<int32_t*>(Zk + (size_t)MR * ZSTR);        // [RT]
    u64* tau = reinterpret_cast<u64*>(reinterpret_cast<unsigned char*>(Ids) + align_up((size_t)RT * 4, 16));  // [MR]
    int* cnt = reinterpret_cast<int*>(tau + MR);                              // [MR]
    float* vmax = reinterpret_cast<float*>(cnt + MR);                         // [MR]

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int row0 = blockIdx.x * RT;
    const int n_valid = min(RT, V_act - row0);

    for (int i = tid; i < RT; i += NT) {
        const int r = row0 + i;
        Ids[i] = (r < V_act) ? (ids ? ids[r] : r) : 0x7fffffff;
    }

    const uint16_t* wp[RGW];
#pragma unroll
    for (int rg = 0; rg < RGW; ++rg) {
        int r = row0 + (w * RGW + rg) * 16 + n16;
        r = min(r, V_act - 1);                         // tail slab: duplicate a valid row, masked later
        wp[rg] = W + (size_t)r * d + g * 8;
    }

    f32x4 acc[RGW][MB];
#pragma unroll
    for (int rg = 0; rg < RGW; ++rg)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[rg][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nchunks = (d + KC - 1) / KC;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    u32x4 hreg[HP];
    u32x4 wa[RGW][KSTEPS], wb[RGW][KSTEPS];

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
    auto load_w_step = [&](u32x4 (&dst)[RGW][KSTEPS], int c, int s) {
        const int koff = c * KC + s * 32;
#pragma unroll
        for (int rg = 0; rg < RGW; ++rg) {
            if constexpr (FULLK) {
                dst[rg][s] = wsrc[rg][koff / 8];
            } else {
                const bool in = koff + g * 8 < d;
                const u32x4 v = *(wsrc[rg] + ((in ? koff + g * 8 : d - 8) - g * 8) / 8);
                dst[rg][s] = in ? v : zero4;
            }
        }
    };
    auto load_b = [&](bf16x8 (&b)[MB], int buf, int s) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            b[mb] = *reinterpret_cast<const bf16x8*>(Hs + ((size_t)buf * MR + mb * 16 + n16) * kHStride + s * 32 + g * 8);
    };
    auto mfma_step = [&](u32x4 (&cur)[RGW][KSTEPS], const bf16x8 (&b)[MB], int s) {
#pragma unroll
        for (int rg = 0; rg < RGW; ++rg) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, cur[rg][s]);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                acc[rg][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b[mb], acc[rg][mb], 0, 0, 0);
        }
    };
    // One chunk: contract `cur` (loaded one chunk earlier) against the h chunk in LDS buffer `buf`
    // while the next chunk's W rows stream into `nxt` and its h pieces into the other buffer.
    // PREFETCH is a compile-time flag so that the steady-state loop has no branch in it.
    auto chunk = [&](u32x4 (&cur)[RGW][KSTEPS], u32x4 (&nxt)[RGW][KSTEPS], int buf, int c, auto prefetch) {
        constexpr bool PREFETCH = decltype(prefetch)::value;
        bf16x8 b0[MB], b1[MB];
        if constexpr (PREFETCH) load_h(c + 1);
        load_b(b0, buf, 0);
#pragma unroll
        for (int s = 0; s < KSTEPS; s += 2) {
            if constexpr (PREFETCH) load_w_step(nxt, c + 1, s);
            load_b(b1, buf, s + 1);
            __builtin_amdgcn_sched_barrier(0);      // keep the prefetch ahead of the MFMAs it overlaps
            mfma_step(cur, b0, s);
            if constexpr (PREFETCH) load_w_step(nxt, c + 1, s + 1);
            if (s + 2 < KSTEPS) load_b(b0, buf, s + 2);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(cur, b1, s + 1);
        }
        if constexpr (PREFETCH) store_h(buf ^ 1);
        lds_barrier();
    };
    using yes = std::true_type;
    using no = std::false_type;

    load_h(0);
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) load_w_step(wa, 0, s);
    store_h(0);
    lds_barrier();
    int c = 0;
    for (; c + 2 < nchunks; c += 2) {           // chunks c and c+1 both have a successor
        chunk(wa, wb, 0, c, yes{});
        chunk(wb, wa, 1, c + 1, yes{});
    }
    if (nchunks - c == 2) {
        chunk(wa, wb, 0, c, yes{});
        chunk(wb, wa, 1, c + 1, no{});
    } else {
        chunk(wa, wb, 0, c, no{});
    }
    // every wave is past its last read of Hs (the loop ends on a barrier): region U is free

    // ---- slab epilogue: logits -> sortable keys in LDS
#pragma unroll
    for (int rg = 0; rg < RGW; ++rg) {
        const int rl = (w * RGW + rg) * 16 + 4 * g;
        const int4 id4 = *reinterpret_cast<const int4*>(Ids + rl);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = mb * 16 + n16;
            u64* dst = Zk + (size_t)m * ZSTR + rl;
            ulonglong2 lo, hi;
            lo.x = make_key(acc[rg][mb][0], id4.x);
            lo.y = make_key(acc[rg][mb][1], id4.y);
            hi.x = make_key(acc[rg][mb][2], id4.z);
            hi.y = make_key(acc[rg][mb][3], id4.w);
            *reinterpret_cast<ulonglong2*>(dst) = lo;
            *reinterpret_cast<ulonglong2*>(dst + 2) = hi;
        }
    }
    if (tid < MR) { cnt[tid] = 0; tau[tid] = 0; }
    __syncthreads();

    // ---- pass 1: maxima of G interleaved groups per draft row
    const int npairs = rows * G;
    for (int p = tid; p < npairs; p += NT) {
        const int m = p / G, s = p - m * G;
        const u64* zr = Zk + (size_t)m * ZSTR;
        u64 mx = 0;
        for (int i = s; i < n_valid; i += G) { const u64 v = zr[i]; mx = v > mx ? v : mx; }
        gkey[(size_t)m * G + s] = mx;
    }
    __syncthreads();
    // ---- pass 2a: tau[m] = k-th largest group maximum (a lower bound of the slab's k-th best key,
    //      because the group maxima are G >= k distinct slab entries); vmax[m] = slab maximum
    for (int p = tid; p < npairs; p += NT) {
        const int m = p / G, s = p - m * G;
        const u64* gk = gkey + (size_t)m * G;
        const u64 mine = gk[s];
        int rank = 0;
        u64 top = 0;
        for (int j = 0; j < G; ++j) {
            const u64 o = gk[j];
            rank += (o > mine) || (o == mine && j < s);
            top = o > top ? o : top;
        }
        if (rank == k - 1) tau[m] = mine;
        if (s == 0) vmax[m] = key_value(top);
    }
    __syncthreads();
    // ---- pass 2b: keep entries >= tau (at least k of them if the slab has k), sum exp(z - vmax)
    for (int p = tid; p < npairs; p += NT) {
        const int m = p / G, s = p - m * G;
        const u64* zr = Zk + (size_t)m * ZSTR;
        const u64 t = tau[m];
        const float vm = vmax[m];
        float sum = 0.f;
        for (int i = s; i < n_valid; i += G) {
            const u64 v = zr[i];
            sum += __expf(key_value(v) - vm);
            if (v >= t) {
                const int pos = atomicAdd(&cnt[m], 1);
                surv[(size_t)m * RT + pos] = (uint16_t)i;
            }
        }
        gsum[(size_t)m * G + s] = sum;
    }
    __syncthreads();
    // ---- pass 3: exact rank among the survivors; write the k best, the stats
    const size_t out_row = (size_t)blockIdx.x * kMTile;
    for (int p = tid; p < rows * n_valid; p += NT) {
        const int m = p / n_valid, q = p - m * n_valid;
        const int c = cnt[m];
        if (q >= c) continue;
        const u64* zr = Zk + (size_t)m * ZSTR;
        const uint16_t* sv = surv + (size_t)m * RT;
        const u64 mine = zr[sv[q]];
        int rank = 0;
        for (int j = 0; j < c; ++j) {
            const u64 o = zr[sv[j]];
            rank += (o > mine) || (o == mine && j < q);
        }
        u64* outk = part_keys + (out_row + m) * k;
        if (rank < k) outk[rank] = mine;
        if (q == 0) {
            for (int j = c; j < k; ++j) outk[j] = 0;               // slab holds fewer than k rows
            const float* gs = gsum + (size_t)m * G;
            float sum = 0.f;
            for (int j = 0; j < G; ++j) sum += gs[j];
            part_stats[out_row + m] = make_float2(vmax[m], sum);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Pass 2: one workgroup per draft row merges the slab partials:
//   logZ = M + log(sum_t s_t * exp(m_t - M)),  M = max_t m_t
//   top-k = the k largest of all slab candidates (keys are unique, so the order is total).
// Candidates come from up to two partial sets (a shared core and a per-sequence extension
// in the batched variant).  The candidate stream is filtered against the running k-th best
// and merged in batches by exact rank counting.
struct PartialSet {
    const u64* keys;        // [n_slabs][64][k]
    const float2* stats;    // [n_slabs][64]
    int n_slabs;
    int row_base;           // draft row of this launch's block 0 inside the set's 64-row pass
};

constexpr int kMergeThreads = 256;

__global__ void __launch_bounds__(kMergeThreads)
lmhead_merge_kernel(PartialSet A, PartialSet B, int k,
                    float* __restrict__ out_vals, int32_t* __restrict__ out_ids,
                    float* __restrict__ out_logz, int out_row0) {
    constexpr int NT = kMergeThreads;
    __shared__ u64 run[2][kKMax];
    __shared__ u64 pend[2 * NT + kKMax];
    __shared__ int npend;
    __shared__ float red_m[NT], red_s[NT];

    const int tid = threadIdx.x;
    const int out_row = out_row0 + blockIdx.x;

    // ---- log-normaliser
    float mx = -INFINITY;
    for (int set = 0; set < 2; ++set) {
        const PartialSet& P = set ? B : A;
        const int slot = P.row_base + blockIdx.x;
        for (int t = tid; t < P.n_slabs; t += NT) mx = fmaxf(mx, P.stats[(size_t)t * kMTile + slot].x);
    }
    red_m[tid] = mx;
    __syncthreads();
    for (int o = NT / 2; o > 0; o >>= 1) {
        if (tid < o) red_m[tid] = fmaxf(red_m[tid], red_m[tid + o]);
        __syncthreads();
    }
    const float gmax = red_m[0];
    float sum = 0.f;
    for (int set = 0; set < 2; ++set) {
        const PartialSet& P = set ? B : A;
        const int slot = P.row_base + blockIdx.x;
        for (int t = tid; t < P.n_slabs; t += NT) {
            const float2 st = P.stats[(size_t)t * kMTile + slot];
            sum += st.y * __expf(st.x - gmax);
        }
    }
    red_s[tid] = sum;
    __syncthreads();
    for (int o = NT / 2; o > 0; o >>= 1) {
        if (tid < o) red_s[tid] += red_s[tid + o];
        __syncthreads();
    }
    if (tid == 0) out_logz[out_row] = gmax + __logf(red_s[0]);

    // ---- top-k over all candidates
    if (tid == 0) npend = 0;
    int nrun = 0;            // entries in run[cur], sorted descending
    int cur = 0;
    u64 thr = 0;             // current k-th best (0 until k candidates were seen)
    __syncthreads();

    auto flush = [&]() {
        // merge run[cur][0..nrun) with pend[0..npend) into run[cur^1]; all threads call it
        const int np = npend;
        const int total = nrun + np;
        for (int e = tid; e < total; e += NT) {
            const u64 mine = e < nrun ? run[cur][e] : pend[e - nrun];
            int rank = 0;
            for (int j = 0; j < nrun; ++j) { const u64 o = run[cur][j]; rank += (o > mine) || (o == mine && j < e); }
            for (int j = 0; j < np; ++j) { const u64 o = pend[j]; rank += (o > mine) || (o == mine && j + nrun < e); }
            if (rank < k) run[cur ^ 1][rank] = mine;
        }
        __syncthreads();
        cur ^= 1;
        nrun = total < k ? total : k;
        thr = nrun == k ? run[cur][k - 1] : 0;
        if (tid == 0) npend = 0;
        __syncthreads();
    };

    for (int set = 0; set < 2; ++set) {
        const PartialSet& P = set ? B : A;
        const int slot = P.row_base + blockIdx.x;
        const int ncand = P.n_slabs * k;
        for (int base = 0; base < ncand; base += NT) {
            const int c = base + tid;
            if (c < ncand) {
                const int t = c / k, j = c - t * k;
                const u64 key = P.keys[((size_t)t * kMTile + slot) * k + j];
                if (key > thr) pend[atomicAdd(&npend, 1)] = key;
            }
            __syncthreads();
            const int np_now = npend;        // same value in every thread ...
            __syncthreads();                 // ... because nobody appends before all have read it
            if (np_now > NT) flush();
        }
    }
    if (npend > 0) flush();                  // uniform: no append since the last barrier
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

template <int NW, int RGW, int MB, bool FULLK>
hipError_t launch_partials_k(const Plan& p, const void* h, int rows, int d, const void* W,
                             const int32_t* ids, int V_act, int k, void* keys, void* stats,
                             hipStream_t stream);

template <int NW, int RGW, int MB>
hipError_t launch_partials_t(const Plan& p, const void* h, int rows, int d, const void* W,
                             const int32_t* ids, int V_act, int k, void* keys, void* stats,
                             hipStream_t stream) {
    if (d % kKC == 0) return launch_partials_k<NW, RGW, MB, true>(p, h, rows, d, W, ids, V_act, k, keys, stats, stream);
    return launch_partials_k<NW, RGW, MB, false>(p, h, rows, d, W, ids, V_act, k, keys, stats, stream);
}

template <int NW, int RGW, int MB, bool FULLK>
hipError_t launch_partials_k(const Plan& p, const void* h, int rows, int d, const void* W,
                             const int32_t* ids, int V_act, int k, void* keys, void* stats,
                             hipStream_t stream) {
    auto kern = lmhead_partials_kernel<NW, RGW, MB, FULLK>;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || !attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < kMaxDevices) attr_set[dev] = true;
    }
    hipLaunchKernelGGL(kern, dim3(p.n_slabs), dim3(NW * 64), p.lds_bytes, stream,
                       static_cast<const uint16_t*>(h), rows, d, static_cast<const uint16_t*>(W), ids,
                       V_act, k, p.groups, static_cast<u64*>(keys), static_cast<float2*>(stats));
    return hipGetLastError();
}

template <int NW, int RGW>
hipError_t launch_partials_mb(const Plan& p, const void* h, int rows, int d, const void* W,
                              const int32_t* ids, int V_act, int k, void* keys, void* stats,
                              hipStream_t stream) {
    switch (p.mb) {
        case 1: return launch_partials_t<NW, RGW, 1>(p, h, rows, d, W, ids, V_act, k, keys, stats, stream);
        case 2: return launch_partials_t<NW, RGW, 2>(p, h, rows, d, W, ids, V_act, k, keys, stats, stream);
        case 4: return launch_partials_t<NW, RGW, 4>(p, h, rows, d, W, ids, V_act, k, keys, stats, stream);
        default: return hipErrorInvalidValue;
    }
}
}  // namespace

hipError_t launch_partials(const Plan& p, const void* h, int rows, int d, const void* W,
                           const int32_t* ids, int V_act, int k, void* keys, void* stats,
                           hipStream_t stream) {
#define EVOSPEC_SHAPE(NW_, RGW_)                                                               \
    if (p.nw == NW_ && p.rgw == RGW_)                                                          \
        return launch_partials_mb<NW_, RGW_>(p, h, rows, d, W, ids, V_act, k, keys, stats, stream);
    EVOSPEC_SHAPE(4, 1) EVOSPEC_SHAPE(5, 1) EVOSPEC_SHAPE(6, 1) EVOSPEC_SHAPE(7, 1) EVOSPEC_SHAPE(8, 1)
    EVOSPEC_SHAPE(9, 1) EVOSPEC_SHAPE(10, 1) EVOSPEC_SHAPE(12, 1) EVOSPEC_SHAPE(8, 2)
#undef EVOSPEC_SHAPE
    return hipErrorInvalidValue;
}

hipError_t launch_merge(const MergeSet& a, const MergeSet& b, int k, float* out_vals, int32_t* out_ids,
                        float* out_logz, int out_row0, int nrows, hipStream_t stream) {
    PartialSet A{static_cast<const u64*>(a.keys), static_cast<const float2*>(a.stats), a.n_slabs, a.row_base};
    PartialSet B{static_cast<const u64*>(b.keys), static_cast<const float2*>(b.stats), b.n_slabs, b.row_base};
    hipLaunchKernelGGL(lmhead_merge_kernel, dim3(nrows), dim3(kMergeThreads), 0, stream, A, B, k,
                       out_vals, out_ids, out_logz, out_row0);
    return hipGetLastError();
}

hipError_t launch_gather(const void* W_lm, int V, int d, const int32_t* src_ids, const int32_t* slots,
                         int n, void* W_act, int32_t* act_ids, int V_act, hipStream_t stream) {
    const int grid = n < 8192 ? n : 8192;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(grid), dim3(256), 0, stream,
                       static_cast<const uint4*>(W_lm), V, d / 8, src_ids, slots, n,
                       static_cast<uint4*>(W_act), act_ids, V_act);
    return hipGetLastError();
}

hipError_t run_validate_ids(const int32_t* ids, int n, int V, hipStream_t stream, int* bad) {
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
