// Retained-support KL gate of Path B (EvoSpec paper, Sec. "Online parameter update", Eq. 5 and
// the admission rule around it; Algorithm 1, Path B): per verification event, the K_logit largest
// target logits are kept; the draft model's logits on the same ids (Eq. 1: h_draft . W_LM[i]) and
// the temperature T_KD turn both into distributions p, q on that support; the event is admitted
// when D_KL(p || q) exceeds the gate.
//
// Four launches:
//  1. kl_select_slices_kernel, one workgroup of 16 wavefronts per (eighth of the vocabulary, event),
//     two of them per compute unit: every thread loads its share of the slice once (all requests in
//     flight together, the values stay in registers) and takes its maximum; a value that K of these
//     1024 maxima reach (the q-th largest of every wavefront, found bit by bit) is a lower bound of the
//     slice's K-th largest logit, so the logits that reach it (a few hundred) go to the workspace as
//     64-bit (logit, id) keys.  If more than 2048 reach it (masses of equal logits), radix select on
//     the key instead (11 bits per pass, histogram in LDS, a pass is skipped as soon as the bin that
//     holds the K-th key is taken whole) leaves exactly K;
//  2. kl_select_final_kernel, one workgroup per event: the K-th largest of the maxima that pairs
//     of threads hold of the slices' candidates (a bitonic sort over half the workgroup) bounds
//     the answer, the survivors (a few more than K) are sorted the same way: the support, by
//     decreasing key;
//  3. kl_draft_logits_kernel, one workgroup of 4 wavefronts per 16 support rows of an event, so that
//     the E x K rows of W_LM (the bulk of the bytes) are spread over the whole GPU: a wavefront
//     takes 4 rows at a time, 16 bytes per lane and load, h in LDS;
//  4. kl_divergence_kernel, one wavefront per event: log-sum-exp of both logit vectors and D_KL.
// Bytes per event: the target logits once, K rows of W_LM once.  Stages 1 and 2 are bound by
// latencies and by instruction issue on the few compute units they occupy, stage 3 by HBM.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"
#include "launch.hpp"

namespace evospec {

namespace {
constexpr int kKlThreads = 1024;
constexpr int kKlMaxK = 256;
constexpr int kKlBits = 11;
constexpr int kKlBins = 1 << kKlBits;
constexpr int kKlCand = 2048;                 // candidates the common path can rank

__device__ __forceinline__ float wave_sum(float x) { return evospec::wave_sum(x, (int)(threadIdx.x & 63)); }
__device__ __forceinline__ float wave_max(float x) { return evospec::wave_max(x, (int)(threadIdx.x & 63)); }

// Wave 0 only: the bin (from the top) in which the cumulative count of hist reaches `need`;
// the number of entries in higher bins goes to *above_out, the bin's own count to *count (set by
// the one lane that owns the bin, left alone by the others).
__device__ __forceinline__ void find_bin(const uint32_t* hist, int lane, int need,
                                         int* bin, int* above_out, int* count) {
    // lane l owns bins [32 (63 - l), +32), so lane 0 holds the largest
    const int b0 = 32 * (63 - lane);
    uint32_t c[32];
#pragma unroll
    for (int j = 0; j < 32; j += 4) {
        const u32x4 q = *reinterpret_cast<const u32x4*>(hist + b0 + j);
        c[j] = q[0]; c[j + 1] = q[1]; c[j + 2] = q[2]; c[j + 3] = q[3];
    }
    uint32_t tot = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) tot += c[j];
    uint32_t incl = tot;                                     // inclusive prefix over lanes 0..lane
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    const uint32_t above = incl - tot;                       // entries in bins owned by lower lanes (larger bins)
    if (above < (uint32_t)need && incl >= (uint32_t)need) {  // exactly one lane
        uint32_t acc = above;
        bool found = false;
#pragma unroll
        for (int j = 31; j >= 0; --j) {
            if (!found && acc + c[j] >= (uint32_t)need) { *bin = b0 + j; *above_out = (int)acc; *count = (int)c[j]; found = true; }
            acc += found ? 0u : c[j];
        }
    }
}

// Sorting networks over 32-bit or 64-bit keys (T = uint32_t or u64), one key per thread.
// Compare-exchange with lane ^ STRIDE: the lower lane of a pair keeps the larger key when desc.
template <int STRIDE, typename T>
__device__ __forceinline__ T cmpx_lane(T x, int lane, bool desc) {
    T y;
    if constexpr (sizeof(T) == 8) {
        const uint32_t lo = xor_lane<STRIDE>((uint32_t)x, lane), hi = xor_lane<STRIDE>((uint32_t)(x >> 32), lane);
        y = ((u64)hi << 32) | lo;
    } else {
        y = xor_lane<STRIDE>(x, lane);
    }
    return ((x > y) == (((lane & STRIDE) == 0) == desc)) ? x : y;
}
template <typename T>
__device__ __forceinline__ T merge_in_wave(T x, int lane, bool desc) {
    x = cmpx_lane<32>(x, lane, desc); x = cmpx_lane<16>(x, lane, desc); x = cmpx_lane<8>(x, lane, desc);
    x = cmpx_lane<4>(x, lane, desc);  x = cmpx_lane<2>(x, lane, desc);  x = cmpx_lane<1>(x, lane, desc);
    return x;
}
// Bitonic sort of the 64 keys of a wavefront, 21 register exchanges: lane 0 ends with the largest
// when desc, with the smallest otherwise.
template <typename T>
__device__ __forceinline__ T sort_in_wave(T x, int lane, bool desc) {
    x = cmpx_lane<1>(x, lane, (lane & 2) == 0);
    x = cmpx_lane<2>(x, lane, (lane & 4) == 0);  x = cmpx_lane<1>(x, lane, (lane & 4) == 0);
    x = cmpx_lane<4>(x, lane, (lane & 8) == 0);  x = cmpx_lane<2>(x, lane, (lane & 8) == 0);
    x = cmpx_lane<1>(x, lane, (lane & 8) == 0);
    x = cmpx_lane<8>(x, lane, (lane & 16) == 0); x = cmpx_lane<4>(x, lane, (lane & 16) == 0);
    x = cmpx_lane<2>(x, lane, (lane & 16) == 0); x = cmpx_lane<1>(x, lane, (lane & 16) == 0);
    x = cmpx_lane<16>(x, lane, (lane & 32) == 0); x = cmpx_lane<8>(x, lane, (lane & 32) == 0);
    x = cmpx_lane<4>(x, lane, (lane & 32) == 0);  x = cmpx_lane<2>(x, lane, (lane & 32) == 0);
    x = cmpx_lane<1>(x, lane, (lane & 32) == 0);
    return merge_in_wave(x, lane, desc);
}
// Bitonic sort of N keys (N = 512 or 1024), one per thread of the first N threads of the workgroup:
// thread t < N returns the (t+1)-th largest (equal keys in any order); every thread of the workgroup
// calls it (the others only meet the barriers).  Steps between lanes of a wavefront are register
// exchanges; the steps between wavefronts go through buf (LDS, [2][N], one barrier each).
// (A radix select of the K-th largest alone was slower: its first histogram pass sends all 1024
// atomic adds to the two or three bins of the common exponent, 3 us per pass.)
template <int N, typename T>
__device__ __forceinline__ T wg_sort_desc(T x, T* buf) {
    static_assert(N % 128 == 0 && N <= kKlThreads, "whole wavefronts");
    const int tid = threadIdx.x, lane = tid & 63;
    const bool act = tid < N;                            // (uniform per wavefront)
    if (act) x = sort_in_wave(x, lane, (tid & 64) == 0);
    int pb = 0;
#pragma unroll
    for (int size = 128; size <= N; size <<= 1) {
        const bool desc = (tid & size) == 0;
#pragma unroll
        for (int stride = size >> 1; stride >= 64; stride >>= 1) {
            if (act) buf[pb * N + tid] = x;
            __syncthreads();
            if (act) {
                const T y = buf[pb * N + (tid ^ stride)];
                x = ((x > y) == (((tid & stride) == 0) == desc)) ? x : y;
            }
            pb ^= 1;                                     // the next step writes the other half
        }
        if (act) x = merge_in_wave(x, lane, desc);
    }
    return x;
}

// The q-th largest (counting repeats, 1 <= q <= 64) of the 64 values of a wavefront: the largest t
// that at least q values reach, found bit by bit.  One vector compare per bit, the rest is scalar:
// with 8 wavefronts per SIMD this costs a fifth of sorting the 64 values.
__device__ __forceinline__ uint32_t wave_kth_largest(uint32_t v, int q) {
    uint32_t t = 0;
#pragma unroll
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t c = t | (1u << bit);
        if (__popcll(__ballot(v >= c)) >= q) t = c;              // (uniform)
    }
    return t;
}
// A lower bound of the K-th largest (counting repeats) of the 1024 values v, one per thread, without
// a selection over the workgroup: with q = ceil(K / 16), each of the 16 wavefronts holds q values at or
// above its own q-th largest, so K values reach the smallest of the 16.  (Looser than the exact K-th
// largest, and a fraction of its cost.)
__device__ __forceinline__ uint32_t kth_bound_1024(uint32_t v, int K, uint32_t* wave_q /*LDS [16]*/) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int q = (K + 15) >> 4;                               // K <= 1024
    const uint32_t s = wave_kth_largest(v, q);
    if (lane == 0) wave_q[w] = s;
    __syncthreads();
    uint32_t t = wave_q[0];
#pragma unroll
    for (int i = 1; i < kKlThreads / 64; ++i) { const uint32_t o = wave_q[i]; t = o < t ? o : t; }
    return t;
}
}  // namespace

// Stage 1 of the selection, one workgroup per (slice g of the vocabulary, event e): the keys of the
// slice that can still be among the event's K largest go to the workspace, unranked:
// ws_keys[(e * G + g) * kKlCand + ...], their number to ws_cnt[e * G + g].
//
// NL > 0: the slice fits NL 16-byte loads per thread (and the logits are 16-byte aligned).  All of
// them are issued before the first is used and the values stay in registers for the second sweep:
// the kernel is bound by memory latency, and a loop of dependent load-then-compare iterations pays
// that latency once per iteration.  NL == 0: any size and alignment, two sweeps over memory.
// (Two workgroups per compute unit, so that the 8 x E workgroups of 60 events run as one round: the
// second launch-bounds figure caps the registers at 64 per lane; the radix path below may spill.)
template <int NL>
__global__ void __launch_bounds__(kKlThreads, 8)
kl_select_slices_kernel(const float* __restrict__ z_target, int V, int K, int G, int slice,
                        u64* __restrict__ ws_keys, int* __restrict__ ws_cnt) {
    __shared__ __align__(16) uint32_t hist[kKlBins];
    __shared__ u64 cand[kKlCand];
    __shared__ int ncand;
    __shared__ u64 prefix_s;
    __shared__ uint32_t wave_q[kKlThreads / 64];
    __shared__ int need_s, done_s;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g = blockIdx.x, e = blockIdx.y;
    const float* z = z_target + (size_t)e * V;
    const int lo = g * slice, hi = min(V, lo + slice);             // slice is a multiple of 4
    const int Kl = min(K, hi - lo);                                // the slice's own K largest suffice
    u64* out = ws_keys + ((size_t)e * G + g) * kKlCand;
    if (hi <= lo) { if (tid == 0) ws_cnt[e * G + g] = 0; return; }

    if (tid == 0) { done_s = 0; ncand = 0; }

    // ---- common path: the Kl-th largest of the per-thread maxima bounds the slice's Kl-th largest
    // logit from below (plain float compares)
    float mx = -INFINITY;
    bool any = false;
    float4 q[NL > 0 ? NL : 1];
    const bool vec = NL > 0 || ((V & 3) == 0 && (reinterpret_cast<uintptr_t>(z_target) & 15) == 0);
    if constexpr (NL > 0) {
        // (the launcher picks NL > 0 only for aligned logits and a slice that NL loads per thread cover)
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int i = lo + 4 * (tid + j * kKlThreads);
            q[j] = *reinterpret_cast<const float4*>(z + (i < hi ? i : lo));     // past the end: a valid address, masked below
        }
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const bool in = lo + 4 * (tid + j * kKlThreads) < hi;
            if (!in) q[j] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            mx = fmaxf(fmaxf(mx, fmaxf(q[j].x, q[j].y)), fmaxf(q[j].z, q[j].w));
            any = any || in;
        }
    } else if (vec) {
        for (int i = lo + 4 * tid; i < hi; i += 4 * kKlThreads) {
            const float4 v = *reinterpret_cast<const float4*>(z + i);
            mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
            any = true;
        }
    } else {
        for (int i = lo + tid; i < hi; i += kKlThreads) { mx = fmaxf(mx, z[i]); any = true; }
    }
    // (absent threads contribute 0, below every real value)
    const uint32_t kth = kth_bound_1024(any ? f32_to_ordered(mx) : 0u, Kl, wave_q);
    const float tau0 = kth ? ordered_to_f32(kth) : -INFINITY;      // too few threads saw a logit: keep all
    auto consider = [&](float v, int i) {
        if (v >= tau0) {
            const int p = atomicAdd(&ncand, 1);
            if (p < kKlCand) cand[p] = make_key(v, i);
        }
    };
    if constexpr (NL > 0) {
        // One atomic add per wavefront instead of one per key (they all go to the same counter):
        // a lane's number of keys (<= 4 NL < 64) is summed over the lower lanes bit by bit.
        const float* qf = reinterpret_cast<const float*>(q);
        uint32_t pass = 0;                                       // (4 NL <= 32 bits) bit 4 j + c: component c of load j reaches the bound
#pragma unroll
        for (int x = 0; x < 4 * NL; ++x)
            if (lo + 4 * (tid + (x >> 2) * kKlThreads) < hi && qf[x] >= tau0) pass |= 1u << x;
        const int mine = __popc(pass);
        int before = 0, total = 0;
#pragma unroll
        for (int bit = 0; bit < 6; ++bit) {
            const u64 bal = __ballot((mine >> bit) & 1);
            before += (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u)) << bit;
            total += __popcll(bal) << bit;
        }
        static_assert(4 * NL < 64, "a lane's count fits six bits");
        int base = 0;
        if (total > 0) {
            if (lane == 0) base = atomicAdd(&ncand, total);
            base = __builtin_amdgcn_readfirstlane(base);
        }
        int p = base + before;
#pragma unroll
        for (int x = 0; x < 4 * NL; ++x) {
            if ((pass >> x) & 1u) {
                if (p < kKlCand) cand[p] = make_key(qf[x], lo + 4 * (tid + (x >> 2) * kKlThreads) + (x & 3));
                ++p;
            }
        }
    } else if (vec) {
        for (int i = lo + 4 * tid; i < hi; i += 4 * kKlThreads) {
            const float4 v = *reinterpret_cast<const float4*>(z + i);
            consider(v.x, i); consider(v.y, i + 1); consider(v.z, i + 2); consider(v.w, i + 3);
        }
    } else {
        for (int i = lo + tid; i < hi; i += kKlThreads) consider(z[i], i);
    }
    __syncthreads();
    const int nc = ncand;
    if (nc <= kKlCand) {
        for (int t = tid; t < nc; t += kKlThreads) out[t] = cand[t];
        if (tid == 0) ws_cnt[e * G + g] = nc;
        return;
    }

    // ---- masses of equal logits: radix select on the 64-bit key.  After a pass, prefix holds the
    // top `done` bits of the slice's Kl-th largest key and need the number of keys still to take
    // among those that share them.
    if (tid == 0) { prefix_s = 0; need_s = Kl; }
    __syncthreads();
    int done = 0;
    while (done < 64) {
        const int nb = 64 - done < kKlBits ? 64 - done : kKlBits;
        const int shift = 64 - done - nb;
        for (int i = tid; i < kKlBins; i += kKlThreads) hist[i] = 0;
        __syncthreads();
        const u64 prefix = prefix_s;
        for (int i = lo + tid; i < hi; i += kKlThreads) {
            const u64 key = make_key(z[i], i);
            if (done == 0 || (key >> (64 - done)) == (prefix >> (64 - done)))
                atomicAdd(&hist[(uint32_t)(key >> shift) & ((1u << nb) - 1u)], 1u);
        }
        __syncthreads();
        if (w == 0) {
            int bin = 0, above = 0, count = 0;
            const int need = need_s;
            find_bin(hist, lane, need, &bin, &above, &count);
            if (count > 0) {
                prefix_s = prefix | ((u64)bin << shift);
                need_s = need - above;
                done_s = count == need - above ? 1 : 0;          // the whole bin is taken
            }
        }
        __syncthreads();
        done += nb;
        if (done_s) break;
    }
    // every key >= threshold is one of the Kl largest (keys are distinct; the bits below `done` are 0)
    const u64 thr = prefix_s;
    if (tid == 0) ncand = 0;
    __syncthreads();
    for (int i = lo + tid; i < hi; i += kKlThreads) {
        const u64 key = make_key(z[i], i);
        if (key >= thr) {
            const int p = atomicAdd(&ncand, 1);
            if (p < kKlCand) out[p] = key;
        }
    }
    if (tid == 0) ws_cnt[e * G + g] = Kl;
}

// Stage 2, one workgroup per event: the K largest of the slices' candidates, by decreasing key.
// The same bound (K-th largest of the per-thread maxima, here over at most 16 candidates per
// thread) leaves at most 16 K keys, which are ranked by counting.
__global__ void __launch_bounds__(kKlThreads)
kl_select_final_kernel(const u64* __restrict__ ws_keys, const int* __restrict__ ws_cnt, int G, int K,
                       int32_t* __restrict__ out_support, float* __restrict__ out_zt) {
    __shared__ __align__(16) u64 surv[16 * kKlMaxK];
    __shared__ u64 sorted[kKlMaxK];
    __shared__ u64 tau_s;
    __shared__ int nsurv;
    const int tid = threadIdx.x, e = blockIdx.x;
    if (tid == 0) nsurv = 0;
    // The slices' lists, taken as one sequence, are dealt out to the threads, wavefronts first
    // (entry i to lane (i / 16) % 64 of wavefront i % 16, at most 16 per thread), so that every
    // wavefront gets its share; all loads are requested before the first is used (counts, then
    // keys) and the keys stay in registers.  0: no key.
    constexpr int kMaxG = 8, kPer = kMaxG * kKlCand / kKlThreads;
    int c[kMaxG + 1];                                            // c[g]: entries in the lists before g
    c[0] = 0;
#pragma unroll
    for (int g = 0; g < kMaxG; ++g) c[g + 1] = g < G ? ws_cnt[e * G + g] : 0;
#pragma unroll
    for (int g = 0; g < kMaxG; ++g) c[g + 1] += c[g];
    u64 key[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = (((tid & 63) << 4) | (tid >> 6)) + j * kKlThreads;
        int g = 0, base = 0;
#pragma unroll
        for (int x = 1; x < kMaxG; ++x)
            if (i >= c[x]) { g = x; base = c[x]; }
        key[j] = i < c[kMaxG] ? ws_keys[((size_t)e * G + g) * kKlCand + (i - base)] : 0ull;
    }
    u64 mx = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) mx = key[j] > mx ? key[j] : mx;
    // A bound that at least K keys reach.  First the K-th largest of the 512 maxima of thread pairs
    // (t, t + 512), on the logits alone: a 32-bit sort by half of the wavefronts; K pairs hold a key
    // at or above it, and about 1.3 K keys reach it.  With masses of equal logits more keys can reach it than the list
    // holds; then the K-th largest of the 1024 per-thread maxima on the whole 64-bit key: keys are
    // distinct, so exactly K threads reach that bound and at most kPer K keys do.  (The cheap bound
    // of the slices admits half as many keys again as the first one, and ranking them cost more
    // than this sort: measured.)
    constexpr int kCap = kPer * kKlMaxK;
    constexpr int kHalf = kKlThreads / 2;
    static_assert(kCap * 8 >= 2 * kKlThreads * 8, "the survivors' list doubles as the sort buffer");
    static_assert(kKlMaxK <= kHalf, "the K-th largest of the pair maxima exists");
    {
        uint32_t* b32 = reinterpret_cast<uint32_t*>(surv);
        if (tid >= kHalf) b32[2 * kHalf + tid - kHalf] = (uint32_t)(mx >> 32);      // (behind the sort's two halves)
        __syncthreads();
        uint32_t pm = (uint32_t)(mx >> 32);
        if (tid < kHalf) { const uint32_t o = b32[2 * kHalf + tid]; pm = o > pm ? o : pm; }
        const uint32_t srt = wg_sort_desc<kHalf>(pm, b32);
        if (tid == K - 1) tau_s = (u64)srt << 32;                // 0: fewer than K pairs hold a key: keep all
    }
    for (int attempt = 0;; ++attempt) {
        __syncthreads();                                         // tau_s written, the sort buffer read
        const u64 tau = tau_s;
        __syncthreads();                                         // (tau_s is rewritten in the second attempt)
        // (one atomic add per key: gathering them per wavefront first, as the slices do, costs more here)
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            if (key[j] != 0ull && key[j] >= tau) { const int p = atomicAdd(&nsurv, 1); if (p < kCap) surv[p] = key[j]; }
        }
        __syncthreads();
        if (nsurv <= kCap || attempt == 1) break;                // (uniform: every thread reads the same count)
        __syncthreads();
        if (tid == 0) nsurv = 0;
        const u64 srt = wg_sort_desc<kKlThreads>(mx, surv);
        if (tid == K - 1) tau_s = srt;
    }
    const int ns = nsurv < kCap ? nsurv : kCap;
    if (ns <= kHalf) {
        // The usual case: the survivors fit one key per thread of half the workgroup, and sorting
        // them there is cheaper than counting (every wavefront would read the whole list).
        const u64 mine = tid < ns ? surv[tid] : 0ull;
        __syncthreads();                                         // the list is in registers: its memory becomes the sort buffer
        const u64 srt = wg_sort_desc<kHalf>(mine, surv);
        if (tid < K) sorted[tid] = srt;                          // (ns >= K whenever K keys exist; K <= V is checked by the caller)
    } else {
        // Rank by counting.  A group of P = 1 or 2 adjacent lanes takes two survivors (each key
        // read from LDS serves two compares: the reads are what bounds this loop), every lane of the
        // group its part of the list, 8 keys per step (the loop waits for LDS once per step).
        const int nh = (ns + 1) >> 1;
        int P = 1;
        while (P < 8 && nh * (2 * P) <= kKlThreads) P *= 2;
        const int seg = ((ns + P - 1) / P + 7) & ~7;             // keys per part, whole steps
        const int lane = tid & 63;
        for (int t0 = 0; t0 < nh * P; t0 += kKlThreads) {
            const int idx = t0 + tid, i = idx / P, part = idx - i * P;
            const bool live0 = i < nh, live1 = i + nh < ns;
            const u64 mine0 = live0 ? surv[i] : ~0ull, mine1 = live1 ? surv[i + nh] : ~0ull;
            const int j0 = part * seg, j1 = live0 ? (j0 + seg < ns ? j0 + seg : ns) : 0;
            int r0 = 0, r1 = 0, j = j0;
            for (; j + 8 <= j1; j += 8) {
                ulonglong2 q[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) q[u] = *reinterpret_cast<const ulonglong2*>(surv + j + 2 * u);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    r0 += (q[u].x > mine0) + (q[u].y > mine0);
                    r1 += (q[u].x > mine1) + (q[u].y > mine1);
                }
            }
            for (; j < j1; ++j) { const u64 o = surv[j]; r0 += o > mine0 ? 1 : 0; r1 += o > mine1 ? 1 : 0; }
            // the P lanes of a group are adjacent and aligned: add their counts
            uint32_t r = (uint32_t)r0 | ((uint32_t)r1 << 16);   // (both below 2^13)
            if (P >= 2) r += xor_lane<1>(r, lane);
            if (P >= 4) r += xor_lane<2>(r, lane);
            if (P >= 8) r += xor_lane<4>(r, lane);
            if (part == 0) {
                if (live0 && (int)(r & 0xffffu) < K) sorted[r & 0xffffu] = mine0;
                if (live1 && (int)(r >> 16) < K) sorted[r >> 16] = mine1;
            }
        }
    }
    __syncthreads();
    for (int r = tid; r < K; r += kKlThreads) {
        out_support[(size_t)e * K + r] = key_id(sorted[r]);
        out_zt[(size_t)e * K + r] = key_value(sorted[r]);
    }
}

// Draft logits z_q[e][r] = h_draft[e] . W_lm[support[e][r]] for the 16 rows r = 16 blockIdx.x + ...
__global__ void __launch_bounds__(256)
kl_draft_logits_kernel(const uint16_t* __restrict__ h_draft, int d, const uint16_t* __restrict__ W_lm, int K,
                       const int32_t* __restrict__ support, float* __restrict__ out_zq) {
    extern __shared__ __align__(16) unsigned char kl_smem[];
    uint16_t* hs = reinterpret_cast<uint16_t*>(kl_smem);            // [d] draft hidden state of the event
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int e = blockIdx.y;
    const int r0 = 16 * blockIdx.x + 4 * w;                         // this wavefront's 4 rows
    const int32_t* sup = support + (size_t)e * K;
    const uint16_t* row[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) row[u] = W_lm + (size_t)sup[r0 + u < K ? r0 + u : K - 1] * d;   // past the end: a valid row again
    for (int i = tid; i < d / 8; i += 256)
        reinterpret_cast<u32x4*>(hs)[i] = *(gvec_ptr)(h_draft + (size_t)e * d + 8 * i);
    __syncthreads();
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < d / 8; p0 += 64) {
        const int p = p0 + lane < d / 8 ? p0 + lane : d / 8 - 1;      // ragged end: clamp, then weigh by zero
        const bool live = p0 + lane < d / 8;
        u32x4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = *(gvec_ptr)(row[u] + 8 * p);
        u32x4 b = reinterpret_cast<const u32x4*>(hs)[p];
        if (!live) b = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[u] = fmaf(__uint_as_float(a[u][q] << 16), __uint_as_float(b[q] << 16), acc[u]);
                acc[u] = fmaf(__uint_as_float(a[u][q] & 0xffff0000u), __uint_as_float(b[q] & 0xffff0000u), acc[u]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const float t = wave_sum(acc[u]);
        if (lane == 0 && r0 + u < K) out_zq[(size_t)e * K + r0 + u] = t;
    }
}

// KL = sum_i p_i (a_i - b_i) - logZ_a + logZ_b with a = z_t / T, b = z_q / T; one wavefront per event.
__global__ void __launch_bounds__(64)
kl_divergence_kernel(const float* __restrict__ zt, const float* __restrict__ zq, int K, float inv_T,
                     float* __restrict__ out_kl) {
    const int lane = threadIdx.x, e = blockIdx.x;
    zt += (size_t)e * K;
    zq += (size_t)e * K;
    float ma = -INFINITY, mb = -INFINITY;
    for (int r = lane; r < K; r += 64) {
        ma = fmaxf(ma, zt[r] * inv_T);
        mb = fmaxf(mb, zq[r] * inv_T);
    }
    ma = wave_max(ma);
    mb = wave_max(mb);
    float sa = 0.f, sb = 0.f, cross = 0.f;
    for (int r = lane; r < K; r += 64) {
        const float a = zt[r] * inv_T, b = zq[r] * inv_T;
        const float ea = __expf(a - ma);
        sa += ea;
        sb += __expf(b - mb);
        cross += ea * (a - b);
    }
    sa = wave_sum(sa); sb = wave_sum(sb); cross = wave_sum(cross);
    if (lane == 0) out_kl[e] = cross / sa - (ma + __logf(sa)) + (mb + __logf(sb));
}

int kl_gate_slices(int V) { return V >= 32768 ? 8 : 1; }

size_t kl_gate_workspace_bytes(int E, int V) {
    const size_t G = (size_t)kl_gate_slices(V);
    return (size_t)E * G * kKlCand * 8 + ((size_t)E * G * 4 + 255) / 256 * 256;
}

hipError_t launch_kl_gate(const float* z_target, int E, int V, const void* h_draft, int d, const void* W_lm,
                          int K, float T, int32_t* out_support, float* out_zt, float* out_zq, float* out_kl,
                          void* workspace, hipStream_t stream) {
    if (K < 1 || K > kKlMaxK || K > V || d % 8 != 0 || (size_t)d * 2 > 48 * 1024) return hipErrorInvalidValue;
    const int G = kl_gate_slices(V);
    const int slice = ((V + G - 1) / G + 3) / 4 * 4;
    u64* ws_keys = static_cast<u64*>(workspace);
    int* ws_cnt = reinterpret_cast<int*>(ws_keys + (size_t)E * G * kKlCand);
    // 16-byte loads per thread that cover a slice, when the logits allow them
    const bool vec = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(z_target) & 15) == 0;
    const int per_thread = (slice / 4 + kKlThreads - 1) / kKlThreads;
    auto slices = kl_select_slices_kernel<0>;
    if (vec && per_thread <= 2) slices = kl_select_slices_kernel<2>;
    else if (vec && per_thread <= 5) slices = kl_select_slices_kernel<5>;
    else if (vec && per_thread <= 8) slices = kl_select_slices_kernel<8>;
    hipLaunchKernelGGL(slices, dim3(G, E), dim3(kKlThreads), 0, stream, z_target, V, K, G, slice, ws_keys, ws_cnt);
    hipLaunchKernelGGL(kl_select_final_kernel, dim3(E), dim3(kKlThreads), 0, stream, ws_keys, ws_cnt, G, K,
                       out_support, out_zt);
    hipLaunchKernelGGL(kl_draft_logits_kernel, dim3((K + 15) / 16, E), dim3(256), (size_t)d * 2, stream,
                       static_cast<const uint16_t*>(h_draft), d, static_cast<const uint16_t*>(W_lm), K, out_support,
                       out_zq);
    hipLaunchKernelGGL(kl_divergence_kernel, dim3(E), dim3(64), 0, stream, out_zt, out_zq, K, 1.0f / T, out_kl);
    return hipGetLastError();
}

}  // namespace evospec
