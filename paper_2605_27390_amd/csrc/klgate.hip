// Retained-support KL gate of Path B (EvoSpec paper, Sec. "Online parameter update", Eq. 5 and
// the admission rule around it; Algorithm 1, Path B): per verification event, the K_logit largest
// target logits are kept; the draft model's logits on the same ids (Eq. 1: h_draft . W_LM[i]) and
// the temperature T_KD turn both into distributions p, q on that support; the event is admitted
// when D_KL(p || q) exceeds the gate.
//
// Four launches:
//  1. kl_select_slices_kernel, one workgroup of 16 wavefronts per (eighth of the vocabulary, event):
//     every thread takes the maximum of its share of the slice; a value that K of these 1024 maxima
//     reach (from one sort per wavefront) is a lower bound of the slice's K-th largest logit, so the
//     logits that reach it (a few hundred) go to the workspace as 64-bit (logit, id) keys.  If more than 2048 reach it (masses
//     of equal logits), radix select on the key instead (11 bits per pass, histogram in LDS, a pass
//     is skipped as soon as the bin that holds the K-th key is taken whole) leaves exactly K;
//  2. kl_select_final_kernel, one workgroup per event: the same bound over the slices' candidates,
//     the survivors ranked by counting: the support, by decreasing key;
//  3. kl_draft_logits_kernel, one workgroup of 4 wavefronts per 16 support rows of an event, so that
//     the E x K rows of W_LM (the bulk of the bytes) are spread over the whole GPU: a wavefront
//     takes 4 rows at a time, 16 bytes per lane and load, h in LDS;
//  4. kl_divergence_kernel, one wavefront per event: log-sum-exp of both logit vectors and D_KL.
// Latency bound: per event the target logits are read twice (they stay in L2) and K rows of W_LM once.
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

// The K-th largest (counting repeats) of the 1024 values v, one per thread, by radix select on
// their top `bits` bits (the rest must be zero); every thread of the workgroup calls it.
__device__ __forceinline__ u64 kth_largest_1024(u64 v, int K, int bits, uint32_t* hist, u64* prefix_s, int* need_s) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid == 0) { *prefix_s = 0; *need_s = K; }
    int done = 0;
    while (done < bits) {
        const int nb = bits - done < kKlBits ? bits - done : kKlBits;
        const int shift = 64 - done - nb;
        for (int i = tid; i < kKlBins; i += kKlThreads) hist[i] = 0;
        __syncthreads();
        const u64 prefix = *prefix_s;
        if (done == 0 || (v >> (64 - done)) == (prefix >> (64 - done)))
            atomicAdd(&hist[(uint32_t)(v >> shift) & ((1u << nb) - 1u)], 1u);
        __syncthreads();
        if (w == 0) {
            int bin = 0, above = 0, count = 0;
            const int need = *need_s;
            find_bin(hist, lane, need, &bin, &above, &count);
            if (count > 0) {
                *prefix_s = prefix | ((u64)bin << shift);
                // 0: the whole bin is taken and the value bits are resolved, so the bound cannot loosen: stop
                *need_s = (count == need - above && done + nb >= 32) ? 0 : need - above;
            }
        }
        __syncthreads();
        done += nb;
        if (*need_s == 0) break;                                 // (prefix with zero low bits bounds exactly K values)
    }
    return *prefix_s;
}

// A lower bound of the K-th largest (counting repeats) of the 1024 values v, one per thread, without
// a selection: every wavefront sorts its 64 values; with q = ceil(K / 16), each of the 16
// wavefronts holds q values at or above its own q-th largest, so K values reach the smallest of the
// 16.  (Looser than the exact K-th largest, which costs three radix passes with their barriers.)
__device__ __forceinline__ u64 kth_bound_1024(u64 v, int K, u64* wave_q /*LDS [16]*/) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int q = (K + 15) >> 4;                               // K <= 1024
    const u64 s = wave_sort_desc(v, lane);
    if (lane == q - 1) wave_q[w] = s;
    __syncthreads();
    u64 t = wave_q[0];
#pragma unroll
    for (int i = 1; i < kKlThreads / 64; ++i) { const u64 o = wave_q[i]; t = o < t ? o : t; }
    return t;
}
}  // namespace

// Stage 1 of the selection, one workgroup per (slice g of the vocabulary, event e): the keys of the
// slice that can still be among the event's K largest go to the workspace, unranked:
// ws_keys[(e * G + g) * kKlCand + ...], their number to ws_cnt[e * G + g].
__global__ void __launch_bounds__(kKlThreads)
kl_select_slices_kernel(const float* __restrict__ z_target, int V, int K, int G, int slice,
                        u64* __restrict__ ws_keys, int* __restrict__ ws_cnt) {
    __shared__ __align__(16) uint32_t hist[kKlBins];
    __shared__ u64 cand[kKlCand];
    __shared__ int ncand;
    __shared__ u64 prefix_s;
    __shared__ u64 wave_q[kKlThreads / 64];
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
    // logit from below (plain float compares; 16-byte loads when the logits are 16-byte aligned)
    const bool vec = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(z_target) & 15) == 0;
    float mx = -INFINITY;
    bool any = false;
    if (vec) {
        for (int i = lo + 4 * tid; i < hi; i += 4 * kKlThreads) {
            const float4 q = *reinterpret_cast<const float4*>(z + i);
            mx = fmaxf(fmaxf(mx, fmaxf(q.x, q.y)), fmaxf(q.z, q.w));
            any = true;
        }
    } else {
        for (int i = lo + tid; i < hi; i += kKlThreads) { mx = fmaxf(mx, z[i]); any = true; }
    }
    // (absent threads contribute 0, below every real value)
    const u64 kth = kth_bound_1024(any ? (u64)f32_to_ordered(mx) << 32 : 0ull, Kl, wave_q);
    const float tau0 = kth ? ordered_to_f32((uint32_t)(kth >> 32)) : -INFINITY;   // too few threads saw a logit: keep all
    auto consider = [&](float v, int i) {
        if (v >= tau0) {
            const int p = atomicAdd(&ncand, 1);
            if (p < kKlCand) cand[p] = make_key(v, i);
        }
    };
    if (vec) {
        for (int i = lo + 4 * tid; i < hi; i += 4 * kKlThreads) {
            const float4 q = *reinterpret_cast<const float4*>(z + i);
            consider(q.x, i); consider(q.y, i + 1); consider(q.z, i + 2); consider(q.w, i + 3);
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
    __shared__ __align__(16) uint32_t hist[kKlBins];
    __shared__ int need_s;
    __shared__ u64 surv[16 * kKlMaxK];
    __shared__ u64 sorted[kKlMaxK];
    __shared__ u64 tau_s;
    __shared__ int nsurv;
    const int tid = threadIdx.x, e = blockIdx.x;
    if (tid == 0) nsurv = 0;
    u64 mx = 0;
    for (int g = 0; g < G; ++g) {
        const int n = ws_cnt[e * G + g];
        const u64* lst = ws_keys + ((size_t)e * G + g) * kKlCand;
        for (int i = tid; i < n; i += kKlThreads) { const u64 key = lst[i]; mx = key > mx ? key : mx; }
    }
    __syncthreads();
    const u64 tau = kth_largest_1024(mx, K, 64, hist, &tau_s, &need_s);   // 0: fewer than K threads hold a key: keep all
    for (int g = 0; g < G; ++g) {
        const int n = ws_cnt[e * G + g];
        const u64* lst = ws_keys + ((size_t)e * G + g) * kKlCand;
        for (int i = tid; i < n; i += kKlThreads) {
            const u64 key = lst[i];
            if (key >= tau) { const int p = atomicAdd(&nsurv, 1); if (p < 16 * kKlMaxK) surv[p] = key; }
        }
    }
    __syncthreads();
    const int ns = nsurv < 16 * kKlMaxK ? nsurv : 16 * kKlMaxK;
    for (int t = tid; t < ns; t += kKlThreads) {
        const u64 mine = surv[t];
        int r = 0;
        for (int j = 0; j < ns; ++j) r += surv[j] > mine ? 1 : 0;
        if (r < K) sorted[r] = mine;
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
    hipLaunchKernelGGL(kl_select_slices_kernel, dim3(G, E), dim3(kKlThreads), 0, stream, z_target, V, K, G, slice,
                       ws_keys, ws_cnt);
    hipLaunchKernelGGL(kl_select_final_kernel, dim3(E), dim3(kKlThreads), 0, stream, ws_keys, ws_cnt, G, K,
                       out_support, out_zt);
    hipLaunchKernelGGL(kl_draft_logits_kernel, dim3((K + 15) / 16, E), dim3(256), (size_t)d * 2, stream,
                       static_cast<const uint16_t*>(h_draft), d, static_cast<const uint16_t*>(W_lm), K, out_support,
                       out_zq);
    hipLaunchKernelGGL(kl_divergence_kernel, dim3(E), dim3(64), 0, stream, out_zt, out_zq, K, 1.0f / T, out_kl);
    return hipGetLastError();
}

}  // namespace evospec
