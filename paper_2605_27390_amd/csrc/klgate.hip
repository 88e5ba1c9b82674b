// Retained-support KL gate of Path B (EvoSpec paper, Sec. "Online parameter update", Eq. 5 and
// the admission rule around it; Algorithm 1, Path B): per verification event, the K_logit largest
// target logits are kept; the draft model's logits on the same ids (Eq. 1: h_draft . W_LM[i]) and
// the temperature T_KD turn both into distributions p, q on that support; the event is admitted
// when D_KL(p || q) exceeds the gate.
//
// One workgroup of 16 wavefronts per event, everything in one launch:
//  1. exact selection of the K largest (logit, id) keys.  Common path, two sweeps: every thread
//     takes the maximum of its share; the K-th largest of these 1024 maxima is a lower bound of the
//     K-th largest key, so the keys that reach it (a few hundred) are collected and ranked by
//     counting.  If more than 2048 reach it (masses of equal logits), radix select on the 64-bit
//     key instead (11 bits per pass, histogram in LDS, a pass is skipped as soon as the bin that
//     holds the K-th key is taken whole), then a collecting sweep and the same ranking;
//  2. draft logits: one wavefront per support row, 16 bytes per lane and load, h in LDS;
//  3. log-sum-exp of both logit vectors and the divergence, by one wavefront.
// Latency bound: per event it reads the target logits a few times (they stay in L2) and K rows
// of W_LM.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"
#include "launch.hpp"

namespace evospec {

namespace {
constexpr int kKlThreads = 1024;
constexpr int kKlWaves = kKlThreads / 64;
constexpr int kKlMaxK = 256;
constexpr int kKlBits = 11;
constexpr int kKlBins = 1 << kKlBits;
constexpr int kKlCand = 2048;                 // candidates the common path can rank

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
}  // namespace

__global__ void __launch_bounds__(kKlThreads)
kl_gate_kernel(const float* __restrict__ z_target, int V, const uint16_t* __restrict__ h_draft, int d,
               const uint16_t* __restrict__ W_lm, int K, float inv_T,
               int32_t* __restrict__ out_support, float* __restrict__ out_zt, float* __restrict__ out_zq,
               float* __restrict__ out_kl) {
    extern __shared__ __align__(16) unsigned char kl_smem[];
    uint16_t* hs = reinterpret_cast<uint16_t*>(kl_smem);            // [d] draft hidden state
    __shared__ uint32_t hist[kKlBins];
    __shared__ u64 sel[kKlMaxK], sorted[kKlMaxK];
    __shared__ u64 tmax[kKlThreads], cand[kKlCand];
    __shared__ u64 tau0_s;
    __shared__ int ncand;
    __shared__ float zq_s[kKlMaxK];
    __shared__ uint32_t lane_tot[64];
    __shared__ u64 prefix_s;
    __shared__ int need_s, nsel, done_s;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int e = blockIdx.x;
    const float* z = z_target + (size_t)e * V;

    for (int i = tid; i < d / 8; i += kKlThreads)
        reinterpret_cast<u32x4*>(hs)[i] = *(gvec_ptr)(h_draft + (size_t)e * d + 8 * i);
    if (tid == 0) { prefix_s = 0; need_s = K; nsel = 0; done_s = 0; ncand = 0; tau0_s = 0; }

    // ---- 1a. common path: bound from the per-thread maxima
    {
        u64 mx = 0;
        for (int i = tid; i < V; i += kKlThreads) {
            const u64 key = make_key(z[i], i);
            mx = key > mx ? key : mx;
        }
        tmax[tid] = mx;
    }
    __syncthreads();
    {
        const u64 mine = tmax[tid];
        int r = 0;
        for (int j = 0; j < kKlThreads; ++j) r += tmax[j] > mine ? 1 : 0;
        if (mine != 0 && r == K - 1) tau0_s = mine;              // keys are distinct: one thread at most
    }
    __syncthreads();
    const u64 tau0 = tau0_s;                                     // 0: fewer than K threads saw a key
    for (int i = tid; i < V; i += kKlThreads) {
        const u64 key = make_key(z[i], i);
        if (key >= tau0) {
            const int p = atomicAdd(&ncand, 1);
            if (p < kKlCand) cand[p] = key;
        }
    }
    __syncthreads();
    const int nc = ncand;
    if (nc <= kKlCand) {
        for (int t = tid; t < nc; t += kKlThreads) {
            const u64 mine = cand[t];
            int r = 0;
            for (int j = 0; j < nc; ++j) r += cand[j] > mine ? 1 : 0;
            if (r < K) sorted[r] = mine;
        }
    } else {

    // ---- 1. radix select: after a pass, prefix holds the top `done` bits of the K-th largest key
    // and need the number of keys still to take among those that share them
    int done = 0;
    while (done < 64) {
        const int nb = 64 - done < kKlBits ? 64 - done : kKlBits;
        const int shift = 64 - done - nb;
        for (int i = tid; i < kKlBins; i += kKlThreads) hist[i] = 0;
        __syncthreads();
        const u64 prefix = prefix_s;
        for (int i = tid; i < V; i += kKlThreads) {
            const u64 key = make_key(z[i], i);
            if (done == 0 || (key >> (64 - done)) == (prefix >> (64 - done)))
                atomicAdd(&hist[(uint32_t)(key >> shift) & ((1u << nb) - 1u)], 1u);
        }
        __syncthreads();
        if (w == 0) {
            // bins from the top: lane l owns bins [32 (63 - l), +32), so lane 0 holds the largest
            const int need = need_s;
            const int b0 = 32 * (63 - lane);
            uint32_t tot = 0;
            for (int j = 0; j < 32; ++j) tot += hist[b0 + j];
            lane_tot[lane] = tot;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            uint32_t above = 0;                                  // keys in bins owned by lower lanes (larger bins)
            for (int j = 0; j < lane; ++j) above += lane_tot[j];
            if (above < (uint32_t)need && above + tot >= (uint32_t)need) {   // exactly one lane
                uint32_t acc = above;
                for (int j = 31; j >= 0; --j) {
                    const uint32_t c = hist[b0 + j];
                    if (acc + c >= (uint32_t)need) {
                        prefix_s = prefix | ((u64)(b0 + j) << shift);
                        need_s = need - (int)acc;
                        done_s = (c == (uint32_t)need - acc) ? 1 : 0;    // the whole bin is taken
                        break;
                    }
                    acc += c;
                }
            }
        }
        __syncthreads();
        done += nb;
        if (done_s) break;
    }
    // every key >= threshold is one of the K largest (keys are distinct; the bits below `done` are 0)
    const u64 thr = prefix_s;
    for (int i = tid; i < V; i += kKlThreads) {
        const u64 key = make_key(z[i], i);
        if (key >= thr) {
            const int p = atomicAdd(&nsel, 1);
            if (p < kKlMaxK) sel[p] = key;
        }
    }
    __syncthreads();
    if (tid < K) {
        const u64 mine = sel[tid];
        int r = 0;
        for (int j = 0; j < K; ++j) r += sel[j] > mine ? 1 : 0;
        sorted[r] = mine;
    }
    }   // radix path
    __syncthreads();

    // ---- 2. draft logits on the support: wavefront w takes rows w, w + 16, ..., four at a time so
    // that their loads are in flight together
    for (int r0 = w; r0 < K; r0 += 4 * kKlWaves) {
        const uint16_t* row[4];
        float acc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + u * kKlWaves;
            row[u] = W_lm + (size_t)key_id(sorted[r < K ? r : r0]) * d;      // past the end: a valid row again
            acc[u] = 0.f;
        }
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
            const int r = r0 + u * kKlWaves;
            if (lane == 0 && r < K) zq_s[r] = t;
        }
    }
    __syncthreads();

    // ---- 3. divergence: KL = sum_i p_i ((a_i - b_i)) - logZ_a + logZ_b with a = z_t / T, b = z_q / T
    if (w == 0) {
        float ma = -INFINITY, mb = -INFINITY;
        for (int r = lane; r < K; r += 64) {
            ma = fmaxf(ma, key_value(sorted[r]) * inv_T);
            mb = fmaxf(mb, zq_s[r] * inv_T);
        }
        ma = wave_max(ma);
        mb = wave_max(mb);
        float sa = 0.f, sb = 0.f, cross = 0.f;
        for (int r = lane; r < K; r += 64) {
            const float a = key_value(sorted[r]) * inv_T, b = zq_s[r] * inv_T;
            const float ea = __expf(a - ma);
            sa += ea;
            sb += __expf(b - mb);
            cross += ea * (a - b);
        }
        sa = wave_sum(sa); sb = wave_sum(sb); cross = wave_sum(cross);
        if (lane == 0) out_kl[e] = cross / sa - (ma + __logf(sa)) + (mb + __logf(sb));
    }
    for (int r = tid; r < K; r += kKlThreads) {
        out_support[(size_t)e * K + r] = key_id(sorted[r]);
        out_zt[(size_t)e * K + r] = key_value(sorted[r]);
        out_zq[(size_t)e * K + r] = zq_s[r];
    }
}

hipError_t launch_kl_gate(const float* z_target, int E, int V, const void* h_draft, int d, const void* W_lm,
                          int K, float T, int32_t* out_support, float* out_zt, float* out_zq, float* out_kl,
                          hipStream_t stream) {
    if (K < 1 || K > kKlMaxK || K > V || d % 8 != 0 || (size_t)d * 2 > 48 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kl_gate_kernel, dim3(E), dim3(kKlThreads), (size_t)d * 2, stream, z_target, V,
                       static_cast<const uint16_t*>(h_draft), d, static_cast<const uint16_t*>(W_lm), K, 1.0f / T,
                       out_support, out_zt, out_zq, out_kl);
    return hipGetLastError();
}

}  // namespace evospec
