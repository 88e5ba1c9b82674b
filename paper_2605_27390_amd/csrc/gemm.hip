// Large-M variant of the restricted head (Eq. 1 of the EvoSpec paper on the active set of Eq. 3):
// with hundreds of draft rows in flight (batched serving, one shared core for all sequences) the
// projection is a dense contraction and bound by the matrix cores, not by the stream of W_act.
//
// One workgroup of four wavefronts (one per SIMD) computes a 256 x 256 tile of z = W_act h^T
// (256 active rows x 256 draft rows) over the whole hidden dimension.  Both operands travel
// HBM/L2 -> LDS with direct-to-LDS loads (no staging registers) in chunks of 32 hidden elements
// through a ring of four stages; every wavefront owns a 128 x 128 quadrant = 8 x 8 accumulators
// of v_mfma_f32_16x16x32_bf16, which fill the 256 accumulation registers of a lane, and reads
// the operands of the next chunk from LDS while the matrix cores work on the current one.
// The logits never leave the registers: each wavefront reduces its quadrant, per draft row, to
// the same partial the streaming kernel leaves per slab (max, sum-exp, k best keys), for a
// "slab" of its 128 rows.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "common.hpp"
#include "launch.hpp"
#include "plan.hpp"

namespace evospec {

namespace {

constexpr int kGK = kGemmKChunk;              // hidden elements per chunk (one MFMA k-step)
constexpr int kGStages = 4;                   // ring of LDS stages
constexpr int kGOperandBytes = kGemmTile * kGK * 2;           // 16 KB: 256 rows x 64 B, no padding
constexpr int kGStageBytes = 2 * kGOperandBytes;              // W_act rows, then h rows
constexpr size_t kGLds = (size_t)kGStages * kGStageBytes;     // 128 KB
constexpr int kGLoads = kGemmTile / 16 / 4;                   // direct-to-LDS loads per wavefront, operand and chunk
constexpr int kGEpiBytes = 16 * kGemmSlab * 8 + kGemmSlab * 4;   // per wavefront: key lists, ids

static_assert(kGLds <= (size_t)kLdsLimit, "operand ring exceeds the LDS of a compute unit");
static_assert(4 * kGEpiBytes <= (int)kGLds, "epilogue lists alias the operand ring");
static_assert(kGLoads == 4, "four wavefronts share 16 blocks of 16 rows");

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// A row of a stage holds 32 hidden elements = four 16-byte pieces.  Piece p of row r sits in
// slot p ^ swz(r).  The 16 lanes of an MFMA operand read take one piece of 16 consecutive rows:
// with this swizzle any 8 consecutive rows fall into 8 different 16-byte columns of a 128-byte
// bank window and any 16 into 16 different columns of a 256-byte window, so the read is free of
// bank conflicts for either bank count.  The direct-to-LDS load writes lane L of a wavefront to
// byte 16 L of a 1 KB block (16 rows), so the swizzle is applied on the source side: the lane
// that fills (row, slot) fetches piece slot ^ swz(row).
__device__ __forceinline__ int swz(int row) { return (((row & 15) >> 1) + ((row & 15) >> 3)) & 3; }

// Accumulators are pinned to the accumulation registers: with all 256 of them live, the
// register allocator must not be left to shuffle them through the other file.
__device__ __forceinline__ void mfma_acc(f32x4& c, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

}  // namespace

__global__ void __launch_bounds__(256, 1)
lmhead_gemm_kernel(const uint16_t* __restrict__ h, int M, int d,
                   const uint16_t* __restrict__ W, const int32_t* __restrict__ ids, int V_act, int k,
                   int m_tiles, u64* __restrict__ part_keys, float2* __restrict__ part_stats) {
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int wv = w >> 1, wm = w & 1;                             // quadrant: active-row half, draft-row half

    // Workgroups are handed to the 8 XCDs round robin; renumber them so that the m_tiles tiles
    // that read the same 256 rows of W_act run on one XCD (one L2) at about the same time.
    const int nb = gridDim.x, b = blockIdx.x;
    const int xcd = b & 7, full = nb >> 3, rem = nb & 7;
    const int logical = xcd * full + (xcd < rem ? xcd : rem) + (b >> 3);
    const int tile_v = logical / m_tiles, tile_m = logical - tile_v * m_tiles;
    const int v0 = tile_v * kGemmTile, m0 = tile_m * kGemmTile;

    // direct-to-LDS loads of this wavefront: blocks of 16 rows number 4 w + i of either operand
    const uint16_t* asrc[kGLoads];
    const uint16_t* bsrc[kGLoads];
#pragma unroll
    for (int i = 0; i < kGLoads; ++i) {
        const int r = (4 * w + i) * 16 + (lane >> 2);
        const int piece = (lane & 3) ^ swz(r);
        asrc[i] = W + (size_t)min(v0 + r, V_act - 1) * d + piece * 8;      // rows past the end repeat
        bsrc[i] = h + (size_t)min(m0 + r, M - 1) * d + piece * 8;          // the last one, masked later
    }
    const int nchunks = d / kGK;                                   // d is a multiple of kGK here
    // Load number j (0..7) of chunk c: block i = j/2 of W_act rows (j even) or of h rows (j odd).
    // Chunks past the end repeat the last one into a stage nobody reads again, which keeps the
    // number of loads in flight, and with it every wait below, the same in every iteration.
    auto issue_one = [&](int c, int j) {
        const size_t koff = (size_t)min(c, nchunks - 1) * kGK;
        unsigned char* dst = smem + (c & (kGStages - 1)) * kGStageBytes + (j & 1) * kGOperandBytes +
                             (4 * w + (j >> 1)) * 1024;
        const uint16_t* src = ((j & 1) ? bsrc[j >> 1] : asrc[j >> 1]) + koff;
        __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 16, 0, 0);
    };

    f32x4 acc[8][8];
#pragma unroll
    for (int rg = 0; rg < 8; ++rg)
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) acc[rg][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // operand reads: lane (n16, g) takes piece g of row n16 of each 16-row block of its quadrant
    const int a_rd = (wv * 128 + n16) * (kGK * 2) + ((g ^ swz(n16)) * 16);
    const int b_rd = kGOperandBytes + (wm * 128 + n16) * (kGK * 2) + ((g ^ swz(n16)) * 16);
    bf16x8 opa[2][8], opb[2][8];
    auto read_a = [&](auto SET, int c, int i) {
        opa[decltype(SET)::value][i] = *reinterpret_cast<const bf16x8*>(
            smem + (c & (kGStages - 1)) * kGStageBytes + a_rd + i * 16 * (kGK * 2));
    };
    auto read_b = [&](auto SET, int c, int i) {
        opb[decltype(SET)::value][i] = *reinterpret_cast<const bf16x8*>(
            smem + (c & (kGStages - 1)) * kGStageBytes + b_rd + i * 16 * (kGK * 2));
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;

    // One chunk: 64 MFMAs on the operands in registers (set CUR); in the gaps, the 16 operand
    // reads of chunk c+1 (into set 1 - CUR) and the 8 loads of chunk c+4 (into the stage of
    // chunk c, which every wavefront finished reading before the barrier).  At the top, chunks up
    // to c+3 have been requested, in order, 8 loads each: chunk c+1 has landed once at most 16
    // loads are outstanding.
    auto step = [&](auto CUR, int c) {
        constexpr int P = decltype(CUR)::value;
        using NXT = std::integral_constant<int, 1 - P>;
        asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");
#pragma unroll
        for (int rg = 0; rg < 8; ++rg) {
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) mfma_acc(acc[rg][mb], opa[P][rg], opb[P][mb]);
#pragma unroll
            for (int q = 3 * rg; q < 3 * rg + 3 && q < 16; ++q) {
                // (a stage past the last chunk holds stale data that is never used)
                if (q & 1) read_a(NXT{}, c + 1, q >> 1);
                else read_b(NXT{}, c + 1, q >> 1);
            }
            issue_one(c + 4, rg);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };

#pragma unroll
    for (int c = 0; c < kGStages; ++c)
#pragma unroll
        for (int j = 0; j < 8; ++j) issue_one(c, j);
    // chunk 0 must have landed before its operands are read
    asm volatile("s_waitcnt vmcnt(24)\n\ts_barrier" ::: "memory");
#pragma unroll
    for (int i = 0; i < 8; ++i) { read_b(S0{}, 0, i); read_a(S0{}, 0, i); }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 7" ::: "memory");

    int c = 0;
    for (; c + 1 < nchunks; c += 2) {
        step(S0{}, c);
        step(S1{}, c + 1);
    }
    if (c < nchunks) step(S0{}, c);
    // the last MFMAs drain before the accumulators are read; the ring is dead once the trailing
    // loads have landed and every wavefront is here
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- epilogue: wave-local from here on; the operand buffers are dead (all waves are past the
    // last barrier), each wavefront takes its own piece of them
    const int vrow0 = v0 + wv * kGemmSlab;
    const int nvalid = min(kGemmSlab, V_act - vrow0);
    if (nvalid <= 0) return;                                       // quadrant wholly past the active set
    const int slab = tile_v * (kGemmTile / kGemmSlab) + wv;
    unsigned char* my = smem + (size_t)w * kGEpiBytes;
    u64* list = reinterpret_cast<u64*>(my);                        // [16][128] surviving keys per draft row
    int32_t* Ids = reinterpret_cast<int32_t*>(my + 16 * kGemmSlab * 8);   // [128]

#pragma unroll
    for (int i = 0; i < kGemmSlab / 64; ++i) {
        const int r = vrow0 + lane + 64 * i;
        Ids[lane + 64 * i] = r < V_act ? (ids ? ids[r] : r) : 0x7fffffff;
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    // lane's entries: active row (within the quadrant) 16 rg + 4 g + j  <->  bit 4 rg + j
    int32_t idv[32];
    uint32_t vmask = 0;
#pragma unroll
    for (int rg = 0; rg < 8; ++rg) {
        const int4 q = *reinterpret_cast<const int4*>(Ids + rg * 16 + 4 * g);
        idv[4 * rg + 0] = q.x; idv[4 * rg + 1] = q.y; idv[4 * rg + 2] = q.z; idv[4 * rg + 3] = q.w;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (rg * 16 + 4 * g + j < nvalid) vmask |= 1u << (4 * rg + j);
    }

#pragma unroll
    for (int mb = 0; mb < 8; ++mb) {
        const int m = m0 + wm * 128 + mb * 16 + n16;
        const bool m_ok = m < M;
        float v[32];
#pragma unroll
        for (int rg = 0; rg < 8; ++rg)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[4 * rg + j] = ((vmask >> (4 * rg + j)) & 1u) ? acc[rg][mb][j] : -INFINITY;

        // statistics of the quadrant's 128 logits of draft row m (4 lanes x 32 entries)
        float t[8];
#pragma unroll
        for (int rg = 0; rg < 8; ++rg)
            t[rg] = fmaxf(fmaxf(v[4 * rg], v[4 * rg + 1]), fmaxf(v[4 * rg + 2], v[4 * rg + 3]));
        float vmax = t[0];
#pragma unroll
        for (int rg = 1; rg < 8; ++rg) vmax = fmaxf(vmax, t[rg]);
        vmax = fmaxf(vmax, __shfl_xor(vmax, 16));
        vmax = fmaxf(vmax, __shfl_xor(vmax, 32));
        float se = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) se += __expf(v[i] - vmax);
        se += __shfl_xor(se, 16);
        se += __shfl_xor(se, 32);
        const size_t slot = (size_t)slab * M + (m_ok ? m : 0);
        if (g == 0 && m_ok) part_stats[slot] = make_float2(vmax, se);

        // lower bound of the k-th best logit: the k-th largest distinct maximum of the 32 groups
        // of 4 entries (k rounds of "take the maximum, strike it out"); with more than 32 wanted,
        // or fewer distinct maxima than k, every valid entry is ranked
        float tau = -INFINITY;
        if (k <= 32) {
            for (int r = 0; r < k; ++r) {
                float lm = t[0];
#pragma unroll
                for (int rg = 1; rg < 8; ++rg) lm = fmaxf(lm, t[rg]);
                lm = fmaxf(lm, __shfl_xor(lm, 16));
                lm = fmaxf(lm, __shfl_xor(lm, 32));
                tau = lm;
#pragma unroll
                for (int rg = 0; rg < 8; ++rg) t[rg] = t[rg] >= lm ? -INFINITY : t[rg];
            }
        }
        uint32_t mask = 0;
#pragma unroll
        for (int i = 0; i < 32; ++i) mask |= (v[i] >= tau ? 1u : 0u) << i;
        mask &= vmask;
        const int cnt = __popc(mask);
        const int c0 = __shfl(cnt, n16), c1 = __shfl(cnt, n16 + 16), c2 = __shfl(cnt, n16 + 32),
                  c3 = __shfl(cnt, n16 + 48);
        const int base = (g > 0 ? c0 : 0) + (g > 1 ? c1 : 0) + (g > 2 ? c2 : 0);
        const int L = c0 + c1 + c2 + c3;                           // <= 128
        u64* mine = list + n16 * kGemmSlab;
#pragma unroll
        for (int i = 0; i < 32; ++i)
            if ((mask >> i) & 1u) mine[base + __popc(mask & ((1u << i) - 1u))] = make_key(v[i], idv[i]);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

        // exact rank of every survivor among the survivors of its draft row (keys are distinct)
        u64* dst = part_keys + slot * k;
        for (int e = g; e < L; e += 4) {
            const u64 key = mine[e];
            int rank = 0;
            for (int f = 0; f < L; ++f) rank += mine[f] > key ? 1 : 0;
            if (rank < k && m_ok) dst[rank] = key;
        }
        if (m_ok)
            for (int r = L + g; r < k; r += 4) dst[r] = 0;         // fewer than k rows in this slab
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

hipError_t launch_gemm_partials(const void* h, int M, int d, const void* W, const int32_t* ids, int V_act,
                                int k, void* keys, void* stats, hipStream_t stream) {
    const int v_tiles = (V_act + kGemmTile - 1) / kGemmTile;
    const int m_tiles = (M + kGemmTile - 1) / kGemmTile;
    if (d % kGK != 0 || d < kGK) return hipErrorInvalidValue;      // callers route such d elsewhere
    auto kern = lmhead_gemm_kernel;
    constexpr int kMaxDevices = 64;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || !attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGLds);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < kMaxDevices) attr_set[dev] = true;
    }
    hipLaunchKernelGGL(kern, dim3(v_tiles * m_tiles), dim3(256), kGLds, stream,
                       static_cast<const uint16_t*>(h), M, d, static_cast<const uint16_t*>(W), ids, V_act, k,
                       m_tiles, static_cast<u64*>(keys), static_cast<float2*>(stats));
    return hipGetLastError();
}

}  // namespace evospec
