// Large-M variant of the restricted head (Eq. 1 of the EvoSpec paper on the active set of Eq. 3):
// with hundreds of draft rows in flight (batched serving, one shared core for all sequences) the
// projection is a dense contraction and bound by the matrix cores, not by the stream of W_act.
//
// One workgroup of four wavefronts (one per SIMD) computes a 256 x 256 tile of z = W_act h^T
// (256 active rows x 256 draft rows) over the whole hidden dimension.  Both operands travel
// HBM/L2 -> LDS with direct-to-LDS loads (no staging registers, whole 128-byte lines per request)
// in chunks of 32 hidden elements through a ring of four stages, filled two at a time.  Every
// wavefront owns a 128 x 128 quadrant = 8 x 8 accumulators of v_mfma_f32_16x16x32_bf16, which
// fill the 256 accumulation registers of a lane, and reads the operands of the next chunk from
// LDS while the matrix cores work on the current one.  The logits never leave the registers:
// each wavefront reduces its quadrant, per draft row, to a partial for a "slab" of its 128 rows:
// (max, sum-exp) and the logits that can still be among the row's k best, unranked, as
// (logit, id) pairs; the merge kernel ranks them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

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
constexpr int kGFastLen = 16;                 // list length the staged common path of the epilogue handles
constexpr int kGEpiBytes = 16 * kGemmSlab * 8 + 64 * 32 * 4 + kGemmSlab * 4;   // per wavefront: lists, parked logits, ids
static_assert(8 * 16 * kGFastLen * 8 + 64 * 8 <= 16 * kGemmSlab * 8 + 64 * 32 * 4, "staged lists and spare slots fit");
constexpr size_t kGLdsTotal = kGLds > 4ull * kGEpiBytes ? kGLds : 4ull * kGEpiBytes;

static_assert(kGLds <= (size_t)kLdsLimit, "operand ring exceeds the LDS of a compute unit");
static_assert(kGLdsTotal <= (size_t)kLdsLimit, "epilogue lists exceed the LDS of a compute unit");

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// A row of a chunk holds 32 hidden elements = four 16-byte pieces, rows are stored in blocks of 8
// (see the kernel).  Piece p of row r sits in slot p ^ swz(r).  The 16 lanes of an MFMA operand
// read take one piece of 16 consecutive rows: with this swizzle any 8 consecutive rows fall into 8 different 16-byte columns of a 128-byte
// bank window and any 16 into 16 different columns of a 256-byte window, so the read is free of
// bank conflicts for either bank count (consecutive rows are 64 bytes apart inside a block, blocks
// 1 KB apart).  The direct-to-LDS load writes lane L of a wavefront to byte 16 L of a 1 KB block, so
// the swizzle is applied on the source side: the lane that fills (row, slot) fetches piece
// slot ^ swz(row).
__device__ __forceinline__ int swz(int row) { return (((row & 15) >> 1) + ((row & 15) >> 3)) & 3; }

// Accumulators are pinned to the accumulation registers: with all 256 of them live, the
// register allocator must not be left to shuffle them through the other file.
__device__ __forceinline__ void mfma_acc(f32x4& c, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// The 4 lanes n16, n16+16, n16+32, n16+48 (one per 16-lane row of the wavefront) hold the four
// quarters of a draft row's logits.  v_permlane16_swap exchanges the odd rows of its first operand
// with the even rows of the second, v_permlane32_swap the upper half of the first with the lower
// half of the second: applied to two copies of x they hand every lane both members of its pair of
// rows, then of its pair of halves.
// Eight independent values at a time, stage by stage (the scheduler is fenced in between).
__device__ __forceinline__ void quad_max8(float (&x)[8]) {
    float y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x[i]), __float_as_uint(x[i]), false, false);
        x[i] = __uint_as_float(a[0]); y[i] = __uint_as_float(a[1]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = fmaxf(x[i], y[i]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x[i]), __float_as_uint(x[i]), false, false);
        x[i] = __uint_as_float(b[0]); y[i] = __uint_as_float(b[1]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = fmaxf(x[i], y[i]);
    __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ void quad_sum8(float (&x)[8]) {
    float y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x[i]), __float_as_uint(x[i]), false, false);
        x[i] = __uint_as_float(a[0]); y[i] = __uint_as_float(a[1]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] += y[i];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x[i]), __float_as_uint(x[i]), false, false);
        x[i] = __uint_as_float(b[0]); y[i] = __uint_as_float(b[1]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] += y[i];
    __builtin_amdgcn_sched_barrier(0);
}
// q[r] = x of the lane in row r (lane n16 + 16 r)
__device__ __forceinline__ void quad_all(uint32_t x, uint32_t (&q)[4]) {
    const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);      // a[0]: rows {0,0,2,2}, a[1]: rows {1,1,3,3}
    const auto e = __builtin_amdgcn_permlane32_swap(a[0], a[0], false, false);  // e[0]: row 0 everywhere, e[1]: row 2
    const auto o = __builtin_amdgcn_permlane32_swap(a[1], a[1], false, false);  // o[0]: row 1 everywhere, o[1]: row 3
    q[0] = e[0]; q[1] = o[0]; q[2] = e[1]; q[3] = o[1];
}

}  // namespace

// PACKED: W is in operand-tile layout (plan.hpp): a wave-level load then takes one whole 1 KB
// operand block (16 rows x 32 hidden elements), which lands in LDS in the order the lanes read it.
template <bool PACKED>
__global__ void __launch_bounds__(256, 1)
lmhead_gemm_kernel(const uint16_t* __restrict__ h, int M, int d,
                   const uint16_t* __restrict__ W, const int32_t* __restrict__ ids, int V_act, int k, int list_len,
                   int m_tiles, u64* __restrict__ part_keys, float2* __restrict__ part_stats) {
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform: keeps LDS destinations scalar
    const int n16 = lane & 15, g = lane >> 4;
    const int wv = w >> 1, wm = w & 1;                             // quadrant: active-row half, draft-row half

    // Workgroups are handed to the 8 XCDs round robin; renumber them so that the m_tiles tiles
    // that read the same 256 rows of W_act run on one XCD (one L2) at about the same time.
    const int nb = gridDim.x, b = blockIdx.x;
    const int xcd = b & 7, full = nb >> 3, rem = nb & 7;
    const int logical = xcd * full + (xcd < rem ? xcd : rem) + (b >> 3);
    const int tile_v = logical / m_tiles, tile_m = logical - tile_v * m_tiles;
    const int v0 = tile_v * kGemmTile, m0 = tile_m * kGemmTile;

    // Direct-to-LDS loads fetch whole 128-byte lines: one wave-level load takes, for 8 rows, the
    // 64 bytes of an even chunk (lanes 0-31) and of the following odd chunk (lanes 32-63).  The
    // ring therefore consists of 2 pair-stages of 64 KB; in a pair-stage, operand o, block b of 8
    // rows: bytes [o * 32 KB + b * 1 KB, +1 KB) = [chunk parity][row][slot].
    constexpr int kPairBytes = 2 * kGStageBytes;                   // 64 KB
    constexpr int kPLoads = kGemmTile / 8 / 4;                     // 8 blocks of 8 rows per wavefront and operand
    const uint16_t* asrc[kPLoads];
    const uint16_t* bsrc[kPLoads];
#pragma unroll
    for (int i = 0; i < kPLoads; ++i) {
        const int r = (kPLoads * w + i) * 8 + ((lane >> 2) & 7);
        const int piece = (lane & 3) ^ swz(r);
        const int half = lane >> 5;
        if constexpr (PACKED) {
            // block B = 8 w + i of the pair-stage: k-step parity B & 1 of the 16-row tile B >> 1
            const int B = kPLoads * w + i;
            const int tile = min((v0 >> 4) + (B >> 1), (V_act - 1) >> 4);            // tiles past the end repeat the last
            asrc[i] = W + (size_t)tile * kPackRows * packed_d(d) + (B & 1) * (16 * kGK) + lane * 8;
        } else {
            asrc[i] = W + (size_t)min(v0 + r, V_act - 1) * d + half * kGK + piece * 8;   // rows past the end repeat
        }
        bsrc[i] = h + (size_t)min(m0 + r, M - 1) * d + half * kGK + piece * 8;       // the last one, masked later
    }
    const int nchunks = d / kGK;                                   // even: d is a multiple of 64 here
    const int npairs = nchunks / 2;
    // Load number j (0..15) of pair p: block j/2 of this wavefront's W_act rows (j even) or h rows (j odd).
    // Pairs past the end repeat the last one into a stage nobody reads again.
    auto issue_one = [&](int p, int j) {
        const size_t koff = (size_t)min(p, npairs - 1) * (2 * kGK);
        unsigned char* dst = smem + (p & 1) * kPairBytes + (j & 1) * (2 * kGOperandBytes) + (kPLoads * w + (j >> 1)) * 1024;
        // (a k-step of a packed tile is 16 rows x 32 elements long)
        const uint16_t* src = (j & 1) ? bsrc[j >> 1] + koff : asrc[j >> 1] + (PACKED ? koff * 16 : koff);
        __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 16, 0, 0);
    };

    f32x4 acc[8][8];
#pragma unroll
    for (int rg = 0; rg < 8; ++rg)
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) acc[rg][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // operand reads: lane (n16, g) takes piece g of row n16 of each 16-row block of its quadrant;
    // row R of an operand sits in block R / 8 at row R % 8
    auto row_off = [&](int R) { return (R >> 3) * 1024 + (R & 7) * 64; };
    const int a_rd = PACKED ? wv * 128 * 128 + lane * 16 : row_off(wv * 128 + n16) + ((g ^ swz(n16)) * 16);
    constexpr int kAParity = PACKED ? 1024 : 512;                  // second chunk of a pair, W side
    const int b_rd = 2 * kGOperandBytes + row_off(wm * 128 + n16) + ((g ^ swz(n16)) * 16);
    bf16x8 opa[2][8], opb[2][8];
    auto stage_of = [&](int c) { return ((c >> 1) & 1) * kPairBytes + (c & 1) * 512; };
    auto read_a = [&](auto SET, int c, int i) {
        opa[decltype(SET)::value][i] = *reinterpret_cast<const bf16x8*>(smem + ((c >> 1) & 1) * kPairBytes + (c & 1) * kAParity + a_rd + i * 2048);
    };
    auto read_b = [&](auto SET, int c, int i) {
        opb[decltype(SET)::value][i] = *reinterpret_cast<const bf16x8*>(smem + stage_of(c) + b_rd + i * 2048);
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;

    // One chunk: 64 MFMAs on the operands in registers (set CUR); in the gaps, the 16 operand
    // reads of chunk c+1 (into set 1 - CUR) and, in odd chunks, the 16 loads of the pair (c+3, c+4)
    // into the pair-stage of chunks (c-1, c), which every wavefront finished reading before the
    // barrier.  An odd chunk needs the pair (c+1, c+2), requested two chunks ago and the youngest
    // request: wait for everything.  An even chunk needs its own pair, which its predecessor needed too.
    auto step = [&](auto CUR, int c) {
        constexpr int P = decltype(CUR)::value;
        using NXT = std::integral_constant<int, 1 - P>;
        if (P == 1) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        else asm volatile("s_barrier" ::: "memory");
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
            if (P == 1) { issue_one((c + 3) >> 1, 2 * rg); issue_one((c + 3) >> 1, 2 * rg + 1); }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };

#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int j = 0; j < 16; ++j) issue_one(p, j);
    // pair 0 must have landed before its operands are read
    asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");
#pragma unroll
    for (int i = 0; i < 8; ++i) { read_b(S0{}, 0, i); read_a(S0{}, 0, i); }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 7" ::: "memory");

    for (int c = 0; c < nchunks; c += 2) {
        step(S0{}, c);
        step(S1{}, c + 1);
    }
    // the last MFMAs drain before the accumulators are read; the ring is dead once the trailing
    // loads have landed and every wavefront is here
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- epilogue: wave-local from here on; the operand buffers are dead (all waves are past the
    // last barrier), each wavefront takes its own piece of them
    const int vrow0 = v0 + wv * kGemmSlab;
    const int nvalid = min(kGemmSlab, V_act - vrow0);
    if (nvalid <= 0) return;                                       // quadrant wholly past the active set
    const int slab = tile_v * (kGemmTile / kGemmSlab) + wv;
    const int n_slabs = (V_act + kGemmSlab - 1) / kGemmSlab;    // lists are laid out [draft row][slab][slot]
    unsigned char* my = smem + (size_t)w * kGEpiBytes;
    // common path: [8][16][16] staged lists of all blocks, then one spare slot per lane;
    // rare path (afterwards, same bytes): [16][128] full lists of one block, then [64][32] parked logits
    u64* flist = reinterpret_cast<u64*>(my);
    u64* list = reinterpret_cast<u64*>(my);
    float* zpark = reinterpret_cast<float*>(my + 16 * kGemmSlab * 8);
    int32_t* Ids = reinterpret_cast<int32_t*>(my + kGEpiBytes - kGemmSlab * 4);   // [128]

#pragma unroll
    for (int i = 0; i < kGemmSlab / 64; ++i) {
        const int r = vrow0 + lane + 64 * i;
        Ids[lane + 64 * i] = r < V_act ? (ids ? ids[r] : r) : 0x7fffffff;
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    // lane's entries: active row (within the quadrant) 16 rg + 4 g + j  <->  bit 4 rg + j
    uint32_t vmask = 0;
#pragma unroll
    for (int rg = 0; rg < 8; ++rg)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (rg * 16 + 4 * g + j < nvalid) vmask |= 1u << (4 * rg + j);
    if (nvalid < kGemmSlab) {                                      // ragged last slab: rows past the end never win
#pragma unroll
        for (int rg = 0; rg < 8; ++rg)
#pragma unroll
            for (int mb = 0; mb < 8; ++mb)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (!((vmask >> (4 * rg + j)) & 1u)) acc[rg][mb][j] = -INFINITY;
    }

    // A wavefront runs alone on its SIMD here, so nothing hides a latency but its own independent
    // work: every phase below runs over all 8 blocks of 16 draft rows before the next one starts.
    // Lane (n16, g) holds, for draft row n16 of block mb, the 32 logits acc[0..7][mb][0..3]; the
    // row's 128 logits are spread over the 4 lanes g = 0..3, which exchange values with the
    // row-swap instructions (no LDS round trip).

    // (an empty statement that "rewrites" the accumulators where they sit: copies read into
    // ordinary registers by one phase are dropped instead of being carried, and spilled, to the next)
    auto repin = [&]() {
#pragma unroll
        for (int rg = 0; rg < 8; ++rg)
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) asm volatile("" : "+a"(acc[rg][mb]));
    };
    repin();
    // Dependent vector instructions of one wavefront issue many cycles apart, so each phase is
    // written as stages over the 8 independent blocks (8 instructions per stage) and the
    // scheduler is fenced between stages so that it keeps them that way.
#define EVOSPEC_FENCE() __builtin_amdgcn_sched_barrier(0)
#define EVOSPEC_MB(body) _Pragma("unroll") for (int mb = 0; mb < 8; ++mb) { body; } EVOSPEC_FENCE();

    // -- phase 1: maxima of the 32 groups of 4 logits of every row, and the row maximum
    float t[8][8], vm[8];
#pragma unroll
    for (int rg = 0; rg < 8; ++rg) {
        float p0[8], p1[8];
        EVOSPEC_MB(p0[mb] = fmaxf(acc[rg][mb][0], acc[rg][mb][1]))
        EVOSPEC_MB(p1[mb] = fmaxf(acc[rg][mb][2], acc[rg][mb][3]))
        EVOSPEC_MB(t[mb][rg] = fmaxf(p0[mb], p1[mb]))
    }
    {
        float p0[8], p1[8], p2[8], p3[8];
        EVOSPEC_MB(p0[mb] = fmaxf(t[mb][0], t[mb][1]))
        EVOSPEC_MB(p1[mb] = fmaxf(t[mb][2], t[mb][3]))
        EVOSPEC_MB(p2[mb] = fmaxf(t[mb][4], t[mb][5]))
        EVOSPEC_MB(p3[mb] = fmaxf(t[mb][6], t[mb][7]))
        EVOSPEC_MB(p0[mb] = fmaxf(p0[mb], p1[mb]))
        EVOSPEC_MB(p2[mb] = fmaxf(p2[mb], p3[mb]))
        EVOSPEC_MB(vm[mb] = fmaxf(p0[mb], p2[mb]))
        quad_max8(vm);
    }

    // -- phase 2: lower bound of every row's k-th best logit.  Each lane sorts its 8 group maxima;
    // k rounds then take the largest head of the row's 4 lanes and pop it wherever it is the head:
    // at least k group maxima, hence k logits, reach the last value taken.  With more than 32
    // wanted, or fewer groups than k, the bound stays at -inf and every valid entry is kept.
    float tau[8];
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) tau[mb] = -INFINITY;
    if (k <= 32) {
#define EVOSPEC_CE(I, J) { float hi[8]; EVOSPEC_MB(hi[mb] = fmaxf(t[mb][I], t[mb][J])) \
                           EVOSPEC_MB(t[mb][J] = fminf(t[mb][I], t[mb][J])) EVOSPEC_MB(t[mb][I] = hi[mb]) }
        EVOSPEC_CE(0, 1) EVOSPEC_CE(2, 3) EVOSPEC_CE(4, 5) EVOSPEC_CE(6, 7)
        EVOSPEC_CE(0, 2) EVOSPEC_CE(1, 3) EVOSPEC_CE(4, 6) EVOSPEC_CE(5, 7)
        EVOSPEC_CE(1, 2) EVOSPEC_CE(5, 6) EVOSPEC_CE(0, 4) EVOSPEC_CE(3, 7)
        EVOSPEC_CE(1, 5) EVOSPEC_CE(2, 6)
        EVOSPEC_CE(1, 4) EVOSPEC_CE(3, 6)
        EVOSPEC_CE(2, 4) EVOSPEC_CE(3, 5)
        EVOSPEC_CE(3, 4)
#undef EVOSPEC_CE
        for (int r = 0; r < k; ++r) {
            EVOSPEC_MB(tau[mb] = t[mb][0])
            quad_max8(tau);
            // pop the head where it is the value just taken: all ones / zero select, no compare chain
            uint32_t pop[8];
            EVOSPEC_MB(pop[mb] = t[mb][0] == tau[mb] ? ~0u : 0u)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                EVOSPEC_MB(const uint32_t cur = __float_as_uint(t[mb][i]);
                           const uint32_t nxt = i < 7 ? __float_as_uint(t[mb][i + 1]) : 0xff800000u;
                           t[mb][i] = __uint_as_float((pop[mb] & nxt) | (~pop[mb] & cur)))
            }
        }
    }

    repin();
    // -- phase 3: sum of exponentials, exp(z - vm) = 2^(z log2(e) - vm log2(e)), two running sums per block
    uint32_t mask[8];
    float se[8];
    {
        float nvm[8], s0[8], s1[8];
        EVOSPEC_MB(nvm[mb] = -vm[mb] * 1.44269504f; s0[mb] = 0.f; s1[mb] = 0.f)
#pragma unroll
        for (int rg = 0; rg < 8; ++rg) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float x[8];
                EVOSPEC_MB(x[mb] = __builtin_fmaf(acc[rg][mb][j], 1.44269504f, nvm[mb]))
                EVOSPEC_MB(x[mb] = __builtin_amdgcn_exp2f(x[mb]))
                if (j & 1) { EVOSPEC_MB(s1[mb] += x[mb]) } else { EVOSPEC_MB(s0[mb] += x[mb]) }
            }
        }
        EVOSPEC_MB(se[mb] = s0[mb] + s1[mb])
        quad_sum8(se);
    }
    repin();
    // -- phase 3b: survivor masks without a compare per entry: the sign of (logit - bound) is
    // shifted in, last entry first, so that entry i ends up as bit i ("below the bound")
    {
        uint32_t below[8];
        EVOSPEC_MB(below[mb] = 0u)
#pragma unroll
        for (int i = 31; i >= 0; --i) {
            float df[8];
            EVOSPEC_MB(df[mb] = acc[i >> 2][mb][i & 3] - tau[mb])
            EVOSPEC_MB(below[mb] = __builtin_amdgcn_alignbit(below[mb], __float_as_uint(df[mb]), 31))
        }
        EVOSPEC_MB(mask[mb] = ~below[mb] & vmask)
    }
    const int mrow0 = m0 + wm * 128 + n16;                         // draft row of block 0
#pragma unroll
    for (int mb = 0; mb < 8; ++mb)
        if (g == 0 && mrow0 + 16 * mb < M) part_stats[(size_t)(mrow0 + 16 * mb) * n_slabs + slab] = make_float2(vm[mb], se[mb]);

    // survivors per lane (<= 32), four blocks to a register; from the 4 lanes of a row: the offset
    // of this lane's survivors in the row's list and the list length L (<= 128), still packed
    uint32_t basep[2], Lp[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        const uint32_t pk = __popc(mask[4 * hf]) | (__popc(mask[4 * hf + 1]) << 8) | (__popc(mask[4 * hf + 2]) << 16) |
                            (__popc(mask[4 * hf + 3]) << 24);
        uint32_t q[4];
        quad_all(pk, q);
        basep[hf] = (g > 0 ? q[0] : 0u) + (g > 1 ? q[1] : 0u) + (g > 2 ? q[2] : 0u);
        Lp[hf] = q[0] + q[1] + q[2] + q[3];
    }
    // blocks in which every row's survivors fit a list go straight out (wave-uniform choice)
    uint32_t fast = 0;
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) {
        const int L = (Lp[mb >> 2] >> (8 * (mb & 3))) & 0xff;
        if (list_len == kGFastLen && __ballot(L > kGFastLen) == 0) fast |= 1u << mb;
    }

    repin();
    int32_t idv[32];                                               // full-vocabulary ids of the lane's entries
#pragma unroll
    for (int rg = 0; rg < 8; ++rg) {
        const int4 q = *reinterpret_cast<const int4*>(Ids + rg * 16 + 4 * g);
        idv[4 * rg + 0] = q.x; idv[4 * rg + 1] = q.y; idv[4 * rg + 2] = q.z; idv[4 * rg + 3] = q.w;
    }
    // -- phase 4: the survivors of every row, as (logit, id) pairs in no particular order, are
    // gathered into the row's 16-slot list in LDS (empty slots: all ones) and the lists copied to the
    // workspace a full line at a time; the merge ranks.  No branch or compare per entry: an entry
    // that is not a survivor goes to the lane's spare slot.
    {
        const u32x4 ones = {~0u, ~0u, ~0u, ~0u};
#pragma unroll
        for (int it = 0; it < 8 * 16 * kGFastLen * 8 / 1024; ++it)
            *reinterpret_cast<u32x4*>(my + (it * 64 + lane) * 16) = ones;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const uint32_t spare_a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) u64*)(flist + 8 * 16 * kGFastLen + lane);
        uint32_t mk[8], rel[8];                                    // survivor mask; row list start - spare slot (bytes)
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) {
            const int base = (basep[mb >> 2] >> (8 * (mb & 3))) & 0xff;
            mk[mb] = ((fast >> mb) & 1u) ? mask[mb] : 0u;
            rel[mb] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) u64*)(flist + (mb * 16 + n16) * kGFastLen + base) - spare_a;
        }
        EVOSPEC_FENCE();
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            uint32_t at[8], sel[8];
            EVOSPEC_MB(at[mb] = mk[mb] & ((1u << i) - 1u))
            EVOSPEC_MB(at[mb] = __popc(at[mb]))
            EVOSPEC_MB(sel[mb] = (uint32_t)__builtin_amdgcn_sbfe((int)mk[mb], i, 1))
            EVOSPEC_MB(at[mb] = rel[mb] + 8u * at[mb])
            EVOSPEC_MB(at[mb] &= sel[mb])
            EVOSPEC_MB(at[mb] += spare_a)
            EVOSPEC_MB(*(__attribute__((address_space(3))) u64*)(uintptr_t)at[mb] =
                           ((u64)__float_as_uint(acc[i >> 2][mb][i & 3]) << 32) | (uint32_t)idv[i])
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // piece p = 64 it + lane of the staged lists: block p / 128, row (p / 8) % 16, 16 bytes p % 8
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int mb = it >> 1, r16 = ((it & 1) << 3) | (lane >> 3);
            const int m = m0 + wm * 128 + 16 * mb + r16;
            const u32x4 q = *reinterpret_cast<const u32x4*>(my + (it * 64 + lane) * 16);
            if (((fast >> mb) & 1u) && m < M)
                *reinterpret_cast<u32x4*>(part_keys + ((size_t)m * n_slabs + slab) * kGFastLen + 2 * (lane & 7)) = q;
        }
    }
#undef EVOSPEC_MB
#undef EVOSPEC_FENCE
    if (fast == 0xffu) return;
    repin();

    // -- rare path, block by block: a row with more survivors than a list holds (many equal logits,
    // or k close to or above the number of groups).  The block's logits are parked in LDS so that
    // one rolled copy of the code serves all blocks: keys of the survivors into per-row lists,
    // exact rank among the row's survivors, the k best kept.
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");            // the staged lists have been read
    float* zbuf = zpark + lane * 32;
    for (int mbr = 0; mbr < 8; ++mbr) {
        if ((fast >> mbr) & 1u) continue;
        uint32_t mk = 0;
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) {
            if (mb != mbr) continue;                               // uniform
            mk = mask[mb];
#pragma unroll
            for (int rg = 0; rg < 8; ++rg) *reinterpret_cast<f32x4*>(zbuf + 4 * rg) = acc[rg][mb];
        }
        const int base = (basep[mbr >> 2] >> (8 * (mbr & 3))) & 0xff;
        const int L = (Lp[mbr >> 2] >> (8 * (mbr & 3))) & 0xff;
        const int m = mrow0 + 16 * mbr;
        const bool m_ok = m < M;
        u64* mine = list + n16 * kGemmSlab;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        int pos = base;
        for (int i = 0; i < 32; ++i) {
            if ((mk >> i) & 1u) mine[pos++] = make_key(zbuf[i], Ids[(i >> 2) * 16 + 4 * g + (i & 3)]);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        u64* dst = part_keys + ((size_t)(m_ok ? m : 0) * n_slabs + slab) * list_len;
        for (int e = g; e < L; e += 4) {
            const u64 key = mine[e];
            int rank = 0;
            for (int f = 0; f < L; ++f) rank += mine[f] > key ? 1 : 0;
            if (rank < k && m_ok) dst[rank] = ((u64)__float_as_uint(key_value(key)) << 32) | (uint32_t)key_id(key);
        }
        if (m_ok)
            for (int r = (L < k ? L : k) + g; r < list_len; r += 4) dst[r] = ~0ull;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

hipError_t launch_gemm_partials(const void* h, int M, int d, const void* W, const int32_t* ids, int V_act,
                                int k, void* keys, void* stats, hipStream_t stream, bool packed) {
    const int v_tiles = (V_act + kGemmTile - 1) / kGemmTile;
    const int m_tiles = (M + kGemmTile - 1) / kGemmTile;
    if (d % (2 * kGK) != 0 || d < 2 * kGK) return hipErrorInvalidValue;      // callers route such d elsewhere
    auto kern = packed ? lmhead_gemm_kernel<true> : lmhead_gemm_kernel<false>;
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> attr_set[kMaxDevices] = {};      // concurrent first calls may both set the (idempotent) attribute
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || !attr_set[dev].load(std::memory_order_acquire)) {
        for (auto kf : {lmhead_gemm_kernel<true>, lmhead_gemm_kernel<false>}) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(kf),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGLdsTotal);
            if (e != hipSuccess) return e;
        }
        if (dev >= 0 && dev < kMaxDevices) attr_set[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(v_tiles * m_tiles), dim3(256), kGLdsTotal, stream,
                       static_cast<const uint16_t*>(h), M, d, static_cast<const uint16_t*>(W), ids, V_act, k, gemm_list_len(k),
                       m_tiles, static_cast<u64*>(keys), static_cast<float2*>(stats));
    return hipGetLastError();
}

}  // namespace evospec
