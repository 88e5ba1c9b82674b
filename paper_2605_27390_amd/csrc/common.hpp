// Types and device helpers shared by the HIP kernels of the active-vocabulary LM head.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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
    const uint32_t u = __float_as_uint(f + 0.0f);       // -0 -> +0 so that the two tie
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);   // negative: flip all bits, else the sign
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

// One set of per-slab partial results as the merge kernel reads it: the list of (slab L, row
// slot r) starts at keys + L * key_slab + r * key_row, its statistics are stats[L * stat_slab + r * stat_row].
struct PartialSet {
    const u64* keys;
    const float2* stats;
    int n_slabs;
    int row_base;           // slot of this launch's block 0 inside the set's row dimension
    size_t key_slab, key_row;       // strides in u64
    size_t stat_slab, stat_row;     // strides in float2
    int list_len;           // key slots per list (>= k); empty slots hold 0
    int sorted;             // lists hold keys, descending (slot 0 is the maximum); else (logit, id)
                            // pairs in any order, all ones = empty
};

// x of lane (lane ^ STRIDE), STRIDE a power of two below 64, without a trip through LDS (a
// ds_bpermute costs its full latency at every step of a dependent chain: 42 of them made the sort
// below 3,500 cycles long).  Strides 1 and 2 are quad permutes; 4 is a mirror of each group of 8
// lanes (lane ^ 7) followed by a reversal within quads (lane ^ 3); 8 is a rotation by 8 within the
// 16-lane row; 16 and 32 are the row / half swaps of gfx950: v_permlane16_swap(x, x) returns the even
// rows' values in all rows and the odd rows' values in all rows, v_permlane32_swap(x, x) the lower and
// the upper half.
template <int STRIDE>
__device__ __forceinline__ uint32_t xor_lane(uint32_t x, int lane) {
    static_assert(STRIDE == 1 || STRIDE == 2 || STRIDE == 4 || STRIDE == 8 || STRIDE == 16 || STRIDE == 32, "stride");
    if constexpr (STRIDE == 1) {
        return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0xB1, 0xF, 0xF, false);      // quad_perm [1,0,3,2]
    } else if constexpr (STRIDE == 2) {
        return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x4E, 0xF, 0xF, false);      // quad_perm [2,3,0,1]
    } else if constexpr (STRIDE == 4) {
        const int m = __builtin_amdgcn_update_dpp((int)x, (int)x, 0x141, 0xF, 0xF, false);        // row_half_mirror
        return (uint32_t)__builtin_amdgcn_update_dpp(m, m, 0x1B, 0xF, 0xF, false);                // quad_perm [3,2,1,0]
    } else if constexpr (STRIDE == 8) {
        return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x128, 0xF, 0xF, false);     // row_ror:8
    } else if constexpr (STRIDE == 16) {
        const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return (lane & 16) ? a[0] : a[1];
    } else {
        const auto a = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        return (lane & 32) ? a[0] : a[1];
    }
}
__device__ __forceinline__ float wave_max(float x, int lane) {
    x = fmaxf(x, __uint_as_float(xor_lane<1>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(xor_lane<2>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(xor_lane<4>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(xor_lane<8>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(xor_lane<16>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(xor_lane<32>(__float_as_uint(x), lane)));
    return x;
}
// Sum over the wavefront in a fixed butterfly order (the same bits in every lane and every launch).
__device__ __forceinline__ float wave_sum(float x, int lane) {
    x += __uint_as_float(xor_lane<1>(__float_as_uint(x), lane));
    x += __uint_as_float(xor_lane<2>(__float_as_uint(x), lane));
    x += __uint_as_float(xor_lane<4>(__float_as_uint(x), lane));
    x += __uint_as_float(xor_lane<8>(__float_as_uint(x), lane));
    x += __uint_as_float(xor_lane<16>(__float_as_uint(x), lane));
    x += __uint_as_float(xor_lane<32>(__float_as_uint(x), lane));
    return x;
}

// Bitonic sort of one key per lane across the wavefront, descending: lane 0 ends with the largest.
// 21 compare-exchange steps; equal keys (only the empty key 0 repeats) may end in any order.
template <int SIZE, int STRIDE>
__device__ __forceinline__ u64 bitonic_step(u64 x, int lane) {
    const uint32_t lo = xor_lane<STRIDE>((uint32_t)x, lane), hi = xor_lane<STRIDE>((uint32_t)(x >> 32), lane);
    const u64 y = ((u64)hi << 32) | lo;
    const bool lower = (lane & STRIDE) == 0;             // this lane is the smaller index of its pair
    const bool desc = (lane & SIZE) == 0;                // its block is being sorted downwards
    const bool gt = x > y;
    return (gt == (lower == desc)) ? x : y;              // lower lane of a descending block keeps the larger
}
__device__ __forceinline__ u64 wave_sort_desc(u64 x, int lane) {
    x = bitonic_step<2, 1>(x, lane);
    x = bitonic_step<4, 2>(x, lane);  x = bitonic_step<4, 1>(x, lane);
    x = bitonic_step<8, 4>(x, lane);  x = bitonic_step<8, 2>(x, lane);  x = bitonic_step<8, 1>(x, lane);
    x = bitonic_step<16, 8>(x, lane); x = bitonic_step<16, 4>(x, lane); x = bitonic_step<16, 2>(x, lane);
    x = bitonic_step<16, 1>(x, lane);
    x = bitonic_step<32, 16>(x, lane); x = bitonic_step<32, 8>(x, lane); x = bitonic_step<32, 4>(x, lane);
    x = bitonic_step<32, 2>(x, lane);  x = bitonic_step<32, 1>(x, lane);
    x = bitonic_step<64, 32>(x, lane); x = bitonic_step<64, 16>(x, lane); x = bitonic_step<64, 8>(x, lane);
    x = bitonic_step<64, 4>(x, lane);  x = bitonic_step<64, 2>(x, lane);  x = bitonic_step<64, 1>(x, lane);
    return x;
}

}  // namespace evospec
