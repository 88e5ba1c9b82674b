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

// Bitonic sort of one key per lane across the wavefront, descending: lane 0 ends with the largest.
// 21 compare-exchange steps; equal keys (only the empty key 0 repeats) may end in any order.
__device__ __forceinline__ u64 wave_sort_desc(u64 x, int lane) {
#pragma unroll
    for (int size = 2; size <= 64; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)x, stride), hi = __shfl_xor((uint32_t)(x >> 32), stride);
            const u64 y = ((u64)hi << 32) | lo;
            const bool lower = (lane & stride) == 0;         // this lane is the smaller index of its pair
            const bool desc = (lane & size) == 0;            // its block is being sorted downwards
            const bool gt = x > y;
            x = (gt == (lower == desc)) ? x : y;             // lower lane of a descending block keeps the larger
        }
    }
    return x;
}

}  // namespace evospec
