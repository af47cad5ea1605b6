// Device-side helpers shared by the HIP kernels of libjx (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define JX_WAVE 64
#define JX_NONE_ID 0xFFFFFFFFu
#define JX_EMPTY_KEY 0xFFFFFFFFFFFFFFFFull

namespace jx {

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// Make LDS traffic of the lanes of one wavefront visible to each other.  A
// wavefront executes its LDS instructions in order, so only the compiler has
// to be stopped from reordering around this point.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// number of set bits of m in lanes below the calling lane
__device__ __forceinline__ int prefix_count(uint64_t m) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t readlane32(uint32_t v, int l) { return __builtin_amdgcn_readlane(v, l); }

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int l) {
    uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, l);
    uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

template <typename T>
__device__ __forceinline__ T shfl_xor(T v, int m) {
    return __shfl_xor(v, m, 64);
}

// sum over aligned groups of W lanes (W power of two <= 64); every lane of the
// group ends up with the total
template <int W, typename T>
__device__ __forceinline__ T group_sum(T v) {
#pragma unroll
    for (int m = 1; m < W; m <<= 1) v += shfl_xor(v, m);
    return v;
}

// Order-preserving map float -> uint32 (total order of the reals, -0 < +0).
__device__ __forceinline__ uint32_t f32_to_ordered(float f) {
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_f32(uint32_t o) {
    uint32_t b = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(b);
}

// Frontier key: [63:32] ordered distance, [31:1] id, [0] expanded flag.
// Comparing keys with bit 0 forced to 1 compares (distance, id).
__device__ __forceinline__ uint64_t make_key(uint32_t dist_code, uint32_t id) {
    return ((uint64_t)dist_code << 32) | ((uint64_t)id << 1);
}
__device__ __forceinline__ uint32_t key_id(uint64_t k) { return (uint32_t)(k & 0xFFFFFFFFull) >> 1; }
__device__ __forceinline__ uint32_t key_dist(uint64_t k) { return (uint32_t)(k >> 32); }

__device__ __forceinline__ uint4 load16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

}  // namespace jx
