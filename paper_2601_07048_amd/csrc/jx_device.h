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

// One 32-bit value from another lane through the data-parallel-primitive path
// (no LDS traffic).  CTRL: 0xB1 = quad_perm [1,0,3,2] (lane ^ 1), 0x4E =
// quad_perm [2,3,0,1] (lane ^ 2), 0x141 = row_half_mirror (lane -> 7 - lane in
// each group of 8), 0x140 = row_mirror (lane -> 15 - lane in each row of 16).
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

template <typename T>
__device__ __forceinline__ T bits_add(T a, uint32_t b_bits);
template <>
__device__ __forceinline__ uint32_t bits_add<uint32_t>(uint32_t a, uint32_t b) { return a + b; }
template <>
__device__ __forceinline__ int32_t bits_add<int32_t>(int32_t a, uint32_t b) { return a + (int32_t)b; }
template <>
__device__ __forceinline__ float bits_add<float>(float a, uint32_t b) { return a + __uint_as_float(b); }

template <typename T>
__device__ __forceinline__ uint32_t to_bits(T v);
template <>
__device__ __forceinline__ uint32_t to_bits<uint32_t>(uint32_t v) { return v; }
template <>
__device__ __forceinline__ uint32_t to_bits<int32_t>(int32_t v) { return (uint32_t)v; }
template <>
__device__ __forceinline__ uint32_t to_bits<float>(float v) { return __float_as_uint(v); }

// Sum over aligned groups of W lanes (W power of two <= 64); every lane of the
// group ends up with the total.  The first four steps stay inside a row of 16
// lanes and use DPP: after the lane^1 and lane^2 steps all four lanes of a
// quad hold the same partial sum, so the mirror patterns (which pair each lane
// with a lane of the other quad / the other half-row) complete the butterfly.
template <int W, typename T>
__device__ __forceinline__ T group_sum(T v) {
    if (W >= 2) v = bits_add<T>(v, dpp_u32<0xB1>(to_bits<T>(v)));
    if (W >= 4) v = bits_add<T>(v, dpp_u32<0x4E>(to_bits<T>(v)));
    if (W >= 8) v = bits_add<T>(v, dpp_u32<0x141>(to_bits<T>(v)));
    if (W >= 16) v = bits_add<T>(v, dpp_u32<0x140>(to_bits<T>(v)));
    if (W >= 32) v += shfl_xor(v, 16);
    if (W >= 64) v += shfl_xor(v, 32);
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
