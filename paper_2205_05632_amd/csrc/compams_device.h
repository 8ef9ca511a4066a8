// Device-side helpers for the gfx950 kernels of libcompams (wave64 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace compams {

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

// 64-bit mask of the lanes of this wavefront for which p holds.
__device__ __forceinline__ uint64_t ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// Number of set bits of mask that belong to lanes below the calling lane.
__device__ __forceinline__ uint32_t count_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint32_t popc64(uint64_t m) { return static_cast<uint32_t>(__popcll(m)); }

// Value of lane 0 made wave-uniform.
__device__ __forceinline__ uint32_t first_lane(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Magnitude key of Definition 1's ordering: the fp32 pattern without its sign bit.
__device__ __forceinline__ uint32_t key_of_bits(uint32_t bits) { return bits & 0x7fffffffu; }

// Inclusive wave prefix sum (64 lanes).
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    const uint32_t o = __shfl_up(v, s, 64);
    if (lane_id() >= static_cast<uint32_t>(s)) v += o;
  }
  return v;
}

// Exclusive prefix sum over a workgroup of NT threads (NT a multiple of 64, at most 1024).
// scratch must hold NT/64 + 1 words.  Returns the exclusive prefix; *total gets the workgroup sum.
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
  constexpr int NW = NT / 64;
  const uint32_t incl = wave_incl_scan(v);
  const uint32_t w = threadIdx.x >> 6;
  __syncthreads();  // scratch may still be read from a previous call
  if (lane_id() == 63) scratch[w] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const uint32_t t = scratch[i];
    if (static_cast<uint32_t>(i) < w) before += t;
    all += t;
  }
  *total = all;
  return before + incl - v;
}

// Bitwise OR over each aligned group of 8 lanes, left in all 8 of them.  Data-parallel-primitive moves
// (quad permutes, then the mirror of each half row) instead of LDS-routed shuffles: three VALU
// instructions, no memory-counter waits.
__device__ __forceinline__ uint32_t or_over_8_lanes(uint32_t w) {
  w |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(w), 0xB1, 0xF, 0xF, true));   // lanes ^ 1
  w |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(w), 0x4E, 0xF, 0xF, true));   // lanes ^ 2
  w |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(w), 0x141, 0xF, 0xF, true));  // 7 - lane
  return w;
}

// 128-bit streaming (non-temporal) access for data that is touched once per step.
typedef float f4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream4(const float* p) {
  const f4v v = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream4(float* p, const float4& x) {
  f4v v;
  v.x = x.x; v.y = x.y; v.z = x.z; v.w = x.w;
  __builtin_nontemporal_store(v, reinterpret_cast<f4v*>(p));
}

// theta, m, v, vhat are touched once per step.  CACHED: an ordinary access, which leaves the line in the memory-side
// cache for the next step; else a streaming one.
template <bool CACHED>
__device__ __forceinline__ float4 load_state4(const float* p) {
  if constexpr (CACHED) return *reinterpret_cast<const float4*>(p);
  else return load_stream4(p);
}
template <bool CACHED>
__device__ __forceinline__ void store_state4(float* p, const float4& x) {
  if constexpr (CACHED) *reinterpret_cast<float4*>(p) = x;
  else store_stream4(p, x);
}

// A value that is the same in every lane, moved to a scalar register: conditions on it become scalar branches
// and it can be an operand of every lane's arithmetic without a register per lane.
__device__ __forceinline__ uint32_t uniform_u32(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// A table entry at a wave-uniform index, read through the scalar path: the tables read this way (block offsets,
// chunk-to-block map, the previous step's means and list offsets, a row's carried-over guess) are not
// written by the kernel that reads them, and a scalar load has its own counter, so waiting for it does not mean
// waiting for the vector loads that are in flight (a vector load here stalled the stream once per chunk); what
// it returns sits in scalar registers.
typedef const __attribute__((address_space(4))) uint32_t* ScalarTable;
__device__ __forceinline__ uint32_t table_u32(const uint32_t* p, uint32_t i) {
  return reinterpret_cast<ScalarTable>(reinterpret_cast<uintptr_t>(p))[i];
}
// Eight consecutive words of such a table (32-byte aligned) with one scalar load.
typedef uint32_t U32x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ U32x8 table_u32x8(const uint32_t* p) {
  return *reinterpret_cast<const __attribute__((address_space(4))) U32x8*>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ float table_f32(const float* p, uint32_t i) {
  return __uint_as_float(table_u32(reinterpret_cast<const uint32_t*>(p), i));
}
}  // namespace compams
