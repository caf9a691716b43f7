// Wavefront (64 lanes) and workgroup primitives shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;
typedef int64_t i64;
typedef int32_t i32;
typedef unsigned __int128 u128;
typedef __int128 i128;

#define CCLD_WAVE 64

namespace ccld {

__device__ __forceinline__ u32 lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// number of set bits of m below the calling lane
__device__ __forceinline__ u32 mbcnt64(u64 m) {
  return __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
}

__device__ __forceinline__ u64 ballot64(bool p) { return __ballot(p); }

__device__ __forceinline__ u64 shfl_u64(u64 v, int src) {
  u32 lo = __shfl((u32)v, src, CCLD_WAVE), hi = __shfl((u32)(v >> 32), src, CCLD_WAVE);
  return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl_up_u64(u64 v, int d) {
  u32 lo = __shfl_up((u32)v, d, CCLD_WAVE), hi = __shfl_up((u32)(v >> 32), d, CCLD_WAVE);
  return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int m) {
  u32 lo = __shfl_xor((u32)v, m, CCLD_WAVE), hi = __shfl_xor((u32)(v >> 32), m, CCLD_WAVE);
  return ((u64)hi << 32) | lo;
}

// inclusive prefix sum over the wavefront
__device__ __forceinline__ u32 wave_inclusive_sum(u32 v) {
  u32 lane = lane_id();
#pragma unroll
  for (int off = 1; off < CCLD_WAVE; off <<= 1) {
    u32 y = __shfl_up(v, off, CCLD_WAVE);
    if (lane >= (u32)off) v += y;
  }
  return v;
}
__device__ __forceinline__ u32 wave_sum(u32 v) {
#pragma unroll
  for (int m = CCLD_WAVE / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, CCLD_WAVE);
  return v;
}
__device__ __forceinline__ u64 wave_max_u64(u64 v) {
#pragma unroll
  for (int m = CCLD_WAVE / 2; m >= 1; m >>= 1) { u64 o = shfl_xor_u64(v, m); v = o > v ? o : v; }
  return v;
}

// Exclusive prefix sum of one value per thread over a workgroup of THREADS threads.
// s_wave: THREADS/64 words of LDS.  *total receives the workgroup sum.  Contains barriers;
// s_wave may be reused after return.
template <int THREADS>
__device__ __forceinline__ u32 block_exclusive_sum(u32 v, u32* s_wave, u32* total) {
  constexpr int NW = THREADS / CCLD_WAVE;
  u32 lane = lane_id(), wave = threadIdx.x / CCLD_WAVE;
  u32 inc = wave_inclusive_sum(v);
  if (lane == CCLD_WAVE - 1) s_wave[wave] = inc;
  __syncthreads();
  u32 base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) { u32 x = s_wave[w]; if ((u32)w < wave) base += x; tot += x; }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

__device__ __forceinline__ int bits_for(u64 max_value) {   // bits needed to store 0..max_value
  return max_value == 0 ? 0 : 64 - __clzll((long long)max_value);
}

}  // namespace ccld
