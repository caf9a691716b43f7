// Ordered selection (stream compaction) of the indices i in [0, n) that satisfy a predicate:
// per-tile counts, a one-workgroup scan, ordered emission.
#pragma once
#include "ccld_internal.h"
#include "device_utils.h"
#include "window_kernels.h"

namespace ccld {

// generic ordered selection of indices i in [0, n) with pred(i)
template <class Pred>
__global__ __launch_bounds__(256) void k_select_count(Pred pred, u32 n, u32* tile_counts) {
  __shared__ u32 s_wave[4];
  const u32 base = blockIdx.x * SEL_TILE;
  u32 c = 0;
#pragma unroll 1
  for (int r = 0; r < SEL_TILE / 256; ++r) {
    const u32 i = base + r * 256 + threadIdx.x;
    if (i < n) c += pred(i) ? 1u : 0u;
  }
  u32 tot;
  block_exclusive_sum<256>(c, s_wave, &tot);
  if (threadIdx.x == 0) tile_counts[blockIdx.x] = tot;
}
template <class Pred>
__global__ __launch_bounds__(256) void k_select_emit(Pred pred, u32 n, const u32* tile_counts, u32* out) {
  __shared__ u32 s_wave[4];
  const u32 base = blockIdx.x * SEL_TILE;
  u32 carry = tile_counts[blockIdx.x];
#pragma unroll 1
  for (int r = 0; r < SEL_TILE / 256; ++r) {
    const u32 i = base + r * 256 + threadIdx.x;
    const bool p = i < n && pred(i);
    u32 tot;
    const u32 ex = block_exclusive_sum<256>(p ? 1u : 0u, s_wave, &tot);
    if (p) out[carry + ex] = i;
    carry += tot;
  }
}
template <class Pred>
inline void run_select(hipStream_t st, Pred pred, u32 n, u32* tile_counts, u32* out, u64* total_out) {
  const u32 nt = (n + SEL_TILE - 1) / SEL_TILE;
  if (n) hipLaunchKernelGGL(k_select_count<Pred>, dim3(nt), dim3(256), 0, st, pred, n, tile_counts);
  launch_scan_tiles(st, tile_counts, nt, total_out);
  if (n) hipLaunchKernelGGL(k_select_emit<Pred>, dim3(nt), dim3(256), 0, st, pred, n, (const u32*)tile_counts, out);
}


}  // namespace ccld
