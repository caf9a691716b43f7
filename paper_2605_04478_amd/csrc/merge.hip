// Retain-and-merge kernels for windows of several batches (gfx950).
#include "merge.h"
#include "device_utils.h"
#include "window_kernels.h"

namespace ccld {

constexpr int RET_TILE = 2048;       // entries per workgroup of the retain pass (256 threads x 8)

__device__ __forceinline__ bool still_there(const RetainArgs& a, u32 slot) {
  u32 off = slot >= a.exp_lo ? slot - a.exp_lo : slot + a.cap - a.exp_lo;      // distance past the expired range's start
  return off >= a.exp_n;
}
__device__ __forceinline__ u64 rebase(const RetainArgs& a, u64 k) {
  const int mb = a.from.mb;
  const u64 slot = k & (((u64)1 << mb) - 1);
  const u64 seq = ((k >> mb) & (((u64)1 << a.from.ws) - 1)) + a.from.seq_base;
  const u64 comm = k >> (mb + a.from.ws);
  return (comm << (mb + a.to.ws)) | ((seq - a.to.seq_base) << mb) | slot;
}

// Entry e of a tile belongs to thread e % 256 in round e / 256, so loads and stores are coalesced; an
// entry's place among the tile's kept entries = kept entries of the earlier rounds + of the earlier
// wavefronts of its round + of the lower lanes of its wavefront.
__global__ __launch_bounds__(256) void k_retain_count(RetainArgs a) {
  __shared__ u32 s_wave[4];
  const u32 base = blockIdx.x * RET_TILE;
  u32 c = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const u32 i = base + k * 256 + threadIdx.x;
    c += (i < a.n && still_there(a, a.idx[i])) ? 1u : 0u;
  }
  u32 tot;
  block_exclusive_sum<256>(c, s_wave, &tot);
  if (threadIdx.x == 0) a.tile_counts[blockIdx.x] = tot;
}
__global__ __launch_bounds__(256) void k_retain_emit(RetainArgs a) {
  __shared__ u32 s_cnt[8][4];
  const u32 base = blockIdx.x * RET_TILE, tid = threadIdx.x, lane = lane_id(), wave = tid / CCLD_WAVE;
  u32 slot[8], below[8];
  u64 key[8];
  bool keep[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const u32 i = base + k * 256 + tid;
    slot[k] = 0; key[k] = 0;
    if (i < a.n) { slot[k] = a.idx[i]; key[k] = a.key[i]; }
    keep[k] = i < a.n && still_there(a, slot[k]);
    const u64 m = ballot64(keep[k]);
    below[k] = (u32)__popcll(m & (((u64)1 << lane) - 1));
    if (lane == 0) s_cnt[k][wave] = (u32)__popcll(m);
  }
  __syncthreads();
  u32 run = a.tile_counts[blockIdx.x];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    u32 before = run;
#pragma unroll
    for (int w = 0; w < 4; ++w) { const u32 cw = s_cnt[k][w]; if ((u32)w < wave) before += cw; run += cw; }
    if (keep[k]) { a.key_out[before + below[k]] = rebase(a, key[k]); a.idx_out[before + below[k]] = slot[k]; }
  }
}
void launch_retain(hipStream_t st, const RetainArgs& a) {
  if (a.n == 0) return;
  const u32 nt = (a.n + RET_TILE - 1) / RET_TILE;
  hipLaunchKernelGGL(k_retain_count, dim3(nt), dim3(256), 0, st, a);
  launch_scan_tiles(st, a.tile_counts, nt, a.total_out);
  hipLaunchKernelGGL(k_retain_emit, dim3(nt), dim3(256), 0, st, a);
}

// ---- merge ----------------------------------------------------------------------------------
// Merge path: output position d splits into a entries of the first sequence and d - a of the second,
// a = the smallest count for which the next entry of the first sequence is greater than the last one
// taken from the second.  A workgroup produces MERGE_TILE outputs from the slices between two such
// splits, staged in LDS; every thread then finds its own split inside the slices and merges eight.
constexpr int MERGE_TILE = 2048;
template <class KA, class KB>
__device__ __forceinline__ u32 merge_split(KA ka, u32 na, KB kb, u32 nb, u32 d) {
  u32 lo = d > nb ? d - nb : 0u, hi = d < na ? d : na;
  while (lo < hi) {
    const u32 mid = (lo + hi) >> 1;
    if (ka(mid) <= kb(d - 1 - mid)) lo = mid + 1; else hi = mid;
  }
  return lo;
}
// splits of the tile boundaries: one thread per boundary
__global__ __launch_bounds__(256) void k_merge_splits(const u64* __restrict__ ka, u32 na, const u64* __restrict__ kb, u32 nb,
                                                      u32 n_tiles, u32* __restrict__ split) {
  const u32 t = blockIdx.x * 256 + threadIdx.x;
  if (t > n_tiles) return;
  const u64 total = (u64)na + nb;
  const u32 d = (u64)t * MERGE_TILE < total ? t * MERGE_TILE : (u32)total;
  split[t] = merge_split([&](u32 i) { return ka[i]; }, na, [&](u32 i) { return kb[i]; }, nb, d);
}
__global__ __launch_bounds__(256) void k_merge(const u64* __restrict__ ka, const u32* __restrict__ ia, u32 na,
                                               const u64* __restrict__ kb, const u32* __restrict__ ib, u32 nb,
                                               const u32* __restrict__ split, u64* __restrict__ ko, u32* __restrict__ io) {
  __shared__ u64 s_ka[MERGE_TILE], s_kb[MERGE_TILE];
  __shared__ u32 s_ia[MERGE_TILE], s_ib[MERGE_TILE];
  const u32 tid = threadIdx.x, total = na + nb;
  const u32 d0 = blockIdx.x * MERGE_TILE, d1 = d0 + MERGE_TILE < total ? d0 + MERGE_TILE : total;
  const u32 a0 = split[blockIdx.x], a1 = split[blockIdx.x + 1], b0 = d0 - a0, b1 = d1 - a1;
  const u32 la = a1 - a0, lb = b1 - b0;                      // la + lb = d1 - d0 <= MERGE_TILE
  for (u32 i = tid; i < la; i += 256) { s_ka[i] = ka[a0 + i]; s_ia[i] = ia[a0 + i]; }
  for (u32 i = tid; i < lb; i += 256) { s_kb[i] = kb[b0 + i]; s_ib[i] = ib[b0 + i]; }
  __syncthreads();
  const u32 n_out = d1 - d0;
  const u32 e0 = tid * 8 < n_out ? tid * 8 : n_out, e1 = e0 + 8 < n_out ? e0 + 8 : n_out;
  u32 x = merge_split([&](u32 i) { return s_ka[i]; }, la, [&](u32 i) { return s_kb[i]; }, lb, e0);
  u32 y = e0 - x;
  u64 ok[8];
  u32 oi[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    ok[k] = 0; oi[k] = 0;
    if (e0 + k < e1) {
      const bool take_a = y >= lb || (x < la && s_ka[x] <= s_kb[y]);
      if (take_a) { ok[k] = s_ka[x]; oi[k] = s_ia[x]; ++x; }
      else { ok[k] = s_kb[y]; oi[k] = s_ib[y]; ++y; }
    }
  }
  __syncthreads();
  // the merged tile goes through LDS once more so that it leaves in coalesced stores
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (e0 + k < e1) { s_ka[e0 + k] = ok[k]; s_ia[e0 + k] = oi[k]; }
  __syncthreads();
  for (u32 i = tid; i < n_out; i += 256) { ko[d0 + i] = s_ka[i]; io[d0 + i] = s_ia[i]; }
}
void launch_merge(hipStream_t st, const uint64_t* ka, const uint32_t* ia, uint32_t na, const uint64_t* kb,
                  const uint32_t* ib, uint32_t nb, uint32_t* split, uint64_t* ko, uint32_t* io) {
  const uint64_t total = (uint64_t)na + nb;
  if (total == 0) return;
  const uint32_t n_tiles = (uint32_t)((total + MERGE_TILE - 1) / MERGE_TILE);
  hipLaunchKernelGGL(k_merge_splits, dim3((n_tiles + 1 + 255) / 256), dim3(256), 0, st, ka, na, kb, nb, n_tiles, split);
  hipLaunchKernelGGL(k_merge, dim3(n_tiles), dim3(256), 0, st, ka, ia, na, kb, ib, nb, (const uint32_t*)split, ko, io);
}

}  // namespace ccld
