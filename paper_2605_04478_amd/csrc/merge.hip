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
// Key of an entry of the previous order in the new window's format.  An entry whose operation counter lies
// outside the new window's range has left the window (every record still there lies inside): it takes the
// smallest or the largest key of its communicator, so that the whole previous order, entries that left
// included, is still a non-decreasing sequence.
__device__ __forceinline__ u64 rebase(const RetainArgs& a, u64 k) {
  const int mb = a.from.mb;
  const u64 slot = k & (((u64)1 << mb) - 1);
  const u64 seq = ((k >> mb) & (((u64)1 << a.from.ws) - 1)) + a.from.seq_base;
  const u64 top = (k >> (mb + a.from.ws)) << (mb + a.to.ws);
  if (seq < a.to.seq_base) return top;
  const u64 rel = seq - a.to.seq_base;
  if ((rel >> a.to.ws) != 0) return top | (((u64)1 << (mb + a.to.ws)) - 1);
  return top | (rel << mb) | slot;
}

// entries of every tile of RET_TILE that are still in the window
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

// ---- merge ----------------------------------------------------------------------------------
// Merge path: output position d splits into x entries of the first sequence and d - x of the second,
// x = the smallest count for which the next entry of the first sequence is greater than the last one
// taken from the second.  The first sequence is the whole previous order (re-based keys), the second
// the sorted new records.  A workgroup merges the slices between two such splits, staged in LDS: every
// thread finds its own split inside the slices and merges eight entries; the entries that left the
// window are dropped as the tile is written, at the position that the kept entries before it fix.
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
__global__ __launch_bounds__(256) void k_merge_splits(RetainArgs a, const u64* __restrict__ kb, u32 nb, u32 n_tiles,
                                                      u32* __restrict__ split) {
  const u32 t = blockIdx.x * 256 + threadIdx.x;
  if (t > n_tiles) return;
  const u64 total = (u64)a.n + nb;
  const u32 d = (u64)t * MERGE_TILE < total ? t * MERGE_TILE : (u32)total;
  split[t] = merge_split([&](u32 i) { return rebase(a, a.key[i]); }, a.n, [&](u32 i) { return kb[i]; }, nb, d);
}
__global__ __launch_bounds__(256) void k_merge(RetainArgs a, const u64* __restrict__ kb, const u32* __restrict__ ib, u32 nb,
                                               const u32* __restrict__ split) {
  __shared__ u64 s_k[MERGE_TILE];        // the first sequence's slice, then the second's; later the tile that leaves
  __shared__ u32 s_i[MERGE_TILE];
  __shared__ u32 s_wave[4];
  static_assert(MERGE_TILE == 8 * 256 && RET_TILE == 8 * 256, "eight entries per thread");
  const u32 tid = threadIdx.x, total = a.n + nb;
  const u32 d0 = blockIdx.x * MERGE_TILE, d1 = d0 + MERGE_TILE < total ? d0 + MERGE_TILE : total;
  const u32 a0 = split[blockIdx.x], a1 = split[blockIdx.x + 1], b0 = d0 - a0, b1 = d1 - a1;
  const u32 la = a1 - a0, lb = b1 - b0, n_out = d1 - d0;     // la + lb = n_out <= MERGE_TILE
  // kept entries of the previous order before a0: whole tiles from the scanned counts, the rest counted here.
  // Every load of the workgroup is issued before the first one is waited for.
  const u32 t0 = a0 / RET_TILE;
  const u32 whole = a.tile_counts[t0];
  u32 pv[8], iv[8];
  u64 kv[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const u32 i = t0 * RET_TILE + k * 256 + tid;
    pv[k] = i < a0 ? a.idx[i] : 0u;
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const u32 j = k * 256 + tid;
    kv[k] = 0; iv[k] = 0;
    if (j < la) { kv[k] = a.key[a0 + j]; iv[k] = a.idx[a0 + j]; }
    else if (j < n_out) { kv[k] = kb[b0 + (j - la)]; iv[k] = ib[b0 + (j - la)]; }
  }
  u32 part = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) part += (t0 * RET_TILE + k * 256 + tid < a0 && still_there(a, pv[k])) ? 1u : 0u;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const u32 j = k * 256 + tid;
    if (j < n_out) { s_k[j] = j < la ? rebase(a, kv[k]) : kv[k]; s_i[j] = iv[k]; }
  }
  u32 before_a;
  block_exclusive_sum<256>(part, s_wave, &before_a);          // its barriers also publish the slices
  const u32 out0 = whole + before_a + b0;
  const u64* s_kb = s_k + la;
  const u32* s_ib = s_i + la;
  const u32 e0 = tid * 8 < n_out ? tid * 8 : n_out, e1 = e0 + 8 < n_out ? e0 + 8 : n_out;
  u32 x = merge_split([&](u32 i) { return s_k[i]; }, la, [&](u32 i) { return s_kb[i]; }, lb, e0);
  u32 y = e0 - x;
  u64 ok[8];
  u32 oi[8];
  u32 keep = 0, n_keep = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    ok[k] = 0; oi[k] = 0;
    if (e0 + k < e1) {
      const bool take_a = y >= lb || (x < la && s_k[x] <= s_kb[y]);
      if (take_a) { ok[k] = s_k[x]; oi[k] = s_i[x]; ++x; }
      else { ok[k] = s_kb[y]; oi[k] = s_ib[y]; ++y; }
      if (!take_a || still_there(a, oi[k])) { keep |= 1u << k; ++n_keep; }
    }
  }
  u32 tile_keep;
  u32 pos = block_exclusive_sum<256>(n_keep, s_wave, &tile_keep);    // barrier: every thread has read its entries
  // the kept entries go through LDS once more so that they leave in coalesced stores
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (keep & (1u << k)) { s_k[pos] = ok[k]; s_i[pos] = oi[k]; ++pos; }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const u32 i = k * 256 + tid;
    if (i < tile_keep) { a.key_out[out0 + i] = s_k[i]; a.idx_out[out0 + i] = s_i[i]; }
  }
}
void launch_merge_kept(hipStream_t st, const RetainArgs& a, const uint64_t* kb, const uint32_t* ib, uint32_t nb,
                       uint32_t* split) {
  const uint64_t total = (uint64_t)a.n + nb;
  if (total == 0) return;
  const u32 nt = (a.n + RET_TILE - 1) / RET_TILE;
  if (nt) hipLaunchKernelGGL(k_retain_count, dim3(nt), dim3(256), 0, st, a);
  launch_scan_tiles(st, a.tile_counts, nt, a.total_out);
  const uint32_t n_tiles = (uint32_t)((total + MERGE_TILE - 1) / MERGE_TILE);
  hipLaunchKernelGGL(k_merge_splits, dim3((n_tiles + 1 + 255) / 256), dim3(256), 0, st, a, kb, nb, n_tiles, split);
  hipLaunchKernelGGL(k_merge, dim3(n_tiles), dim3(256), 0, st, a, kb, ib, nb, (const uint32_t*)split);
}

}  // namespace ccld
