// Dense placement for gfx950: the layout of the (communicator, operation counter, member slot) grid
// from the window's counter ranges, and the partition pass that moves every payload row into the fine
// bucket of its cell (Section 5.1: all ranks of a communicator bump the same operation counter, so
// the cell of a record follows from its Trace ID alone).
#include "dense.h"
#include "device_utils.h"

namespace ccld {

// ---- layout ------------------------------------------------------------------------------------------
// One workgroup: per communicator the rounds in the window, its fine buckets and its rows of the
// collective table (exclusive scans over the communicators).  The layout is infeasible (the caller then
// sorts) when a communicator is larger than a fine bucket, when the grid needs more fine buckets than
// the row array holds (counters that are far apart), or when two neighbouring coarse buckets of the
// batch span more fine buckets than a partition workgroup addresses.
__global__ __launch_bounds__(1024) void k_dense_layout(DenseArgs d) {
  __shared__ u32 s_wave[1024 / CCLD_WAVE];
  __shared__ u32 s_bad;
  const u32 tid = threadIdx.x;
  if (tid == 0) s_bad = 0;
  __syncthreads();
  u64 fb_carry = 0, seg_carry = 0;
  bool bad = false;
  for (u32 base = 0; base < d.n_comms; base += 1024) {
    const u32 c = base + tid;
    u32 rounds = 0, nfb = 0, rpb = 1;
    u64 mn = 0;
    if (c < d.n_comms) {
      const u64 mx = d.range[2 * c], inv = d.range[2 * c + 1];
      const u32 size = d.comm_size[c];
      if (size > DENSE_B) bad = true;
      else rpb = DENSE_B / size;
      if (mx | inv) {
        mn = ~inv;
        const u64 r = mx - mn + 1;                     // mx >= mn; r == 0 only for the full 64-bit range
        if (r == 0 || r > 0x7FFFFFFFull) bad = true;
        else { rounds = (u32)r; nfb = (rounds + rpb - 1) / rpb; }
      }
    }
    u32 tf, ts;
    const u32 ef = block_exclusive_sum<1024>(nfb, s_wave, &tf);
    const u32 es = block_exclusive_sum<1024>(rounds, s_wave, &ts);
    if (c < d.n_comms) {
      CommLayout L;
      L.seq_min = mn; L.fb_base = (u32)(fb_carry + ef); L.rpb = rpb; L.rounds = rounds; L.seg_base = (u32)(seg_carry + es);
      d.lay[c] = L;
    }
    fb_carry += tf; seg_carry += ts;
    // more rounds than records means a round without any record: the sort handles such windows
    if (fb_carry > d.fine_cap || seg_carry > d.n) bad = true;               // uniform: both sums are
  }
  if (tid == 0) {
    CommLayout L;
    L.seq_min = 0; L.fb_base = (u32)(fb_carry > d.fine_cap ? d.fine_cap : fb_carry); L.rpb = 1; L.rounds = 0;
    L.seg_base = (u32)seg_carry;
    d.lay[d.n_comms] = L;
  }
  if (bad) atomicOr(&s_bad, 1u);
  __threadfence_block();
  __syncthreads();
  // two neighbouring coarse buckets must fit the partition workgroup's table
  if (!s_bad) {
    bool wide = false;
    for (u32 b = tid; b < d.n_buckets; b += 1024) {
      u64 c0 = (u64)b << d.bshift, c1 = (u64)(b + 2) << d.bshift;
      if (c0 > d.n_comms) c0 = d.n_comms;
      if (c1 > d.n_comms) c1 = d.n_comms;
      if (d.lay[c1].fb_base - d.lay[c0].fb_base > DENSE_SPAN) wide = true;
    }
    if (wide) atomicOr(&s_bad, 1u);
  }
  __syncthreads();
  if (tid == 0) {
    d.hdr[DH_FEASIBLE] = s_bad ? 0u : 1u;
    d.hdr[DH_N_FINE] = s_bad ? 0u : (u32)fb_carry;
    d.hdr[DH_N_SEG] = s_bad ? 0u : (u32)seg_carry;
    if (s_bad) atomicOr((unsigned long long*)&d.counters[CNT_STATUS], (unsigned long long)DS_DENSE_FALLBACK);
    else d.counters[CNT_NSEG] = seg_carry;
  }
}

void launch_dense_layout(hipStream_t st, const DenseArgs& d) {
  hipLaunchKernelGGL(k_dense_layout, dim3(1), dim3(1024), 0, st, d);
}

// ---- partition --------------------------------------------------------------------------------------
// fine bucket and cell of a record from its ingest key
struct FineCell { u32 f, word; };      // word = cell << 4 | slot << 15 (op is OR-ed in by the caller)
__device__ __forceinline__ FineCell fine_cell_of(const DenseArgs& d, u64 key, u64 lo_mask, u32 slot_mask) {
  const u32 comm = d.kf.cb ? (u32)(key >> (64 - d.kf.cb)) : 0u;
  const u64 seq = (key & lo_mask) >> d.kf.mb;
  const u32 slot = (u32)key & slot_mask;
  const CommLayout L = d.lay[comm];
  const u32 rel = (u32)(seq - L.seq_min);
  const u32 fr = rel / L.rpb;
  const u32 rr = rel - fr * L.rpb;
  FineCell o;
  o.f = L.fb_base + fr;
  const u32 cell = rr * d.comm_size[comm] + slot;
  o.word = (cell << 4) | (slot << 15);
  return o;
}

// first index i in [0, n] with base[i] > v, minus one: the bucket that holds record v
__device__ __forceinline__ u32 bucket_of(const u32* __restrict__ base, u32 n_buckets, u32 v) {
  u32 lo = 0, hi = n_buckets;
  while (lo < hi) { const u32 m = (lo + hi) >> 1; if (base[m] <= v) lo = m + 1; else hi = m; }
  return lo ? lo - 1 : 0;
}

// One workgroup per slice of the batch.  The batch lies in coarse-bucket order (communicator >> bshift),
// so the fine buckets of a slice form one short range [f_lo, f_hi).  The workgroup counts its records
// per fine bucket, reserves one contiguous run of rows in each (one atomic per bucket), then takes
// PART_CHUNK records per round: it ranks them per bucket in LDS, stages the rows in (bucket, rank)
// order and writes them out with consecutive lanes on consecutive 16-byte pieces.  Pieces of a line
// that the round writes completely leave with the streaming hint, which keeps them from displacing
// the partially written lines at the buckets' frontiers from the L2.
constexpr u32 PART_THREADS = 1024;
constexpr u32 PART_U = 3;          // 3,072 records per round (96 KB of staged rows): the longest runs the LDS allows
constexpr u32 PART_CHUNK = PART_THREADS * PART_U;
__global__ __launch_bounds__(PART_THREADS) void k_dense_partition(DenseArgs d) {
  extern __shared__ uint4 s_dyn[];      // [2 PART_CHUNK] staged row halves | [PART_CHUNK] destinations | 3 x [DENSE_SPAN] tables
  __shared__ u32 s_wave[PART_THREADS / CCLD_WAVE];
  __shared__ u32 s_total;
  if (d.hdr[DH_FEASIBLE] == 0) return;
  uint4* s_row = s_dyn;
  u32* s_p = reinterpret_cast<u32*>(s_row + 2 * PART_CHUNK);
  u32* s_rc = s_p + PART_CHUNK;         // records per bucket: of the slice first, then of each round
  u32* s_pre = s_rc + DENSE_SPAN;       // exclusive scan of the round's counts
  u32* s_dst = s_pre + DENSE_SPAN;      // next free row of this workgroup's run in every bucket (~0: no room)
  const u32 tid = threadIdx.x;
  const u64 per = (((u64)d.n + gridDim.x - 1) / gridDim.x + PART_CHUNK - 1) / PART_CHUNK * PART_CHUNK;
  const u64 lo64 = per * blockIdx.x;
  if (lo64 >= d.n) return;
  const u32 lo = (u32)lo64, hi = (u32)((lo64 + per) < d.n ? (lo64 + per) : d.n);
  const u64 lo_mask = d.kf.cb > 0 ? (((u64)1 << (64 - d.kf.cb)) - 1) : ~0ull;
  const u32 slot_mask = d.kf.mb < 32 ? (1u << d.kf.mb) - 1 : ~0u;
  // fine buckets this slice can hold
  u32 f_lo, span;
  {
    const u32 b0 = bucket_of(d.bucket_base, d.n_buckets, lo), b1 = bucket_of(d.bucket_base, d.n_buckets, hi - 1);
    u64 c0 = (u64)b0 << d.bshift, c1 = (u64)(b1 + 1) << d.bshift;
    if (c0 > d.n_comms) c0 = d.n_comms;
    if (c1 > d.n_comms) c1 = d.n_comms;
    f_lo = d.lay[c0].fb_base;
    span = d.lay[c1].fb_base - f_lo;
  }
  if (span > DENSE_SPAN) {        // more than two coarse buckets in one slice: leave it to the sort
    if (tid == 0) atomicOr((unsigned long long*)&d.counters[CNT_STATUS], (unsigned long long)DS_DENSE_FALLBACK);
    return;
  }
  for (u32 i = tid; i < span; i += PART_THREADS) s_rc[i] = 0;
  __syncthreads();
  const u64* __restrict__ wkey = d.win_key;
  const uint4* __restrict__ wrow = reinterpret_cast<const uint4*>(d.win_row);
  auto phys = [&](u32 j) -> u32 { u32 p = d.head + j; if (p >= d.cap) p -= d.cap; return p; };
  // 1. records of the slice per fine bucket (the keys only)
  for (u32 j0 = lo + tid; j0 < hi; j0 += PART_THREADS * 4) {
    u64 k[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const u32 j = j0 + u * PART_THREADS;
      k[u] = j < hi ? wkey[phys(j)] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const u32 j = j0 + u * PART_THREADS;
      if (j < hi) {
        const u32 fi = fine_cell_of(d, k[u], lo_mask, slot_mask).f - f_lo;
        if (fi < span) atomicAdd(&s_rc[fi], 1u);
      }
    }
  }
  __syncthreads();
  // 2. one run of rows per bucket; a bucket that would overflow holds a duplicate key
  bool over = false;
  for (u32 i = tid; i < span; i += PART_THREADS) {
    const u32 cnt = s_rc[i];
    u32 dst = ~0u;
    if (cnt) {
      const u32 start = atomicAdd(&d.fill[f_lo + i], cnt);
      if ((u64)start + cnt <= DENSE_STRIDE) dst = (f_lo + i) * DENSE_STRIDE + start;
      else over = true;
    }
    s_dst[i] = dst;
    s_rc[i] = 0;
  }
  if (over) atomicOr((unsigned long long*)&d.counters[CNT_STATUS], (unsigned long long)DS_DUPLICATE);
  __syncthreads();
  // 3. rounds
  uint4* __restrict__ out = reinterpret_cast<uint4*>(d.rows);
  u64 key[PART_U], nkey[PART_U];
  uint4 r0[PART_U], r1[PART_U], n0[PART_U], n1[PART_U];
  auto load_round = [&](u32 base, u64 (&K)[PART_U], uint4 (&A)[PART_U], uint4 (&B)[PART_U]) {
#pragma unroll
    for (u32 u = 0; u < PART_U; ++u) {
      const u32 j = base + u * PART_THREADS + tid;
      if (j < hi) {
        const u32 p = phys(j);
        K[u] = __builtin_nontemporal_load(wkey + p);
        typedef u32 u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow + 2ull * p));
        const u32x4 b = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow + 2ull * p + 1));
        A[u] = make_uint4(a.x, a.y, a.z, a.w); B[u] = make_uint4(b.x, b.y, b.z, b.w);
      }
    }
  };
  load_round(lo, key, r0, r1);
  for (u32 base = lo; base < hi; base += PART_CHUNK) {
    u32 fi[PART_U], at[PART_U], word[PART_U];
    bool on[PART_U];
    if (base + PART_CHUNK < hi) load_round(base + PART_CHUNK, nkey, n0, n1);
#pragma unroll
    for (u32 u = 0; u < PART_U; ++u) {
      on[u] = base + u * PART_THREADS + tid < hi;
      if (!on[u]) continue;
      const FineCell fc = fine_cell_of(d, key[u], lo_mask, slot_mask);
      fi[u] = fc.f - f_lo; word[u] = fc.word;
      on[u] = fi[u] < span && s_dst[fi[u]] != ~0u;
      if (on[u]) at[u] = atomicAdd(&s_rc[fi[u]], 1u);
    }
    __syncthreads();
    {     // exclusive scan of the round's counts: consecutive buckets per thread
      constexpr u32 PER = (DENSE_SPAN + PART_THREADS - 1) / PART_THREADS;
      u32 v[PER], sum = 0;
#pragma unroll
      for (u32 i = 0; i < PER; ++i) { const u32 b = PER * tid + i; v[i] = b < span ? s_rc[b] : 0u; sum += v[i]; }
      u32 tot;
      u32 ex = block_exclusive_sum<PART_THREADS>(sum, s_wave, &tot);
#pragma unroll
      for (u32 i = 0; i < PER; ++i) { const u32 b = PER * tid + i; if (b < span) s_pre[b] = ex; ex += v[i]; }
      if (tid == 0) s_total = tot;
    }
    __syncthreads();
#pragma unroll
    for (u32 u = 0; u < PART_U; ++u) {
      if (!on[u]) continue;
      const u32 q = s_pre[fi[u]] + at[u];
      s_p[q] = s_dst[fi[u]] + at[u];
      s_row[2 * q] = r0[u];
      s_row[2 * q + 1] = make_uint4(r1[u].x, r1[u].y, (r1[u].z & 15u) | word[u], r1[u].w);
    }
    __syncthreads();
    const u32 total = s_total;
    typedef u32 u32x4 __attribute__((ext_vector_type(4)));
    for (u32 i = tid; i < 2 * total; i += PART_THREADS) {
      const u64 D = 2ull * s_p[i >> 1] + (i & 1);
      const u32 o = (u32)(D & 7);
      bool full = false;
      if (i >= o && i + 7 - o < 2 * total) {
        const u32 a = i - o, b = i + 7 - o;
        full = (2ull * s_p[a >> 1] + (a & 1) == D - o) && (2ull * s_p[b >> 1] + (b & 1) == D + 7 - o);
      }
      const uint4 v = s_row[i];
      if (full) { u32x4 vv = {v.x, v.y, v.z, v.w}; __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>(out + D)); }
      else out[D] = v;
    }
    // the runs grow; the round's counts go back to zero
    for (u32 i = tid; i < span; i += PART_THREADS) {
      const u32 c = s_rc[i];
      if (c) { s_dst[i] += c; s_rc[i] = 0; }
    }
    __syncthreads();
#pragma unroll
    for (u32 u = 0; u < PART_U; ++u) { key[u] = nkey[u]; r0[u] = n0[u]; r1[u] = n1[u]; }
  }
}

// ---- fine bucket descriptors ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_dense_desc(DenseArgs d) {
  if (d.hdr[DH_FEASIBLE] == 0) return;
  const u32 f = blockIdx.x * 256 + threadIdx.x;
  if (f >= d.hdr[DH_N_FINE]) return;
  // the communicator whose fine buckets include f: the last one whose first bucket is <= f
  u32 lo = 0, hi = d.n_comms;
  while (lo < hi) { const u32 m = (lo + hi) >> 1; if (d.lay[m].fb_base <= f) lo = m + 1; else hi = m; }
  const u32 c = lo - 1;
  const CommLayout L = d.lay[c];
  const u32 r0 = (f - L.fb_base) * L.rpb;
  FineDesc D;
  D.comm = c; D.size = d.comm_size[c];
  D.K = (L.rounds - r0) < L.rpb ? (L.rounds - r0) : L.rpb;
  D.rec0 = d.fill[f]; D.cnt = d.fill[f + 1] - D.rec0;
  D.srow0 = L.seg_base + r0;
  D.rel0 = L.seq_min + r0 - d.seq_base;
  d.desc[f] = D;
}
void launch_dense_desc(hipStream_t st, const DenseArgs& d) {
  hipLaunchKernelGGL(k_dense_desc, dim3((d.fine_cap + 255) / 256), dim3(256), 0, st, d);
}

void launch_dense_partition(hipStream_t st, const DenseArgs& d) {
  if (d.n == 0) return;
  const size_t lds = (size_t)PART_CHUNK * (32 + 4) + (size_t)DENSE_SPAN * 12;
  static bool raised = false;
  if (!raised) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dense_partition), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    raised = true;
  }
  hipLaunchKernelGGL(k_dense_partition, dim3(DENSE_PART_BLOCKS), dim3(PART_THREADS), lds, st, d);
}

}  // namespace ccld
