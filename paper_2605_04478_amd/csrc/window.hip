// Window analysis kernels for gfx950: ingest (validation, keys, bucketed placement), collective
// heads per tile, compaction of the late-rank flags, per-rank blame, the slow-detection rules
// (Eq. 1-4) per detection group, and hang alerts.  The per-collective statistics are in
// segments.hip, the sort in radix_sort.hip.
#include "window_kernels.h"
#include "device_utils.h"
#include "select.h"

namespace ccld {

constexpr i64 T_INFLIGHT = INT64_MAX;

__device__ __forceinline__ void atomic_or_u64(u64* p, u64 v) { atomicOr((unsigned long long*)p, (unsigned long long)v); }
__device__ __forceinline__ u64 atomic_add_u64(u64* p, u64 v) {
  return atomicAdd((unsigned long long*)p, (unsigned long long)v);
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill_u64(u64* p, u64 n, u64 v) {
  for (u64 i = (u64)blockIdx.x * 256 + threadIdx.x; i < n; i += (u64)gridDim.x * 256) p[i] = v;
}
__global__ __launch_bounds__(256) void k_fill_u32(u32* p, u64 n, u32 v) {
  for (u64 i = (u64)blockIdx.x * 256 + threadIdx.x; i < n; i += (u64)gridDim.x * 256) p[i] = v;
}
static void launch_fill_u32(hipStream_t st, uint32_t* p, uint64_t n, uint32_t v) {
  if (n == 0) return;
  u32 g = (u32)((n + 255) / 256); if (g > 4096) g = 4096;
  hipLaunchKernelGGL(k_fill_u32, dim3(g), dim3(256), 0, st, p, n, v);
}
void launch_fill_u64(hipStream_t st, uint64_t* p, uint64_t n, uint64_t v) {
  if (n == 0) return;
  u32 g = (u32)((n + 255) / 256); if (g > 4096) g = 4096;
  hipLaunchKernelGGL(k_fill_u64, dim3(g), dim3(256), 0, st, p, n, v);
}

// ------------------------------------------------------------------------------------------
// Ingest: validate each record, key it by Trace ID (communicator id, operation counter) plus
// rank, store key and payload row at the window's tail.
// Records per communicator bucket in each workgroup's slice of the batch (first half of the
// two-step placement below).
// With RANGE the kernel also reads the operation counters and leaves, per communicator, the batch's
// largest counter and the largest complement of one (i.e. ~smallest) in a.range (zeroed before): the
// dense placement lays the window out from these.
template <bool RANGE>
__global__ __launch_bounds__(256) void k_ingest_hist(IngestArgs a, u32 n_comms) {
  extern __shared__ u32 s_cnt[];
  // [n_buckets] counts, then (RANGE) [n_comms][2] extreme counters, 8-byte aligned
  unsigned long long* s_rng = reinterpret_cast<unsigned long long*>(s_cnt + ((a.n_buckets + 1) & ~1u));
  for (u32 b = threadIdx.x; b < a.n_buckets; b += 256) s_cnt[b] = 0;
  if (RANGE) for (u32 i = threadIdx.x; i < 2 * n_comms; i += 256) s_rng[i] = 0;
  // the batch's header starts from zero (the placement kernel, next on the stream, accumulates into it)
  if (blockIdx.x == 0 && threadIdx.x == 0) { a.meta->status = 0; a.meta->max_seq = 0; a.meta->max_inv_seq = 0; a.meta->pad = 0; }
  __syncthreads();
  const u64 chunk = a.chunk / a.hist_split;
  const u64 i_end = (chunk * (blockIdx.x + 1)) < a.n ? chunk * (blockIdx.x + 1) : a.n;
  const u32* __restrict__ in_comm = a.comm;
  const u64* __restrict__ in_seq = a.seq;
  for (u64 i0 = chunk * blockIdx.x + threadIdx.x; i0 < i_end; i0 += 256 * 8) {
    u32 c[8];
    u64 q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool on = i0 + (u64)u * 256 < i_end;
      c[u] = on ? __builtin_nontemporal_load(in_comm + i0 + (u64)u * 256) : 0xFFFFFFFFu;
      if (RANGE) q[u] = on ? __builtin_nontemporal_load(in_seq + i0 + (u64)u * 256) : 0ull;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (i0 + (u64)u * 256 < i_end) {
        atomicAdd(&s_cnt[c[u] < n_comms ? (c[u] >> a.bshift) : 0u], 1u);
        if (RANGE && c[u] < n_comms) {
          atomicMax(&s_rng[2 * c[u]], (unsigned long long)q[u]);
          atomicMax(&s_rng[2 * c[u] + 1], (unsigned long long)~q[u]);
        }
      }
  }
  __syncthreads();
  for (u32 b = threadIdx.x; b < a.n_buckets; b += 256) a.table[(u64)b * gridDim.x + blockIdx.x] = s_cnt[b];
  if (RANGE)
    for (u32 i = threadIdx.x; i < 2 * n_comms; i += 256)
      if (s_rng[i]) atomicMax((unsigned long long*)&a.range[i], s_rng[i]);
}
// exclusive scan of every bucket's row of per-workgroup counts (row length <= 2048)
__global__ __launch_bounds__(256) void k_ingest_scan(u32* table, u32* totals, u32 n_blocks) {
  __shared__ u32 s_wave[4];
  u32* row = table + (u64)blockIdx.x * n_blocks;
  u32 v[8], sum = 0;
  const u32 i0 = threadIdx.x * 8;
#pragma unroll
  for (int k = 0; k < 8; ++k) { v[k] = (i0 + k) < n_blocks ? row[i0 + k] : 0u; sum += v[k]; }
  u32 tot;
  u32 ex = block_exclusive_sum<256>(sum, s_wave, &tot);
#pragma unroll
  for (int k = 0; k < 8; ++k) { if ((i0 + k) < n_blocks) row[i0 + k] = ex; ex += v[k]; }
  if (threadIdx.x == 0) totals[blockIdx.x] = tot;
}

// Validation and key of one record (Trace ID = communicator id + operation counter, then the rank's
// member slot).  mem = the rank's packed membership row when the topology has one (memb4 != null).
__device__ __forceinline__ u64 ingest_key(u32 r, u32 c, u64 sq, u32 op, i64 te, i64 tx, const uint4& mem,
                                          const uint4* memb4, const DeviceTopology& T, const KeyFormat& kf,
                                          u32 slot_mask, u64& status, u64& maxseq, u64& maxinv) {
  u64 key = 0;
  if (c >= T.n_comms) {
    status |= DS_UNKNOWN_COMM;
    return key;
  }
  bool member = false;
  u32 slot = 0;
  if (memb4) {
    const u32 w = c == (mem.x >> kf.mb) ? mem.x : c == (mem.y >> kf.mb) ? mem.y : c == (mem.z >> kf.mb) ? mem.z : mem.w;
    member = c == (w >> kf.mb);
    slot = w & slot_mask;
  } else if (r < T.n_ranks) {
    for (u32 q = T.rank_comm_off[r]; q < T.rank_comm_off[r + 1]; ++q)
      if (T.rank_comms[q] == c) { member = true; slot = T.rank_slots[q]; }
  }
  if (!member) status |= DS_NOT_MEMBER;
  if (op >= CCLD_OP_MAX || te < 0 || te == T_INFLIGHT || tx < te) status |= DS_RANGE;
  if (kf.sb < 64 && (sq >> kf.sb) != 0) {
    status |= DS_KEY_WIDTH;
  } else {
    key = (kf.cb ? ((u64)c << (64 - kf.cb)) : 0ull) | (sq << kf.mb) | (u64)slot;
    maxseq = sq > maxseq ? sq : maxseq;
    maxinv = ~sq > maxinv ? ~sq : maxinv;
  }
  return key;
}

// status bits and the extreme operation counters of a workgroup leave through one set of atomics
template <int THREADS>
__device__ __forceinline__ void ingest_publish(u64 status, u64 maxseq, u64 maxinv, u64* s_status, u64* s_max,
                                               u64* s_inv, BatchMeta* meta) {
  u64 st = status;
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) st |= shfl_xor_u64(st, m);
  u64 mx = wave_max_u64(maxseq), mi = wave_max_u64(maxinv);
  const u32 lane = lane_id(), wave = threadIdx.x / CCLD_WAVE;
  if (lane == 0) { s_status[wave] = st; s_max[wave] = mx; s_inv[wave] = mi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    u64 S = 0, M = 0, I = 0;
    for (int w = 0; w < THREADS / CCLD_WAVE; ++w) {
      S |= s_status[w]; M = s_max[w] > M ? s_max[w] : M; I = s_inv[w] > I ? s_inv[w] : I;
    }
    if (S) atomic_or_u64(&meta->status, S);
    if (M) atomicMax((unsigned long long*)&meta->max_seq, (unsigned long long)M);
    if (I) atomicMax((unsigned long long*)&meta->max_inv_seq, (unsigned long long)I);
  }
}

// Validates and keys every record and stores it in the window.  Inside the batch's slot range the
// records are placed grouped by communicator bucket (the order inside a bucket is arbitrary), so
// that the analysis, which walks the window in (communicator, ...) order, gathers its payload rows
// from a small region at a time instead of from the whole window.
// THREADS = 512 with LDS_TABLE keeps a copy of the ranks' packed membership rows in LDS (16 bytes per
// rank): with records in random order that lookup is a gather with no locality, cheaper from LDS
// than from the L2.
template <int THREADS, bool LDS_TABLE>
__global__ __launch_bounds__(THREADS) void k_ingest(IngestArgs a, DeviceTopology T, KeyFormat kf) {
  constexpr int U = 4;               // records per thread in flight
  extern __shared__ uint4 s_dyn[];   // [n_ranks] membership rows (LDS_TABLE), then the buckets' next free slots
  __shared__ u64 s_status[THREADS / CCLD_WAVE], s_max[THREADS / CCLD_WAVE], s_inv[THREADS / CCLD_WAVE];
  u32* s_off = reinterpret_cast<u32*>(s_dyn + (LDS_TABLE ? T.n_ranks : 0u));
  for (u32 b = threadIdx.x; b < a.n_buckets; b += THREADS)
    s_off[b] = a.bucket_base[b] + a.table[((u64)b * gridDim.x + blockIdx.x) * a.hist_split];
  if (LDS_TABLE) {
    const uint4* __restrict__ g = reinterpret_cast<const uint4*>(T.rank_memb4);
    for (u32 r = threadIdx.x; r < T.n_ranks; r += THREADS) s_dyn[r] = g[r];
  }
  __syncthreads();
  u64 status = 0, maxseq = 0, maxinv = 0;      // maxinv = ~(smallest operation counter)
  const u32* __restrict__ in_rank = a.rank;
  const u32* __restrict__ in_comm = a.comm;
  const u64* __restrict__ in_seq = a.seq;
  const uint8_t* __restrict__ in_op = a.op;
  const u64* __restrict__ in_bytes = a.bytes;
  const i64* __restrict__ in_te = a.t_enter;
  const i64* __restrict__ in_tx = a.t_exit;
  u64* __restrict__ out_key = a.win_key;
  Row* __restrict__ out_row = a.win_row;
  const uint4* __restrict__ memb4 = reinterpret_cast<const uint4*>(T.rank_memb4);
  const u32 slot_mask = kf.mb < 32 ? (1u << kf.mb) - 1 : ~0u;
  // every workgroup walks one contiguous slice of the batch, so its nine streams advance page by page
  const u64 chunk = a.chunk;
  const u64 i_end = (chunk * (blockIdx.x + 1)) < a.n ? chunk * (blockIdx.x + 1) : a.n;
  for (u64 i0 = chunk * blockIdx.x + threadIdx.x; i0 < i_end; i0 += THREADS * U) {
    u32 r[U], c[U], op[U];
    u64 sq[U], nb[U];
    i64 te[U], tx[U];
    uint4 mem[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u64 i = i0 + (u64)u * THREADS;
      if (i < i_end) {
        r[u] = __builtin_nontemporal_load(in_rank + i); c[u] = __builtin_nontemporal_load(in_comm + i);
        sq[u] = __builtin_nontemporal_load(in_seq + i); op[u] = __builtin_nontemporal_load(in_op + i);
        nb[u] = __builtin_nontemporal_load(in_bytes + i);
        te[u] = __builtin_nontemporal_load(in_te + i); tx[u] = __builtin_nontemporal_load(in_tx + i);
      }
    }
    // the communicators of each rank with its member slot in each: one 16-byte row of words
    // comm << mb | slot when no rank is in more than four communicators
#pragma unroll
    for (int u = 0; u < U; ++u) {
      mem[u] = make_uint4(~0u, ~0u, ~0u, ~0u);
      if (i0 + (u64)u * THREADS < i_end && memb4 && r[u] < T.n_ranks) mem[u] = LDS_TABLE ? s_dyn[r[u]] : memb4[r[u]];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u64 i = i0 + (u64)u * THREADS;
      if (i >= i_end) continue;
      const u64 key = ingest_key(r[u], c[u], sq[u], op[u], te[u], tx[u], mem[u], memb4, T, kf, slot_mask, status, maxseq,
                                 maxinv);
      const u32 at = atomicAdd(&s_off[c[u] < T.n_comms ? (c[u] >> a.bshift) : 0u], 1u);
      u64 p = (u64)a.tail + at;
      if (p >= a.cap) p -= a.cap;
      out_key[p] = key;
      Row rw;
      rw.t_enter = te[u]; rw.t_exit = tx[u]; rw.bytes = nb[u]; rw.op = op[u];
      rw.pad = a.seqno0 + (u32)i;          // arrival number of the record (modulo 2^32)
      out_row[p] = rw;
    }
  }
  ingest_publish<THREADS>(status, maxseq, maxinv, s_status, s_max, s_inv, a.meta);
}
// Large batches: the same placement with the write-out regrouped in LDS.  A workgroup takes CHUNK
// records per round, gives each its slot in its bucket (LDS atomic, as above), then stages keys and
// rows in LDS ordered by (bucket, slot) and writes them out with consecutive lanes on consecutive
// 16-byte pieces: every bucket's share of the round leaves as one contiguous run instead of one
// scattered 40-byte store per lane.  At most INGEST_STAGED_BUCKETS buckets.
template <int THREADS, bool LDS_TABLE>
__global__ __launch_bounds__(THREADS) void k_ingest_staged(IngestArgs a, DeviceTopology T, KeyFormat kf) {
  constexpr int U = 2;
  constexpr u32 CHUNK = THREADS * U;
  // [n_ranks] membership rows (LDS_TABLE) | [2 CHUNK] row halves | [CHUNK] keys | [CHUNK] window slots
  extern __shared__ uint4 s_dyn[];
  __shared__ u64 s_status[THREADS / CCLD_WAVE], s_max[THREADS / CCLD_WAVE], s_inv[THREADS / CCLD_WAVE];
  __shared__ u32 s_off[INGEST_STAGED_BUCKETS], s_start[INGEST_STAGED_BUCKETS], s_pre[INGEST_STAGED_BUCKETS], s_total;
  __shared__ u32 s_scan[THREADS / CCLD_WAVE];
  uint4* s_row = s_dyn + (LDS_TABLE ? T.n_ranks : 0u);
  u64* s_key = reinterpret_cast<u64*>(s_row + 2 * CHUNK);
  u32* s_p = reinterpret_cast<u32*>(s_key + CHUNK);
  const u32 tid = threadIdx.x;
  if (tid < a.n_buckets) {
    const u32 o = a.bucket_base[tid] + a.table[((u64)tid * gridDim.x + blockIdx.x) * a.hist_split];
    s_off[tid] = o; s_start[tid] = o;
  }
  if (LDS_TABLE) {
    const uint4* __restrict__ g = reinterpret_cast<const uint4*>(T.rank_memb4);
    for (u32 r = tid; r < T.n_ranks; r += THREADS) s_dyn[r] = g[r];
  }
  __syncthreads();
  u64 status = 0, maxseq = 0, maxinv = 0;
  const u32* __restrict__ in_rank = a.rank;
  const u32* __restrict__ in_comm = a.comm;
  const u64* __restrict__ in_seq = a.seq;
  const uint8_t* __restrict__ in_op = a.op;
  const u64* __restrict__ in_bytes = a.bytes;
  const i64* __restrict__ in_te = a.t_enter;
  const i64* __restrict__ in_tx = a.t_exit;
  u64* __restrict__ out_key = a.win_key;
  uint4* __restrict__ out_row = reinterpret_cast<uint4*>(a.win_row);
  const uint4* __restrict__ memb4 = reinterpret_cast<const uint4*>(T.rank_memb4);
  const u32 slot_mask = kf.mb < 32 ? (1u << kf.mb) - 1 : ~0u;
  const u64 i_begin = a.chunk * blockIdx.x;
  const u64 i_end = (a.chunk * (blockIdx.x + 1)) < a.n ? a.chunk * (blockIdx.x + 1) : a.n;
  // the next round's columns are loaded while this round is staged and written out
  u32 r[U], c[U], op[U], nr[U], nc[U], nop[U];
  u64 sq[U], nb[U], nsq[U], nnb[U];
  i64 te[U], tx[U], nte[U], ntx[U];
  auto load_round = [&](u64 base, u32 (&R)[U], u32 (&C)[U], u64 (&S)[U], u32 (&O)[U], u64 (&B)[U], i64 (&E)[U], i64 (&X)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u64 i = base + (u64)u * THREADS + tid;
      if (i < i_end) {
        R[u] = __builtin_nontemporal_load(in_rank + i); C[u] = __builtin_nontemporal_load(in_comm + i);
        S[u] = __builtin_nontemporal_load(in_seq + i); O[u] = __builtin_nontemporal_load(in_op + i);
        B[u] = __builtin_nontemporal_load(in_bytes + i);
        E[u] = __builtin_nontemporal_load(in_te + i); X[u] = __builtin_nontemporal_load(in_tx + i);
      }
    }
  };
  load_round(i_begin, r, c, sq, op, nb, te, tx);
  for (u64 base = i_begin; base < i_end; base += CHUNK) {        // uniform over the workgroup
    u32 at[U], bk[U];
    u64 key[U];
    bool on[U];
#pragma unroll
    for (int u = 0; u < U; ++u) on[u] = base + (u64)u * THREADS + tid < i_end;
    load_round(base + CHUNK, nr, nc, nsq, nop, nnb, nte, ntx);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!on[u]) continue;
      uint4 mem = make_uint4(~0u, ~0u, ~0u, ~0u);
      if (memb4 && r[u] < T.n_ranks) mem = LDS_TABLE ? s_dyn[r[u]] : memb4[r[u]];
      key[u] = ingest_key(r[u], c[u], sq[u], op[u], te[u], tx[u], mem, memb4, T, kf, slot_mask, status, maxseq, maxinv);
      bk[u] = c[u] < T.n_comms ? (c[u] >> a.bshift) : 0u;
      at[u] = atomicAdd(&s_off[bk[u]], 1u);
    }
    __syncthreads();
    // this round's records per bucket -> where each bucket's run starts in the staging order
    if (a.n_buckets <= CCLD_WAVE) {
      if (tid < CCLD_WAVE) {
        const u32 cnt = tid < a.n_buckets ? s_off[tid] - s_start[tid] : 0u;
        const u32 inc = wave_inclusive_sum(cnt);
        s_pre[tid] = inc - cnt;
        if (tid == CCLD_WAVE - 1) s_total = inc;
      }
      __syncthreads();
    } else {
      const u32 cnt = tid < a.n_buckets ? s_off[tid] - s_start[tid] : 0u;
      u32 tot;
      const u32 ex = block_exclusive_sum<THREADS>(cnt, s_scan, &tot);
      if (tid < a.n_buckets) s_pre[tid] = ex;
      if (tid == 0) s_total = tot;
      __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!on[u]) continue;
      const u32 q = s_pre[bk[u]] + (at[u] - s_start[bk[u]]);
      u64 p = (u64)a.tail + at[u];
      if (p >= a.cap) p -= a.cap;
      s_p[q] = (u32)p;
      s_key[q] = key[u];
      const u64 last = (u64)op[u] | ((u64)(a.seqno0 + (u32)(base + (u64)u * THREADS + tid)) << 32);   // op, arrival number
      s_row[2 * q] = make_uint4((u32)te[u], (u32)((u64)te[u] >> 32), (u32)tx[u], (u32)((u64)tx[u] >> 32));
      s_row[2 * q + 1] = make_uint4((u32)nb[u], (u32)(nb[u] >> 32), (u32)last, (u32)(last >> 32));
    }
    __syncthreads();
    const u32 total = s_total;
    // Pieces of a line that this round writes completely leave with the streaming hint: they do not stay in
    // the L2, where they would displace the partially written lines at the buckets' frontiers before the
    // next round completes them.
    {
      typedef u32 u32x4 __attribute__((ext_vector_type(4)));
      for (u32 i = tid; i < 2 * total; i += THREADS) {
        const u64 D = 2ull * s_p[i >> 1] + (i & 1);
        const u32 o = (u32)(D & 7);
        bool full = false;
        if (i >= o && i + 7 - o < 2 * total) {
          const u32 lo = i - o, hi = i + 7 - o;
          full = (2ull * s_p[lo >> 1] + (lo & 1) == D - o) && (2ull * s_p[hi >> 1] + (hi & 1) == D + 7 - o);
        }
        const uint4 v = s_row[i];
        if (full) { u32x4 vv = {v.x, v.y, v.z, v.w}; __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>(out_row + D)); }
        else out_row[D] = v;
      }
      for (u32 q = tid; q < total; q += THREADS) {
        const u32 D = s_p[q];
        const u32 o = D & 15;
        bool full = false;
        if (q >= o && q + 15 - o < total) full = (s_p[q - o] == D - o) && (s_p[q + 15 - o] == D + 15 - o);
        if (full) __builtin_nontemporal_store(s_key[q], out_key + D);
        else out_key[D] = s_key[q];
      }
    }
    if (tid < a.n_buckets) s_start[tid] = s_off[tid];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      r[u] = nr[u]; c[u] = nc[u]; sq[u] = nsq[u]; op[u] = nop[u]; nb[u] = nnb[u]; te[u] = nte[u]; tx[u] = ntx[u];
    }
  }
  ingest_publish<THREADS>(status, maxseq, maxinv, s_status, s_max, s_inv, a.meta);
}

void launch_ingest(hipStream_t st, const IngestArgs& a_in, const DeviceTopology& T, const KeyFormat& kf) {
  if (a_in.n == 0) return;
  IngestArgs a = a_in;
  u64 g = (a.n + 255) / 256;
  if (g > INGEST_BLOCKS) g = INGEST_BLOCKS;
  a.hist_split = 1;
  const bool range = a.range != nullptr;
  const size_t lds = sizeof(u32) * a.n_buckets;
  const size_t lds_hist = sizeof(u32) * ((a.n_buckets + 1) & ~1u) + (range ? (size_t)16 * T.n_comms : 0);
  // large batches: one 1,024-thread workgroup per compute unit with the write-out regrouped in LDS, the
  // membership rows in LDS too when they fit beside the staging area; four counting workgroups per
  // placement workgroup
  const bool staged = a.n >= (1u << 22) && a.n_buckets <= INGEST_STAGED_BUCKETS;
  const size_t stage_bytes = (size_t)2048 * (32 + 8 + 4);
  const bool staged_table = staged && T.rank_memb4 && (u64)T.n_ranks * 16 + stage_bytes <= 156 * 1024;
  // otherwise, large batches over few enough ranks: half as many workgroups of twice the size, each with the
  // membership rows in LDS (two workgroups per compute unit)
  const bool lds_table = !staged && T.rank_memb4 && (u64)T.n_ranks * 16 + lds <= 72 * 1024 && a.n >= (1u << 22);
  if (staged) { g = 256; a.hist_split = 4; }
  else if (lds_table) g = (g + 1) / 2;
  const u64 unit = 256ull * a.hist_split;
  a.chunk = ((a.n + g - 1) / g + unit - 1) / unit * unit;
  const u32 g_hist = (u32)(g * a.hist_split);
  if (range) hipLaunchKernelGGL(k_ingest_hist<true>, dim3(g_hist), dim3(256), lds_hist, st, a, T.n_comms);
  else hipLaunchKernelGGL(k_ingest_hist<false>, dim3(g_hist), dim3(256), lds_hist, st, a, T.n_comms);
  hipLaunchKernelGGL(k_ingest_scan, dim3(a.n_buckets), dim3(256), 0, st, a.table, a.bucket_base, g_hist);
  launch_scan_tiles(st, a.bucket_base, a.n_buckets, a.scratch_total);
  static bool raised = false;       // more than 64 KB of dynamic LDS has to be asked for once
  if (!raised) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_ingest<512, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_ingest_staged<1024, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 156 * 1024);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_ingest_staged<1024, false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    raised = true;
  }
  if (staged_table)
    hipLaunchKernelGGL((k_ingest_staged<1024, true>), dim3((u32)g), dim3(1024), stage_bytes + (size_t)T.n_ranks * 16, st, a, T, kf);
  else if (staged)
    hipLaunchKernelGGL((k_ingest_staged<1024, false>), dim3((u32)g), dim3(1024), stage_bytes, st, a, T, kf);
  else if (lds_table)
    hipLaunchKernelGGL((k_ingest<512, true>), dim3((u32)g), dim3(512), lds + (size_t)T.n_ranks * 16, st, a, T, kf);
  else
    hipLaunchKernelGGL((k_ingest<256, false>), dim3((u32)g), dim3(256), lds, st, a, T, kf);
}

// ------------------------------------------------------------------------------------------
// In-place exclusive scan of per-tile counts by one workgroup; counts[n_tiles] and *total_out
// receive the total.
constexpr int SCAN_PER = 8;          // consecutive counts per thread and round
__device__ __forceinline__ void scan_load(const u32* counts, u32 i0, u32 n_tiles, bool vec, u32 (&v)[SCAN_PER]) {
  if (vec && i0 + SCAN_PER <= n_tiles) {
    const uint4 a = *reinterpret_cast<const uint4*>(counts + i0), b = *reinterpret_cast<const uint4*>(counts + i0 + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) v[k] = (i0 + k) < n_tiles ? counts[i0 + k] : 0u;
  }
}
__global__ __launch_bounds__(1024) void k_scan_tiles(u32* counts, u32 n_tiles, u64* total_out) {
  static_assert(SCAN_PER == 8, "two 16-byte pieces per thread");
  __shared__ u32 s_wave[1024 / CCLD_WAVE];
  const bool vec = (reinterpret_cast<uintptr_t>(counts) & 15) == 0;
  u32 carry = 0;
  u32 v[SCAN_PER], nv[SCAN_PER];
  scan_load(counts, threadIdx.x * SCAN_PER, n_tiles, vec, v);
  for (u32 b = 0; b < n_tiles; b += 1024 * SCAN_PER) {
    const u32 i0 = b + threadIdx.x * SCAN_PER;
    // the next round's counts are on their way while this round is scanned and stored
    scan_load(counts, i0 + 1024 * SCAN_PER, n_tiles, vec, nv);
    u32 sum = 0;
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) sum += v[k];
    u32 tot;
    u32 ex = carry + block_exclusive_sum<1024>(sum, s_wave, &tot);
    if (vec && i0 + SCAN_PER <= n_tiles) {
      u32 o[SCAN_PER];
#pragma unroll
      for (int k = 0; k < SCAN_PER; ++k) { o[k] = ex; ex += v[k]; }
      *reinterpret_cast<uint4*>(counts + i0) = make_uint4(o[0], o[1], o[2], o[3]);
      *reinterpret_cast<uint4*>(counts + i0 + 4) = make_uint4(o[4], o[5], o[6], o[7]);
    } else {
#pragma unroll
      for (int k = 0; k < SCAN_PER; ++k) { if ((i0 + k) < n_tiles) counts[i0 + k] = ex; ex += v[k]; }
    }
    carry += tot;
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) v[k] = nv[k];
  }
  if (threadIdx.x == 0) { counts[n_tiles] = carry; *total_out = carry; }
}
void launch_scan_tiles(hipStream_t st, uint32_t* counts, uint32_t n_tiles, uint64_t* total_out) {
  hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(1024), 0, st, counts, n_tiles, total_out);
}

// ------------------------------------------------------------------------------------------
// ------------------------------------------------------------------------------------------
// Ordered compaction of the flagged records into the flag list.
// eight consecutive flag bytes of one thread, as one 8-byte load where the tile is full
__device__ __forceinline__ u64 load_flags8(const uint8_t* __restrict__ f, u32 j0, u32 n) {
  if (j0 + 8 <= n && (reinterpret_cast<uintptr_t>(f + j0) & 7) == 0) return *reinterpret_cast<const u64*>(f + j0);
  u64 v = 0;
  for (u32 k = 0; k < 8; ++k) if (j0 + k < n) v |= (u64)f[j0 + k] << (8 * k);
  return v;
}
static_assert(SEL_TILE == 256 * 8, "one 8-byte piece of the flag bytes per thread");
__global__ __launch_bounds__(256) void k_flag_count(FlagArgs a) {
  __shared__ u32 s_wave[4];
  const u64 v = load_flags8(a.rec_flag, blockIdx.x * SEL_TILE + threadIdx.x * 8, a.n);
  u32 c = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) c += ((v >> (8 * k)) & 0xFF) != 0;
  u32 tot;
  block_exclusive_sum<256>(c, s_wave, &tot);
  if (threadIdx.x == 0) a.tile_flags[blockIdx.x] = tot;
}
__global__ __launch_bounds__(256) void k_flag_emit(FlagArgs a) {
  __shared__ u32 s_wave[4];
  const u32 j0 = blockIdx.x * SEL_TILE + threadIdx.x * 8;
  const int mb = a.sf.mb;
  const u64 mmask = ((u64)1 << mb) - 1, smask = ((u64)1 << a.sf.ws) - 1;
  const u64 v = load_flags8(a.rec_flag, j0, a.n);
  u32 c = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) c += ((v >> (8 * k)) & 0xFF) != 0;
  u32 tot;
  u32 k_out = a.tile_flags[blockIdx.x] + block_exclusive_sum<256>(c, s_wave, &tot);
  if (c == 0) return;
  for (u32 b = 0; b < 8; ++b) {
    const u32 f = (u32)(v >> (8 * b)) & 0xFF;
    if (!f) continue;
    const u32 j = j0 + b, k = k_out++;
    a.flag_pos[k] = j;
    if (a.flag && k < a.flag_cap) {
      const u64 key = a.key[j];
      const u32 comm = (u32)(key >> (mb + a.sf.ws));
      a.flag[(u64)CCLD_FLG_COMM * a.flag_cap + k] = (i64)comm;
      a.flag[(u64)CCLD_FLG_SEQ * a.flag_cap + k] = (i64)(((key >> mb) & smask) + a.sf.seq_base);
      a.flag[(u64)CCLD_FLG_RANK * a.flag_cap + k] =
          (i64)rank_of_slot(a.member_off, a.members_sorted, comm, (u32)(key & mmask));
      a.flag[(u64)CCLD_FLG_KIND * a.flag_cap + k] = (i64)f;
      a.flag[(u64)CCLD_FLG_LAG_ENTER * a.flag_cap + k] = a.flag_lag[j];
      a.flag[(u64)CCLD_FLG_LAG_EXIT * a.flag_cap + k] = a.flag_lag[a.cap_n + j];
    }
  }
}
void launch_flag_compact(hipStream_t st, const FlagArgs& a) {
  const u32 nt = (a.n + SEL_TILE - 1) / SEL_TILE;
  if (a.n) hipLaunchKernelGGL(k_flag_count, dim3(nt), dim3(256), 0, st, a);
  launch_scan_tiles(st, a.tile_flags, nt, &a.counters[CNT_NFLAG]);
  if (a.n) hipLaunchKernelGGL(k_flag_emit, dim3(nt), dim3(256), 0, st, a);
}

// ------------------------------------------------------------------------------------------
// One pass over the sorted keys for two results.
// (1) Collective heads per tile of SEG_TILE keys (a head = the first key of a (communicator,
//     operation counter) pair); equal neighbours are duplicates.
// (2) Records per rank.  The keys are sorted by communicator, so a workgroup's slice of them covers a
//     short run of communicators: it counts (communicator, member slot) pairs in an LDS table that
//     spans as many communicators as fit, then adds every non-zero cell to its rank's (zeroed) blame
//     column with one integer atomic.  A slice that covers more communicators takes several rounds.
constexpr u32 RC_CELLS = 8192;
constexpr u32 RC_MAX_TILES = 1024 + 8;      // tiles of one workgroup's slice (the launch keeps slices within 1024 tiles)
__global__ __launch_bounds__(256) void k_keys_pass(const u64* __restrict__ key, u32 n, SqueezedFormat sf,
                                                   const u32* __restrict__ member_off,
                                                   const u32* __restrict__ members_sorted,
                                                   const u32* __restrict__ comm_size, u32 n_ranks,
                                                   i64* __restrict__ blame, u32* __restrict__ tile_heads,
                                                   u64* __restrict__ counters) {
  __shared__ u32 s_h[RC_CELLS];
  __shared__ u32 s_tile[RC_MAX_TILES];
  __shared__ u32 s_end;
  const int mb = sf.mb, cshift = sf.mb + sf.ws;
  const u64 mmask = ((u64)1 << mb) - 1;
  const u32 slots = mb >= 13 ? RC_CELLS : (1u << mb);         // member slots covered by one round
  const u32 width = RC_CELLS / slots;                         // communicators covered by one round
  const u32 n_sub = mb >= 13 ? (1u << (mb - 13)) : 1u;        // rounds needed to cover every slot
  // slices of whole tiles
  const u64 per = (((u64)n + gridDim.x - 1) / gridDim.x + SEG_TILE - 1) / SEG_TILE * SEG_TILE;
  const u64 lo64 = per * blockIdx.x;
  if (lo64 >= n) return;
  const u32 lo = (u32)lo64, hi = (u32)((lo64 + per) < n ? (lo64 + per) : n);
  const u32 my_tiles = (hi - lo + SEG_TILE - 1) / SEG_TILE;
  for (u32 i = threadIdx.x; i < my_tiles; i += 256) s_tile[i] = 0;
  unsigned long long* out = (unsigned long long*)(blame + (u64)CCLD_BLM_N_RECORDS * n_ranks);
  bool dup = false;
  u32 pos = lo;
  while (pos < hi) {
    const u32 c0 = (u32)(key[pos] >> cshift);
    u32 end = hi;
    for (u32 sub = 0; sub < n_sub; ++sub) {
      const u32 s0 = sub * slots;
      for (u32 i = threadIdx.x; i < RC_CELLS; i += 256) s_h[i] = 0;
      if (threadIdx.x == 0) s_end = hi;
      __syncthreads();
      // eight keys per thread in flight; the keys are sorted, so the first one past the table's
      // communicators ends this thread's walk (that key is taken up by the next round)
      bool more = true;
      for (u32 j0 = pos + threadIdx.x; more && j0 < hi; j0 += 256 * 8) {
        u64 k[8], kp[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const u32 j = j0 + u * 256;
          k[u] = j < hi ? __builtin_nontemporal_load(key + j) : ~0ull;
        }
        // the key before each one sits in the lane below (a lane walks on no longer than the lanes
        // below it, so that lane is active); a wave's first lane reads it from memory
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const u32 j = j0 + u * 256;
          kp[u] = __shfl_up((unsigned long long)k[u], 1);
          if ((threadIdx.x & 63) == 0) kp[u] = (j < hi && j > 0) ? key[j - 1] : ~0ull;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const u32 j = j0 + u * 256;
          if (!more || j >= hi) continue;
          const u32 c = (u32)(k[u] >> cshift);
          if (c - c0 >= width) { atomicMin(&s_end, j); more = false; continue; }
          if (sub == 0) {
            if (j == 0 || (k[u] >> mb) != (kp[u] >> mb)) atomicAdd(&s_tile[(j - lo) / SEG_TILE], 1u);
            else dup |= (k[u] == kp[u]);
          }
          const u32 slot = (u32)(k[u] & mmask);
          if (slot - s0 < slots) atomicAdd(&s_h[(c - c0) * slots + (slot - s0)], 1u);
        }
      }
      __syncthreads();
      for (u32 i = threadIdx.x; i < RC_CELLS; i += 256) {
        const u32 v = s_h[i];
        if (!v) continue;
        const u32 c = c0 + i / slots, slot = s0 + i % slots;
        if (slot < comm_size[c]) atomicAdd(&out[members_sorted[member_off[c] + slot]], (unsigned long long)v);
      }
      end = s_end;
      __syncthreads();
    }
    pos = end;
  }
  for (u32 i = threadIdx.x; i < my_tiles; i += 256) tile_heads[lo / SEG_TILE + i] = s_tile[i];
  if (dup) atomic_or_u64(&counters[CNT_STATUS], DS_DUPLICATE);
}
void launch_keys_pass(hipStream_t st, const uint64_t* key, uint32_t n, const SqueezedFormat& sf,
                      const DeviceTopology& T, int64_t* blame, uint32_t* tile_heads, uint64_t* counters) {
  if (n == 0) return;
  uint32_t blocks = std::min<uint32_t>((n + 4095) / 4096, RANKCOUNT_BLOCKS);
  const uint32_t max_slice = (RC_MAX_TILES - 8) * (uint32_t)SEG_TILE;        // the per-tile counters of one slice fit in LDS
  blocks = std::max<uint32_t>(blocks, (uint32_t)(((uint64_t)n + max_slice - 1) / max_slice));
  hipLaunchKernelGGL(k_keys_pass, dim3(blocks), dim3(256), 0, st, key, n, sf, T.member_off, T.members_sorted,
                     T.size, T.n_ranks, blame, tile_heads, counters);
}

// Blame: key every flag by its rank, sort, then one wavefront per rank sums its run.
__global__ __launch_bounds__(256) void k_blame_keys(const u64* __restrict__ key, const u32* __restrict__ flag_pos,
                                                    u32 n_flag, SqueezedFormat sf, const u32* __restrict__ member_off,
                                                    const u32* __restrict__ members_sorted, u64* __restrict__ out_key) {
  const u32 k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n_flag) return;
  const u64 kk = key[flag_pos[k]];
  out_key[k] = rank_of_slot(member_off, members_sorted, (u32)(kk >> (sf.mb + sf.ws)), (u32)(kk & (((u64)1 << sf.mb) - 1)));
}
void launch_blame_keys(hipStream_t st, const uint64_t* key, const uint32_t* flag_pos, uint32_t n_flag,
                       const SqueezedFormat& sf, const DeviceTopology& T, uint64_t* out_key) {
  if (n_flag)
    hipLaunchKernelGGL(k_blame_keys, dim3((n_flag + 255) / 256), dim3(256), 0, st, key, flag_pos, n_flag, sf,
                       T.member_off, T.members_sorted, out_key);
}
// ends of every rank's run in the sorted flag keys: run[r] = first, run[n_ranks + r] = one past the
// last (both zero for a rank without a flag; the array is cleared before)
__global__ __launch_bounds__(256) void k_blame_runs(const u64* __restrict__ skey, u32 n_flag, u32 n_ranks,
                                                    u32* __restrict__ run) {
  const u32 q = blockIdx.x * 256 + threadIdx.x;
  if (q >= n_flag) return;
  const u64 r = skey[q];
  if (q == 0 || skey[q - 1] != r) run[r] = q;
  if (q + 1 == n_flag || skey[q + 1] != r) run[n_ranks + r] = q + 1;
}
// gridDim.y workgroups per rank: the rank's run in the sorted flag keys is dealt to them in pieces of 1,024
// flags, four flags per thread in flight (a faulty rank's run is tens of thousands of flags long).  The
// table was cleared before; the integer sums do not depend on the order of the additions.
__global__ __launch_bounds__(256) void k_blame_reduce(const u32* __restrict__ run, const u32* __restrict__ sidx,
                                                      const u32* __restrict__ flag_pos,
                                                      const uint8_t* __restrict__ rec_flag,
                                                      const i64* __restrict__ flag_lag, u64 cap_n, u32 n_ranks,
                                                      i64* __restrict__ blame) {
  __shared__ unsigned long long s_acc[4];
  const u32 r = blockIdx.x, tid = threadIdx.x;
  const u32 first = run[r], last = run[n_ranks + r];
  if ((u64)first + (u64)blockIdx.y * 1024 >= last) return;
  if (tid < 4) s_acc[tid] = 0;
  __syncthreads();
  u64 ne = 0, nx = 0, se = 0, sx = 0;
  for (u64 q1 = (u64)first + blockIdx.y * 1024 + tid; q1 < last; q1 += 1024ull * gridDim.y) {
    const u32 q0 = (u32)q1;
    u32 j[4], f[4];
    i64 le[4], lx[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) j[u] = (u64)q0 + u * 256 < last ? flag_pos[sidx[q0 + u * 256]] : 0xFFFFFFFFu;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      f[u] = 0; le[u] = 0; lx[u] = 0;
      if (j[u] != 0xFFFFFFFFu) { f[u] = rec_flag[j[u]]; le[u] = flag_lag[j[u]]; lx[u] = flag_lag[cap_n + j[u]]; }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (f[u] & CCLD_FLAG_LATE_ENTER) { ne += 1; se += (u64)le[u]; }
      if (f[u] & CCLD_FLAG_LATE_EXIT) { nx += 1; sx += (u64)lx[u]; }
    }
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    ne += shfl_xor_u64(ne, m); nx += shfl_xor_u64(nx, m); se += shfl_xor_u64(se, m); sx += shfl_xor_u64(sx, m);
  }
  if (lane_id() == 0) {
    atomicAdd(&s_acc[CCLD_BLM_N_LATE_ENTER], (unsigned long long)ne);
    atomicAdd(&s_acc[CCLD_BLM_N_LATE_EXIT], (unsigned long long)nx);
    atomicAdd(&s_acc[CCLD_BLM_SUM_LAG_ENTER], (unsigned long long)se);
    atomicAdd(&s_acc[CCLD_BLM_SUM_LAG_EXIT], (unsigned long long)sx);
  }
  __syncthreads();
  if (tid < 4 && s_acc[tid])
    atomicAdd(reinterpret_cast<unsigned long long*>(&blame[(u64)tid * n_ranks + r]), s_acc[tid]);
}
static_assert(CCLD_BLM_N_LATE_ENTER == 0 && CCLD_BLM_N_LATE_EXIT == 1 && CCLD_BLM_SUM_LAG_ENTER == 2 &&
              CCLD_BLM_SUM_LAG_EXIT == 3, "blame column order");
void launch_blame_reduce(hipStream_t st, const uint64_t* skey, const uint32_t* sidx, uint32_t n_flag,
                         const uint32_t* flag_pos, const uint8_t* rec_flag, const int64_t* flag_lag,
                         uint64_t cap_n, uint32_t n_ranks, uint32_t* run, int64_t* blame) {
  launch_fill_u32(st, run, 2ull * n_ranks, 0u);
  hipLaunchKernelGGL(k_blame_runs, dim3((n_flag + 255) / 256), dim3(256), 0, st, skey, n_flag, n_ranks, run);
  // no run is longer than n_flag: a few thousand flags need no second workgroup per rank
  const u32 split = std::min<u32>(std::max<u32>(n_flag / 4096, 1), 8);
  hipLaunchKernelGGL(k_blame_reduce, dim3(n_ranks, split), dim3(256), 0, st, (const u32*)run, sidx, flag_pos, rec_flag,
                     flag_lag, cap_n, n_ranks, blame);
}

// order[] = ranks by (flags descending, summed lag descending, rank ascending).  Ranks with any
// flag come first and only they need ranking: a wavefront per flagged rank counts the flagged
// ranks that precede it.  The ranks without a flag follow in ascending order.
struct PredBlamed {
  const i64 *ne, *nx;
  bool want;
  __device__ bool operator()(u32 r) const { return ((ne[r] + nx[r]) != 0) == want; }
};
__global__ __launch_bounds__(256) void k_blame_order(const i64* __restrict__ blame, u32 n_ranks,
                                                     const u32* __restrict__ lists, const u64* __restrict__ counters,
                                                     u32* __restrict__ order) {
  const u32 nb = (u32)counters[CNT_NBLAMED];
  const u32 lane = lane_id();
  const i64* NE = blame + (u64)CCLD_BLM_N_LATE_ENTER * n_ranks;
  const i64* NX = blame + (u64)CCLD_BLM_N_LATE_EXIT * n_ranks;
  const i64* SE = blame + (u64)CCLD_BLM_SUM_LAG_ENTER * n_ranks;
  const i64* SX = blame + (u64)CCLD_BLM_SUM_LAG_EXIT * n_ranks;
  for (u32 q = blockIdx.x * 4 + threadIdx.x / CCLD_WAVE; q < nb; q += gridDim.x * 4) {
    const u32 r = lists[q];
    const i64 myn = NE[r] + NX[r];
    const i64 mys = (i64)((u64)SE[r] + (u64)SX[r]);
    u32 before = 0;
    for (u32 i = lane; i < nb; i += CCLD_WAVE) {
      const u32 o = lists[i];
      const i64 on = NE[o] + NX[o];
      const i64 os = (i64)((u64)SE[o] + (u64)SX[o]);
      before += (on > myn) || (on == myn && (os > mys || (os == mys && o < r)));
    }
    before = wave_sum(before);
    if (lane == 0) order[before] = r;
  }
  const u32 stride = gridDim.x * 256;
  for (u32 i = blockIdx.x * 256 + threadIdx.x; i < n_ranks - nb; i += stride) order[nb + i] = lists[n_ranks + i];
}
void launch_blame_order(hipStream_t st, const int64_t* blame, uint32_t n_ranks, uint32_t* lists,
                        uint32_t* tile_counts, uint64_t* counters, uint32_t* order) {
  PredBlamed p{blame + (u64)CCLD_BLM_N_LATE_ENTER * n_ranks, blame + (u64)CCLD_BLM_N_LATE_EXIT * n_ranks, true};
  run_select(st, p, n_ranks, tile_counts, lists, &counters[CNT_NBLAMED]);
  p.want = false;
  run_select(st, p, n_ranks, tile_counts, lists + n_ranks, &counters[CNT_NCLEAN]);
  const u32 blocks = std::min<u32>((n_ranks + 3) / 4, 4096);
  hipLaunchKernelGGL(k_blame_order, dim3(std::max<u32>(blocks, 1)), dim3(256), 0, st, blame, n_ranks,
                     (const u32*)lists, (const u64*)counters, order);
}

// the blame table and its order handed to the caller: one launch for both
__global__ __launch_bounds__(256) void k_blame_out(const i64* __restrict__ blame, const u32* __restrict__ order_in,
                                                   u32 n_ranks, i64* __restrict__ table_out, u32* __restrict__ order_out) {
  const u64 nt = (u64)CCLD_BLM_NCOL * n_ranks, stride = (u64)gridDim.x * 256;
  for (u64 i = (u64)blockIdx.x * 256 + threadIdx.x; i < nt; i += stride) {
    if (table_out) table_out[i] = blame[i];
    if (order_out && i < n_ranks) order_out[i] = order_in[i];
  }
}
void launch_blame_out(hipStream_t st, const int64_t* blame, const uint32_t* order_in, uint32_t n_ranks, int64_t* table_out,
                      uint32_t* order_out) {
  if (n_ranks == 0 || (!table_out && !order_out)) return;
  const u64 nt = (u64)CCLD_BLM_NCOL * n_ranks;
  const u32 blocks = (u32)std::min<u64>((nt + 255) / 256, 2048);
  hipLaunchKernelGGL(k_blame_out, dim3(blocks), dim3(256), 0, st, blame, order_in, n_ranks, table_out, order_out);
}

// ------------------------------------------------------------------------------------------
// The detection-group key of every collective was written with its statistics: (communicator, op,
// floor(log2 bytes)) for a usable one, one value past every real key otherwise.  The table is in
// (communicator, operation counter) order, so a stable sort by this key lists every group's rounds in
// ascending operation counter, with the collectives that take no part at the end.
// number of usable collectives = position of the first key past the groups in the sorted keys
__global__ void k_group_bound(const u64* __restrict__ skey, u32 n_rows, u64 no_group, u64* __restrict__ counters) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  u32 lo = 0, hi = n_rows;
  while (lo < hi) { const u32 m = (lo + hi) / 2; if (skey[m] < no_group) lo = m + 1; else hi = m; }
  counters[CNT_NUSABLE] = lo;
}
struct PredGroupHead {
  const u64* skey; u64 no_group;
  __device__ bool operator()(u32 i) const { return skey[i] != no_group && (i == 0 || skey[i] != skey[i - 1]); }
};
void launch_group_heads(hipStream_t st, const uint64_t* skey, uint32_t n_rows, uint64_t no_group, uint32_t* tile_counts,
                        uint32_t* group_first, uint64_t* counters) {
  PredGroupHead p{skey, no_group};
  hipLaunchKernelGGL(k_group_bound, dim3(1), dim3(64), 0, st, skey, n_rows, no_group, counters);
  run_select(st, p, n_rows, tile_counts, group_first, &counters[CNT_NGROUP]);
}

// Eq. 1: baseline = mean of T_max over the first m rounds (m = min(tbase_rounds, rounds within the
// warm-up span)); Eq. 2: the window's round of largest T_max - T_min; Eq. 3: slow iff (T_max - T_base)/
// T_base > theta; Eq. 4: P = (T_max - T_min)/(T_max - T_base) against alpha / beta; repetition counter.
// All ratios cross-multiplied.  The numbers of groups and of usable collectives are read from the
// device counters, so the host does not have to learn them before this launch.
// T threads per group: one wavefront walks all groups and leaves those longer than GROUP_LONG rounds on a
// list (BIG = false); a second launch takes that list with a full workgroup per group (BIG = true).
constexpr u32 GROUP_LONG = GROUP_LONG_MIN;
template <int T, bool BIG>
__global__ __launch_bounds__(T) void k_group_eval(GroupArgs a, const u64* __restrict__ skey,
                                                    const u32* __restrict__ sidx,
                                                    const u32* __restrict__ group_first, u32* __restrict__ long_list) {
  __shared__ u32 s_i0, s_istar, s_kstar;
  __shared__ unsigned long long s_sum, s_best;
  const u32 tid = threadIdx.x;
  // a data error or an abandoned dense placement found by an earlier kernel of this analysis: the tables are
  // not valid and the detection state must stay as it is
  if (a.counters[CNT_STATUS] != 0) return;
  const u32 n_group = (u32)a.counters[CNT_NGROUP], n_usable = (u32)a.counters[CNT_NUSABLE];
  const u32 n_work = BIG ? (u32)a.counters[CNT_NLONG] : n_group;
  const i64* SEQ = a.seg + (u64)CCLD_SEG_SEQ * a.seg_cap;
  const i64* EMIN = a.seg + (u64)CCLD_SEG_ENTER_MIN * a.seg_cap;
  const i64* DMAX = a.seg + (u64)CCLD_SEG_DUR_MAX * a.seg_cap;
  const i64* DMIN = a.seg + (u64)CCLD_SEG_DUR_MIN * a.seg_cap;
  auto seq_of = [&](u32 i) -> u64 { return (u64)SEQ[sidx[i]]; };
  for (u32 w = blockIdx.x; w < n_work; w += gridDim.x) {
    const u32 g = BIG ? long_list[w] : w;
    const u32 f = group_first[g], e = (g + 1 < n_group) ? group_first[g + 1] : n_usable;
    if (!BIG && e - f > GROUP_LONG) {
      if (tid == 0) long_list[(u32)atomic_add_u64(&a.counters[CNT_NLONG], 1)] = g;
      continue;
    }
    const u64 gid = skey[f];                               // (comm*OP_MAX + op)*CLS + cls
    GroupState* G = a.gstate + gid;
    const GroupState g0 = *G;
    if (tid == 0) { s_i0 = e; s_istar = e; s_kstar = e; s_sum = 0; s_best = 0; }
    __syncthreads();
    // rounds not yet visited by Eq. 1 form a suffix (ascending operation counters): compare the last
    // round first; a fully visited group needs no search
    const bool any_new = seq_of(e - 1) + 1 > g0.baselined_wm;
    if (any_new) {
      // the first hit of a thread's ascending walk is its smallest, one atomic per thread
      u32 mine = e;
      for (u32 i = f + tid; i < e; i += T)
        if (seq_of(i) + 1 > g0.baselined_wm) { mine = i; break; }
      if (mine < e) atomicMin(&s_i0, mine);
    }
    // Eq. 2 needs the largest range; the first rounds of every thread stay in registers for the
    // second look below
    constexpr int KEEP = 4;
    unsigned long long kept[KEEP];
    {
      unsigned long long mine = 0;
#pragma unroll
      for (int j = 0; j < KEEP; ++j) {
        const u32 i = f + tid + (u32)T * j;
        kept[j] = i < e ? (unsigned long long)a.range_c[sidx[i]] : 0ull;
        mine = kept[j] > mine ? kept[j] : mine;
      }
      for (u32 i = f + tid + (u32)T * KEEP; i < e; i += T) {
        const unsigned long long v = (unsigned long long)a.range_c[sidx[i]];
        mine = v > mine ? v : mine;
      }
      if (mine) atomicMax(&s_best, mine);
    }
    __syncthreads();
    const u32 i0 = s_i0;
    const i64 t0 = (g0.cnt == 0 && i0 < e) ? EMIN[sidx[i0]] : g0.t0;
    if (!g0.frozen) {
      for (u32 i = i0 + tid; i < e; i += T) {
        const u32 s = sidx[i];
        const u64 q = i - i0;
        if ((u64)g0.cnt + q >= (u64)a.p.tbase_rounds || EMIN[s] - t0 > a.p.tbase_warmup_ns) atomicMin(&s_istar, i);
      }
    }
    const unsigned long long best = s_best;
    {
      u32 first = e;
#pragma unroll
      for (int j = KEEP - 1; j >= 0; --j) {
        const u32 i = f + tid + (u32)T * j;
        if (i < e && kept[j] == best) first = i;
      }
      if (first == e)
        for (u32 i = f + tid + (u32)T * KEEP; i < e; i += T)
          if ((unsigned long long)a.range_c[sidx[i]] == best) { first = i; break; }
      if (first < e) atomicMin(&s_kstar, first);
    }
    __syncthreads();
    const u32 istar = s_istar;
    if (!g0.frozen) {
      unsigned long long part = 0;
      for (u32 i = i0 + tid; i < istar; i += T) part += (unsigned long long)DMAX[sidx[i]];
      if (part) atomicAdd(&s_sum, part);
    }
    __syncthreads();
    if (tid == 0) {
    GroupState n = g0;
    if (!g0.frozen && i0 < e) {
      n.t0 = t0;
      n.sum = (i64)((u64)g0.sum + (u64)s_sum);
      n.cnt = g0.cnt + (istar - i0);
      if (istar > i0) n.baseline_last_seq = seq_of(istar - 1);
      if (istar < e) { n.frozen = 1; n.tbase_dyn = n.sum / (i64)n.cnt; }
    }
    if (i0 < e) n.baselined_wm = seq_of(e - 1) + 1;
    const u32 ks = s_kstar;
    const u32 sx = sidx[ks];
    const u64 rseq = seq_of(ks);
    const i64 tmax = DMAX[sx], tmin = DMIN[sx];
    const bool dynamic = n.frozen && rseq > n.baseline_last_seq;
    const i64 tbase = dynamic ? n.tbase_dyn : a.p.tbase_init_ns;
    const bool slow = (i128)(tmax - tbase) * (i128)a.p.theta_den > (i128)a.p.theta_num * (i128)tbase;
    int cls = CCLD_SLOW_NONE;
    i64 root1 = CCLD_NO_RANK;
    if (slow) {
      const i128 num = (i128)(tmax - tmin) * (i128)a.p.ab_den, den = (i128)(tmax - tbase);
      if (num > (i128)a.p.beta_num * den) cls = CCLD_SLOW_S1_COMPUTATION;
      else if (num < (i128)a.p.alpha_num * den) cls = CCLD_SLOW_S2_COMMUNICATION;
      else cls = CCLD_SLOW_S3_MIXED;
      if (cls != CCLD_SLOW_S2_COMMUNICATION) root1 = a.seg[(u64)CCLD_SEG_ARGMIN_RANK * a.seg_cap + sx];
      if (rseq + 1 > n.detected_wm) { n.repeats += 1; n.detected_wm = rseq + 1; }
    }
    *G = n;
    if (g < a.group_cap) {
      i64* O = a.group;
      const u64 C = a.group_cap;
      O[CCLD_GRP_COMM * C + g] = (i64)(gid / (CCLD_OP_MAX * GROUP_CLS));
      O[CCLD_GRP_OP * C + g] = (i64)((gid / GROUP_CLS) % CCLD_OP_MAX);
      O[CCLD_GRP_CLS * C + g] = (i64)(gid % GROUP_CLS);
      O[CCLD_GRP_N_USABLE * C + g] = (i64)(e - f);
      O[CCLD_GRP_RSTAR_SEQ * C + g] = (i64)rseq;
      O[CCLD_GRP_TMAX * C + g] = tmax;
      O[CCLD_GRP_TMIN * C + g] = tmin;
      O[CCLD_GRP_TBASE * C + g] = tbase;
      O[CCLD_GRP_STATIC * C + g] = dynamic ? 0 : 1;
      O[CCLD_GRP_FROZEN * C + g] = n.frozen;
      O[CCLD_GRP_M * C + g] = n.cnt;
      O[CCLD_GRP_SLOW * C + g] = slow ? 1 : 0;
      O[CCLD_GRP_CLASS * C + g] = cls;
      O[CCLD_GRP_ROOT_S1 * C + g] = root1;
      // communication-slow root (Eq. 4): the communicator's member of minimal SendRate / RecvRate
      O[CCLD_GRP_ROOT_S2 * C + g] = (cls == CCLD_SLOW_S2_COMMUNICATION || cls == CCLD_SLOW_S3_MIXED)
                                        ? a.rate_root[gid / (CCLD_OP_MAX * GROUP_CLS)] : (i64)CCLD_NO_RANK;
      O[CCLD_GRP_REPEATS * C + g] = n.repeats;
      O[CCLD_GRP_LOCATE * C + g] = (slow && n.repeats >= a.p.repeat_threshold) ? 1 : 0;
    }
    }
    __syncthreads();       // the shared cells are reused by the next group
  }
}
void launch_group_eval(hipStream_t st, const GroupArgs& a, const uint64_t* skey, const uint32_t* sidx,
                       const uint32_t* group_first, uint32_t* long_list) {
  hipLaunchKernelGGL((k_group_eval<64, false>), dim3(256 * 16), dim3(64), 0, st, a, skey, sidx, group_first, long_list);
  hipLaunchKernelGGL((k_group_eval<256, true>), dim3(256 * 4), dim3(256), 0, st, a, skey, sidx, group_first, long_list);
}

// ------------------------------------------------------------------------------------------
// Hang alerts: a collective with an operation in flight longer than the threshold, barriers
// excepted; class by the first two questions of the hang decision tree.
struct PredAlert {
  const i64 *inflight, *state, *imin;
  i64 now, thr;
  __device__ bool operator()(u32 s) const {
    return inflight[s] > 0 && !(state[s] & CCLD_SEG_BARRIER) && now - imin[s] > thr;
  }
};
void launch_alert_select(hipStream_t st, const AlertArgs& a) {
  PredAlert p{a.seg + (u64)CCLD_SEG_INFLIGHT * a.seg_cap, a.seg + (u64)CCLD_SEG_STATE * a.seg_cap,
              a.seg + (u64)CCLD_SEG_INFLIGHT_ENTER_MIN * a.seg_cap, a.now_ns, a.hang_threshold_ns};
  run_select(st, p, a.n_seg, a.tile_counts, a.alert_list, &a.counters[CNT_NALERT]);
}

// candidates of one alert, in ascending rank order; EMIT = false only counts them
template <bool EMIT>
__global__ __launch_bounds__(256) void k_alert_cand(AlertArgs a, u32 n_alert) {
  __shared__ u32 s_wave[4];
  const u32 al = blockIdx.x, tid = threadIdx.x;
  const u32 s = a.alert_list[al];
  const u64 C = a.seg_cap;
  const u32 comm = (u32)a.seg[CCLD_SEG_COMM * C + s];
  const u32 nn = (u32)a.seg[CCLD_SEG_N * C + s], ninfl = (u32)a.seg[CCLD_SEG_INFLIGHT * C + s];
  const u32 first = (u32)a.seg[CCLD_SEG_FIRST * C + s];
  const u32 size = a.topo.size[comm], moff = a.topo.member_off[comm];
  const u64 mmask = ((u64)1 << a.sf.mb) - 1;      // key slot = position among the members in ascending rank order
  const u32 off = EMIT ? a.alert_ncand[al] : 0u;
  int cls;
  u32 total = 0;
  if (nn < size) {
    cls = CCLD_HANG_H1_NOT_ENTERED;          // members with no record for this operation counter
    for (u32 q0 = 0; q0 < size; q0 += 256) {
      const u32 q = q0 + tid;
      bool miss = false;
      u32 r = 0;
      if (q < size) {
        r = a.topo.members_sorted[moff + q];
        u32 lo = first, hi = first + nn;
        while (lo < hi) { const u32 m = (lo + hi) / 2; if ((u32)(a.key[m] & mmask) < q) lo = m + 1; else hi = m; }
        miss = !(lo < first + nn && (u32)(a.key[lo] & mmask) == q);
      }
      u32 tot;
      const u32 ex = block_exclusive_sum<256>(miss ? 1u : 0u, s_wave, &tot);
      if (EMIT && miss && (u64)off + total + ex < a.cand_cap) a.cand[off + total + ex] = (i64)r;
      total += tot;
    }
  } else if (ninfl < nn) {
    cls = CCLD_HANG_H2_INCONSISTENT;         // everyone entered; the ranks that completed are the root
    for (u32 j0 = 0; j0 < nn; j0 += 256) {
      const u32 j = j0 + tid;
      bool done = false;
      u32 r = 0;
      if (j < nn) {
        r = a.topo.members_sorted[moff + (u32)(a.key[first + j] & mmask)];
        done = a.row[a.idx[first + j]].t_exit != T_INFLIGHT;
      }
      u32 tot;
      const u32 ex = block_exclusive_sum<256>(done ? 1u : 0u, s_wave, &tot);
      if (EMIT && done && (u64)off + total + ex < a.cand_cap) a.cand[off + total + ex] = (i64)r;
      total += tot;
    }
  } else {
    cls = CCLD_HANG_H3_HARDWARE;             // all hung: needs the Send/Recv counters
  }
  if (tid != 0) return;
  if (!EMIT) { a.alert_ncand[al] = total; return; }
  if (al < a.alert_cap) {
    const u64 A = a.alert_cap;
    a.alert[CCLD_ALR_COMM * A + al] = comm;
    a.alert[CCLD_ALR_SEQ * A + al] = a.seg[CCLD_SEG_SEQ * C + s];
    a.alert[CCLD_ALR_AGE * A + al] = a.now_ns - a.seg[CCLD_SEG_INFLIGHT_ENTER_MIN * C + s];
    a.alert[CCLD_ALR_CLASS * A + al] = cls;
    a.alert[CCLD_ALR_NCAND * A + al] = total;
    a.alert[CCLD_ALR_CAND_OFF * A + al] = off;
  }
}
void launch_alert_candidates(hipStream_t st, const AlertArgs& a, uint32_t n_alert) {
  if (n_alert == 0) return;
  hipLaunchKernelGGL(k_alert_cand<false>, dim3(n_alert), dim3(256), 0, st, a, n_alert);
  launch_scan_tiles(st, a.alert_ncand, n_alert, &a.counters[CNT_NCAND]);
  hipLaunchKernelGGL(k_alert_cand<true>, dim3(n_alert), dim3(256), 0, st, a, n_alert);
}

// ------------------------------------------------------------------------------------------
// position of every sorted record in the window's arrival order: its arrival number minus that of
// the window's oldest record (both modulo 2^32)
__global__ __launch_bounds__(256) void k_perm(const u32* __restrict__ idx, const Row* __restrict__ row, u32 n,
                                              u32 seqno_head, u32* perm) {
  const u32 j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  perm[j] = row[idx[j]].pad - seqno_head;
}
void launch_perm(hipStream_t st, const uint32_t* idx, const Row* row, uint32_t n, uint32_t seqno_head, uint32_t* perm) {
  if (n) hipLaunchKernelGGL(k_perm, dim3((n + 255) / 256), dim3(256), 0, st, idx, row, n, seqno_head, perm);
}

}  // namespace ccld
