// Hang location from progress-counter snapshots for gfx950: rows are placed into a dense grid
// [member slot][channel][snapshot], one wavefront per (rank, communicator) scans its channels'
// time series, one workgroup per communicator applies the hang decision tree and builds the
// ring / tree wait-for edges, victims are filtered across communicators, and the edges are
// walked to the roots.
#include <algorithm>
#include <cstring>
#include <mutex>

#include "ccld_internal.h"
#include "device_utils.h"
#include "select.h"
#include "window_kernels.h"

using namespace ccld;

namespace ccld {

struct HangArgs {
  // rows
  const u32 *snap, *rank, *comm, *channel;
  const u64* seq_posted;
  const u32 *sent, *recv;
  u64 n_rows;
  u32 n_snap, n_ch;
  int mb;             // bits of the position field in the packed membership words
  DeviceTopology T;
  u64 n_members;
  // grid
  u64* cell;          // [n_members * n_ch * n_snap][2]
  u32* cnt;           // presence bitmap, one bit per cell
  int exact;          // 1: the bitmap is kept (duplicates and gaps told apart); 0: cells start from an all-ones fill and a
                      //    cell that still holds it is suspect
  // tables
  i64* pair;          // [CCLD_HPAIR_NCOL][n_members]
  i64* hcomm;         // [CCLD_HCOMM_NCOL][n_comms]
  int* wait_slot;
  uint8_t* cand;
  u64* layer_max;
  u64* counters;
  u32 stall_snapshots, fifo_depth;
  // two-step placement of large grids: rows regrouped by region of 2^rb cells
  ulonglong2* part_pay;   // [n_regions << rb] cell contents
  u32* part_idx;          // [n_regions << rb] cell number inside the region
  u32* part_fill;         // [n_regions] rows received
  int rb;
  u32 n_regions;
};

#define PAIR(a, col, p) (a.pair[(u64)(col) * a.n_members + (p)])
#define HCOMM(a, col, c) (a.hcomm[(u64)(col) * a.T.n_comms + (c)])

// slot of rank r inside communicator c, or -1
__device__ __forceinline__ int slot_of(const DeviceTopology& T, u32 c, u32 r) {
  const u32 off = T.member_off[c], n = T.size[c];
  u32 lo = 0, hi = n;
  while (lo < hi) { const u32 m = (lo + hi) / 2; if (T.members_sorted[off + m] < r) lo = m + 1; else hi = m; }
  if (lo < n && T.members_sorted[off + lo] == r) return (int)T.sorted_slot[off + lo];
  return -1;
}

// Row of the snapshot grid (member index) of rank r in communicator c, or -1.  m: the rank's packed row of
// rank_cell4 when that table exists (words comm << pb | member index), else of rank_memb4 (comm << mb | sorted
// position), else unused.
__device__ __forceinline__ i64 grid_row_of(const HangArgs& a, u32 c, u32 r, const uint4& m) {
  if (r >= a.T.n_ranks) return -1;
  if (a.T.rank_cell4) {
    const int pb = a.T.pb;
    const u32 w = c == (m.x >> pb) ? m.x : c == (m.y >> pb) ? m.y : c == (m.z >> pb) ? m.z : m.w;
    return c == (w >> pb) ? (i64)(w & ((1u << pb) - 1u)) : -1;
  }
  int slot = -1;
  if (a.T.rank_memb4) {
    const u32 mmask = a.mb < 32 ? (1u << a.mb) - 1 : ~0u;
    const u32 w = c == (m.x >> a.mb) ? m.x : c == (m.y >> a.mb) ? m.y : c == (m.z >> a.mb) ? m.z : m.w;
    if (c == (w >> a.mb)) slot = (int)a.T.sorted_slot[a.T.member_off[c] + (w & mmask)];
  } else {
    slot = slot_of(a.T, c, r);
  }
  return slot < 0 ? -1 : (i64)a.T.member_off[c] + slot;
}
__device__ __forceinline__ uint4 grid_row_lookup(const HangArgs& a, u32 r) {
  const uint4* __restrict__ t = reinterpret_cast<const uint4*>(a.T.rank_cell4 ? a.T.rank_cell4 : a.T.rank_memb4);
  return (t && r < a.T.n_ranks) ? t[r] : make_uint4(~0u, ~0u, ~0u, ~0u);
}

// Status of one cell as the per-member passes read it.  With the bitmap: its bit.  Without: a cell that still
// holds the all-ones fill was (almost certainly) never written; the caller then repeats the placement with the
// bitmap, which tells a gap from a duplicate and from a row that really holds that pattern.
__device__ __forceinline__ u64 cell_status(const HangArgs& a, u64 cell, u64 w0, u64 w1) {
  if (a.exact) return ((a.cnt[cell >> 5] >> (cell & 31)) & 1u) ? 0 : (u64)DS_SNAPSHOT_GAP;
  return (w0 == ~0ull && w1 == ~0ull) ? (u64)DS_SUSPECT : 0;
}

// ---- place every row in its cell ------------------------------------------------------------
template <bool EXACT>
__global__ __launch_bounds__(256) void k_hang_place(HangArgs a) {
  constexpr int U = 4;               // rows per thread in flight
  u64 status = 0;
  ulonglong2* __restrict__ cell2 = reinterpret_cast<ulonglong2*>(a.cell);
  const u64 stride = (u64)gridDim.x * 256;
  for (u64 i0 = (u64)blockIdx.x * 256 + threadIdx.x; i0 < a.n_rows; i0 += stride * U) {
    u32 c[U], r[U], ch[U], sn[U], se[U], rv[U];
    u64 sq[U];
    bool on[U];
    // the seven columns are read once: streaming loads
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u64 i = i0 + stride * u;
      on[u] = i < a.n_rows;
      if (on[u]) {
        c[u] = __builtin_nontemporal_load(a.comm + i); r[u] = __builtin_nontemporal_load(a.rank + i);
        ch[u] = __builtin_nontemporal_load(a.channel + i); sn[u] = __builtin_nontemporal_load(a.snap + i);
        sq[u] = __builtin_nontemporal_load(a.seq_posted + i);
        se[u] = __builtin_nontemporal_load(a.sent + i); rv[u] = __builtin_nontemporal_load(a.recv + i);
      }
    }
    uint4 m[U];
#pragma unroll
    for (int u = 0; u < U; ++u) m[u] = on[u] ? grid_row_lookup(a, r[u]) : make_uint4(~0u, ~0u, ~0u, ~0u);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!on[u]) continue;
      if (c[u] >= a.T.n_comms) { status |= DS_UNKNOWN_COMM; continue; }
      const i64 p = grid_row_of(a, c[u], r[u], m[u]);
      if (p < 0) { status |= DS_NOT_MEMBER; continue; }
      if (ch[u] >= a.n_ch || sn[u] >= a.n_snap) { status |= DS_RANGE; continue; }
      const u64 k = ((u64)p * a.n_ch + ch[u]) * a.n_snap + sn[u];
      cell2[k] = make_ulonglong2(sq[u], (u64)se[u] | ((u64)rv[u] << 32));
      if (EXACT) {
        // presence bitmap (one bit per cell: small enough to stay in cache); a bit already set is a duplicate
        const u32 bit = 1u << (k & 31);
        if (atomicOr(&a.cnt[k >> 5], bit) & bit) status |= DS_DUPLICATE;
      }
    }
  }
  u64 st = status;
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) st |= shfl_xor_u64(st, m);
  if (lane_id() == 0 && st) atomicOr((unsigned long long*)&a.counters[CNT_STATUS], (unsigned long long)st);
}

// ---- placement of large grids in two steps ---------------------------------------------------------
// Rows arrive in any order, so placing them directly sends one 16-byte store per row to a random line of a
// grid that is far larger than the L2.  Here the rows are first regrouped by region of 2^rb cells (at most
// PART_REGIONS regions; a round's rows of one region leave as one run), then every region's rows are placed
// by workgroups that run side by side on one XCD, so that the eight cells of a line meet in that XCD's L2
// and reach memory as whole lines.  A region takes at most 2^rb rows; more can only arrive with duplicate
// cells, which the caller's exact pass reports.
constexpr u32 PART_REGIONS = 256;
constexpr int PART_THREADS = 512, PART_U = 4;
constexpr u32 PART_CHUNK = PART_THREADS * PART_U;
constexpr u32 PLACE_ROWS = 256;           // rows per workgroup of the second step (one per thread)

__global__ __launch_bounds__(PART_THREADS) void k_hang_part(HangArgs a, u64 chunk) {
  extern __shared__ ulonglong2 s_pay[];                    // [PART_CHUNK] contents | [PART_CHUNK] cell numbers | [PART_CHUNK] destinations
  u32* s_idx = reinterpret_cast<u32*>(s_pay + PART_CHUNK);
  u32* s_dst = s_idx + PART_CHUNK;
  __shared__ u32 s_cnt[PART_REGIONS], s_pre[PART_REGIONS], s_base[PART_REGIONS], s_scan[PART_THREADS / CCLD_WAVE], s_total;
  const u32 tid = threadIdx.x;
  u64 status = 0;
  const u32 cap = 1u << a.rb, kmask = cap - 1;
  const u64 i_begin = chunk * blockIdx.x;
  const u64 i_end = chunk * (blockIdx.x + 1) < a.n_rows ? chunk * (blockIdx.x + 1) : a.n_rows;
  if (tid < PART_REGIONS) s_cnt[tid] = 0;
  __syncthreads();
  u32 c[PART_U], r[PART_U], ch[PART_U], sn[PART_U], se[PART_U], rv[PART_U];
  u64 sq[PART_U];
  u32 nc[PART_U], nr[PART_U], nch[PART_U], nsn[PART_U], nse[PART_U], nrv[PART_U];
  u64 nsq[PART_U];
  auto load_round = [&](u64 base, u32 (&C)[PART_U], u32 (&R)[PART_U], u32 (&CH)[PART_U], u32 (&SN)[PART_U], u64 (&SQ)[PART_U],
                        u32 (&SE)[PART_U], u32 (&RV)[PART_U]) {
#pragma unroll
    for (int u = 0; u < PART_U; ++u) {
      const u64 i = base + (u64)u * PART_THREADS + tid;
      if (i < i_end) {
        C[u] = __builtin_nontemporal_load(a.comm + i); R[u] = __builtin_nontemporal_load(a.rank + i);
        CH[u] = __builtin_nontemporal_load(a.channel + i); SN[u] = __builtin_nontemporal_load(a.snap + i);
        SQ[u] = __builtin_nontemporal_load(a.seq_posted + i);
        SE[u] = __builtin_nontemporal_load(a.sent + i); RV[u] = __builtin_nontemporal_load(a.recv + i);
      }
    }
  };
  load_round(i_begin, c, r, ch, sn, sq, se, rv);
  for (u64 base = i_begin; base < i_end; base += PART_CHUNK) {       // uniform over the workgroup
    u32 at[PART_U], reg[PART_U], kin[PART_U];
    bool on[PART_U];
#pragma unroll
    for (int u = 0; u < PART_U; ++u) on[u] = base + (u64)u * PART_THREADS + tid < i_end;
    load_round(base + PART_CHUNK, nc, nr, nch, nsn, nsq, nse, nrv);     // the next round's columns are on their way meanwhile
    uint4 m[PART_U];
#pragma unroll
    for (int u = 0; u < PART_U; ++u) m[u] = on[u] ? grid_row_lookup(a, r[u]) : make_uint4(~0u, ~0u, ~0u, ~0u);
#pragma unroll
    for (int u = 0; u < PART_U; ++u) {
      if (!on[u]) continue;
      on[u] = false;
      if (c[u] >= a.T.n_comms) { status |= DS_UNKNOWN_COMM; continue; }
      const i64 p = grid_row_of(a, c[u], r[u], m[u]);
      if (p < 0) { status |= DS_NOT_MEMBER; continue; }
      if (ch[u] >= a.n_ch || sn[u] >= a.n_snap) { status |= DS_RANGE; continue; }
      const u64 k = ((u64)p * a.n_ch + ch[u]) * a.n_snap + sn[u];
      reg[u] = (u32)(k >> a.rb); kin[u] = (u32)k & kmask;
      at[u] = atomicAdd(&s_cnt[reg[u]], 1u);
      on[u] = true;
    }
    __syncthreads();
    {
      const u32 cnt = tid < a.n_regions ? s_cnt[tid] : 0u;
      u32 tot;
      const u32 ex = block_exclusive_sum<PART_THREADS>(cnt, s_scan, &tot);
      if (tid < a.n_regions) {
        s_pre[tid] = ex;
        s_base[tid] = cnt ? atomicAdd(&a.part_fill[tid], cnt) : 0u;
      }
      if (tid == 0) s_total = tot;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PART_U; ++u) {
      if (!on[u]) continue;
      const u32 q = s_pre[reg[u]] + at[u];
      const u32 pos = s_base[reg[u]] + at[u];
      if (pos >= cap) status |= DS_SUSPECT;              // more rows than cells: some cell is written twice
      s_dst[q] = pos < cap ? ((reg[u] << a.rb) + pos) : ~0u;
      s_idx[q] = kin[u];
      s_pay[q] = make_ulonglong2(sq[u], (u64)se[u] | ((u64)rv[u] << 32));
    }
    __syncthreads();
    const u32 total = s_total;
    for (u32 i = tid; i < total; i += PART_THREADS) {
      const u32 D = s_dst[i];
      if (D == ~0u) continue;
      // pieces of a line that this round writes completely leave with the streaming hint
      const u32 o = D & 7;
      const bool full = i >= o && i + 7 - o < total && s_dst[i - o] == D - o && s_dst[i + 7 - o] == D + 7 - o;
      const ulonglong2 v = s_pay[i];
      if (full) {
        typedef u64 u64x2 __attribute__((ext_vector_type(2)));
        u64x2 vv = {v.x, v.y};
        __builtin_nontemporal_store(vv, reinterpret_cast<u64x2*>(a.part_pay + D));
      } else {
        a.part_pay[D] = v;
      }
      a.part_idx[D] = s_idx[i];
    }
    if (tid < PART_REGIONS) s_cnt[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PART_U; ++u) { c[u] = nc[u]; r[u] = nr[u]; ch[u] = nch[u]; sn[u] = nsn[u]; sq[u] = nsq[u]; se[u] = nse[u]; rv[u] = nrv[u]; }
  }
  u64 st = status;
#pragma unroll
  for (int m2 = 32; m2 >= 1; m2 >>= 1) st |= shfl_xor_u64(st, m2);
  if (lane_id() == 0 && st) atomicOr((unsigned long long*)&a.counters[CNT_STATUS], (unsigned long long)st);
}

// Second step: workgroup i runs on XCD i % 8 (workgroups are dealt to the XCDs in turn); XCD x takes the regions
// x, x + 8, ... one after the other, wpr consecutive workgroups of the XCD per region.
__global__ __launch_bounds__(256) void k_hang_place_regions(HangArgs a, u32 wpr) {
  const u32 xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const u32 reg = xcd + 8 * (j / wpr), part = j % wpr;
  if (reg >= a.n_regions) return;
  const u32 cap = 1u << a.rb;
  const u32 have = a.part_fill[reg];
  const u32 cnt = have < cap ? have : cap;
  ulonglong2* __restrict__ cell2 = reinterpret_cast<ulonglong2*>(a.cell) + ((u64)reg << a.rb);
  const ulonglong2* __restrict__ pay = a.part_pay + ((u64)reg << a.rb);
  const u32* __restrict__ idx = a.part_idx + ((u64)reg << a.rb);
  const u32 i = part * PLACE_ROWS + threadIdx.x;
  if (i >= cnt) return;
  typedef u64 u64x2 __attribute__((ext_vector_type(2)));
  const u32 k = __builtin_nontemporal_load(idx + i);                 // read once: streaming loads
  const u64x2 t = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(pay + i));
  cell2[k] = make_ulonglong2(t.x, t.y);
}

// ---- per (rank, communicator): stalled, operation counter, chunk totals, onset -------------------
// One wavefront per member slot; lanes read consecutive snapshots of one channel.
__global__ __launch_bounds__(256) void k_hang_pairs(HangArgs a) {
  const u32 lane = lane_id();
  const u64 p = (u64)blockIdx.x * 4 + threadIdx.x / CCLD_WAVE;
  if (p >= a.n_members) return;
  const u32 L = a.n_snap - 1, W = a.stall_snapshots;
  const bool can_stall = L >= W;
  bool stalled = can_stall;
  u64 seq = 0, S = 0, R = 0;
  u32 onset = 0;
  u64 status = 0;
  for (u32 ch = 0; ch < a.n_ch; ++ch) {
    const u64 base = (p * a.n_ch + ch) * a.n_snap;
    const u64 sL0 = a.cell[2 * (base + L)], sL1 = a.cell[2 * (base + L) + 1];
    if (can_stall) {
      const u64 o0 = a.cell[2 * (base + L - W)], o1 = a.cell[2 * (base + L - W) + 1];
      if (o0 != sL0 || o1 != sL1) stalled = false;
    }
    u32 last_diff = 0;        // 1 + the last snapshot whose state differs from the final one
    for (u32 s0 = 0; s0 < a.n_snap; s0 += CCLD_WAVE) {
      const u32 s = s0 + lane;
      bool diff = false;
      if (s < a.n_snap) {
        const u64 w0 = a.cell[2 * (base + s)], w1 = a.cell[2 * (base + s) + 1];
        diff = w0 != sL0 || w1 != sL1;
        status |= cell_status(a, base + s, w0, w1);
      }
      const u64 m = ballot64(diff);
      if (m) last_diff = s0 + (64 - (u32)__clzll((long long)m));
    }
    onset = last_diff > onset ? last_diff : onset;
    seq = sL0 > seq ? sL0 : seq;
    S += sL1 & 0xFFFFFFFFull;
    R += sL1 >> 32;
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) status |= shfl_xor_u64(status, m);
  if (lane == 0) {
    if (status) atomicOr((unsigned long long*)&a.counters[CNT_STATUS], (unsigned long long)status);
    // communicator of this slot: the last one whose offset is <= p
    u32 lo = 0, hi = a.T.n_comms;
    while (hi - lo > 1) { const u32 m = (lo + hi) / 2; if (a.T.member_off[m] <= p) lo = m; else hi = m; }
    PAIR(a, CCLD_HPAIR_RANK, p) = a.T.members[p];
    PAIR(a, CCLD_HPAIR_COMM, p) = lo;
    PAIR(a, CCLD_HPAIR_STALLED, p) = stalled ? 1 : 0;
    PAIR(a, CCLD_HPAIR_ENTERED, p) = 0;
    PAIR(a, CCLD_HPAIR_SEQ, p) = (i64)seq;
    PAIR(a, CCLD_HPAIR_SENT, p) = (i64)S;
    PAIR(a, CCLD_HPAIR_RECV, p) = (i64)R;
    PAIR(a, CCLD_HPAIR_WAITS_ON, p) = CCLD_NO_RANK;
    PAIR(a, CCLD_HPAIR_HOPS, p) = -1;
    PAIR(a, CCLD_HPAIR_ONSET, p) = onset;
    a.wait_slot[p] = -1;
    a.cand[p] = 0;
    a.layer_max[p] = 0;
  }
}

// ---- per communicator: entered, idle test, decision tree, wait-for edges ------------------------
__global__ __launch_bounds__(256) void k_hang_comm(HangArgs a) {
  __shared__ unsigned long long s_seqmax, s_minsum, s_minrecv, s_worst;
  __shared__ u32 s_flags, s_best, s_ncand;      // flags: 1 not all entered, 2 any stalled, 4 not all stalled, 8 not idle
  const u32 c = blockIdx.x, tid = threadIdx.x;
  const u32 n = a.T.size[c], off = a.T.member_off[c];
  const bool tree = a.T.algo[c] == CCLD_ALGO_TREE;
  if (tid == 0) { s_seqmax = 0; s_minsum = ~0ull; s_minrecv = ~0ull; s_worst = 0; s_flags = 0; s_best = 0xFFFFFFFFu; s_ncand = 0; }
  __syncthreads();
  {     // every thread reduces its own members first: one LDS atomic per thread, not per member
    unsigned long long mine = 0;
    for (u32 q = tid; q < n; q += 256) {
      const unsigned long long v = (unsigned long long)PAIR(a, CCLD_HPAIR_SEQ, off + q);
      mine = v > mine ? v : mine;
    }
    if (tid < n) atomicMax(&s_seqmax, mine);
  }
  __syncthreads();
  const u64 seq_max = s_seqmax;
  // depth of a slot in the tree (layers are contiguous in BFS order)
  auto depth_of = [&](u32 q) -> u32 {
    u32 d = 0;
    if (tree) { int cur = (int)q; while (a.T.tree_parent[off + cur] >= 0) { cur = a.T.tree_parent[off + cur]; ++d; } }
    return d;
  };
  {
    u32 fl = 0;
    unsigned long long minsum = ~0ull;
    for (u32 q = tid; q < n; q += 256) {
      const u64 p = off + q;
      const bool entered = (u64)PAIR(a, CCLD_HPAIR_SEQ, p) == seq_max;
      PAIR(a, CCLD_HPAIR_ENTERED, p) = entered ? 1 : 0;
      if (!entered) fl |= 1 | 8;
      if (PAIR(a, CCLD_HPAIR_STALLED, p)) fl |= 2; else fl |= 4;
      // identical totals across comparable ranks: every adjacent pair of the same layer
      if (q > 0 && (!tree || depth_of(q) == depth_of(q - 1)) &&
          (PAIR(a, CCLD_HPAIR_SENT, p) != PAIR(a, CCLD_HPAIR_SENT, p - 1) ||
           PAIR(a, CCLD_HPAIR_RECV, p) != PAIR(a, CCLD_HPAIR_RECV, p - 1)))
        fl |= 8;
      const unsigned long long sum = (unsigned long long)(PAIR(a, CCLD_HPAIR_SENT, p) + PAIR(a, CCLD_HPAIR_RECV, p));
      minsum = sum < minsum ? sum : minsum;
      if (tree) atomicMax((unsigned long long*)&a.layer_max[off + depth_of(q)], sum);
    }
    if (fl) atomicOr(&s_flags, fl);
    if (tid < n) atomicMin(&s_minsum, minsum);
  }
  __syncthreads();
  // fewest SendCount + RecvCount, then fewest received, then smallest rank
  {
    const unsigned long long ms = s_minsum;
    unsigned long long mr = ~0ull;
    for (u32 q = tid; q < n; q += 256)
      if ((u64)(PAIR(a, CCLD_HPAIR_SENT, off + q) + PAIR(a, CCLD_HPAIR_RECV, off + q)) == ms) {
        const unsigned long long v = (unsigned long long)PAIR(a, CCLD_HPAIR_RECV, off + q);
        mr = v < mr ? v : mr;
      }
    if (mr != ~0ull) atomicMin(&s_minrecv, mr);
  }
  __syncthreads();
  {
    const unsigned long long ms = s_minsum, mr = s_minrecv;
    u32 best = 0xFFFFFFFFu;
    for (u32 q = tid; q < n; q += 256)
      if ((u64)(PAIR(a, CCLD_HPAIR_SENT, off + q) + PAIR(a, CCLD_HPAIR_RECV, off + q)) == ms &&
          (u64)PAIR(a, CCLD_HPAIR_RECV, off + q) == mr) {
        const u32 rk = (u32)PAIR(a, CCLD_HPAIR_RANK, off + q);
        best = rk < best ? rk : best;
      }
    if (best != 0xFFFFFFFFu) atomicMin(&s_best, best);
  }
  __syncthreads();
  const u32 flags = s_flags;
  const bool all_entered = !(flags & 1), any_stalled = flags & 2, all_stalled = !(flags & 4), idle_ok = !(flags & 8);
  const bool hung = !idle_ok && any_stalled;
  int cls = 0;
  if (hung) cls = !all_entered ? CCLD_HANG_H1_NOT_ENTERED : (!all_stalled ? CCLD_HANG_H2_INCONSISTENT : CCLD_HANG_H3_HARDWARE);
  if (tid == 0) {
    HCOMM(a, CCLD_HCOMM_COMM, c) = c;
    HCOMM(a, CCLD_HCOMM_HUNG, c) = hung ? 1 : 0;
    HCOMM(a, CCLD_HCOMM_CLASS, c) = cls;
    HCOMM(a, CCLD_HCOMM_SEQ_MAX, c) = (i64)seq_max;
    HCOMM(a, CCLD_HCOMM_ROOT_BY_COUNT, c) = hung ? (i64)s_best : CCLD_NO_RANK;
    HCOMM(a, CCLD_HCOMM_NCAND, c) = 0;
  }
  if (!hung) return;
  if (cls == CCLD_HANG_H1_NOT_ENTERED) {
    for (u32 q = tid; q < n; q += 256) if (!PAIR(a, CCLD_HPAIR_ENTERED, off + q)) a.cand[off + q] = 1;
    return;
  }
  if (cls == CCLD_HANG_H2_INCONSISTENT) {
    for (u32 q = tid; q < n; q += 256) if (!PAIR(a, CCLD_HPAIR_STALLED, off + q)) a.cand[off + q] = 1;
    return;
  }
  // all entered, all hung
  if (!tree) {
    for (u32 q = tid; q < n; q += 256) {
      const u32 pred = (q + n - 1) % n, succ = (q + 1) % n;
      const i64 Rq = PAIR(a, CCLD_HPAIR_RECV, off + q), Sq = PAIR(a, CCLD_HPAIR_SENT, off + q);
      if (n > 1 && Rq >= PAIR(a, CCLD_HPAIR_SENT, off + pred)) {
        PAIR(a, CCLD_HPAIR_WAITS_ON, off + q) = PAIR(a, CCLD_HPAIR_RANK, off + pred);
        a.wait_slot[off + q] = (int)pred;
      } else if (n > 1 && Sq - PAIR(a, CCLD_HPAIR_RECV, off + succ) >= (i64)a.fifo_depth) {
        PAIR(a, CCLD_HPAIR_WAITS_ON, off + q) = PAIR(a, CCLD_HPAIR_RANK, off + succ);
        a.wait_slot[off + q] = (int)succ;
      } else {
        a.cand[off + q] = 1;
        atomicAdd(&s_ncand, 1u);
      }
    }
  } else {
    for (u32 q = tid; q < n; q += 256) {
      const u64 def = a.layer_max[off + depth_of(q)] - (u64)(PAIR(a, CCLD_HPAIR_SENT, off + q) + PAIR(a, CCLD_HPAIR_RECV, off + q));
      atomicMax(&s_worst, (unsigned long long)def);
    }
    __syncthreads();
    const u64 worst = s_worst;
    if (worst > 0)
      for (u32 q = tid; q < n; q += 256) {
        const u64 def = a.layer_max[off + depth_of(q)] - (u64)(PAIR(a, CCLD_HPAIR_SENT, off + q) + PAIR(a, CCLD_HPAIR_RECV, off + q));
        if (def == worst) { a.cand[off + q] = 1; atomicAdd(&s_ncand, 1u); }
      }
  }
  __syncthreads();
  if (s_ncand == 0)      // a pure cycle: the rank with the fewest counts
    for (u32 q = tid; q < n; q += 256) if ((u32)PAIR(a, CCLD_HPAIR_RANK, off + q) == s_best) a.cand[off + q] = 1;
}

// ---- a not-entered rank that has entered another hung communicator is a victim --------------------
__global__ __launch_bounds__(256) void k_hang_filter(HangArgs a) {
  const u64 p = (u64)blockIdx.x * 256 + threadIdx.x;
  if (p >= a.n_members || !a.cand[p]) return;
  const u32 c = (u32)PAIR(a, CCLD_HPAIR_COMM, p), r = (u32)PAIR(a, CCLD_HPAIR_RANK, p);
  if (HCOMM(a, CCLD_HCOMM_CLASS, c) != CCLD_HANG_H1_NOT_ENTERED) return;
  for (u32 k = a.T.rank_comm_off[r]; k < a.T.rank_comm_off[r + 1]; ++k) {
    const u32 c2 = a.T.rank_comms[k];
    if (c2 == c || !HCOMM(a, CCLD_HCOMM_HUNG, c2)) continue;
    const int q2 = slot_of(a.T, c2, r);
    if (q2 >= 0 && PAIR(a, CCLD_HPAIR_ENTERED, (u64)a.T.member_off[c2] + q2)) { a.cand[p] = 2; return; }   // 2 = dropped
  }
}

// ---- hops along the wait-for edges to a root; candidates per communicator ---------------------------
__global__ __launch_bounds__(256) void k_hang_hops(HangArgs a) {
  const u64 p = (u64)blockIdx.x * 256 + threadIdx.x;
  if (p >= a.n_members) return;
  const u32 c = (u32)PAIR(a, CCLD_HPAIR_COMM, p);
  if (a.cand[p] == 1) atomicAdd((unsigned long long*)&HCOMM(a, CCLD_HCOMM_NCAND, c), 1ull);
  if (!HCOMM(a, CCLD_HCOMM_HUNG, c)) return;
  const u32 off = a.T.member_off[c], n = a.T.size[c];
  u32 cur = (u32)(p - off);
  i64 hops = 0;
  while (true) {
    if (a.cand[off + cur] == 1) break;
    const int w = a.wait_slot[off + cur];
    if (w < 0 || hops >= (i64)n) { hops = -1; break; }
    cur = (u32)w;
    ++hops;
  }
  PAIR(a, CCLD_HPAIR_HOPS, p) = hops;
}

struct PredRoot {
  const uint8_t* cand;
  __device__ bool operator()(u32 p) const { return cand[p] == 1; }
};
struct PredHung {
  const i64* hung;
  __device__ bool operator()(u32 c) const { return hung[c] != 0; }
};

__global__ __launch_bounds__(256) void k_hang_root_keys(HangArgs a, const u32* list, u32 n_root, int cb, u64* key) {
  const u32 k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n_root) return;
  const u32 p = list[k];
  key[k] = ((u64)PAIR(a, CCLD_HPAIR_RANK, p) << cb) | (u64)PAIR(a, CCLD_HPAIR_COMM, p);
}
__global__ __launch_bounds__(256) void k_hang_root_emit(HangArgs a, const u32* list, const u32* sidx, u32 n_root,
                                                        i64* root, u64 root_cap) {
  const u32 k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n_root || k >= root_cap) return;
  const u32 p = list[sidx[k]];
  const u32 c = (u32)PAIR(a, CCLD_HPAIR_COMM, p);
  root[CCLD_HROOT_RANK * root_cap + k] = PAIR(a, CCLD_HPAIR_RANK, p);
  root[CCLD_HROOT_COMM * root_cap + k] = c;
  root[CCLD_HROOT_CLASS * root_cap + k] = HCOMM(a, CCLD_HCOMM_CLASS, c);
}

// copy the first `rows` rows of every column of a column-major table into a table of another capacity
__global__ __launch_bounds__(256) void k_copy_table(const i64* src, u64 src_cap, i64* dst, u64 dst_cap, u64 rows, int ncol) {
  const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * (u64)ncol) return;
  const u64 col = i / rows, r = i % rows;
  dst[col * dst_cap + r] = src[col * src_cap + r];
}

// ---- SendRate / RecvRate: count changes per operation (Section 4.1.2) ------------------------------
#define RPAIR(a, col, p) (a.pair[(u64)(col) * a.n_members + (p)])
#define RCOMM(a, col, c) (a.hcomm[(u64)(col) * a.T.n_comms + (c)])

// One wavefront per member slot, lanes on consecutive snapshots of one channel.  A run of equal
// operation counters is committed when the next run starts, so the open last run never counts.
__global__ __launch_bounds__(256) void k_rate_pairs(HangArgs a) {
  const u32 lane = lane_id();
  const u64 p = (u64)blockIdx.x * 4 + threadIdx.x / CCLD_WAVE;
  if (p >= a.n_members) return;
  u64 ops_s = 0, chg_s = 0, ops_r = 0, chg_r = 0, status = 0;
  const u64 below = ((u64)1 << lane) - 1;                // lanes before this one
  for (u32 ch = 0; ch < a.n_ch; ++ch) {
    const u64 base = (p * a.n_ch + ch) * a.n_snap;
    u64 c_seq = 0, c_cnt = 0;                            // last sample of the previous chunk
    u32 pend_s = 0, pend_r = 0;                          // changes seen so far in the run that is still open
    for (u32 s0 = 0; s0 < a.n_snap; s0 += CCLD_WAVE) {
      const u32 s = s0 + lane;
      const bool in = s < a.n_snap;
      u64 seq = 0, cnt = 0;
      if (in) {
        seq = a.cell[2 * (base + s)]; cnt = a.cell[2 * (base + s) + 1];
        status |= cell_status(a, base + s, seq, cnt);
      }
      u64 pseq = shfl_u64(seq, (int)lane - 1), pcnt = shfl_u64(cnt, (int)lane - 1);
      if (lane == 0) { pseq = c_seq; pcnt = c_cnt; }
      const bool start = in && (s == 0 || seq != pseq);
      if (start) pcnt = 0;                               // a run's first sample is compared with zero
      const u64 B = ballot64(start);
      const u64 Cs = ballot64(in && (u32)cnt != (u32)pcnt);
      const u64 Cr = ballot64(in && (u32)(cnt >> 32) != (u32)(pcnt >> 32));
      if (B == 0) {
        pend_s += (u32)__popcll(Cs); pend_r += (u32)__popcll(Cr);
      } else {
        const u32 last = 63 - (u32)__clzll((long long)B);             // start of the run still open
        const u64 closed = ((u64)1 << last) - 1;                      // samples of runs that close here
        // this lane's run begins at the highest start at or below it (or came in from the last chunk)
        const u64 Bat = B & (below | ((u64)1 << lane));
        const bool carried = Bat == 0;
        const u32 rs = carried ? 0u : 63 - (u32)__clzll((long long)Bat);
        const u64 run_before = below & ~(((u64)1 << rs) - 1);         // lanes of my run before me
        const bool mine = ((closed >> lane) & 1) != 0;
        const bool first_s = mine && ((Cs >> lane) & 1) && (Cs & run_before) == 0 && !(carried && pend_s);
        const bool first_r = mine && ((Cr >> lane) & 1) && (Cr & run_before) == 0 && !(carried && pend_r);
        const u32 first_start = (u32)__builtin_ctzll(B);
        // the carried run closes at the chunk's first start: it is one operation if it had a change
        // earlier, else if one of its lanes here is a first change (counted below)
        ops_s += (u64)__popcll(ballot64(first_s)) + ((pend_s && first_start <= last) ? 1 : 0);
        ops_r += (u64)__popcll(ballot64(first_r)) + ((pend_r && first_start <= last) ? 1 : 0);
        chg_s += pend_s + (u64)__popcll(Cs & closed);
        chg_r += pend_r + (u64)__popcll(Cr & closed);
        pend_s = (u32)__popcll(Cs & ~closed); pend_r = (u32)__popcll(Cr & ~closed);
      }
      c_seq = shfl_u64(seq, 63); c_cnt = shfl_u64(cnt, 63);
    }
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) status |= shfl_xor_u64(status, m);
  if (lane == 0) {
    if (status) atomicOr((unsigned long long*)&a.counters[CNT_STATUS], (unsigned long long)status);
    u32 lo = 0, hi = a.T.n_comms;
    while (hi - lo > 1) { const u32 m = (lo + hi) / 2; if (a.T.member_off[m] <= p) lo = m; else hi = m; }
    RPAIR(a, CCLD_RATE_RANK, p) = a.T.members[p];
    RPAIR(a, CCLD_RATE_COMM, p) = lo;
    RPAIR(a, CCLD_RATE_OPS_SEND, p) = (i64)ops_s;
    RPAIR(a, CCLD_RATE_CHANGES_SEND, p) = (i64)chg_s;
    RPAIR(a, CCLD_RATE_OPS_RECV, p) = (i64)ops_r;
    RPAIR(a, CCLD_RATE_CHANGES_RECV, p) = (i64)chg_r;
  }
}

// a rate (ops / changes, rank); changes == 0 means "no rate" and loses against everything
struct RateCand { u64 ops, chg; u32 rank; };
__device__ __forceinline__ bool rate_less(const RateCand& x, const RateCand& y) {
  if (x.chg == 0) return false;
  if (y.chg == 0) return true;
  const u128 l = (u128)x.ops * (u128)y.chg, r = (u128)y.ops * (u128)x.chg;
  if (l != r) return l < r;
  return x.rank < y.rank;
}

// One workgroup per communicator: the member of minimal SendRate, RecvRate, and of both kinds.
__global__ __launch_bounds__(256) void k_rate_comm(HangArgs a, i64* __restrict__ rate_root) {
  __shared__ RateCand s_best[3][256];
  const u32 c = blockIdx.x, tid = threadIdx.x;
  const u32 off = a.T.member_off[c], n = a.T.size[c];
  RateCand best[3] = {{0, 0, 0xFFFFFFFFu}, {0, 0, 0xFFFFFFFFu}, {0, 0, 0xFFFFFFFFu}};
  for (u32 q = tid; q < n; q += 256) {
    const u64 p = (u64)off + q;
    const u32 rk = (u32)RPAIR(a, CCLD_RATE_RANK, p);
    const RateCand snd{(u64)RPAIR(a, CCLD_RATE_OPS_SEND, p), (u64)RPAIR(a, CCLD_RATE_CHANGES_SEND, p), rk};
    const RateCand rcv{(u64)RPAIR(a, CCLD_RATE_OPS_RECV, p), (u64)RPAIR(a, CCLD_RATE_CHANGES_RECV, p), rk};
    if (rate_less(snd, best[0])) best[0] = snd;
    if (rate_less(rcv, best[1])) best[1] = rcv;
    if (rate_less(snd, best[2])) best[2] = snd;
    if (rate_less(rcv, best[2])) best[2] = rcv;
  }
  for (int k = 0; k < 3; ++k) s_best[k][tid] = best[k];
  __syncthreads();
  for (u32 w = 128; w >= 1; w >>= 1) {
    if (tid < w)
      for (int k = 0; k < 3; ++k)
        if (rate_less(s_best[k][tid + w], s_best[k][tid])) s_best[k][tid] = s_best[k][tid + w];
    __syncthreads();
  }
  if (tid == 0) {
    RCOMM(a, CCLD_RCOMM_COMM, c) = c;
    RCOMM(a, CCLD_RCOMM_ROOT_SEND, c) = s_best[0][0].chg ? (i64)s_best[0][0].rank : (i64)CCLD_NO_RANK;
    RCOMM(a, CCLD_RCOMM_ROOT_RECV, c) = s_best[1][0].chg ? (i64)s_best[1][0].rank : (i64)CCLD_NO_RANK;
    const i64 root = s_best[2][0].chg ? (i64)s_best[2][0].rank : (i64)CCLD_NO_RANK;
    RCOMM(a, CCLD_RCOMM_ROOT, c) = root;
    rate_root[c] = root;
  }
}

// ---- Probing Frames (Section 5.1) -------------------------------------------------------------------
struct FrameArgs {
  const uint8_t* frames;
  const u32* frame_rank;
  u64 n_frames;
  u32 n_ch, snap;
  int mb;
  DeviceTopology T;
  u64 n_members;
  u64* last;          // [n_members][CCLD_FRAME_CHANNELS][2]
  u32* seen;          // ranks that delivered a frame
  u64* counters;
};

// member slot of rank r in communicator c (r < n_ranks), or -1
__device__ __forceinline__ int member_slot(const DeviceTopology& T, int mb, u32 c, u32 r) {
  if (T.rank_memb4) {
    const uint4 m = reinterpret_cast<const uint4*>(T.rank_memb4)[r];
    const u32 w = c == (m.x >> mb) ? m.x : c == (m.y >> mb) ? m.y : c == (m.z >> mb) ? m.z : m.w;
    if (c != (w >> mb)) return -1;
    return (int)T.sorted_slot[T.member_off[c] + (w & (mb < 32 ? (1u << mb) - 1 : ~0u))];
  }
  return slot_of(T, c, r);
}

// One wavefront per frame, lane = 8 * block + channel.  CHECK: the validity checks only.  Otherwise:
// the block that holds the rank's latest kernel on its communicator replaces the remembered state.
template <bool CHECK>
__global__ __launch_bounds__(256) void k_frames(FrameArgs a) {
  const u32 lane = lane_id();
  const u64 f = (u64)blockIdx.x * 4 + threadIdx.x / CCLD_WAVE;
  if (f >= a.n_frames) return;
  const uint8_t* F = a.frames + f * CCLD_FRAME_BYTES;
  const u32 b = lane / CCLD_FRAME_CHANNELS, ch = lane % CCLD_FRAME_CHANNELS;
  const u32 r = a.frame_rank[f];
  const u32 nch = reinterpret_cast<const u32*>(F)[4];
  const uint4 tid4 = *reinterpret_cast<const uint4*>(F + CCLD_FRAME_HEADER_BYTES + b * CCLD_FRAME_BLOCK_BYTES);
  const uint4 cnt4 = *reinterpret_cast<const uint4*>(F + CCLD_FRAME_HEADER_BYTES + b * CCLD_FRAME_BLOCK_BYTES + 16 + ch * 16);
  const u32 comm = tid4.x;
  const bool written = (tid4.y & 1u) != 0;
  const u64 opc = (u64)tid4.z | ((u64)tid4.w << 32);
  const u64 sent = (u64)cnt4.x | ((u64)cnt4.y << 32), recv = (u64)cnt4.z | ((u64)cnt4.w << 32);
  if (CHECK) {
    u64 status = 0;
    if (nch > CCLD_FRAME_CHANNELS) status |= DS_RANGE;
    if (lane == 0 && r < a.T.n_ranks) {
      const u32 bit = 1u << (r & 31);
      if (atomicOr(&a.seen[r >> 5], bit) & bit) status |= DS_DUPLICATE;
    }
    if (written) {
      if (comm >= a.T.n_comms) {
        status |= DS_UNKNOWN_COMM;
      } else {
        if (r >= a.T.n_ranks || member_slot(a.T, a.mb, comm, r) < 0) status |= DS_NOT_MEMBER;
        if (ch < nch && (sent > 0xFFFFFFFFull || recv > 0xFFFFFFFFull)) status |= DS_RANGE;
      }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) status |= shfl_xor_u64(status, m);
    if (lane == 0 && status) atomicOr((unsigned long long*)&a.counters[CNT_STATUS], (unsigned long long)status);
    return;
  }
  // a later kernel of this rank on the same communicator in another block of the frame?
  bool loses = false;
#pragma unroll
  for (u32 b2 = 0; b2 < CCLD_FRAME_BLOCKS; ++b2) {
    const u32 c2 = __shfl(comm, (int)(b2 * CCLD_FRAME_CHANNELS), CCLD_WAVE);
    const u32 w2 = __shfl(written ? 1u : 0u, (int)(b2 * CCLD_FRAME_CHANNELS), CCLD_WAVE);
    const u64 o2 = shfl_u64(opc, (int)(b2 * CCLD_FRAME_CHANNELS));
    if (b2 != b && w2 && c2 == comm && (o2 > opc || (o2 == opc && b2 > b))) loses = true;
  }
  if (!written || loses) return;
  const int slot = member_slot(a.T, a.mb, comm, r);
  const u64 p = (u64)a.T.member_off[comm] + (u32)slot;
  u64* L = a.last + (p * CCLD_FRAME_CHANNELS + ch) * 2;
  if (opc < L[0]) return;                                  // what is remembered is newer
  L[0] = opc;
  L[1] = ch < nch ? ((sent & 0xFFFFFFFFull) | (recv << 32)) : 0ull;
}

// one snapshot row per member slot and channel, from the remembered state
__global__ __launch_bounds__(256) void k_frame_rows(FrameArgs a, ccld_snapshot_rows o) {
  const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.n_members * a.n_ch) return;
  const u64 p = i / a.n_ch;
  const u32 ch = (u32)(i % a.n_ch);
  u32 lo = 0, hi = a.T.n_comms;
  while (hi - lo > 1) { const u32 m = (lo + hi) / 2; if (a.T.member_off[m] <= p) lo = m; else hi = m; }
  const u64* L = a.last + (p * CCLD_FRAME_CHANNELS + ch) * 2;
  o.snap[i] = a.snap; o.rank[i] = a.T.members[p]; o.comm[i] = lo; o.channel[i] = ch;
  o.seq_posted[i] = L[0]; o.chunks_sent[i] = (u32)L[1]; o.chunks_recv[i] = (u32)(L[1] >> 32);
}

}  // namespace ccld

#define HIP_TRY(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); return CCLD_E_HIP; } } while (0)

static ccld_status hang_status(uint64_t bits) {
  if (bits & DS_UNKNOWN_COMM) return CCLD_E_UNKNOWN_COMM;
  if (bits & DS_NOT_MEMBER) return CCLD_E_RANK_NOT_MEMBER;
  if (bits & DS_RANGE) return CCLD_E_RANGE;
  if (bits & DS_DUPLICATE) return CCLD_E_DUPLICATE_KEY;
  if (bits & DS_SNAPSHOT_GAP) return CCLD_E_SNAPSHOT_GAP;
  return CCLD_OK;
}

// Device memory the hang and rate passes work in, beyond their inputs and outputs: either carved from the
// context's workspace or from the library's static device array.
struct HangScratch {
  uint64_t* counters;        // [CNT_COUNT]
  uint64_t* cell;            // [n_cell][2]
  uint32_t* cnt;             // presence bitmap, one bit per cell
  int64_t* pair;             // [CCLD_HPAIR_NCOL][n_members]
  int64_t* hcomm;            // [CCLD_HCOMM_NCOL][n_comms]
  int32_t* wait_slot;        // [n_members]
  uint8_t* cand;             // [n_members]
  uint64_t* layer_max;       // [n_members]
  uint32_t* root_list;       // [n_members + 1]
  uint32_t* tiles_a;         // [n_members / SEL_TILE + 2] per-tile counts of the root selection
  uint32_t* tiles_b;         // [n_comms / SEL_TILE + 2] per-tile counts of the hung-communicator selection
  uint32_t* comm_list;       // [n_comms] hung communicators
  SortBuffers sb;            // root list sort: n_members items
  uint64_t* keyC;            // [n_members]
  uint64_t sort_cap;
  uint8_t* stage;            // [stage_bytes] staging for host-resident rows, or null
  uint64_t stage_bytes;
  bool fill_kernels;         // clear with fill kernels instead of hipMemsetAsync
};

static HangScratch scratch_of_context(ccld_ctx* c) {
  HangScratch S;
  S.counters = c->counters; S.cell = c->h_cell; S.cnt = c->h_cnt; S.pair = c->h_pair; S.hcomm = c->h_comm;
  S.wait_slot = c->h_wait_slot; S.cand = c->h_cand; S.layer_max = c->h_layer_max; S.root_list = c->h_root_list;
  S.tiles_a = c->tile_flags; S.tiles_b = c->tile_heads; S.comm_list = c->alert_list;
  S.sb.key[0] = c->sb.key[0]; S.sb.idx[0] = c->sb.idx[0]; S.sb.key[1] = c->sb.key[1]; S.sb.idx[1] = c->sb.idx[1];
  S.sb.table = c->table2; S.sb.totals = c->totals2;
  S.keyC = c->keyC; S.sort_cap = c->sort_cap; S.stage = c->h_stage; S.stage_bytes = c->snap_cap * 32; S.fill_kernels = false;
  return S;
}

static hipError_t clear_bytes(hipStream_t st, void* p, int value, uint64_t bytes, bool fill_kernels) {
  if (!fill_kernels) return hipMemsetAsync(p, value, bytes, st);
  launch_fill_u64(st, (uint64_t*)p, (bytes + 7) / 8, value ? ~0ull : 0ull);     // regions are padded to 256 bytes
  return hipGetLastError();
}

// Stages host-resident rows, clears the grid's presence counts and places every row in its cell.
static hipError_t place_snapshots(ccld_ctx* c, const HangScratch& S, const ccld_snapshots* sn, uint64_t n_rows,
                                  uint64_t n_cell, HangArgs& a, bool exact) {
  hipStream_t st = c->stream;
  std::memset(&a, 0, sizeof(a));
  hipError_t e = hipSuccess;
  if (sn->on_device) {
    a.snap = sn->snap; a.rank = sn->rank; a.comm = sn->comm; a.channel = sn->channel;
    a.seq_posted = sn->seq_posted; a.sent = sn->chunks_sent; a.recv = sn->chunks_recv;
  } else if (n_rows) {
    uint64_t* d_seq = (uint64_t*)S.stage;
    uint32_t* d32 = (uint32_t*)(d_seq + n_rows);
    const uint32_t* src[6] = {sn->snap, sn->rank, sn->comm, sn->channel, sn->chunks_sent, sn->chunks_recv};
    if ((e = hipMemcpyAsync(d_seq, sn->seq_posted, 8 * n_rows, hipMemcpyHostToDevice, st)) != hipSuccess) return e;
    for (int i = 0; i < 6; ++i)
      if ((e = hipMemcpyAsync(d32 + i * n_rows, src[i], 4 * n_rows, hipMemcpyHostToDevice, st)) != hipSuccess) return e;
    a.seq_posted = d_seq; a.snap = d32; a.rank = d32 + n_rows; a.comm = d32 + 2 * n_rows; a.channel = d32 + 3 * n_rows;
    a.sent = d32 + 4 * n_rows; a.recv = d32 + 5 * n_rows;
  }
  a.n_rows = n_rows; a.n_snap = sn->n_snapshots; a.n_ch = sn->n_channels; a.T = c->topo; a.mb = c->kf.mb; a.n_members = c->n_members;
  a.cell = S.cell; a.cnt = S.cnt; a.pair = S.pair; a.hcomm = S.hcomm; a.wait_slot = S.wait_slot;
  a.cand = S.cand; a.layer_max = S.layer_max; a.counters = S.counters;
  a.stall_snapshots = c->p.stall_snapshots; a.fifo_depth = c->p.fifo_depth;

  c->prof.begin(CCLD_PROF_HANG_PLACE);
  if ((e = clear_bytes(st, S.counters, 0, sizeof(uint64_t) * CNT_COUNT, S.fill_kernels)) != hipSuccess) return e;
  a.exact = exact ? 1 : 0;
  if (exact) e = clear_bytes(st, S.cnt, 0, sizeof(uint32_t) * ((n_cell + 31) / 32), S.fill_kernels);
  else e = clear_bytes(st, S.cell, 0xFF, 16 * n_cell, S.fill_kernels);
  if (e != hipSuccess) return e;
  // large grids whose rows are already on the device (the staging area is free then) are placed in two steps
  int rb = 16;
  while ((n_cell >> rb) >= PART_REGIONS && rb < 31) ++rb;
  const uint64_t n_regions = (n_cell + ((uint64_t)1 << rb) - 1) >> rb;
  const bool two_step = !exact && sn->on_device && S.stage && n_rows >= ((uint64_t)1 << 20) && n_cell < ((uint64_t)1 << 31) &&
                        (n_regions << rb) * 20 <= S.stage_bytes && n_regions <= PART_REGIONS;
  if (n_rows && two_step) {
    a.rb = rb; a.n_regions = (uint32_t)n_regions;
    a.part_pay = reinterpret_cast<ulonglong2*>(S.stage);
    a.part_idx = reinterpret_cast<uint32_t*>(S.stage + (n_regions << rb) * 16);
    a.part_fill = S.cnt;                       // the presence bitmap is not in use in this mode
    if ((e = clear_bytes(st, S.cnt, 0, sizeof(uint32_t) * PART_REGIONS, S.fill_kernels)) != hipSuccess) return e;
    uint64_t g = (n_rows + PART_CHUNK - 1) / PART_CHUNK; if (g > 1024) g = 1024;
    uint64_t chunk = (n_rows + g - 1) / g;
    chunk = (chunk + PART_CHUNK - 1) / PART_CHUNK * PART_CHUNK;
    static bool raised = false;       // more than 64 KB of dynamic LDS has to be asked for once
    constexpr size_t part_lds = (size_t)PART_CHUNK * (16 + 4 + 4);
    if (!raised) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hang_part), hipFuncAttributeMaxDynamicSharedMemorySize, (int)part_lds);
      raised = true;
    }
    hipLaunchKernelGGL(k_hang_part, dim3((uint32_t)g), dim3(PART_THREADS), part_lds, st, a, chunk);
    const uint32_t wpr = (uint32_t)((((uint64_t)1 << rb) + PLACE_ROWS - 1) / PLACE_ROWS);
    const uint64_t g2 = 8 * ((n_regions + 7) / 8) * wpr;
    hipLaunchKernelGGL(k_hang_place_regions, dim3((uint32_t)g2), dim3(256), 0, st, a, wpr);
  } else if (n_rows) {
    uint64_t g = (n_rows + 255) / 256; if (g > 4096) g = 4096;
    if (exact) hipLaunchKernelGGL(k_hang_place<true>, dim3((uint32_t)g), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(k_hang_place<false>, dim3((uint32_t)g), dim3(256), 0, st, a);
  }
  c->prof.split(CCLD_PROF_HANG_PLACE, CCLD_PROF_HANG);
  return hipSuccess;
}

// argument checks shared by the hang entry points; *n_cell receives the grid size
static ccld_status check_hang_args(ccld_ctx* c, const ccld_snapshots* sn, uint64_t n_rows, ccld_hang_result* o,
                                   uint64_t* n_cell) {
  if (!c || !sn || !o) return CCLD_E_NULL;
  o->n_root = o->n_pair = o->n_hung_comm = 0;
  o->status = CCLD_OK;
  if (!o->root && o->root_cap) return o->status = CCLD_E_NULL;
  if (n_rows && (!sn->snap || !sn->rank || !sn->comm || !sn->channel || !sn->seq_posted || !sn->chunks_sent || !sn->chunks_recv))
    return o->status = CCLD_E_NULL;
  if (sn->n_snapshots == 0 || sn->n_channels == 0) return o->status = CCLD_E_BAD_ARG;
  *n_cell = c->n_members * sn->n_channels * sn->n_snapshots;
  return CCLD_OK;
}

// the hang pass proper, on scratch memory S (n_cell cells and n_rows rows fit it)
static ccld_status locate_hang_on(ccld_ctx* c, const HangScratch& S, const ccld_snapshots* sn, uint64_t n_rows,
                                  uint64_t n_cell, ccld_hang_result* o) {
  hipStream_t st = c->stream;
  HangArgs a;
  const uint32_t nm = (uint32_t)c->n_members;
  // One row per cell is the normal case: the rows are placed without the presence bitmap (its atomics are a
  // third of the placement's time) and the per-member pass looks for cells that nobody wrote.  If it finds one
  // and no row was refused for a worse reason, or if the row count already rules the normal case out, the
  // placement is repeated with the bitmap, which tells duplicates from gaps.
  for (bool exact = n_rows != n_cell;; exact = true) {
    HIP_TRY(place_snapshots(c, S, sn, n_rows, n_cell, a, exact));
    hipLaunchKernelGGL(k_hang_pairs, dim3((nm + 3) / 4), dim3(256), 0, st, a);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpyAsync(c->h_pinned, S.counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (exact || c->h_pinned[CNT_STATUS] != (uint64_t)DS_SUSPECT) break;
    c->prof.end(CCLD_PROF_HANG);
  }
  if (c->h_pinned[CNT_STATUS]) { c->prof.end(CCLD_PROF_HANG); c->prof.collect(); return o->status = hang_status(c->h_pinned[CNT_STATUS]); }

  hipLaunchKernelGGL(k_hang_comm, dim3(c->topo.n_comms), dim3(256), 0, st, a);
  hipLaunchKernelGGL(k_hang_filter, dim3((nm + 255) / 256), dim3(256), 0, st, a);
  hipLaunchKernelGGL(k_hang_hops, dim3((nm + 255) / 256), dim3(256), 0, st, a);
  // roots in (rank, communicator) order
  PredRoot pr{S.cand};
  run_select(st, pr, nm, S.tiles_a, S.root_list, &S.counters[CNT_NCAND]);
  PredHung ph{S.hcomm + (uint64_t)CCLD_HCOMM_HUNG * c->topo.n_comms};
  run_select(st, ph, c->topo.n_comms, S.tiles_b, S.comm_list, &S.counters[CNT_NALERT]);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(c->h_pinned, S.counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  const uint32_t n_root = (uint32_t)c->h_pinned[CNT_NCAND];
  o->n_root = n_root;
  o->n_hung_comm = c->h_pinned[CNT_NALERT];
  o->n_pair = c->n_members;
  if (n_root && o->root_cap) {
    const SortBuffers& sb2 = S.sb;
    if (n_root > S.sort_cap) return o->status = CCLD_E_CAPACITY;
    hipLaunchKernelGGL(k_hang_root_keys, dim3((n_root + 255) / 256), dim3(256), 0, st, a, (const u32*)S.root_list, n_root, c->kf.cb, S.keyC);
    KeySource ks; ks.key = S.keyC; ks.head = 0; ks.cap = n_root; ks.squeeze = 0; ks.hi_shift = 0; ks.lo_bits = 0; ks.lo_mask = 0; ks.lo_sub = 0;
    const int r = radix_sort_pairs(st, ks, n_root, sb2, c->kf.cb + c->rank_bits);
    if (r < 0) return o->status = CCLD_E_HIP;
    hipLaunchKernelGGL(k_hang_root_emit, dim3((n_root + 255) / 256), dim3(256), 0, st, a, (const u32*)S.root_list,
                       (const u32*)sb2.idx[r], n_root, o->root, o->root_cap);
  }
  if (o->pair && o->pair_cap) {
    const uint64_t rows = std::min<uint64_t>(o->pair_cap, c->n_members);
    hipLaunchKernelGGL(k_copy_table, dim3((uint32_t)((rows * CCLD_HPAIR_NCOL + 255) / 256)), dim3(256), 0, st,
                       (const i64*)S.pair, c->n_members, o->pair, o->pair_cap, rows, (int)CCLD_HPAIR_NCOL);
  }
  if (o->comm && o->comm_cap) {
    const uint64_t rows = std::min<uint64_t>(o->comm_cap, c->topo.n_comms);
    hipLaunchKernelGGL(k_copy_table, dim3((uint32_t)((rows * CCLD_HCOMM_NCOL + 255) / 256)), dim3(256), 0, st,
                       (const i64*)S.hcomm, (uint64_t)c->topo.n_comms, o->comm, o->comm_cap, rows, (int)CCLD_HCOMM_NCOL);
  }
  c->prof.end(CCLD_PROF_HANG);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(st));
  c->prof.collect();
  if (o->n_root > o->root_cap || (o->pair && o->pair_cap < c->n_members) || (o->comm && o->comm_cap < c->topo.n_comms))
    o->status = CCLD_W_TRUNCATED;
  return o->status;
}

extern "C" ccld_status ccld_locate_hang(ccld_ctx* c, const ccld_snapshots* sn, uint64_t n_rows, ccld_hang_result* o) {
  uint64_t n_cell = 0;
  const ccld_status s = check_hang_args(c, sn, n_rows, o, &n_cell);
  if (s != CCLD_OK) return s;
  if (n_cell > c->snap_cap || n_rows > c->snap_cap) return o->status = CCLD_E_CAPACITY;
  c->inc_ok = false;            // the root list is sorted in the window's sort buffers
  c->chain_ready = false;
  return locate_hang_on(c, scratch_of_context(c), sn, n_rows, n_cell, o);
}

// ---- hang location on the library's static device array ------------------------------------------------
// For callers that cannot allocate device memory and whose context was created without room for snapshots:
// the grid, the per-member and per-communicator tables and the sort buffers of the hang pass live in one
// file-scope device array.  Every GPU the library runs on holds its own copy of the array at its own
// address until the process ends; the address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[CCLD_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {nullptr};     // device address of `scratch` on each GPU
std::mutex g_scratch_mutex;

// device address of the static array on the current device (looked up on the first call per device)
ccld_status static_scratch_address(unsigned char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) { (void)hipGetLastError(); return CCLD_E_HIP; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return CCLD_E_HIP; }
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return CCLD_OK;
}

// Bump allocator over the static array; regions start on 256-byte boundaries and are padded to them.
struct StaticCarver {
  unsigned char* base; uint64_t off;
  template <class T> T* take(uint64_t count) {
    T* p = reinterpret_cast<T*>(base + off);
    off += (count * sizeof(T) + 255) & ~(uint64_t)255;
    return p;
  }
};
}  // namespace

// called by ccld_create with the context's device current: the first look-up happens at set-up
ccld_status ccld_static_scratch_init() {
  unsigned char* p = nullptr;
  return static_scratch_address(&p);
}

extern "C" ccld_status ccld_locate_hang_static(ccld_ctx* c, const ccld_snapshots* sn, uint64_t n_rows,
                                               ccld_hang_result* o) {
  uint64_t n_cell = 0;
  const ccld_status s = check_hang_args(c, sn, n_rows, o, &n_cell);
  if (s != CCLD_OK) return s;
  unsigned char* base = nullptr;
  const ccld_status sa = static_scratch_address(&base);
  if (sa != CCLD_OK) return o->status = sa;
  const uint64_t nm = c->n_members, nc = c->topo.n_comms;
  // every size below is bounded before it is multiplied: a grid beyond the array is refused here
  if (n_cell > CCLD_STATIC_SCRATCH_BYTES / 16 || n_rows > CCLD_STATIC_SCRATCH_BYTES / 32 ||
      nm > CCLD_STATIC_SCRATCH_BYTES / 64 || nc > CCLD_STATIC_SCRATCH_BYTES / 64)
    return o->status = CCLD_E_CAPACITY;
  HangScratch S;
  StaticCarver w{base, 0};
  S.counters = w.take<uint64_t>(CNT_COUNT);
  S.cell = w.take<uint64_t>(2 * n_cell);
  S.cnt = w.take<uint32_t>(n_cell / 32 + 1);
  S.pair = w.take<int64_t>((uint64_t)CCLD_HPAIR_NCOL * nm);
  S.hcomm = w.take<int64_t>((uint64_t)CCLD_HCOMM_NCOL * nc);
  S.wait_slot = w.take<int32_t>(nm);
  S.cand = w.take<uint8_t>(nm);
  S.layer_max = w.take<uint64_t>(nm);
  S.root_list = w.take<uint32_t>(nm + 1);
  S.tiles_a = w.take<uint32_t>(nm / SEL_TILE + 3);
  S.tiles_b = w.take<uint32_t>(nc / SEL_TILE + 3);
  S.comm_list = w.take<uint32_t>(nc + 1);
  for (int i = 0; i < 2; ++i) { S.sb.key[i] = w.take<uint64_t>(nm + 1); S.sb.idx[i] = w.take<uint32_t>(nm + 1); }
  S.sb.table = w.take<uint32_t>(sort_table_words(nm + 1));
  S.sb.totals = w.take<uint32_t>(SORT_RADIX);
  S.keyC = w.take<uint64_t>(nm + 1);
  S.sort_cap = nm;
  S.stage = sn->on_device ? nullptr : w.take<uint8_t>(n_rows * 32);
  S.stage_bytes = sn->on_device ? 0 : n_rows * 32;
  S.fill_kernels = true;
  if (w.off > CCLD_STATIC_SCRATCH_BYTES) return o->status = CCLD_E_CAPACITY;
  return locate_hang_on(c, S, sn, n_rows, n_cell, o);
}

extern "C" ccld_status ccld_progress_rates(ccld_ctx* c, const ccld_snapshots* sn, uint64_t n_rows, ccld_rate_result* o) {
  if (!c || !sn || !o) return CCLD_E_NULL;
  o->n_pair = o->n_comm = 0;
  o->status = CCLD_OK;
  if (n_rows && (!sn->snap || !sn->rank || !sn->comm || !sn->channel || !sn->seq_posted || !sn->chunks_sent || !sn->chunks_recv))
    return o->status = CCLD_E_NULL;
  if (sn->n_snapshots == 0 || sn->n_channels == 0) return o->status = CCLD_E_BAD_ARG;
  const uint64_t n_cell = c->n_members * sn->n_channels * sn->n_snapshots;
  if (n_cell > c->snap_cap || n_rows > c->snap_cap) return o->status = CCLD_E_CAPACITY;
  hipStream_t st = c->stream;
  HangArgs a;
  const uint32_t nm = (uint32_t)c->n_members;
  for (bool exact = n_rows != n_cell;; exact = true) {       // see ccld_locate_hang
    HIP_TRY(place_snapshots(c, scratch_of_context(c), sn, n_rows, n_cell, a, exact));
    if (nm) hipLaunchKernelGGL(k_rate_pairs, dim3((nm + 3) / 4), dim3(256), 0, st, a);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpyAsync(c->h_pinned, c->counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (exact || c->h_pinned[CNT_STATUS] != (uint64_t)DS_SUSPECT) break;
    c->prof.end(CCLD_PROF_HANG);
  }
  if (c->h_pinned[CNT_STATUS]) { c->prof.end(CCLD_PROF_HANG); c->prof.collect(); return o->status = hang_status(c->h_pinned[CNT_STATUS]); }
  if (c->topo.n_comms) hipLaunchKernelGGL(k_rate_comm, dim3(c->topo.n_comms), dim3(256), 0, st, a, c->rate_root);
  o->n_pair = c->n_members;
  o->n_comm = c->topo.n_comms;
  if (o->pair && o->pair_cap) {
    const uint64_t rows = std::min<uint64_t>(o->pair_cap, c->n_members);
    if (rows)
      hipLaunchKernelGGL(k_copy_table, dim3((uint32_t)((rows * CCLD_RATE_NCOL + 255) / 256)), dim3(256), 0, st,
                         (const i64*)c->h_pair, c->n_members, o->pair, o->pair_cap, rows, (int)CCLD_RATE_NCOL);
  }
  if (o->comm && o->comm_cap) {
    const uint64_t rows = std::min<uint64_t>(o->comm_cap, c->topo.n_comms);
    if (rows)
      hipLaunchKernelGGL(k_copy_table, dim3((uint32_t)((rows * CCLD_RCOMM_NCOL + 255) / 256)), dim3(256), 0, st,
                         (const i64*)c->h_comm, (uint64_t)c->topo.n_comms, o->comm, o->comm_cap, rows, (int)CCLD_RCOMM_NCOL);
  }
  c->prof.end(CCLD_PROF_HANG);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(st));
  c->prof.collect();
  if (o->pair_cap < o->n_pair && o->pair) o->status = CCLD_W_TRUNCATED;
  if (o->comm_cap < o->n_comm && o->comm) o->status = CCLD_W_TRUNCATED;
  return o->status;
}

extern "C" ccld_status ccld_reset_frames(ccld_ctx* c) {
  if (!c) return CCLD_E_NULL;
  HIP_TRY(hipMemsetAsync(c->f_last, 0, sizeof(uint64_t) * 2 * CCLD_FRAME_CHANNELS * c->n_members, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  return CCLD_OK;
}

extern "C" ccld_status ccld_decode_frames(ccld_ctx* c, const ccld_frames* fr, const ccld_snapshot_rows* rows,
                                          uint64_t* n_rows) {
  if (!c || !fr || !rows || !n_rows) return CCLD_E_NULL;
  *n_rows = 0;
  if (fr->n_channels == 0 || fr->n_channels > CCLD_FRAME_CHANNELS) return CCLD_E_BAD_ARG;
  if (fr->n_frames && (!fr->frames || !fr->frame_rank)) return CCLD_E_NULL;
  if (!rows->snap || !rows->rank || !rows->comm || !rows->channel || !rows->seq_posted || !rows->chunks_sent ||
      !rows->chunks_recv)
    return CCLD_E_NULL;
  const uint64_t n_out = c->n_members * fr->n_channels;
  if (n_out > rows->capacity) return CCLD_E_CAPACITY;
  hipStream_t st = c->stream;
  FrameArgs a;
  std::memset(&a, 0, sizeof(a));
  if (fr->on_device) {
    if ((reinterpret_cast<uintptr_t>(fr->frames) & 15) != 0) return CCLD_E_BAD_ARG;
    a.frames = fr->frames; a.frame_rank = fr->frame_rank;
  } else if (fr->n_frames) {
    // staging buffer of the snapshot rows: 32 bytes per row of capacity
    const uint64_t need = fr->n_frames * (CCLD_FRAME_BYTES + 4);
    if (need > c->snap_cap * 32) return CCLD_E_CAPACITY;
    uint8_t* d = c->h_stage;
    HIP_TRY(hipMemcpyAsync(d, fr->frames, fr->n_frames * CCLD_FRAME_BYTES, hipMemcpyHostToDevice, st));
    uint32_t* dr = reinterpret_cast<uint32_t*>(d + fr->n_frames * CCLD_FRAME_BYTES);
    HIP_TRY(hipMemcpyAsync(dr, fr->frame_rank, fr->n_frames * 4, hipMemcpyHostToDevice, st));
    a.frames = d; a.frame_rank = dr;
  }
  a.n_frames = fr->n_frames; a.n_ch = fr->n_channels; a.snap = fr->snapshot; a.mb = c->kf.mb; a.T = c->topo;
  a.n_members = c->n_members; a.last = c->f_last; a.seen = c->f_seen; a.counters = c->counters;
  c->prof.begin(CCLD_PROF_FRAMES);
  HIP_TRY(hipMemsetAsync(c->counters, 0, sizeof(uint64_t) * CNT_COUNT, st));
  HIP_TRY(hipMemsetAsync(c->f_seen, 0, sizeof(uint32_t) * (c->topo.n_ranks / 32 + 1), st));
  const uint32_t fblocks = (uint32_t)((fr->n_frames + 3) / 4);
  if (fr->n_frames) hipLaunchKernelGGL(k_frames<true>, dim3(fblocks), dim3(256), 0, st, a);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(c->h_pinned, c->counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (c->h_pinned[CNT_STATUS]) { c->prof.end(CCLD_PROF_FRAMES); c->prof.collect(); return hang_status(c->h_pinned[CNT_STATUS]); }
  if (fr->n_frames) hipLaunchKernelGGL(k_frames<false>, dim3(fblocks), dim3(256), 0, st, a);
  if (n_out) hipLaunchKernelGGL(k_frame_rows, dim3((uint32_t)((n_out + 255) / 256)), dim3(256), 0, st, a, *rows);
  c->prof.end(CCLD_PROF_FRAMES);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(st));
  c->prof.collect();
  *n_rows = n_out;
  return CCLD_OK;
}
