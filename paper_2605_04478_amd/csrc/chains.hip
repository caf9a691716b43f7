// Root cause and secondary effects among the late-entry flags of an analysed window (Section 4.2.2: an
// anomaly may propagate across ranks; the location step separates the rank that triggered it from the
// ranks that pass it on).  Per late-entry flag: the operation its rank ran just before (found by binary
// search over the rounds of each of the rank's communicators, on the rank's own timestamps), the member
// whose late arrival ended that operation late (its parent flag), then pointer jumping to the chain's
// first flag.
#include <algorithm>
#include <cstring>

#include "ccld_internal.h"
#include "device_utils.h"
#include "window_kernels.h"

using namespace ccld;

namespace ccld {

constexpr i64 T_INFLIGHT = INT64_MAX;

struct ChainArgs {
  const u64* key;            // squeezed keys in (communicator, counter, rank) order
  const u32* idx;            // payload row of each sorted record
  const Row* row;
  SqueezedFormat sf;
  DeviceTopology T;
  const i64* seg;            // the analysis's collective table
  u64 seg_cap;
  u32 n_seg;
  const uint8_t* rec_flag;   // by sorted position
  const i64* flag_lag;       // [2][cap_n] lags of the flagged records by sorted position
  u64 cap_n;
  const u32* flag_pos;       // sorted position of the k-th flag
  u32 n_flag;
  u32* comm_first;           // [n_comms + 1] first table row of each communicator
  u32* parent;               // [n_flag] parent flag or ~0
};

// first row of the collective table of every communicator (the table is ordered by communicator)
__global__ __launch_bounds__(256) void k_chain_comm_rows(ChainArgs a) {
  const u32 c = blockIdx.x * 256 + threadIdx.x;
  if (c > a.T.n_comms) return;
  const i64* COMM = a.seg + (u64)CCLD_SEG_COMM * a.seg_cap;
  u32 lo = 0, hi = a.n_seg;
  while (lo < hi) { const u32 m = (lo + hi) >> 1; if ((u32)COMM[m] < c) lo = m + 1; else hi = m; }
  a.comm_first[c] = lo;
}

// sorted position of the record of member slot `slot` in table row `row`, or ~0
__device__ __forceinline__ u32 chain_record_of(const ChainArgs& a, u32 row, u32 slot, u32 size) {
  const u32 first = (u32)a.seg[(u64)CCLD_SEG_FIRST * a.seg_cap + row], n = (u32)a.seg[(u64)CCLD_SEG_N * a.seg_cap + row];
  if (n == size) return first + slot;
  const u64 mmask = ((u64)1 << a.sf.mb) - 1;
  u32 lo = first, hi = first + n;
  while (lo < hi) { const u32 m = (lo + hi) >> 1; if ((u32)(a.key[m] & mmask) < slot) lo = m + 1; else hi = m; }
  return (lo < first + n && (u32)(a.key[lo] & mmask) == slot) ? lo : ~0u;
}

// One thread per flag: the parent of a late entry.
__global__ __launch_bounds__(256) void k_chain_parent(ChainArgs a) {
  const u32 k = blockIdx.x * 256 + threadIdx.x;
  if (k >= a.n_flag) return;
  const u32 j = a.flag_pos[k];
  u32 parent = ~0u;
  if (a.rec_flag[j] & CCLD_FLAG_LATE_ENTER) {
    const int mb = a.sf.mb;
    const u64 mmask = ((u64)1 << mb) - 1;
    const u64 key = a.key[j];
    const u32 comm = (u32)(key >> (mb + a.sf.ws));
    const u32 r = a.T.members_sorted[a.T.member_off[comm] + (u32)(key & mmask)];
    const i64 t = a.row[a.idx[j]].t_enter;
    // the operation this rank ran just before: per communicator of the rank the last round that the rank left
    // before t (its rounds are in time order; a round without a record of the rank is skipped), then the latest
    bool have = false;
    i64 b_exit = 0, b_enter = 0;
    u32 b_comm = 0, b_row = 0;
    for (u32 q = a.T.rank_comm_off[r]; q < a.T.rank_comm_off[r + 1]; ++q) {
      const u32 c2 = a.T.rank_comms[q], slot2 = a.T.rank_slots[q], size2 = a.T.size[c2];
      u32 lo = a.comm_first[c2], hi = a.comm_first[c2 + 1];
      const u32 row_lo = lo;
      bool found = false;
      u32 f_row = 0;
      i64 f_exit = 0, f_enter = 0;
      while (lo < hi) {
        const u32 mid = (lo + hi) >> 1;
        // the nearest round at or below mid in which the rank has a record
        u32 probe = mid, pos = ~0u;
        while (true) {
          pos = chain_record_of(a, probe, slot2, size2);
          if (pos != ~0u || probe == lo) break;
          --probe;
        }
        bool ok = false;
        i64 te = 0, tx = 0;
        if (pos != ~0u) {
          const Row rw = a.row[a.idx[pos]];
          te = rw.t_enter; tx = rw.t_exit;
          ok = pos != j && tx != T_INFLIGHT && tx <= t;
        }
        if (ok) { found = true; f_row = probe; f_exit = tx; f_enter = te; lo = mid + 1; }
        else if (pos == ~0u) lo = mid + 1;       // no record of the rank in [lo, mid]
        else hi = probe;
      }
      (void)row_lo;
      if (!found) continue;
      const bool better = !have || f_exit > b_exit || (f_exit == b_exit && (f_enter > b_enter || (f_enter == b_enter && c2 > b_comm)));
      if (better) { have = true; b_exit = f_exit; b_enter = f_enter; b_comm = c2; b_row = f_row; }
    }
    if (have) {
      // who ended it late: the late entry with the largest lag (ties: smallest rank = first in rank order)
      const u32 first = (u32)a.seg[(u64)CCLD_SEG_FIRST * a.seg_cap + b_row], n = (u32)a.seg[(u64)CCLD_SEG_N * a.seg_cap + b_row];
      u32 m_pos = ~0u;
      i64 m_lag = 0;
      for (u32 p = first; p < first + n; ++p)
        if (a.rec_flag[p] & CCLD_FLAG_LATE_ENTER) {
          const i64 lag = a.flag_lag[p];
          if (m_pos == ~0u || lag > m_lag) { m_pos = p; m_lag = lag; }
        }
      if (m_pos != ~0u) {
        u32 lo = 0, hi = a.n_flag;
        while (lo < hi) { const u32 m = (lo + hi) >> 1; if (a.flag_pos[m] < m_pos) lo = m + 1; else hi = m; }
        parent = lo;
      }
    }
  }
  a.parent[k] = parent;
}

// pointer jumping: anc = current ancestor (a root points to itself), dist = links between the flag and it
__global__ __launch_bounds__(256) void k_chain_init(const u32* parent, u32 n_flag, u32* anc, u32* dist) {
  const u32 k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n_flag) return;
  const u32 p = parent[k];
  anc[k] = p == ~0u ? k : p;
  dist[k] = p == ~0u ? 0u : 1u;
}
__global__ __launch_bounds__(256) void k_chain_jump(const u32* anc_in, const u32* dist_in, u32 n_flag, u32* anc_out, u32* dist_out) {
  const u32 k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n_flag) return;
  const u32 a1 = anc_in[k], a2 = anc_in[a1];
  anc_out[k] = a2;
  dist_out[k] = dist_in[k] + (a2 != a1 ? dist_in[a1] : 0u);
}
// column[idx] += 1 for every lane with `on`, one atomic per distinct idx in the wavefront: a faulty rank's thousands
// of entries would otherwise queue up at one address.  Called by every active lane of the wavefront.
__device__ __forceinline__ void wave_count_by_index(i64* column, u32 idx, bool on) {
  u64 todo = ballot64(on);
  while (todo) {
    const u32 leader = (u32)__builtin_ctzll(todo);
    const u32 v = (u32)__shfl((int)idx, (int)leader, CCLD_WAVE);
    const u64 same = ballot64(on && idx == v);
    if (lane_id() == leader) atomicAdd((unsigned long long*)&column[v], (unsigned long long)__popcll(same));
    todo &= ~same;
  }
}
__global__ __launch_bounds__(256) void k_chain_emit(ChainArgs a, const u32* anc, const u32* dist, i64* chain, u64 chain_cap,
                                                    i64* per_rank) {
  const u32 k = blockIdx.x * 256 + threadIdx.x;
  if (k >= a.n_flag) return;
  const int mb = a.sf.mb;
  const u64 mmask = ((u64)1 << mb) - 1;
  auto rank_at = [&](u32 flag) -> u32 {
    const u64 key = a.key[a.flag_pos[flag]];
    return a.T.members_sorted[a.T.member_off[(u32)(key >> (mb + a.sf.ws))] + (u32)(key & mmask)];
  };
  const u32 root = anc[k], p = a.parent[k];
  const u32 root_rank = rank_at(root);
  if (k < chain_cap) {
    chain[(u64)CCLD_CHN_PARENT * chain_cap + k] = p == ~0u ? -1 : (i64)p;
    chain[(u64)CCLD_CHN_ROOT * chain_cap + k] = (i64)root;
    chain[(u64)CCLD_CHN_ROOT_RANK * chain_cap + k] = (i64)root_rank;
    chain[(u64)CCLD_CHN_DEPTH * chain_cap + k] = (i64)dist[k];
  }
  if (per_rank) {
    const bool on = (a.rec_flag[a.flag_pos[k]] & CCLD_FLAG_LATE_ENTER) != 0;
    const u32 n_ranks = a.T.n_ranks;
    const u32 mine = on ? rank_at(k) : 0u;
    wave_count_by_index(per_rank + (u64)CCLD_CHR_ROOT_ENTRIES * n_ranks, mine, on && p == ~0u);
    wave_count_by_index(per_rank + (u64)CCLD_CHR_SECONDARY_ENTRIES * n_ranks, mine, on && p != ~0u);
    wave_count_by_index(per_rank + (u64)CCLD_CHR_CAUSED * n_ranks, root_rank, on);
  }
}

}  // namespace ccld

#define HIP_TRY(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); return CCLD_E_HIP; } } while (0)

extern "C" ccld_status ccld_flag_chains(ccld_ctx* c, const ccld_window_result* w, ccld_chain_result* o) {
  if (!c || !w || !o) return CCLD_E_NULL;
  o->n_chain = 0;
  o->status = CCLD_OK;
  if (o->chain_cap && !o->chain) return o->status = CCLD_E_NULL;
  // the tables and the order of the most recent analysis must still be there
  if (!c->chain_ready || w->seg != c->last_seg || w->seg_cap != c->last_seg_cap || w->n_seg != c->last_n_seg ||
      w->n_flag != c->last_n_flag)
    return o->status = CCLD_E_BAD_ARG;
  if (w->n_seg > w->seg_cap) return o->status = CCLD_E_CAPACITY;      // a truncated table cannot be searched
  hipStream_t st = c->stream;
  const uint32_t n_flag = (uint32_t)c->last_n_flag, n_ranks = c->topo.n_ranks;
  o->n_chain = n_flag;
  if (o->per_rank) HIP_TRY(hipMemsetAsync(o->per_rank, 0, sizeof(int64_t) * CCLD_CHR_NCOL * (uint64_t)n_ranks, st));
  if (n_flag) {
    ChainArgs a;
    std::memset(&a, 0, sizeof(a));
    a.key = c->sb.key[c->sorted_buf]; a.idx = c->sb.idx[c->sorted_buf]; a.row = c->last_rows; a.sf = c->sf; a.T = c->topo;
    a.seg = w->seg; a.seg_cap = w->seg_cap; a.n_seg = (uint32_t)w->n_seg;
    a.rec_flag = c->last_rec_flag; a.flag_lag = c->flag_lag; a.cap_n = c->cap; a.flag_pos = c->flag_pos; a.n_flag = n_flag;
    a.comm_first = c->chain_first; a.parent = c->group_first;
    // scratch that the analysis no longer needs: the third sort buffer pair and the alert candidate counts
    uint32_t* anc[2] = {reinterpret_cast<uint32_t*>(c->keyC), reinterpret_cast<uint32_t*>(c->keyC) + n_flag};
    uint32_t* dist[2] = {c->idxC, c->alert_ncand};
    const uint32_t blocks = (n_flag + 255) / 256;
    hipLaunchKernelGGL(k_chain_comm_rows, dim3((c->topo.n_comms + 256) / 256), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_chain_parent, dim3(blocks), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_chain_init, dim3(blocks), dim3(256), 0, st, (const u32*)a.parent, n_flag, anc[0], dist[0]);
    int cur = 0;
    for (uint64_t reach = 1; reach < n_flag; reach *= 2) {        // after i rounds every flag has looked 2^i links up
      hipLaunchKernelGGL(k_chain_jump, dim3(blocks), dim3(256), 0, st, (const u32*)anc[cur], (const u32*)dist[cur], n_flag,
                         anc[1 - cur], dist[1 - cur]);
      cur = 1 - cur;
    }
    hipLaunchKernelGGL(k_chain_emit, dim3(blocks), dim3(256), 0, st, a, (const u32*)anc[cur], (const u32*)dist[cur], o->chain,
                       o->chain_cap, o->per_rank);
  }
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(st));
  if (o->n_chain > o->chain_cap) o->status = CCLD_W_TRUNCATED;
  return o->status;
}
