// Per-collective statistics for gfx950.  Collectives of up to 64 records are packed side by side
// into the lanes of a wavefront and sorted there with a bitonic network whose exchanges are DPP
// row operations wherever the lane pattern allows, which yields minimum, exact lower median
// (order statistic floor((n-1)/2)), maximum, and then the median absolute deviation.  Collectives
// of 65 to 512 records take a wavefront each with 2, 4 or 8 values per lane in registers, those of
// up to 16,384 records a workgroup each with a bitonic sort in LDS (k_seg_team, k_seg_large), and longer ones
// the counting selection of k_seg_big.
#include "window_kernels.h"
#include "dense.h"
#include "device_utils.h"

namespace ccld {

constexpr i64 T_INFLIGHT = INT64_MAX;
constexpr int SEG_WAVE_MAX = 64;     // longest collective handled inside one wavefront's registers
constexpr int SEG_MULTI_MAX = 512;   // longest collective one wavefront sorts in registers (eight values per lane)
constexpr int SEG_TEAM_MAX = 2048;   // longest collective a workgroup of 256 threads sorts in LDS (three arrays)
constexpr int SEG_LARGE_MAX = 16384; // longest collective a workgroup of 1,024 threads sorts in LDS (one array of 128 KB)

__device__ __forceinline__ u64 atomic_add_u64(u64* p, u64 v) {
  return atomicAdd((unsigned long long*)p, (unsigned long long)v);
}

__device__ __forceinline__ void seg_put(const SegArgs& a, int col, u32 srow, i64 v) {
  if (srow < a.seg_cap) a.seg[(u64)col * a.seg_cap + srow] = v;
}
// detection-group key and intra-round range T_max - T_min (Eq. 2) of one collective
__device__ __forceinline__ void seg_group_of(const SegArgs& a, bool usable, u32 comm, u32 op, u64 nb, i64 dmax, i64 dmin,
                                             u64* key, i64* range) {
  *key = a.no_group;
  *range = 0;
  if (usable) {
    const u64 cls = 63 - __clzll((long long)(nb | 1));
    *key = ((u64)comm * CCLD_OP_MAX + op) * GROUP_CLS + cls;
    *range = dmax - dmin;
  }
}
__device__ __forceinline__ void seg_put_group(const SegArgs& a, u32 srow, bool usable, u32 comm, u32 op, u64 nb,
                                              i64 dmax, i64 dmin) {
  u64 key;
  i64 range;
  seg_group_of(a, usable, comm, op, nb, dmax, dmin, &key, &range);
  a.gkey[srow] = key;
  a.range_c[srow] = range;
}
__device__ __forceinline__ i64 absdiff(i64 a, i64 b) { return a >= b ? a - b : b - a; }
// payload row of the j-th record in (communicator, counter, rank) order; the op word's upper bits belong
// to the dense placement
__device__ __forceinline__ Row load_row(const SegArgs& a, u32 j) {
  Row r = a.row[a.idx[j]];
  r.op &= 15u;
  return r;
}
__device__ __forceinline__ bool is_late(i64 lag, i64 floor_ns, u32 knum, u32 kden, i64 mad) {
  return lag > floor_ns && (i128)lag * (i128)kden > (i128)knum * (i128)mad;
}
__device__ __forceinline__ void seg_put_empty_stats(const SegArgs& a, u32 srow) {
  for (int c = CCLD_SEG_ENTER_MIN; c <= CCLD_SEG_DUR_MAX; ++c) seg_put(a, c, srow, 0);
  seg_put(a, CCLD_SEG_ARGMIN_RANK, srow, CCLD_NO_RANK);
  seg_put(a, CCLD_SEG_ARGMAX_RANK, srow, CCLD_NO_RANK);
}


// ---- lane exchanges ------------------------------------------------------------------------
// value held by lane (lane ^ M)
template <int M>
__device__ __forceinline__ u32 xor_lane_u32(u32 v) {
  const int s = (int)v;
  // every lane of these patterns reads a valid lane, so no previous value has to be kept: the plain
  // DPP move needs no copy of the destination first
  if constexpr (M == 1) return (u32)__builtin_amdgcn_mov_dpp(s, 0xB1, 0xF, 0xF, true);        // quad_perm [1,0,3,2]
  else if constexpr (M == 2) return (u32)__builtin_amdgcn_mov_dpp(s, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
  else if constexpr (M == 3) return (u32)__builtin_amdgcn_mov_dpp(s, 0x1B, 0xF, 0xF, true);   // quad_perm [3,2,1,0]
  else if constexpr (M == 7) return (u32)__builtin_amdgcn_mov_dpp(s, 0x141, 0xF, 0xF, true);  // row_half_mirror
  else if constexpr (M == 15) return (u32)__builtin_amdgcn_mov_dpp(s, 0x140, 0xF, 0xF, true); // row_mirror
  else if constexpr (M == 8) return (u32)__builtin_amdgcn_mov_dpp(s, 0x128, 0xF, 0xF, true);  // row_ror:8
  else if constexpr (M == 4) {
    int t = __builtin_amdgcn_mov_dpp(s, 0x104, 0xF, 0x5, true);           // banks 0,2 read lane + 4 (row_shl:4)
    t = __builtin_amdgcn_update_dpp(t, s, 0x114, 0xF, 0xA, false);        // banks 1,3 read lane - 4 (row_shr:4)
    return (u32)t;
  } else
    return __shfl_xor(v, M, CCLD_WAVE);       // masks that cross a row of 16 lanes
}
template <int M>
__device__ __forceinline__ i64 xor_lane_i64(i64 v) {
  const u32 lo = xor_lane_u32<M>((u32)(u64)v), hi = xor_lane_u32<M>((u32)((u64)v >> 32));
  return (i64)(((u64)hi << 32) | lo);
}
__device__ __forceinline__ i64 shfl_i64(i64 v, int src) { return (i64)shfl_u64((u64)v, src); }

constexpr int high_bit(int m) { int b = 1; while (b * 2 <= m) b *= 2; return b; }

// compare-exchange with lane ^ M: the lane whose top bit of M is clear keeps the smaller value
template <int M>
__device__ __forceinline__ i64 cmpx(i64 v, u32 lane) {
  const i64 p = xor_lane_i64<M>(v);
  const bool upper = (lane & high_bit(M)) != 0;
  return ((p < v) != upper) ? p : v;
}

// ascending sort inside every aligned group of G lanes (bitonic merges: mirror, then halving strides)
template <int G>
__device__ __forceinline__ i64 sort_groups(i64 v, u32 lane) {
  if constexpr (G >= 2) { v = cmpx<1>(v, lane); }
  if constexpr (G >= 4) { v = cmpx<3>(v, lane); v = cmpx<1>(v, lane); }
  if constexpr (G >= 8) { v = cmpx<7>(v, lane); v = cmpx<2>(v, lane); v = cmpx<1>(v, lane); }
  if constexpr (G >= 16) { v = cmpx<15>(v, lane); v = cmpx<4>(v, lane); v = cmpx<2>(v, lane); v = cmpx<1>(v, lane); }
  if constexpr (G >= 32) {
    v = cmpx<31>(v, lane); v = cmpx<8>(v, lane); v = cmpx<4>(v, lane); v = cmpx<2>(v, lane); v = cmpx<1>(v, lane);
  }
  if constexpr (G >= 64) {
    v = cmpx<63>(v, lane); v = cmpx<16>(v, lane); v = cmpx<8>(v, lane); v = cmpx<4>(v, lane);
    v = cmpx<2>(v, lane); v = cmpx<1>(v, lane);
  }
  return v;
}

// ascending sort of a sequence that falls and then rises inside every aligned group of G lanes (one bitonic
// merge: halving strides).  The absolute deviations of sorted values from their median form such a sequence,
// with the empty lanes' largest value at its end.
template <int G>
__device__ __forceinline__ i64 merge_groups(i64 v, u32 lane) {
  if constexpr (G >= 64) v = cmpx<32>(v, lane);
  if constexpr (G >= 32) v = cmpx<16>(v, lane);
  if constexpr (G >= 16) v = cmpx<8>(v, lane);
  if constexpr (G >= 8) v = cmpx<4>(v, lane);
  if constexpr (G >= 4) v = cmpx<2>(v, lane);
  if constexpr (G >= 2) v = cmpx<1>(v, lane);
  return v;
}

// all-reduce inside a group: smallest (d, r) / largest d with the smallest r among equals
template <int G, bool MAXIMUM>
__device__ __forceinline__ void reduce_dur(i64& d, u32& r) {
#define CCLD_DUR_STEP(M)                                                        \
  if constexpr (G > M) {                                                        \
    const i64 od = xor_lane_i64<M>(d);                                          \
    const u32 orr = xor_lane_u32<M>(r);                                         \
    const bool better = MAXIMUM ? (od > d) : (od < d);                          \
    if (better || (od == d && orr < r)) { d = od; r = orr; }                    \
  }
  CCLD_DUR_STEP(1) CCLD_DUR_STEP(2) CCLD_DUR_STEP(4) CCLD_DUR_STEP(8) CCLD_DUR_STEP(16) CCLD_DUR_STEP(32)
#undef CCLD_DUR_STEP
}
template <int G>
__device__ __forceinline__ i64 reduce_min(i64 v) {
#define CCLD_MIN_STEP(M) if constexpr (G > M) { const i64 o = xor_lane_i64<M>(v); v = o < v ? o : v; }
  CCLD_MIN_STEP(1) CCLD_MIN_STEP(2) CCLD_MIN_STEP(4) CCLD_MIN_STEP(8) CCLD_MIN_STEP(16) CCLD_MIN_STEP(32)
#undef CCLD_MIN_STEP
  return v;
}

typedef __attribute__((address_space(3))) i64 lds_i64;      // an LDS word: 32-bit addresses, ds instructions

// What one lane knows about its record before the group-wide statistics.
struct DenseLane {
  i64 e, x;          // arrival, completion (T_INFLIGHT while the operation runs)
  u64 nb;            // bytes
  u32 op, rank;
  bool valid;        // the lane's member has a record in this collective
  u64 pm;            // lanes of this lane's collective whose members have a record
  u32 fl;            // first such lane
  u32 n, first, j;   // records of the collective, sorted position of its first record and of this record
  u32 srow;          // the collective's row of the table
  u32 comm;
  u64 seq;           // operation counter
  // LDS words that take the collective's table row (STAGE_COLS of them) when `staged`; otherwise the row goes
  // straight to the table.  A flag and not a null pointer: LDS address 0 is a valid address (the first staged row).
  lds_i64* stage;
  bool staged;
};
// A staged table row: the 21 columns, then the detection-group key and the range T_max - T_min, at constant
// offsets from the row's pointer.  k_seg_wave keeps the rows STAGE_COLS words apart (an odd stride).  In
// k_dense_stats a row lies in its collective's own cells, a multiple of 256 bytes from its neighbours, and
// starts stage_skew(k) words into that region, so that the lanes that later read one column of 64 rows
// spread over eight bank pairs.
constexpr u32 STAGE_COLS = CCLD_SEG_NCOL + 2, STAGE_REGION = 32;
__device__ __forceinline__ u32 stage_skew(u32 k) { return k & 7u; }
static_assert(STAGE_COLS + 7 <= STAGE_REGION, "a skewed row fits its region");

// Table rows of the collectives of one wavefront pass (called by the first lane of every collective; the rows of a
// pass are consecutive).  A staged row goes to LDS and the workgroup writes it out later; a row that is not staged
// is written here: the columns are written from one wavefront-uniform pointer that steps from column to column,
// plus a 32-bit byte offset per lane: no 64-bit address arithmetic per lane and column, and the kernel arguments need
// not stay in scalar registers across the whole pass (212 spilled scalar registers become 20).  Storing G words of
// a row per instruction from the G lanes of its group (3 instead of 23 store instructions at G = 8) was measured
// too: the selects that bring each lane its word cost more than the stores save (2.18 -> 2.56 ms).
enum { PUT_DIRECT = 0, PUT_STAGED = 1, PUT_EITHER = 2 };     // where a table row goes: known when compiled, or by L.staged
template <int MODE>
__device__ __forceinline__ void dense_put_row(const SegArgs& a, const DenseLane& L, u32 ninfl, bool complete, bool incons,
                                              bool barrier, bool usable, u32 hop, u64 hb, i64 imin, u32 nd, i64 min_e,
                                              i64 med_e, i64 max_e, i64 mad_e, i64 min_x, i64 med_x, i64 max_x, i64 mad_x,
                                              i64 dmin, i64 dmax, u32 rmin, u32 rmax) {
  const u32 srow = L.srow;
  const bool none = nd == 0;            // no completed record: the statistics columns are empty
  if (MODE == PUT_STAGED || (MODE == PUT_EITHER && L.staged)) {
    // the row waits in LDS until the workgroup writes the table column by column, whole lines at a time
    lds_i64* st = L.stage;
    auto put = [&](u32 c, i64 v) { st[c] = v; };
    u64 gk;
    i64 gr;
    seg_group_of(a, usable, L.comm, hop, hb, dmax, dmin, &gk, &gr);
    put(CCLD_SEG_COMM, (i64)L.comm); put(CCLD_SEG_SEQ, (i64)L.seq); put(CCLD_SEG_N, (i64)L.n); put(CCLD_SEG_INFLIGHT, (i64)ninfl);
    put(CCLD_SEG_STATE, (complete ? CCLD_SEG_COMPLETE : 0) | (!incons ? CCLD_SEG_CONSISTENT : 0) |
                            (barrier ? CCLD_SEG_BARRIER : 0) | (usable ? CCLD_SEG_USABLE : 0));
    put(CCLD_SEG_OP, (i64)hop); put(CCLD_SEG_BYTES, (i64)hb);
    put(CCLD_SEG_ENTER_MIN, none ? 0 : min_e); put(CCLD_SEG_ENTER_MED, none ? 0 : med_e);
    put(CCLD_SEG_ENTER_MAX, none ? 0 : max_e); put(CCLD_SEG_ENTER_MAD, none ? 0 : mad_e);
    put(CCLD_SEG_EXIT_MIN, none ? 0 : min_x); put(CCLD_SEG_EXIT_MED, none ? 0 : med_x);
    put(CCLD_SEG_EXIT_MAX, none ? 0 : max_x); put(CCLD_SEG_EXIT_MAD, none ? 0 : mad_x);
    put(CCLD_SEG_DUR_MIN, none ? 0 : dmin); put(CCLD_SEG_DUR_MAX, none ? 0 : dmax);
    put(CCLD_SEG_ARGMIN_RANK, none ? (i64)CCLD_NO_RANK : (i64)rmin); put(CCLD_SEG_ARGMAX_RANK, none ? (i64)CCLD_NO_RANK : (i64)rmax);
    put(CCLD_SEG_INFLIGHT_ENTER_MIN, imin); put(CCLD_SEG_FIRST, (i64)L.first);
    put(CCLD_SEG_NCOL, (i64)gk); put(CCLD_SEG_NCOL + 1, gr);
    return;
  }
  seg_put_group(a, srow, usable, L.comm, hop, hb, dmax, dmin);
  if (srow >= a.seg_cap) return;
  const u32 s0 = (u32)__builtin_amdgcn_readfirstlane((int)srow);      // the first of the pass's rows that fit the table
  const u32 off = (srow - s0) * 8u;
  const u64 stride = a.seg_cap * 8u;
  char* p = reinterpret_cast<char*>(a.seg + s0);
  auto put = [&](i64 v) { *reinterpret_cast<i64*>(p + off) = v; p += stride; };
  static_assert(CCLD_SEG_COMM == 0 && CCLD_SEG_SEQ == 1 && CCLD_SEG_N == 2 && CCLD_SEG_INFLIGHT == 3 && CCLD_SEG_STATE == 4 &&
                CCLD_SEG_OP == 5 && CCLD_SEG_BYTES == 6 && CCLD_SEG_ENTER_MIN == 7 && CCLD_SEG_ENTER_MAD == 10 &&
                CCLD_SEG_EXIT_MIN == 11 && CCLD_SEG_EXIT_MAD == 14 && CCLD_SEG_DUR_MIN == 15 && CCLD_SEG_DUR_MAX == 16 &&
                CCLD_SEG_ARGMIN_RANK == 17 && CCLD_SEG_ARGMAX_RANK == 18 && CCLD_SEG_INFLIGHT_ENTER_MIN == 19 &&
                CCLD_SEG_FIRST == 20 && CCLD_SEG_NCOL == 21, "the columns are written in this order");
  put((i64)L.comm);
  put((i64)L.seq);
  put((i64)L.n);
  put((i64)ninfl);
  put((complete ? CCLD_SEG_COMPLETE : 0) | (!incons ? CCLD_SEG_CONSISTENT : 0) | (barrier ? CCLD_SEG_BARRIER : 0) |
      (usable ? CCLD_SEG_USABLE : 0));
  put((i64)hop);
  put((i64)hb);
  put(none ? 0 : min_e); put(none ? 0 : med_e); put(none ? 0 : max_e); put(none ? 0 : mad_e);
  put(none ? 0 : min_x); put(none ? 0 : med_x); put(none ? 0 : max_x); put(none ? 0 : mad_x);
  put(none ? 0 : dmin); put(none ? 0 : dmax);
  put(none ? (i64)CCLD_NO_RANK : (i64)rmin); put(none ? (i64)CCLD_NO_RANK : (i64)rmax);
  put(imin);
  put((i64)L.first);
}
__device__ __forceinline__ void dense_put_record(const SegArgs& a, u32 j, u32 f, i64 le, i64 lx) {
  a.rec_flag[j] = (uint8_t)f;
  if (a.lag_e) a.lag_e[j] = le;
  if (a.lag_x) a.lag_x[j] = lx;
  if (f) { a.flag_lag[j] = le; a.flag_lag[a.cap_n + j] = lx; }
}

// Statistics of the collectives of one wavefront pass in 64-bit arithmetic (any spread of the times).
template <int G, int MODE>
__device__ __forceinline__ void dense_pass64(const SegArgs& a, const DenseLane& L, u32 size, u32 lane, u32 gbase, u64 gmask) {
  const i64 e = L.e, x = L.x;
  const bool valid = L.valid;
  const bool done = valid && x != T_INFLIGHT;
  const u64 m_infl = ballot64(valid && !done);
  const u32 nd = (u32)__popcll(ballot64(done) & gmask);
  const u32 ninfl = (u32)__popcll(m_infl & gmask);
  const u32 km = nd ? (nd - 1) / 2 : 0, kl = nd ? nd - 1 : 0;
  const i64 se = sort_groups<G>(done ? e : T_INFLIGHT, lane);
  const i64 sx = sort_groups<G>(done ? x : T_INFLIGHT, lane);
  const i64 med_e = shfl_i64(se, gbase + km), med_x = shfl_i64(sx, gbase + km);
  const i64 min_e = shfl_i64(se, gbase), max_e = shfl_i64(se, gbase + kl);
  const i64 min_x = shfl_i64(sx, gbase), max_x = shfl_i64(sx, gbase + kl);
  // deviations of the sorted values: the first nd lanes of a group hold its finished records
  const bool held = lane - gbase < nd;
  const i64 sde = merge_groups<G>(held ? absdiff(se, med_e) : T_INFLIGHT, lane);
  const i64 sdx = merge_groups<G>(held ? absdiff(sx, med_x) : T_INFLIGHT, lane);
  const i64 mad_e = shfl_i64(sde, gbase + km), mad_x = shfl_i64(sdx, gbase + km);
  i64 dmin = done ? x - e : INT64_MAX, dmax = done ? x - e : INT64_MIN;
  u32 rmin = done ? L.rank : 0xFFFFFFFFu, rmax = rmin;
  reduce_dur<G, false>(dmin, rmin);
  reduce_dur<G, true>(dmax, rmax);
  const u64 hb = shfl_u64(L.nb, (int)L.fl);
  const u32 hop = __shfl(L.op, (int)L.fl, CCLD_WAVE);
  const bool incons = (ballot64(valid && (L.nb != hb || L.op != hop)) & gmask) != 0;
  i64 imin = T_INFLIGHT;
  if (m_infl) imin = reduce_min<G>((valid && !done) ? e : T_INFLIGHT);
  if (!valid) return;
  const bool complete = L.n == size && ninfl == 0;
  const bool barrier = hop == CCLD_OP_ALLREDUCE && hb < (u64)a.barrier_bytes;
  const bool usable = complete && !incons && !barrier;
  if (lane == L.fl)
    dense_put_row<MODE>(a, L, ninfl, complete, incons, barrier, usable, hop, hb, imin, nd, min_e, med_e, max_e, mad_e, min_x,
                  med_x, max_x, mad_x, dmin, dmax, rmin, rmax);
  i64 le = 0, lx = 0;
  u32 f = 0;
  if (usable) {
    le = e - med_e; lx = x - med_x;
    if (is_late(le, a.lag_floor, a.kmad_num, a.kmad_den, mad_e)) f |= CCLD_FLAG_LATE_ENTER;
    if (is_late(lx, a.lag_floor, a.kmad_num, a.kmad_den, mad_x)) f |= CCLD_FLAG_LATE_EXIT;
  }
  dense_put_record(a, L.j, f, le, lx);
}

// ---- the same statistics on 32-bit times relative to the collective's first record --------------------
// Inside one collective the arrivals and completions lie within a second or so of each other, so they
// are sorted, compared and subtracted as signed 32-bit offsets from the arrival of the collective's first
// present member (half the instructions of the 64-bit form); the results are turned back into absolute
// times where they are stored.  A pass in which some offset does not fit takes the 64-bit form.
constexpr i32 REL_NONE = 0x7FFFFFFF;         // sorts behind every real offset (those stay below 2^30 in magnitude)

template <int M>
__device__ __forceinline__ i32 cmpx32(i32 v, u32 lane) {
  const i32 p = (i32)xor_lane_u32<M>((u32)v);
  const bool upper = (lane & high_bit(M)) != 0;
  const i32 lo = p < v ? p : v, hi = p < v ? v : p;
  return upper ? hi : lo;
}
template <int G>
__device__ __forceinline__ i32 sort_groups32(i32 v, u32 lane) {
  if constexpr (G >= 2) { v = cmpx32<1>(v, lane); }
  if constexpr (G >= 4) { v = cmpx32<3>(v, lane); v = cmpx32<1>(v, lane); }
  if constexpr (G >= 8) { v = cmpx32<7>(v, lane); v = cmpx32<2>(v, lane); v = cmpx32<1>(v, lane); }
  if constexpr (G >= 16) { v = cmpx32<15>(v, lane); v = cmpx32<4>(v, lane); v = cmpx32<2>(v, lane); v = cmpx32<1>(v, lane); }
  if constexpr (G >= 32) {
    v = cmpx32<31>(v, lane); v = cmpx32<8>(v, lane); v = cmpx32<4>(v, lane); v = cmpx32<2>(v, lane); v = cmpx32<1>(v, lane);
  }
  if constexpr (G >= 64) {
    v = cmpx32<63>(v, lane); v = cmpx32<16>(v, lane); v = cmpx32<8>(v, lane); v = cmpx32<4>(v, lane);
    v = cmpx32<2>(v, lane); v = cmpx32<1>(v, lane);
  }
  return v;
}
template <int G>
__device__ __forceinline__ i32 merge_groups32(i32 v, u32 lane) {
  if constexpr (G >= 64) v = cmpx32<32>(v, lane);
  if constexpr (G >= 32) v = cmpx32<16>(v, lane);
  if constexpr (G >= 16) v = cmpx32<8>(v, lane);
  if constexpr (G >= 8) v = cmpx32<4>(v, lane);
  if constexpr (G >= 4) v = cmpx32<2>(v, lane);
  if constexpr (G >= 2) v = cmpx32<1>(v, lane);
  return v;
}
// all-reduce of an unsigned 64-bit word inside a group
template <int G, bool MAXIMUM>
__device__ __forceinline__ u64 reduce_u64(u64 v) {
#define CCLD_U64_STEP(M)                                                                         \
  if constexpr (G > M) {                                                                         \
    const u64 o = (u64)xor_lane_i64<M>((i64)v);                                                  \
    v = MAXIMUM ? (o > v ? o : v) : (o < v ? o : v);                                             \
  }
  CCLD_U64_STEP(1) CCLD_U64_STEP(2) CCLD_U64_STEP(4) CCLD_U64_STEP(8) CCLD_U64_STEP(16) CCLD_U64_STEP(32)
#undef CCLD_U64_STEP
  return v;
}
// late iff lag > floor and lag * kden > knum * mad, with a 32-bit lag and a non-negative 32-bit mad
__device__ __forceinline__ bool is_late32(i32 lag, i64 floor_ns, u32 knum, u32 kden, i32 mad) {
  if (lag <= 0 || (i64)lag <= floor_ns) return false;       // a lag that is not positive never exceeds knum * mad >= 0
  return (u64)(u32)lag * (u64)kden > (u64)knum * (u64)(u32)mad;
}

template <int G, int MODE>
__device__ __forceinline__ void dense_pass32(const SegArgs& a, const DenseLane& L, i64 ref, i32 er, i32 xr, u32 size,
                                             u32 lane, u32 gbase, u64 gmask) {
  const bool valid = L.valid;
  const bool done = valid && L.x != T_INFLIGHT;
  const u64 m_infl = ballot64(valid && !done);
  const u32 nd = (u32)__popcll(ballot64(done) & gmask);
  const u32 ninfl = (u32)__popcll(m_infl & gmask);
  const u32 km = nd ? (nd - 1) / 2 : 0, kl = nd ? nd - 1 : 0;
  const i32 se = sort_groups32<G>(done ? er : REL_NONE, lane);
  const i32 sx = sort_groups32<G>(done ? xr : REL_NONE, lane);
  const i32 med_e = __shfl(se, (int)(gbase + km), CCLD_WAVE), med_x = __shfl(sx, (int)(gbase + km), CCLD_WAVE);
  const i32 min_e = __shfl(se, (int)gbase, CCLD_WAVE), max_e = __shfl(se, (int)(gbase + kl), CCLD_WAVE);
  const i32 min_x = __shfl(sx, (int)gbase, CCLD_WAVE), max_x = __shfl(sx, (int)(gbase + kl), CCLD_WAVE);
  // deviations of the sorted offsets (the first nd lanes of a group hold its finished records): they fall to zero
  // at the median and rise again, so one merge sorts them
  const bool held = lane - gbase < nd;
  const i32 sde = merge_groups32<G>(held ? (se >= med_e ? se - med_e : med_e - se) : REL_NONE, lane);
  const i32 sdx = merge_groups32<G>(held ? (sx >= med_x ? sx - med_x : med_x - sx) : REL_NONE, lane);
  const i32 mad_e = __shfl(sde, (int)(gbase + km), CCLD_WAVE), mad_x = __shfl(sdx, (int)(gbase + km), CCLD_WAVE);
  // T_min / T_max of the Duration Time with the ranks attaining them (ties: smallest rank): duration and rank
  // travel as one 64-bit word
  const u32 dur = (u32)(xr - er);
  u64 wmin = done ? (((u64)dur << 32) | L.rank) : ~0ull;
  u64 wmax = done ? (((u64)dur << 32) | (u32)~L.rank) : 0ull;
  wmin = reduce_u64<G, false>(wmin);
  wmax = reduce_u64<G, true>(wmax);
  const u64 hb = shfl_u64(L.nb, (int)L.fl);
  const u32 hop = __shfl(L.op, (int)L.fl, CCLD_WAVE);
  const bool incons = (ballot64(valid && (L.nb != hb || L.op != hop)) & gmask) != 0;
  i64 imin = T_INFLIGHT;
  if (m_infl) imin = reduce_min<G>((valid && !done) ? L.e : T_INFLIGHT);
  if (!valid) return;
  const bool complete = L.n == size && ninfl == 0;
  const bool barrier = hop == CCLD_OP_ALLREDUCE && hb < (u64)a.barrier_bytes;
  const bool usable = complete && !incons && !barrier;
  if (lane == L.fl)
    dense_put_row<MODE>(a, L, ninfl, complete, incons, barrier, usable, hop, hb, imin, nd, ref + min_e, ref + med_e, ref + max_e,
                  (i64)mad_e, ref + min_x, ref + med_x, ref + max_x, (i64)mad_x, (i64)(wmin >> 32), (i64)(wmax >> 32),
                  (u32)wmin, ~(u32)wmax);
  i32 le = 0, lx = 0;
  u32 f = 0;
  if (usable) {
    le = er - med_e; lx = xr - med_x;
    if (is_late32(le, a.lag_floor, a.kmad_num, a.kmad_den, mad_e)) f |= CCLD_FLAG_LATE_ENTER;
    if (is_late32(lx, a.lag_floor, a.kmad_num, a.kmad_den, mad_x)) f |= CCLD_FLAG_LATE_EXIT;
  }
  dense_put_record(a, L.j, f, (i64)le, (i64)lx);
}

// ---- collectives of up to 64 records, 64/G of them per wavefront pass --------------------------
constexpr u32 SEG_STAGE_ROWS = 144;      // table rows a tile stages in LDS (a tile of eight-member collectives has 128 or 129)
template <int G>
__device__ __forceinline__ void seg_wave_batches(const SegArgs& a, u32 base, u32 seg0, u32 nheads,
                                                 const unsigned short* s_head, i64* s_stage, u32 lane, u32 wave) {
  constexpr int SPW = CCLD_WAVE / G, NW = SEG_THREADS / CCLD_WAVE;
  const int mb = a.sf.mb;
  const u64 mmask = ((u64)1 << mb) - 1, smask = ((u64)1 << a.sf.ws) - 1;
  const u32 q = lane / G, l = lane % G, gbase = q * G;
  const u64 gmask = (G == 64 ? ~0ull : (((u64)1 << (G & 63)) - 1)) << gbase;
  for (u32 b = wave; b * SPW < nheads; b += NW) {
    const u32 sl = b * SPW + q;
    u32 a0 = 0, n = 0;
    if (sl < nheads) { a0 = s_head[sl]; n = (u32)s_head[sl + 1] - a0; }
    const bool small = n >= 1 && n <= (u32)SEG_WAVE_MAX;
    if (n > (u32)SEG_WAVE_MAX && l == 0) {            // too long for a wavefront: leave it to k_seg_big
      const u64 slot = atomic_add_u64(&a.counters[CNT_NBIG], 1);
      a.big_list[3 * slot] = seg0 + sl;
      a.big_list[3 * slot + 1] = base + a0;
    }
    DenseLane L;
    L.valid = small && l < n;
    L.e = 0; L.x = T_INFLIGHT; L.nb = 0; L.op = 0; L.rank = 0;
    L.first = base + a0; L.j = L.first + l; L.fl = gbase; L.n = n; L.srow = seg0 + sl;
    L.pm = 0;
    // rows beyond the staging area (a tile of many short collectives) go straight to the table
    L.staged = sl < SEG_STAGE_ROWS;
    L.stage = (lds_i64*)s_stage + sl * STAGE_COLS;
    u64 key = 0;
    u32 size = 0;
    if (L.valid) {
      key = a.key[L.j];
      const Row rw = load_row(a, L.j);
      // first member and size of the communicator in one load; the slot -> rank lookup overlaps the row gather
      const uint2 ci = a.comm_info[(u32)(key >> (mb + a.sf.ws))];
      L.rank = a.members_sorted[ci.x + (u32)(key & mmask)];
      size = ci.y;
      L.e = rw.t_enter; L.x = rw.t_exit; L.nb = rw.bytes; L.op = rw.op;
    }
    L.comm = (u32)(key >> (mb + a.sf.ws));
    L.seq = ((key >> mb) & smask) + a.sf.seq_base;
    // offsets from the arrival of the collective's first record
    const i64 ref = shfl_i64(L.e, (int)gbase);
    const i64 oe = L.e - ref, ox = L.x - ref;
    constexpr i64 LIM = (i64)1 << 30;
    const bool wide = L.valid && (oe < -LIM || oe >= LIM || (L.x != T_INFLIGHT && (ox < -LIM || ox >= LIM)));
    if (ballot64(wide) == 0) dense_pass32<G, PUT_EITHER>(a, L, ref, (i32)oe, (i32)ox, size, lane, gbase, gmask);
    else dense_pass64<G, PUT_EITHER>(a, L, size, lane, gbase, gmask);
  }
}

// One workgroup per tile of SEG_TILE sorted records: finds the collectives that start in the
// tile, then its wavefronts take them 64/G at a time (G = the tile's widest short collective,
// rounded up to a power of two).
__global__ __launch_bounds__(SEG_THREADS) void k_seg_wave(SegArgs a) {
  constexpr int OWN = SEG_TILE / SEG_THREADS, NW = SEG_THREADS / CCLD_WAVE;
  __shared__ unsigned short s_head[SEG_TILE + 2];
  __shared__ u32 s_cnt[OWN * NW];
  __shared__ u32 s_halo_head, s_gmax;
  // Table rows of the tile's first SEG_STAGE_ROWS collectives wait here (STAGE_COLS words each: an odd stride, so
  // the lanes that read one column of consecutive rows spread over the banks) and leave column by column at the
  // end, consecutive lanes to consecutive rows: one store instruction per 64 rows and column instead of one per
  // wavefront pass and column.
  __shared__ i64 s_stage[SEG_STAGE_ROWS * STAGE_COLS];
  const u32 tid = threadIdx.x, lane = lane_id(), wave = tid / CCLD_WAVE;
  const u32 tile = blockIdx.x, base = tile * SEG_TILE;
  const u32 rem = a.n - base;                                     // records from the tile's start to the end
  const u32 own = rem < (u32)SEG_TILE ? rem : (u32)SEG_TILE;
  const int mb = a.sf.mb;
  if (tid == 0) { s_halo_head = rem <= (u32)(SEG_TILE + SEG_WAVE_MAX) ? rem : 0xFFFFu; s_gmax = 0; }
  // Heads of the tile.  Position r * SEG_THREADS + tid ascends with (r, wavefront, lane), so a head's index is
  // the number of heads in the (r, wavefront) blocks before its own (16 counts in LDS, one ballot each) plus
  // the heads below its lane: no scan over the workgroup, one barrier.
  bool head[OWN];
  u64 hm[OWN];
#pragma unroll
  for (int r = 0; r < OWN; ++r) {
    const u32 pos = r * SEG_THREADS + tid, j = base + pos;
    head[r] = pos < own && (j == 0 || (a.key[j - 1] >> mb) != (a.key[j] >> mb));
    hm[r] = ballot64(head[r]);
    if (lane == 0) s_cnt[r * NW + wave] = (u32)__popcll(hm[r]);
  }
  __syncthreads();
  u32 before[OWN], acc = 0;
#pragma unroll
  for (int r = 0; r < OWN; ++r) before[r] = 0;
#pragma unroll
  for (int bl = 0; bl < OWN * NW; ++bl) {
    if ((u32)(bl % NW) == wave) before[bl / NW] = acc;
    acc += s_cnt[bl];
  }
  const u32 nheads = acc;
#pragma unroll
  for (int r = 0; r < OWN; ++r)
    if (head[r]) s_head[before[r] + mbcnt64(hm[r])] = (unsigned short)(r * SEG_THREADS + tid);
  // where the tile's last collective ends: the first head within 64 records past the tile
  if (tid <= (u32)SEG_WAVE_MAX) {
    const u32 pos = SEG_TILE + tid;
    if (pos < rem) {
      const u32 j = base + pos;
      if ((a.key[j - 1] >> mb) != (a.key[j] >> mb)) atomicMin(&s_halo_head, pos);
    }
  }
  __syncthreads();
  const u32 halo = s_halo_head & 0xFFFFu;
  if (tid == 0) s_head[nheads] = (unsigned short)halo;
  for (u32 s = tid; s < nheads; s += SEG_THREADS) {
    const u32 n = (s + 1 < nheads ? (u32)s_head[s + 1] : halo) - (u32)s_head[s];
    if (n <= (u32)SEG_WAVE_MAX) atomicMax(&s_gmax, n);
  }
  __syncthreads();
  const u32 gmax = s_gmax, seg0 = a.tile_heads[tile];
  if (gmax <= 2) seg_wave_batches<2>(a, base, seg0, nheads, s_head, s_stage, lane, wave);
  else if (gmax <= 4) seg_wave_batches<4>(a, base, seg0, nheads, s_head, s_stage, lane, wave);
  else if (gmax <= 8) seg_wave_batches<8>(a, base, seg0, nheads, s_head, s_stage, lane, wave);
  else if (gmax <= 16) seg_wave_batches<16>(a, base, seg0, nheads, s_head, s_stage, lane, wave);
  else if (gmax <= 32) seg_wave_batches<32>(a, base, seg0, nheads, s_head, s_stage, lane, wave);
  else seg_wave_batches<64>(a, base, seg0, nheads, s_head, s_stage, lane, wave);
  __syncthreads();
  const u32 staged = nheads < SEG_STAGE_ROWS ? nheads : SEG_STAGE_ROWS;
  for (u32 col = wave; col < STAGE_COLS; col += NW) {
    for (u32 sl = lane; sl < staged; sl += CCLD_WAVE) {
      // a collective of more than 64 records is on the list of the kernels that take those: they write its row
      if ((u32)s_head[sl + 1] - (u32)s_head[sl] > (u32)SEG_WAVE_MAX) continue;
      const i64 v = s_stage[sl * STAGE_COLS + col];
      const u32 srow = seg0 + sl;
      if (col < (u32)CCLD_SEG_NCOL) { if (srow < a.seg_cap) a.seg[(u64)col * a.seg_cap + srow] = v; }
      else if (col == (u32)CCLD_SEG_NCOL) a.gkey[srow] = (u64)v;
      else a.range_c[srow] = v;
    }
  }
}

// ---- collectives of 65 to 512 records: E values per lane, sorted in registers ---------------------
// Element i of the collective sits in register i / 64 of lane i % 64.  Every register is sorted by
// the 64-lane network, then runs of 2, 4, 8 registers are merged: the mirror step pairs register r
// with r ^ (run - 1) and lane l with 63 - l, strides of whole registers need no lane exchange, and
// strides below 64 are the lane exchanges of the 64-lane merge.
template <int E>
__device__ __forceinline__ void sort_multi(i64 (&v)[E], u32 lane) {
#pragma unroll
  for (int r = 0; r < E; ++r) v[r] = sort_groups<64>(v[r], lane);
#pragma unroll
  for (int kb = 2; kb <= E; kb <<= 1) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      if ((r & (kb >> 1)) == 0) {
        const int q = r ^ (kb - 1);
        const i64 b = xor_lane_i64<63>(v[q]);
        const bool sw = b < v[r];
        const i64 lo = sw ? b : v[r], hi = sw ? v[r] : b;
        v[r] = lo;
        v[q] = xor_lane_i64<63>(hi);
      }
    }
#pragma unroll
    for (int jb = kb >> 2; jb >= 1; jb >>= 1) {
#pragma unroll
      for (int r = 0; r < E; ++r) {
        if ((r & jb) == 0) {
          const int q = r | jb;
          const bool sw = v[q] < v[r];
          const i64 lo = sw ? v[q] : v[r], hi = sw ? v[r] : v[q];
          v[r] = lo; v[q] = hi;
        }
      }
    }
#pragma unroll
    for (int r = 0; r < E; ++r) {
      v[r] = cmpx<32>(v[r], lane); v[r] = cmpx<16>(v[r], lane); v[r] = cmpx<8>(v[r], lane);
      v[r] = cmpx<4>(v[r], lane); v[r] = cmpx<2>(v[r], lane); v[r] = cmpx<1>(v[r], lane);
    }
  }
}
// k-th smallest after sort_multi (k uniform across the wavefront)
template <int E>
__device__ __forceinline__ i64 kth_multi(const i64 (&v)[E], u32 k) {
  i64 sel = v[0];
#pragma unroll
  for (int r = 1; r < E; ++r) if ((k >> 6) == (u32)r) sel = v[r];
  return shfl_i64(sel, (int)(k & 63));
}

// Lower median of |value - median| over the nd smallest values of a sorted collective (nd >= 1, km = (nd - 1) / 2,
// all uniform across the wavefront).  The deviations of the values up to the median, walked downwards, and of
// the values above it, walked upwards, are two ascending lists; the km-th smallest of their union is found by
// the split that takes km + 1 entries from the two lists in order, without sorting the deviations.
template <int E>
__device__ __forceinline__ i64 mad_of_sorted(const i64 (&v)[E], u32 nd, u32 km) {
  const i64 med = kth_multi<E>(v, km);
  const u32 nl = km + 1, nr = nd - nl, d = km + 1;
  auto below = [&](u32 j) { return med - kth_multi<E>(v, km - j); };          // j < nl, ascending, below(0) = 0
  auto above = [&](u32 j) { return kth_multi<E>(v, km + 1 + j) - med; };      // j < nr, ascending
  u32 lo = d > nr ? d - nr : 0u, hi = d < nl ? d : nl;
  while (lo < hi) {
    const u32 mid = (lo + hi) >> 1;
    if (below(mid) <= above(d - 1 - mid)) lo = mid + 1; else hi = mid;
  }
  // lo entries come from the lower list, d - lo from the upper one; the largest of them is the answer
  i64 r = lo > 0 ? below(lo - 1) : INT64_MIN;
  if (d - lo > 0) { const i64 u = above(d - lo - 1); r = u > r ? u : r; }
  return r;
}

// One wavefront per listed collective of 32 E + 1 .. 64 E records (E = 1: of 1 .. 64 records; only the dense
// placement lists collectives that short, those of communicators with more than 64 members).
template <int E>
__global__ __launch_bounds__(SEG_THREADS) void k_seg_multi(SegArgs a) {
  constexpr u32 LO = E == 1 ? 1 : 32 * E + 1, HI = 64 * E, NW = SEG_THREADS / CCLD_WAVE;
  const u32 lane = lane_id();
  const int mb = a.sf.mb;
  const u64 mmask = ((u64)1 << mb) - 1, smask = ((u64)1 << a.sf.ws) - 1;
  const u32 nbig = (u32)a.counters[CNT_NBIG];
  for (u32 ent = blockIdx.x * NW + threadIdx.x / CCLD_WAVE; ent < nbig; ent += gridDim.x * NW) {
    const u32 nn = a.big_list[3 * ent + 2];
    if (nn < LO || nn > HI) continue;
    const u32 srow = a.big_list[3 * ent], a0 = a.big_list[3 * ent + 1];
    const u64 k0 = a.key[a0];
    const u32 comm = (u32)(k0 >> (mb + a.sf.ws));
    const u32* ms = a.members_sorted + a.member_off[comm];
    i64 e[E], x[E];
    u32 ninfl = 0, nd = 0;
    bool inc = false;
    i64 imin = T_INFLIGHT, dmin = INT64_MAX, dmax = INT64_MIN;
    u32 rmin = 0xFFFFFFFFu, rmax = 0xFFFFFFFFu;
    u64 hb = 0;
    u32 hop = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const u32 i = r * CCLD_WAVE + lane;
      const bool valid = i < nn;
      e[r] = 0; x[r] = T_INFLIGHT;
      u64 nb = 0;
      u32 op = 0, rank = 0;
      if (valid) {
        const u32 j = a0 + i;
        const u64 key = a.key[j];
        const Row rw = load_row(a, j);
        rank = ms[(u32)(key & mmask)];
        e[r] = rw.t_enter; x[r] = rw.t_exit; nb = rw.bytes; op = rw.op;
      }
      if (r == 0) { hb = shfl_u64(nb, 0); hop = __shfl(op, 0, CCLD_WAVE); }
      inc |= valid && (nb != hb || op != hop);
      const bool done = valid && x[r] != T_INFLIGHT;
      nd += (u32)__popcll(ballot64(done));
      ninfl += (u32)__popcll(ballot64(valid && !done));
      if (valid && !done) imin = e[r] < imin ? e[r] : imin;
      if (done) {
        const i64 d = x[r] - e[r];
        if (d < dmin || (d == dmin && rank < rmin)) { dmin = d; rmin = rank; }
        if (d > dmax || (d == dmax && rank < rmax)) { dmax = d; rmax = rank; }
      }
    }
    const bool incons = ballot64(inc) != 0;
    if (ninfl) imin = reduce_min<64>(imin);
    reduce_dur<64, false>(dmin, rmin);
    reduce_dur<64, true>(dmax, rmax);
    const u32 km = nd ? (nd - 1) / 2 : 0, kl = nd ? nd - 1 : 0;
    // two sorts, arrival and completion; the median of the absolute deviations is selected from each sorted
    // sequence (records still in flight carry the largest value and sort behind the nd finished ones)
    i64 stat_min[2] = {0, 0}, stat_med[2] = {0, 0}, stat_max[2] = {0, 0}, stat_mad[2] = {0, 0};
#pragma unroll 1
    for (int w = 0; w < 2; ++w) {                  // 0 arrival, 1 completion
      i64 v[E];
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const bool done = x[r] != T_INFLIGHT;      // lanes past the end hold the in-flight mark too
        v[r] = !done ? T_INFLIGHT : (w ? x[r] : e[r]);
      }
      sort_multi<E>(v, lane);
      stat_min[w] = kth_multi<E>(v, 0); stat_med[w] = kth_multi<E>(v, km); stat_max[w] = kth_multi<E>(v, kl);
      if (nd) stat_mad[w] = mad_of_sorted<E>(v, nd, km);
    }
    const bool complete = nn == a.comm_size[comm] && ninfl == 0;
    const bool barrier = hop == CCLD_OP_ALLREDUCE && hb < (u64)a.barrier_bytes;
    const bool usable = complete && !incons && !barrier;
    if (lane == 0) {
      seg_put(a, CCLD_SEG_COMM, srow, (i64)comm);
      seg_put(a, CCLD_SEG_SEQ, srow, (i64)(((k0 >> mb) & smask) + a.sf.seq_base));
      seg_put(a, CCLD_SEG_N, srow, (i64)nn);
      seg_put(a, CCLD_SEG_INFLIGHT, srow, (i64)ninfl);
      seg_put(a, CCLD_SEG_STATE, srow,
              (complete ? CCLD_SEG_COMPLETE : 0) | (!incons ? CCLD_SEG_CONSISTENT : 0) |
                  (barrier ? CCLD_SEG_BARRIER : 0) | (usable ? CCLD_SEG_USABLE : 0));
      seg_put(a, CCLD_SEG_OP, srow, (i64)hop);
      seg_put(a, CCLD_SEG_BYTES, srow, (i64)hb);
      seg_put(a, CCLD_SEG_INFLIGHT_ENTER_MIN, srow, imin);
      seg_put(a, CCLD_SEG_FIRST, srow, (i64)a0);
      seg_put_group(a, srow, usable, comm, hop, hb, dmax, dmin);
      if (nd == 0) {
        seg_put_empty_stats(a, srow);
      } else {
        seg_put(a, CCLD_SEG_ENTER_MIN, srow, stat_min[0]); seg_put(a, CCLD_SEG_ENTER_MED, srow, stat_med[0]);
        seg_put(a, CCLD_SEG_ENTER_MAX, srow, stat_max[0]); seg_put(a, CCLD_SEG_ENTER_MAD, srow, stat_mad[0]);
        seg_put(a, CCLD_SEG_EXIT_MIN, srow, stat_min[1]); seg_put(a, CCLD_SEG_EXIT_MED, srow, stat_med[1]);
        seg_put(a, CCLD_SEG_EXIT_MAX, srow, stat_max[1]); seg_put(a, CCLD_SEG_EXIT_MAD, srow, stat_mad[1]);
        seg_put(a, CCLD_SEG_DUR_MIN, srow, dmin); seg_put(a, CCLD_SEG_DUR_MAX, srow, dmax);
        seg_put(a, CCLD_SEG_ARGMIN_RANK, srow, (i64)rmin); seg_put(a, CCLD_SEG_ARGMAX_RANK, srow, (i64)rmax);
      }
    }
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const u32 i = r * CCLD_WAVE + lane;
      if (i >= nn) continue;
      const u32 j = a0 + i;
      i64 le = 0, lx = 0;
      u32 f = 0;
      if (usable) {
        le = e[r] - stat_med[0]; lx = x[r] - stat_med[1];
        if (is_late(le, a.lag_floor, a.kmad_num, a.kmad_den, stat_mad[0])) f |= CCLD_FLAG_LATE_ENTER;
        if (is_late(lx, a.lag_floor, a.kmad_num, a.kmad_den, stat_mad[1])) f |= CCLD_FLAG_LATE_EXIT;
      }
      a.rec_flag[j] = (uint8_t)f;
      if (a.lag_e) a.lag_e[j] = le;
      if (a.lag_x) a.lag_x[j] = lx;
      if (f) { a.flag_lag[j] = le; a.flag_lag[a.cap_n + j] = lx; }
    }
  }
}

// ---- collectives of 65 to SEG_TEAM_MAX records -------------------------------------------------
// length of every listed collective, capped at SEG_LARGE_MAX + 1: one wavefront per entry walks the
// sorted keys from the collective's first record until the (communicator, counter) prefix changes
__global__ __launch_bounds__(SEG_THREADS) void k_seg_lengths(SegArgs a) {
  const u32 nbig = (u32)a.counters[CNT_NBIG];
  const u32 lane = lane_id(), nw = SEG_THREADS / CCLD_WAVE;
  const int mb = a.sf.mb;
  for (u32 ent = blockIdx.x * nw + threadIdx.x / CCLD_WAVE; ent < nbig; ent += gridDim.x * nw) {
    const u32 a0 = a.big_list[3 * ent + 1];
    const u64 pref = a.key[a0] >> mb;
    u32 len = SEG_LARGE_MAX + 1;
    for (u32 o = 1; o <= (u32)SEG_LARGE_MAX + 1; o += CCLD_WAVE) {
      const u64 j = (u64)a0 + o + lane;
      const u64 m = ballot64(j >= a.n || (a.key[j] >> mb) != pref);
      if (m) { len = o + (u32)__builtin_ctzll(m); break; }
    }
    if (lane == 0) a.big_list[3 * ent + 2] = len < (u32)SEG_LARGE_MAX + 1 ? len : (u32)SEG_LARGE_MAX + 1;
  }
}

struct TeamAcc {
  unsigned long long imin;
  long long dmin, dmax;
  u32 ninfl, incons, rmin, rmax;
};

// one compare-exchange step of the network over v[0, P): partner of i is i ^ M, the element whose
// bit HB (the top bit of M) is clear keeps the smaller value
template <u32 TT = SEG_THREADS>
__device__ __forceinline__ void team_cmpx(i64* v, u32 P, u32 M, u32 HB, u32 t) {
  for (u32 p = t; p < P / 2; p += TT) {
    const u32 lo = p & (HB - 1), ia = ((p - lo) << 1) | lo, ib = ia ^ M;
    const i64 va = v[ia], vb = v[ib];
    if (vb < va) { v[ia] = vb; v[ib] = va; }
  }
  __syncthreads();
}
// ascending bitonic sort of v[0, P), P a power of two (same merges as sort_groups, in LDS)
template <u32 TT = SEG_THREADS>
__device__ __forceinline__ void team_sort(i64* v, u32 P, u32 t) {
  for (u32 k = 2; k <= P; k <<= 1) {
    team_cmpx<TT>(v, P, k - 1, k >> 1, t);
    for (u32 j = k >> 2; j; j >>= 1) team_cmpx<TT>(v, P, j, j, t);
  }
}

// One workgroup per collective of 513 to SEG_TEAM_MAX records; arrival and completion times are
// staged in LDS and a third LDS array is sorted four times (arrival, completion, and their absolute
// deviations).
__global__ __launch_bounds__(SEG_THREADS) void k_seg_team(SegArgs a) {
  constexpr u32 TEAMS = 1, TT = SEG_THREADS;
  constexpr u32 CAPN = SEG_TEAM_MAX;
  constexpr u32 LO = (u32)SEG_MULTI_MAX + 1;
  __shared__ i64 s_e[TEAMS][CAPN], s_x[TEAMS][CAPN], s_v[TEAMS][CAPN];
  __shared__ TeamAcc s_acc[TEAMS];
  const u32 team = threadIdx.x / TT, t = threadIdx.x % TT;
  i64 *E = s_e[team], *X = s_x[team], *V = s_v[team];
  TeamAcc& acc = s_acc[team];
  const int mb = a.sf.mb;
  const u64 mmask = ((u64)1 << mb) - 1, smask = ((u64)1 << a.sf.ws) - 1;
  const u32 nbig = (u32)a.counters[CNT_NBIG];
  for (u32 ent = blockIdx.x * TEAMS + team; ent < nbig; ent += gridDim.x * TEAMS) {
    const u32 nn = a.big_list[3 * ent + 2];
    if (nn < LO || nn > CAPN) continue;
    const u32 srow = a.big_list[3 * ent], a0 = a.big_list[3 * ent + 1];
    const u64 k0 = a.key[a0];
    const Row h = load_row(a, a0);
    if (t == 0) {
      acc.imin = (unsigned long long)T_INFLIGHT; acc.dmin = INT64_MAX; acc.dmax = INT64_MIN;
      acc.ninfl = 0; acc.incons = 0; acc.rmin = 0xFFFFFFFFu; acc.rmax = 0xFFFFFFFFu;
    }
    __syncthreads();
    {
      u32 ni = 0, rmin = 0xFFFFFFFFu, rmax = 0xFFFFFFFFu;
      bool inc = false;
      i64 imin = T_INFLIGHT, dmin = INT64_MAX, dmax = INT64_MIN;
      for (u32 i = t; i < nn; i += TT) {
        const u32 j = a0 + i;
        const Row rw = load_row(a, j);
        E[i] = rw.t_enter; X[i] = rw.t_exit;
        inc |= (rw.op != h.op || rw.bytes != h.bytes);
        if (rw.t_exit == T_INFLIGHT) {
          ++ni; imin = rw.t_enter < imin ? rw.t_enter : imin;
        } else {
          const i64 d = rw.t_exit - rw.t_enter;
          const u32 rk = (u32)(a.key[j] & mmask);
          if (d < dmin || (d == dmin && rk < rmin)) { dmin = d; rmin = rk; }
          if (d > dmax || (d == dmax && rk < rmax)) { dmax = d; rmax = rk; }
        }
      }
      if (ni) { atomicAdd(&acc.ninfl, ni); atomicMin(&acc.imin, (unsigned long long)imin); }
      if (inc) atomicOr(&acc.incons, 1u);
      if (rmin != 0xFFFFFFFFu) { atomicMin(&acc.dmin, (long long)dmin); atomicMax(&acc.dmax, (long long)dmax); }
      __syncthreads();
      if (rmin != 0xFFFFFFFFu && dmin == (i64)acc.dmin) atomicMin(&acc.rmin, rmin);
      if (rmax != 0xFFFFFFFFu && dmax == (i64)acc.dmax) atomicMin(&acc.rmax, rmax);
    }
    const u32 ninfl = acc.ninfl, nd = nn - ninfl;
    const u32 km = nd ? (nd - 1) / 2 : 0, kl = nd ? nd - 1 : 0;
    u32 P = 2;
    while (P < nn) P <<= 1;
    for (u32 i = t; i < P; i += TT) V[i] = (i < nn && X[i] != T_INFLIGHT) ? E[i] : T_INFLIGHT;
    __syncthreads();
    team_sort(V, P, t);
    const i64 min_e = V[0], med_e = V[km], max_e = V[kl];
    __syncthreads();
    for (u32 i = t; i < P; i += TT) V[i] = i < nn ? X[i] : T_INFLIGHT;
    __syncthreads();
    team_sort(V, P, t);
    const i64 min_x = V[0], med_x = V[km], max_x = V[kl];
    __syncthreads();
    for (u32 i = t; i < P; i += TT) V[i] = (i < nn && X[i] != T_INFLIGHT) ? absdiff(E[i], med_e) : T_INFLIGHT;
    __syncthreads();
    team_sort(V, P, t);
    const i64 mad_e = V[km];
    __syncthreads();
    for (u32 i = t; i < P; i += TT) V[i] = (i < nn && X[i] != T_INFLIGHT) ? absdiff(X[i], med_x) : T_INFLIGHT;
    __syncthreads();
    team_sort(V, P, t);
    const i64 mad_x = V[km];
    const u32 comm = (u32)(k0 >> (mb + a.sf.ws));
    const bool complete = nn == a.comm_size[comm] && ninfl == 0;
    const bool consistent = acc.incons == 0;
    const bool barrier = h.op == CCLD_OP_ALLREDUCE && h.bytes < (u64)a.barrier_bytes;
    const bool usable = complete && consistent && !barrier;
    if (t == 0) {
      seg_put(a, CCLD_SEG_COMM, srow, (i64)comm);
      seg_put(a, CCLD_SEG_SEQ, srow, (i64)(((k0 >> mb) & smask) + a.sf.seq_base));
      seg_put(a, CCLD_SEG_N, srow, (i64)nn);
      seg_put(a, CCLD_SEG_INFLIGHT, srow, (i64)ninfl);
      seg_put(a, CCLD_SEG_STATE, srow,
              (complete ? CCLD_SEG_COMPLETE : 0) | (consistent ? CCLD_SEG_CONSISTENT : 0) |
                  (barrier ? CCLD_SEG_BARRIER : 0) | (usable ? CCLD_SEG_USABLE : 0));
      seg_put(a, CCLD_SEG_OP, srow, (i64)h.op);
      seg_put(a, CCLD_SEG_BYTES, srow, (i64)h.bytes);
      seg_put(a, CCLD_SEG_INFLIGHT_ENTER_MIN, srow, (i64)acc.imin);
      seg_put(a, CCLD_SEG_FIRST, srow, (i64)a0);
      if (nd == 0) {
        seg_put_empty_stats(a, srow);
      } else {
        seg_put(a, CCLD_SEG_ENTER_MIN, srow, min_e); seg_put(a, CCLD_SEG_ENTER_MED, srow, med_e);
        seg_put(a, CCLD_SEG_ENTER_MAX, srow, max_e); seg_put(a, CCLD_SEG_ENTER_MAD, srow, mad_e);
        seg_put(a, CCLD_SEG_EXIT_MIN, srow, min_x); seg_put(a, CCLD_SEG_EXIT_MED, srow, med_x);
        seg_put(a, CCLD_SEG_EXIT_MAX, srow, max_x); seg_put(a, CCLD_SEG_EXIT_MAD, srow, mad_x);
        seg_put(a, CCLD_SEG_DUR_MIN, srow, (i64)acc.dmin); seg_put(a, CCLD_SEG_DUR_MAX, srow, (i64)acc.dmax);
        const u32* ms = a.members_sorted + a.member_off[comm];
        seg_put(a, CCLD_SEG_ARGMIN_RANK, srow, (i64)ms[acc.rmin]); seg_put(a, CCLD_SEG_ARGMAX_RANK, srow, (i64)ms[acc.rmax]);
      }
    }
    for (u32 i = t; i < nn; i += TT) {
      const u32 j = a0 + i;
      i64 le = 0, lx = 0;
      u32 f = 0;
      if (usable) {
        le = E[i] - med_e; lx = X[i] - med_x;
        if (is_late(le, a.lag_floor, a.kmad_num, a.kmad_den, mad_e)) f |= CCLD_FLAG_LATE_ENTER;
        if (is_late(lx, a.lag_floor, a.kmad_num, a.kmad_den, mad_x)) f |= CCLD_FLAG_LATE_EXIT;
      }
      a.rec_flag[j] = (uint8_t)f;
      if (a.lag_e) a.lag_e[j] = le;
      if (a.lag_x) a.lag_x[j] = lx;
      if (f) { a.flag_lag[j] = le; a.flag_lag[a.cap_n + j] = lx; }
    }
    __syncthreads();     // the staged times and the accumulator are reused by the next collective
  }
}

// One workgroup of 1,024 threads per collective of SEG_TEAM_MAX + 1 to SEG_LARGE_MAX records (a world communicator
// of thousands of ranks): the times are staged in global scratch, and one LDS array of 128 KB is filled and sorted
// four times (arrival, completion, and their absolute deviations from the medians).
constexpr u32 LARGE_THREADS = 1024;
__global__ __launch_bounds__(LARGE_THREADS) void k_seg_large(SegArgs a) {
  extern __shared__ i64 s_large[];          // [SEG_LARGE_MAX]
  __shared__ TeamAcc acc;
  i64* V = s_large;
  const u32 t = threadIdx.x;
  const int mb = a.sf.mb;
  const u64 mmask = ((u64)1 << mb) - 1, smask = ((u64)1 << a.sf.ws) - 1;
  i64* big_e = a.big_ex;
  i64* big_x = a.big_ex + a.cap_n;
  const u32 nbig = (u32)a.counters[CNT_NBIG];
  for (u32 ent = blockIdx.x; ent < nbig; ent += gridDim.x) {
    const u32 nn = a.big_list[3 * ent + 2];
    if (nn <= (u32)SEG_TEAM_MAX || nn > (u32)SEG_LARGE_MAX) continue;
    const u32 srow = a.big_list[3 * ent], a0 = a.big_list[3 * ent + 1];
    const u64 k0 = a.key[a0];
    const Row h = load_row(a, a0);
    if (t == 0) {
      acc.imin = (unsigned long long)T_INFLIGHT; acc.dmin = INT64_MAX; acc.dmax = INT64_MIN;
      acc.ninfl = 0; acc.incons = 0; acc.rmin = 0xFFFFFFFFu; acc.rmax = 0xFFFFFFFFu;
    }
    __syncthreads();
    {
      u32 ni = 0, rmin = 0xFFFFFFFFu, rmax = 0xFFFFFFFFu;
      bool inc = false;
      i64 imin = T_INFLIGHT, dmin = INT64_MAX, dmax = INT64_MIN;
      for (u32 i = t; i < nn; i += LARGE_THREADS) {
        const u32 j = a0 + i;
        const Row rw = load_row(a, j);
        big_e[j] = rw.t_enter; big_x[j] = rw.t_exit;
        inc |= (rw.op != h.op || rw.bytes != h.bytes);
        if (rw.t_exit == T_INFLIGHT) {
          ++ni; imin = rw.t_enter < imin ? rw.t_enter : imin;
        } else {
          const i64 d = rw.t_exit - rw.t_enter;
          const u32 rk = (u32)(a.key[j] & mmask);
          if (d < dmin || (d == dmin && rk < rmin)) { dmin = d; rmin = rk; }
          if (d > dmax || (d == dmax && rk < rmax)) { dmax = d; rmax = rk; }
        }
      }
      if (ni) { atomicAdd(&acc.ninfl, ni); atomicMin(&acc.imin, (unsigned long long)imin); }
      if (inc) atomicOr(&acc.incons, 1u);
      if (rmin != 0xFFFFFFFFu) { atomicMin(&acc.dmin, (long long)dmin); atomicMax(&acc.dmax, (long long)dmax); }
      __threadfence_block();
      __syncthreads();
      if (rmin != 0xFFFFFFFFu && dmin == (i64)acc.dmin) atomicMin(&acc.rmin, rmin);
      if (rmax != 0xFFFFFFFFu && dmax == (i64)acc.dmax) atomicMin(&acc.rmax, rmax);
    }
    const u32 ninfl = acc.ninfl, nd = nn - ninfl;
    const u32 km = nd ? (nd - 1) / 2 : 0, kl = nd ? nd - 1 : 0;
    u32 P = 2;
    while (P < nn) P <<= 1;
    const i64* E = big_e + a0;
    const i64* X = big_x + a0;
    for (u32 i = t; i < P; i += LARGE_THREADS) V[i] = (i < nn && X[i] != T_INFLIGHT) ? E[i] : T_INFLIGHT;
    __syncthreads();
    team_sort<LARGE_THREADS>(V, P, t);
    const i64 min_e = V[0], med_e = V[km], max_e = V[kl];
    __syncthreads();
    for (u32 i = t; i < P; i += LARGE_THREADS) V[i] = i < nn ? X[i] : T_INFLIGHT;
    __syncthreads();
    team_sort<LARGE_THREADS>(V, P, t);
    const i64 min_x = V[0], med_x = V[km], max_x = V[kl];
    __syncthreads();
    for (u32 i = t; i < P; i += LARGE_THREADS) V[i] = (i < nn && X[i] != T_INFLIGHT) ? absdiff(E[i], med_e) : T_INFLIGHT;
    __syncthreads();
    team_sort<LARGE_THREADS>(V, P, t);
    const i64 mad_e = V[km];
    __syncthreads();
    for (u32 i = t; i < P; i += LARGE_THREADS) V[i] = (i < nn && X[i] != T_INFLIGHT) ? absdiff(X[i], med_x) : T_INFLIGHT;
    __syncthreads();
    team_sort<LARGE_THREADS>(V, P, t);
    const i64 mad_x = V[km];
    const u32 comm = (u32)(k0 >> (mb + a.sf.ws));
    const bool complete = nn == a.comm_size[comm] && ninfl == 0;
    const bool consistent = acc.incons == 0;
    const bool barrier = h.op == CCLD_OP_ALLREDUCE && h.bytes < (u64)a.barrier_bytes;
    const bool usable = complete && consistent && !barrier;
    if (t == 0) {
      seg_put(a, CCLD_SEG_COMM, srow, (i64)comm);
      seg_put(a, CCLD_SEG_SEQ, srow, (i64)(((k0 >> mb) & smask) + a.sf.seq_base));
      seg_put(a, CCLD_SEG_N, srow, (i64)nn);
      seg_put(a, CCLD_SEG_INFLIGHT, srow, (i64)ninfl);
      seg_put(a, CCLD_SEG_STATE, srow,
              (complete ? CCLD_SEG_COMPLETE : 0) | (consistent ? CCLD_SEG_CONSISTENT : 0) |
                  (barrier ? CCLD_SEG_BARRIER : 0) | (usable ? CCLD_SEG_USABLE : 0));
      seg_put(a, CCLD_SEG_OP, srow, (i64)h.op);
      seg_put(a, CCLD_SEG_BYTES, srow, (i64)h.bytes);
      seg_put(a, CCLD_SEG_INFLIGHT_ENTER_MIN, srow, (i64)acc.imin);
      seg_put(a, CCLD_SEG_FIRST, srow, (i64)a0);
      if (nd == 0) {
        seg_put_empty_stats(a, srow);
      } else {
        seg_put(a, CCLD_SEG_ENTER_MIN, srow, min_e); seg_put(a, CCLD_SEG_ENTER_MED, srow, med_e);
        seg_put(a, CCLD_SEG_ENTER_MAX, srow, max_e); seg_put(a, CCLD_SEG_ENTER_MAD, srow, mad_e);
        seg_put(a, CCLD_SEG_EXIT_MIN, srow, min_x); seg_put(a, CCLD_SEG_EXIT_MED, srow, med_x);
        seg_put(a, CCLD_SEG_EXIT_MAX, srow, max_x); seg_put(a, CCLD_SEG_EXIT_MAD, srow, mad_x);
        seg_put(a, CCLD_SEG_DUR_MIN, srow, (i64)acc.dmin); seg_put(a, CCLD_SEG_DUR_MAX, srow, (i64)acc.dmax);
        const u32* ms = a.members_sorted + a.member_off[comm];
        seg_put(a, CCLD_SEG_ARGMIN_RANK, srow, (i64)ms[acc.rmin]); seg_put(a, CCLD_SEG_ARGMAX_RANK, srow, (i64)ms[acc.rmax]);
      }
    }
    for (u32 i = t; i < nn; i += LARGE_THREADS) {
      const u32 j = a0 + i;
      i64 le = 0, lx = 0;
      u32 f = 0;
      if (usable) {
        le = E[i] - med_e; lx = X[i] - med_x;
        if (is_late(le, a.lag_floor, a.kmad_num, a.kmad_den, mad_e)) f |= CCLD_FLAG_LATE_ENTER;
        if (is_late(lx, a.lag_floor, a.kmad_num, a.kmad_den, mad_x)) f |= CCLD_FLAG_LATE_EXIT;
      }
      a.rec_flag[j] = (uint8_t)f;
      if (a.lag_e) a.lag_e[j] = le;
      if (a.lag_x) a.lag_x[j] = lx;
      if (f) { a.flag_lag[j] = le; a.flag_lag[a.cap_n + j] = lx; }
    }
    __syncthreads();     // the LDS array and the accumulator are reused by the next collective
  }
}

// Collectives longer than SEG_LARGE_MAX records: one workgroup per collective, values staged in
// global scratch, order statistics by counting with all reads broadcast across the workgroup.
__global__ __launch_bounds__(SEG_THREADS) void k_seg_big(SegArgs a) {
  __shared__ u32 s_end, s_ninfl, s_incons;
  __shared__ unsigned long long s_imin;
  __shared__ i64 s_stat[4];      // med_e, med_x, mad_e, mad_x
  const u32 tid = threadIdx.x;
  const int mb = a.sf.mb;
  const u64 mmask = ((u64)1 << mb) - 1, smask = ((u64)1 << a.sf.ws) - 1;
  i64* big_e = a.big_ex;
  i64* big_x = a.big_ex + a.cap_n;
  const u32 nbig = (u32)a.counters[CNT_NBIG];
  for (u32 ent = blockIdx.x; ent < nbig; ent += gridDim.x) {
    if (a.big_list[3 * ent + 2] <= (u32)SEG_LARGE_MAX) continue;    // a workgroup kernel has taken it
    const u32 srow = a.big_list[3 * ent], a0 = a.big_list[3 * ent + 1];
    const u64 k0 = a.key[a0];
    const u64 pref = k0 >> mb;
    if (tid == 0) { s_end = a.n; s_ninfl = 0; s_incons = 0; s_imin = (unsigned long long)T_INFLIGHT; }
    __syncthreads();
    for (u64 j0 = (u64)a0 + 1;; j0 += SEG_THREADS) {
      const u64 j = j0 + tid;
      if (j < a.n && (a.key[j] >> mb) != pref) atomicMin(&s_end, (u32)j);
      __syncthreads();
      const bool stop = s_end != a.n || j0 + SEG_THREADS >= a.n;
      __syncthreads();
      if (stop) break;
    }
    const u32 b0 = s_end, nn = b0 - a0;
    const Row h = load_row(a, a0);
    {
      u32 ni = 0; bool inc = false; i64 imin = T_INFLIGHT;
      for (u32 j = a0 + tid; j < b0; j += SEG_THREADS) {
        const Row rw = load_row(a, j);
        big_e[j] = rw.t_enter; big_x[j] = rw.t_exit;
        if (rw.t_exit == T_INFLIGHT) { ++ni; imin = rw.t_enter < imin ? rw.t_enter : imin; }
        inc |= (rw.op != h.op || rw.bytes != h.bytes);
      }
      if (ni) { atomicAdd(&s_ninfl, ni); atomicMin(&s_imin, (unsigned long long)imin); }
      if (inc) atomicOr(&s_incons, 1u);
    }
    __threadfence_block();
    __syncthreads();
    const u32 ninfl = s_ninfl, nd = nn - ninfl, km = nd ? (nd - 1) / 2 : 0;
    if (tid == 0) {
      seg_put(a, CCLD_SEG_COMM, srow, (i64)(k0 >> (mb + a.sf.ws)));
      seg_put(a, CCLD_SEG_SEQ, srow, (i64)(((k0 >> mb) & smask) + a.sf.seq_base));
      seg_put(a, CCLD_SEG_N, srow, (i64)nn);
      seg_put(a, CCLD_SEG_INFLIGHT, srow, (i64)ninfl);
      seg_put(a, CCLD_SEG_OP, srow, (i64)h.op);
      seg_put(a, CCLD_SEG_BYTES, srow, (i64)h.bytes);
      seg_put(a, CCLD_SEG_INFLIGHT_ENTER_MIN, srow, (i64)s_imin);
      seg_put(a, CCLD_SEG_FIRST, srow, (i64)a0);
      if (nd == 0) seg_put_empty_stats(a, srow);
    }
    for (u32 i = a0 + tid; i < b0; i += SEG_THREADS) {
      const i64 ei = big_e[i], xi = big_x[i];
      if (xi == T_INFLIGHT) continue;
      const i64 di = xi - ei;
      u32 re = 0, rx = 0, cmin = 0, cmax = 0;
      for (u32 j = a0; j < b0; ++j) {
        const i64 ej = big_e[j], xj = big_x[j];
        if (xj == T_INFLIGHT) continue;
        const i64 dj = xj - ej;
        const bool before = j < i;
        re += (ej < ei) || (ej == ei && before);
        rx += (xj < xi) || (xj == xi && before);
        cmin += (dj < di) || (dj == di && before);
        cmax += (dj > di) || (dj == di && before);
      }
      if (re == km) { s_stat[0] = ei; seg_put(a, CCLD_SEG_ENTER_MED, srow, ei); }
      if (re == 0) seg_put(a, CCLD_SEG_ENTER_MIN, srow, ei);
      if (re == nd - 1) seg_put(a, CCLD_SEG_ENTER_MAX, srow, ei);
      if (rx == km) { s_stat[1] = xi; seg_put(a, CCLD_SEG_EXIT_MED, srow, xi); }
      if (rx == 0) seg_put(a, CCLD_SEG_EXIT_MIN, srow, xi);
      if (rx == nd - 1) seg_put(a, CCLD_SEG_EXIT_MAX, srow, xi);
      const i64 rk = (i64)a.members_sorted[a.member_off[(u32)(k0 >> (mb + a.sf.ws))] + (u32)(a.key[i] & mmask)];
      if (cmin == 0) { seg_put(a, CCLD_SEG_DUR_MIN, srow, di); seg_put(a, CCLD_SEG_ARGMIN_RANK, srow, rk); }
      if (cmax == 0) { seg_put(a, CCLD_SEG_DUR_MAX, srow, di); seg_put(a, CCLD_SEG_ARGMAX_RANK, srow, rk); }
    }
    __syncthreads();
    const i64 me = s_stat[0], mx = s_stat[1];
    for (u32 i = a0 + tid; i < b0; i += SEG_THREADS) {
      const i64 xi = big_x[i];
      if (xi == T_INFLIGHT) continue;
      const i64 dei = absdiff(big_e[i], me), dxi = absdiff(xi, mx);
      u32 rde = 0, rdx = 0;
      for (u32 j = a0; j < b0; ++j) {
        const i64 xj = big_x[j];
        if (xj == T_INFLIGHT) continue;
        const i64 dej = absdiff(big_e[j], me), dxj = absdiff(xj, mx);
        const bool before = j < i;
        rde += (dej < dei) || (dej == dei && before);
        rdx += (dxj < dxi) || (dxj == dxi && before);
      }
      if (rde == km) { s_stat[2] = dei; seg_put(a, CCLD_SEG_ENTER_MAD, srow, dei); }
      if (rdx == km) { s_stat[3] = dxi; seg_put(a, CCLD_SEG_EXIT_MAD, srow, dxi); }
    }
    __syncthreads();
    const u32 comm = (u32)(k0 >> (mb + a.sf.ws));
    const bool complete = nn == a.comm_size[comm] && ninfl == 0;
    const bool consistent = s_incons == 0;
    const bool barrier = h.op == CCLD_OP_ALLREDUCE && h.bytes < (u64)a.barrier_bytes;
    const bool usable = complete && consistent && !barrier;
    if (tid == 0)
      seg_put(a, CCLD_SEG_STATE, srow,
              (complete ? CCLD_SEG_COMPLETE : 0) | (consistent ? CCLD_SEG_CONSISTENT : 0) |
                  (barrier ? CCLD_SEG_BARRIER : 0) | (usable ? CCLD_SEG_USABLE : 0));
    for (u32 i = a0 + tid; i < b0; i += SEG_THREADS) {
      i64 le = 0, lx = 0;
      u32 f = 0;
      if (usable) {
        le = big_e[i] - me; lx = big_x[i] - mx;
        if (is_late(le, a.lag_floor, a.kmad_num, a.kmad_den, s_stat[2])) f |= CCLD_FLAG_LATE_ENTER;
        if (is_late(lx, a.lag_floor, a.kmad_num, a.kmad_den, s_stat[3])) f |= CCLD_FLAG_LATE_EXIT;
      }
      a.rec_flag[i] = (uint8_t)f;
      if (a.lag_e) a.lag_e[i] = le;
      if (a.lag_x) a.lag_x[i] = lx;
      if (f) { a.flag_lag[i] = le; a.flag_lag[a.cap_n + i] = lx; }
    }
    __syncthreads();
  }
}

// group key and range of the collectives that a workgroup analysed (more than SEG_MULTI_MAX records), from
// their rows of the table; a row past the table's capacity is not stored and takes no part in the group stage
__global__ __launch_bounds__(256) void k_seg_group_listed(SegArgs a) {
  const u32 nbig = (u32)a.counters[CNT_NBIG];
  for (u32 ent = blockIdx.x * 256 + threadIdx.x; ent < nbig; ent += gridDim.x * 256) {
    if (a.big_list[3 * ent + 2] <= (u32)SEG_MULTI_MAX) continue;
    const u32 srow = a.big_list[3 * ent];
    if (srow >= a.seg_cap) { a.gkey[srow] = a.no_group; a.range_c[srow] = 0; continue; }
    const u64 C = a.seg_cap;
    const bool usable = (a.seg[(u64)CCLD_SEG_STATE * C + srow] & CCLD_SEG_USABLE) != 0;
    seg_put_group(a, srow, usable, (u32)a.seg[(u64)CCLD_SEG_COMM * C + srow], (u32)a.seg[(u64)CCLD_SEG_OP * C + srow],
                  (u64)a.seg[(u64)CCLD_SEG_BYTES * C + srow], a.seg[(u64)CCLD_SEG_DUR_MAX * C + srow],
                  a.seg[(u64)CCLD_SEG_DUR_MIN * C + srow]);
  }
}

// ---- dense placement: statistics straight from the partitioned rows -----------------------------------
// One workgroup per fine bucket: the bucket's rows (in arrival order) are placed in LDS by grid cell
// (round inside the bucket x member slot), which puts every collective's records side by side in rank
// order with empty cells where a member has no record; the wavefronts then take the collectives
// 64 / G at a time exactly as k_seg_wave does.  The kernel also writes the records' squeezed keys and row
// indices in (communicator, counter, rank) order, which the flag, blame, group and alert stages read, and
// adds the records per rank to the blame table.
constexpr int DENSE_THREADS = 512;

template <int G, bool STAGED>
__device__ __forceinline__ u32 dense_wave_batches(const SegArgs& a, uint4* s_cell, const u32* s_pres,
                                                  const u32* s_pre, u32 K, u32 size, u32 comm, u64 rel0, u32 srow0,
                                                  u32 rec0, u32 row0, u64* __restrict__ skey, u32* __restrict__ sidx,
                                                  u32 lane, u32 wave) {
  constexpr int SPW = CCLD_WAVE / G, NW = DENSE_THREADS / CCLD_WAVE;
  const int mb = a.sf.mb;
  const u32 q = lane / G, l = lane % G, gbase = q * G;
  const u64 gmask = (G == 64 ? ~0ull : (((u64)1 << (G & 63)) - 1)) << gbase;
  const u64 below = ((u64)1 << lane) - 1;
  const u32* __restrict__ ms = a.members_sorted + a.member_off[comm];
  const u32 rank = l < size ? ms[l] : 0u;
  u32 mine = 0;                                    // records seen in this lane's member slot
  for (u32 b = wave; b * SPW < K; b += NW) {
    const u32 k = b * SPW + q;
    const bool in = k < K && l < size;
    const u32 cell = k * size + l;
    DenseLane L;
    L.valid = in && ((s_pres[cell >> 5] >> (cell & 31)) & 1u);
    L.pm = ballot64(L.valid) & gmask;
    L.n = (u32)__popcll(L.pm);
    L.e = 0; L.x = T_INFLIGHT; L.nb = 0; L.op = 0; L.rank = rank; L.comm = comm;
    // the collective's own cells (size x 32 bytes, at least one region) take its row once they are read
    L.staged = STAGED;
    L.stage = (lds_i64*)reinterpret_cast<i64*>(s_cell) + k * size * 4 + stage_skew(k);
    u32 ai = 0;
    if (L.valid) {
      const uint4 h0 = s_cell[2 * cell], h1 = s_cell[2 * cell + 1];
      L.e = (i64)(((u64)h0.y << 32) | h0.x); L.x = (i64)(((u64)h0.w << 32) | h0.z);
      L.nb = ((u64)h1.y << 32) | h1.x; L.op = h1.z & 15u; ai = h1.z >> 4;
      ++mine;
    }
    L.first = rec0 + (k < K ? s_pre[k] : 0u);
    L.j = L.first + (u32)__popcll(L.pm & below);
    L.fl = L.pm ? (u32)__builtin_ctzll(L.pm) : gbase;
    L.srow = srow0 + k;
    const u64 rel = rel0 + k;
    L.seq = rel + a.sf.seq_base;
    if (L.valid) {
      skey[L.j] = ((u64)comm << (mb + a.sf.ws)) | (rel << mb) | (u64)l;
      sidx[L.j] = row0 + ai;
    }
    // offsets from the arrival of the collective's first present member
    const i64 ref = shfl_i64(L.e, (int)L.fl);
    const i64 oe = L.e - ref, ox = L.x - ref;
    constexpr i64 LIM = (i64)1 << 30;
    const bool wide = L.valid && (oe < -LIM || oe >= LIM || (L.x != T_INFLIGHT && (ox < -LIM || ox >= LIM)));
    if (ballot64(wide) == 0) dense_pass32<G, STAGED ? PUT_STAGED : PUT_DIRECT>(a, L, ref, (i32)oe, (i32)ox, size, lane, gbase, gmask);
    else dense_pass64<G, STAGED ? PUT_STAGED : PUT_DIRECT>(a, L, size, lane, gbase, gmask);
  }
  return mine;
}

// One workgroup per fine bucket, two workgroups of eight wavefronts per compute unit (their LDS allows no more):
// while one of them waits for its rows or at a barrier the other one computes.  Measured at the 4,096-rank
// trace: a grid-stride loop over the buckets makes the compiler keep the loop's invariants in some 230
// registers (two wavefronts per SIMD, 2.2 ms; capped at 128 registers it spills, 3.3 ms); one bucket per
// workgroup needs 97 registers, and 512 threads take 1.7 ms (256: 2.0, 384: 2.7, 640: 2.3, 1,024: 2.2 ms).
__global__ __launch_bounds__(DENSE_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_dense_stats(SegArgs a, DenseArgs d, u64* __restrict__ skey,
                                                               u32* __restrict__ sidx, i64* __restrict__ blame,
                                                               u32 n_ranks) {
  constexpr int U = (DENSE_STRIDE + DENSE_THREADS - 1) / DENSE_THREADS;        // rows per thread
  __shared__ uint4 s_cell[2 * DENSE_B];
  __shared__ u32 s_pres[DENSE_B / 32];
  __shared__ unsigned short s_n[DENSE_B];
  __shared__ u32 s_aux[DENSE_B + 4];          // [K] first record of each collective, then [size] records per member slot
  __shared__ u32 s_wave[DENSE_THREADS / CCLD_WAVE];
  if (d.hdr[DH_FEASIBLE] == 0) return;
  const u32 tid = threadIdx.x, lane = lane_id(), wave = tid / CCLD_WAVE;
  const u32 f = blockIdx.x;
  if (f >= d.hdr[DH_N_FINE]) return;
  const uint4* __restrict__ rows4 = reinterpret_cast<const uint4*>(d.rows);
  unsigned long long* nrec = (unsigned long long*)(blame + (u64)CCLD_BLM_N_RECORDS * n_ranks);
  typedef u32 u32x4 __attribute__((ext_vector_type(4)));
  u32x4 h0[U], h1[U];
  auto fetch = [&](u32 f, u32 cnt) {
    const u64 row0 = (u64)f * DENSE_STRIDE;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u32 i = tid + u * DENSE_THREADS;
      if (i < cnt) {
        h0[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rows4 + 2 * (row0 + i)));
        h1[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rows4 + 2 * (row0 + i) + 1));
      }
    }
  };
  auto clamp = [](u32 c) { return c < DENSE_STRIDE ? c : DENSE_STRIDE; };
  const FineDesc D = d.desc[f];
  {
    const u32 c = D.comm, size = D.size, K = D.K, rec0 = D.rec0, cnt = clamp(D.cnt);
    const u32 row0 = f * DENSE_STRIDE;
    u32* s_pre = s_aux;
    u32* s_slot = s_aux + K;
    fetch(f, cnt);                    // the rows are on their way while the bucket's LDS state is cleared
    for (u32 i = tid; i < DENSE_B / 32; i += DENSE_THREADS) s_pres[i] = 0;
    for (u32 i = tid; i < size; i += DENSE_THREADS) s_slot[i] = 0;
    __syncthreads();
    // 1. every row into its cell; a cell taken twice is a duplicate key
    bool dup = D.cnt > DENSE_STRIDE;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u32 i = tid + u * DENSE_THREADS;
      if (i >= cnt) continue;
      const u32 cell = (h1[u].z >> 4) & (DENSE_B - 1);
      if (cell >= K * size) { dup = true; continue; }
      const u32 bit = 1u << (cell & 31);
      if (atomicOr(&s_pres[cell >> 5], bit) & bit) { dup = true; continue; }
      s_cell[2 * cell] = make_uint4(h0[u].x, h0[u].y, h0[u].z, h0[u].w);
      s_cell[2 * cell + 1] = make_uint4(h1[u].x, h1[u].y, (h1[u].z & 15u) | (i << 4), h1[u].w);
    }
    __syncthreads();
    // 2. records per collective, their exclusive scan; a round without any record is a hole in the grid
    for (u32 k = tid; k < K; k += DENSE_THREADS) {
      const u32 b0 = k * size, b1 = b0 + size;      // bits [b0, b1)
      u32 nk = 0;
      for (u32 w = b0 >> 5; w <= (b1 - 1) >> 5; ++w) {
        u32 m = s_pres[w];
        if (w == (b0 >> 5)) m &= ~0u << (b0 & 31);
        if (w == ((b1 - 1) >> 5) && (b1 & 31)) m &= (1u << (b1 & 31)) - 1;
        nk += __popc(m);
      }
      s_n[k] = (unsigned short)nk;
    }
    __syncthreads();
    bool gap = false;
    {
      constexpr int PER = (DENSE_B + DENSE_THREADS - 1) / DENSE_THREADS;
      u32 v[PER], sum = 0;
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const u32 k = PER * tid + i;
        v[i] = k < K ? s_n[k] : 0u;
        gap |= k < K && v[i] == 0;
        sum += v[i];
      }
      u32 tot;
      u32 ex = block_exclusive_sum<DENSE_THREADS>(sum, s_wave, &tot);
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const u32 k = PER * tid + i;
        if (k < K) s_pre[k] = ex;
        ex += v[i];
      }
    }
    __syncthreads();
    u64 bad = (dup ? (u64)DS_DUPLICATE : 0) | (gap ? (u64)DS_DENSE_FALLBACK : 0);
    // 3. the collectives
    const u64 rel0 = D.rel0;
    const u32 srow0 = D.srow0;
    if (size <= (u32)SEG_WAVE_MAX) {
      u32 mine;
      // from eight members on, a collective's cells are large enough to hold its table row
      if (size <= 2) mine = dense_wave_batches<2, false>(a, s_cell, s_pres, s_pre, K, size, c, rel0, srow0, rec0, row0, skey, sidx, lane, wave);
      else if (size <= 4) mine = dense_wave_batches<4, false>(a, s_cell, s_pres, s_pre, K, size, c, rel0, srow0, rec0, row0, skey, sidx, lane, wave);
      else if (size < 8) mine = dense_wave_batches<8, false>(a, s_cell, s_pres, s_pre, K, size, c, rel0, srow0, rec0, row0, skey, sidx, lane, wave);
      else if (size == 8) mine = dense_wave_batches<8, true>(a, s_cell, s_pres, s_pre, K, size, c, rel0, srow0, rec0, row0, skey, sidx, lane, wave);
      else if (size <= 16) mine = dense_wave_batches<16, true>(a, s_cell, s_pres, s_pre, K, size, c, rel0, srow0, rec0, row0, skey, sidx, lane, wave);
      else if (size <= 32) mine = dense_wave_batches<32, true>(a, s_cell, s_pres, s_pre, K, size, c, rel0, srow0, rec0, row0, skey, sidx, lane, wave);
      else mine = dense_wave_batches<64, true>(a, s_cell, s_pres, s_pre, K, size, c, rel0, srow0, rec0, row0, skey, sidx, lane, wave);
      // the lane's member slot is the same in every pass
      u32 G = 2; while (G < size) G <<= 1;
      if (mine) atomicAdd(&s_slot[lane % G], mine);
    } else {
      // communicators of more than 64 members: the records are written out in rank order and every
      // collective goes on the list of the kernels that take long collectives
      const int mb = a.sf.mb;
      for (u32 k = wave; k < K; k += DENSE_THREADS / CCLD_WAVE) {
        const u32 nk = s_n[k];
        if (nk == 0) continue;
        const u32 first = rec0 + s_pre[k];
        u32 run = 0;
        for (u32 s0 = 0; s0 < size; s0 += CCLD_WAVE) {
          const u32 slot = s0 + lane, cell = k * size + slot;
          const bool valid = slot < size && ((s_pres[cell >> 5] >> (cell & 31)) & 1u);
          const u64 pm = ballot64(valid);
          if (valid) {
            const u32 j = first + run + mbcnt64(pm);
            skey[j] = ((u64)c << (mb + a.sf.ws)) | ((rel0 + k) << mb) | (u64)slot;
            sidx[j] = row0 + (s_cell[2 * cell + 1].z >> 4);
            atomicAdd(&s_slot[slot], 1u);
          }
          run += (u32)__popcll(pm);
        }
        if (lane == 0) {
          const u64 at = atomic_add_u64(&a.counters[CNT_NBIG], 1);
          if (at < a.big_cap) {
            a.big_list[3 * at] = srow0 + k; a.big_list[3 * at + 1] = first; a.big_list[3 * at + 2] = nk;
          } else {
            bad |= (u64)DS_DENSE_FALLBACK;      // more listed collectives than the list holds
          }
        }
      }
    }
    if (bad) atomicOr((unsigned long long*)&a.counters[CNT_STATUS], (unsigned long long)bad);
    __syncthreads();
    // the staged table rows: every wavefront writes whole columns, consecutive lanes to consecutive rows
    if (size >= 8 && size <= (u32)SEG_WAVE_MAX) {
      const i64* S = reinterpret_cast<const i64*>(s_cell);
      for (u32 col = wave; col < STAGE_COLS; col += DENSE_THREADS / CCLD_WAVE) {
        for (u32 k = lane; k < K; k += CCLD_WAVE) {
          if (s_n[k] == 0) continue;                   // a round without any record has no row
          const i64 v = S[k * size * 4 + stage_skew(k) + col];
          const u32 srow = srow0 + k;
          if (col < (u32)CCLD_SEG_NCOL) { if (srow < a.seg_cap) a.seg[(u64)col * a.seg_cap + srow] = v; }
          else if (col == (u32)CCLD_SEG_NCOL) a.gkey[srow] = (u64)v;
          else a.range_c[srow] = v;
        }
      }
    }
    // 4. records per rank
    {
      const u32* __restrict__ ms = a.members_sorted + a.member_off[c];
      for (u32 sl = tid; sl < size; sl += DENSE_THREADS) {
        const u32 v = s_slot[sl];
        if (v) atomicAdd(&nrec[ms[sl]], (unsigned long long)v);
      }
    }
  }
}

// the collectives on the list (more than 64 records; from the dense placement also shorter ones)
static void launch_seg_listed(hipStream_t st, const SegArgs& a, bool with_short) {
  // a collective has at most as many records as its communicator has members (a longer one holds a
  // duplicate, which ends the analysis with an error): size classes that cannot occur are not launched
  const uint32_t m = a.max_size;
  if (m <= (uint32_t)SEG_WAVE_MAX) return;
  hipLaunchKernelGGL(k_seg_lengths, dim3(1024), dim3(SEG_THREADS), 0, st, a);
  if (with_short) hipLaunchKernelGGL(k_seg_multi<1>, dim3(2048), dim3(SEG_THREADS), 0, st, a);
  hipLaunchKernelGGL(k_seg_multi<2>, dim3(2048), dim3(SEG_THREADS), 0, st, a);
  if (m > 128) hipLaunchKernelGGL(k_seg_multi<4>, dim3(2048), dim3(SEG_THREADS), 0, st, a);
  if (m > 256) hipLaunchKernelGGL(k_seg_multi<8>, dim3(2048), dim3(SEG_THREADS), 0, st, a);
  if (m > (uint32_t)SEG_MULTI_MAX) hipLaunchKernelGGL(k_seg_team, dim3(1024), dim3(SEG_THREADS), 0, st, a);
  if (m > (uint32_t)SEG_TEAM_MAX) {
    static bool raised = false;       // more than 64 KB of dynamic LDS has to be asked for once
    constexpr size_t lds = sizeof(int64_t) * SEG_LARGE_MAX;
    if (!raised) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_seg_large), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      raised = true;
    }
    hipLaunchKernelGGL(k_seg_large, dim3(512), dim3(LARGE_THREADS), lds, st, a);
  }
  if (m > (uint32_t)SEG_LARGE_MAX) hipLaunchKernelGGL(k_seg_big, dim3(2048), dim3(SEG_THREADS), 0, st, a);
  if (m > (uint32_t)SEG_MULTI_MAX) hipLaunchKernelGGL(k_seg_group_listed, dim3(256), dim3(256), 0, st, a);
}

void launch_dense_stats(hipStream_t st, const SegArgs& a, const DenseArgs& d, uint32_t n_fine, uint64_t* skey,
                        uint32_t* sidx, int64_t* blame, uint32_t n_ranks) {
  if (a.n == 0 || n_fine == 0) return;
  hipLaunchKernelGGL(k_dense_stats, dim3(n_fine), dim3(DENSE_THREADS), 0, st, a, d, skey, sidx, blame, n_ranks);
  launch_seg_listed(st, a, true);
}

void launch_seg_analyze(hipStream_t st, const SegArgs& a) {
  if (a.n == 0) return;
  hipLaunchKernelGGL(k_seg_wave, dim3((a.n + SEG_TILE - 1) / SEG_TILE), dim3(SEG_THREADS), 0, st, a);
  launch_seg_listed(st, a, false);
}

}  // namespace ccld
