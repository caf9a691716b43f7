// extern "C" entry points: context set-up, workspace carving, ingest, window analysis, blame.
#include <algorithm>
#include <cstring>
#include <new>

#include "ccld_internal.h"
#include "window_kernels.h"
#include "merge.h"
#include "dense.h"

using namespace ccld;

#define HIP_TRY(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); return CCLD_E_HIP; } } while (0)

static int bits_for_host(uint64_t v) { int b = 0; while (v) { ++b; v >>= 1; } return b; }

namespace {

// Bump allocator over the caller's workspace; with base == nullptr it only measures.
struct Carver {
  uint8_t* base; uint64_t off;
  template <class T> T* take(uint64_t count) {
    off = (off + 255) & ~(uint64_t)255;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

struct TopoCounts { uint64_t n_members; };

void carve_all(ccld_ctx* c, Carver& w, uint32_t n_ranks, uint32_t n_comms, uint64_t n_members) {
  const uint64_t N = std::max<uint64_t>(c->cap, 1), B = std::max<uint64_t>(c->batch_cap, 1);
  // topology
  c->topo.algo = w.take<uint8_t>(n_comms);
  c->topo.size = w.take<uint32_t>(n_comms);
  c->topo.member_off = w.take<uint32_t>(n_comms);
  c->topo.members = w.take<uint32_t>(n_members);
  c->topo.members_sorted = w.take<uint32_t>(n_members);
  c->topo.sorted_slot = w.take<uint32_t>(n_members);
  c->topo.tree_parent = w.take<int32_t>(n_members);
  c->topo.rank_comm_off = w.take<uint32_t>((uint64_t)n_ranks + 1);
  c->topo.rank_comms = w.take<uint32_t>(n_members);
  c->topo.rank_slots = w.take<uint32_t>(n_members);
  c->topo.rank_memb4 = w.take<uint32_t>(4ull * n_ranks);
  c->topo.rank_cell4 = w.take<uint32_t>(4ull * n_ranks);
  c->comm_info = w.take<uint2>(n_comms);
  // window
  c->win_key = w.take<uint64_t>(N);
  c->win_row = w.take<Row>(N);
  c->batch_meta = w.take<BatchMeta>((uint64_t)c->p.window_batches + 2);
  c->ing_table = w.take<uint32_t>((uint64_t)INGEST_MAX_BUCKETS * INGEST_BLOCKS);
  c->ing_base = w.take<uint32_t>(INGEST_MAX_BUCKETS + 2);
  // sort
  // (the hang pass sorts its root list, at most one entry per communicator member, in these buffers too)
  const uint64_t NS = std::max<uint64_t>(N, n_members);
  c->sort_cap = NS;
  const uint64_t tw = sort_table_words(NS);
  for (int i = 0; i < 2; ++i) { c->sb.key[i] = w.take<uint64_t>(NS); c->sb.idx[i] = w.take<uint32_t>(NS); }
  c->sb.table = w.take<uint32_t>(tw);
  c->sb.totals = w.take<uint32_t>(SORT_RADIX);
  c->keyC = w.take<uint64_t>(NS); c->idxC = w.take<uint32_t>(NS);
  c->table2 = w.take<uint32_t>(tw);
  c->totals2 = w.take<uint32_t>(SORT_RADIX);
  // analysis scratch
  const uint64_t NT = std::max<uint64_t>(N, std::max<uint64_t>(n_members, n_comms));   // the tile-count scratch also serves the hang pass
  const uint64_t seg_tiles = (NT + SEG_TILE - 1) / SEG_TILE, sel_tiles = (NT + SEL_TILE - 1) / SEL_TILE;
  c->tile_heads = w.take<uint32_t>(seg_tiles + 2);
  c->tile_flags = w.take<uint32_t>(sel_tiles + 2);
  c->blame_list = w.take<uint32_t>(2ull * n_ranks);
  c->blame_tiles = w.take<uint32_t>(n_ranks / SEL_TILE + 3);
  c->blame_order = w.take<uint32_t>(n_ranks);
  // per-record scratch of one analysis; nothing in it outlives the next ingest, so a batch that arrives in host
  // memory is staged in the same bytes (48 per record of batch capacity)
  c->stage = w.take<uint8_t>(0);
  const uint64_t scratch_begin = w.off;
  c->rec_flag = w.take<uint8_t>(N);
  c->flag_pos = w.take<uint32_t>(N);
  c->flag_lag = w.take<int64_t>(2 * N);
  c->big_list = w.take<uint32_t>(3 * (N / 65 + 2));
  c->big_ex = w.take<int64_t>(2 * N);
  c->range_c = w.take<int64_t>(N);
  c->group_long = w.take<uint32_t>(N / GROUP_LONG_MIN + 2);
  c->group_first = w.take<uint32_t>(N + 1);
  c->alert_list = w.take<uint32_t>(NT);
  c->alert_ncand = w.take<uint32_t>(N + 2);
  if (w.off - scratch_begin < B * 48) (void)w.take<uint8_t>(B * 48 - (w.off - scratch_begin));
  c->gstate = w.take<GroupState>((uint64_t)n_comms * GROUP_SLOTS);
  c->chain_first = w.take<uint32_t>((uint64_t)n_comms + 2);
  // the counters and the blame table are cleared together at the start of every analysis
  c->counters = w.take<uint64_t>(CNT_COUNT);
  c->blame = w.take<int64_t>((uint64_t)CCLD_BLM_NCOL * n_ranks);
  // dense placement: counter ranges, layout, fine-bucket fill counts and the partitioned rows (room for an
  // eighth more cells than records, and one partly filled fine bucket per communicator)
  c->fine_cap = 0;
  c->comm_range = nullptr; c->d_lay = nullptr; c->d_hdr = nullptr; c->d_fill = nullptr; c->d_rows = nullptr; c->d_desc = nullptr;
  if (c->dense_capable) {
    c->fine_cap = (uint32_t)((N + N / 8) / DENSE_B + n_comms + 16);
    c->comm_range = w.take<uint64_t>(2ull * n_comms);
    c->d_lay = w.take<CommLayout>((uint64_t)n_comms + 1);
    c->d_hdr = w.take<uint32_t>(DH_COUNT);
    c->d_fill = w.take<uint32_t>((uint64_t)c->fine_cap + 4);
    c->d_rows = w.take<Row>((uint64_t)c->fine_cap * DENSE_STRIDE);
    c->d_desc = w.take<FineDesc>((uint64_t)c->fine_cap);
  }
  // hang location
  const uint64_t SN = std::max<uint64_t>(c->snap_cap, 1);
  c->n_members = n_members;
  c->rate_root = w.take<int64_t>(n_comms);
  c->h_cell = w.take<uint64_t>(2 * SN);
  c->h_cnt = w.take<uint32_t>(SN / 32 + 1);
  c->h_pair = w.take<int64_t>((uint64_t)CCLD_HPAIR_NCOL * n_members);
  c->h_comm = w.take<int64_t>((uint64_t)CCLD_HCOMM_NCOL * n_comms);
  c->h_wait_slot = w.take<int32_t>(n_members);
  c->h_cand = w.take<uint8_t>(n_members);
  c->h_layer_max = w.take<uint64_t>(n_members);
  c->h_root_list = w.take<uint32_t>(n_members + 1);
  c->f_last = w.take<uint64_t>(2ull * CCLD_FRAME_CHANNELS * n_members);
  c->f_seen = w.take<uint32_t>(n_ranks / 32 + 1);
  c->h_stage = w.take<uint8_t>(SN * 32);
}

ccld_status check_params(const ccld_params* p) {
  if (!p) return CCLD_E_NULL;
  if (p->tbase_rounds < 1 || p->theta_den < 1 || p->ab_den < 1 || p->kmad_den < 1 || p->tbase_warmup_ns < 0 ||
      p->window_batches < 1 || p->window_batches > 4096 || p->hang_threshold_ns < 0 ||
      p->placement > CCLD_PLACEMENT_DENSE)
    return CCLD_E_BAD_ARG;
  return CCLD_OK;
}

ccld_status check_topology(const ccld_topology* t, uint64_t* n_members) {
  if (!t) return CCLD_E_NULL;
  if (t->n_ranks == 0 || t->n_comms == 0) return CCLD_E_BAD_TOPOLOGY;
  if (!t->algo || !t->size || !t->member_off || !t->members) return CCLD_E_NULL;
  uint64_t total = 0;
  for (uint32_t c = 0; c < t->n_comms; ++c) {
    if (t->size[c] == 0 || t->algo[c] > CCLD_ALGO_TREE) return CCLD_E_BAD_TOPOLOGY;
    if (t->member_off[c] != total) return CCLD_E_BAD_TOPOLOGY;     // packed CSR
    total += t->size[c];
    if (total > 0xFFFFFFFFull) return CCLD_E_BAD_TOPOLOGY;
  }
  for (uint32_t c = 0; c < t->n_comms; ++c) {
    std::vector<uint32_t> m(t->members + t->member_off[c], t->members + t->member_off[c] + t->size[c]);
    std::sort(m.begin(), m.end());
    for (size_t i = 0; i < m.size(); ++i)
      if (m[i] >= t->n_ranks || (i > 0 && m[i] == m[i - 1])) return CCLD_E_BAD_TOPOLOGY;
    if (t->algo[c] == CCLD_ALGO_TREE) {
      if (!t->tree_parent) return CCLD_E_BAD_TOPOLOGY;
      int roots = 0;
      for (uint32_t q = 0; q < t->size[c]; ++q) {
        int32_t par = t->tree_parent[t->member_off[c] + q];
        if (par < 0) ++roots;
        else if ((uint32_t)par >= q) return CCLD_E_BAD_TOPOLOGY;   // BFS order: parents come first
      }
      if (roots != 1 || t->tree_parent[t->member_off[c]] >= 0) return CCLD_E_BAD_TOPOLOGY;
      std::vector<uint32_t> depth(t->size[c], 0);                  // BFS order: layers are contiguous
      for (uint32_t q = 1; q < t->size[c]; ++q) {
        depth[q] = depth[t->tree_parent[t->member_off[c] + q]] + 1;
        if (depth[q] < depth[q - 1]) return CCLD_E_BAD_TOPOLOGY;
      }
    }
  }
  *n_members = total;
  return CCLD_OK;
}

// Windows of one batch can be analysed by dense placement when every communicator fits a fine bucket and
// the counting kernel's LDS holds a counter range per communicator.
bool dense_capable(const ccld_params* p, const ccld_topology* t) {
  if (p->placement != CCLD_PLACEMENT_DENSE || p->window_batches != 1 || t->n_comms > DENSE_MAX_COMMS) return false;
  for (uint32_t k = 0; k < t->n_comms; ++k) if (t->size[k] > DENSE_B) return false;
  return true;
}

ccld_status data_status(uint64_t bits) {
  if (bits & DS_UNKNOWN_COMM) return CCLD_E_UNKNOWN_COMM;
  if (bits & DS_NOT_MEMBER) return CCLD_E_RANK_NOT_MEMBER;
  if (bits & DS_RANGE) return CCLD_E_RANGE;
  if (bits & DS_KEY_WIDTH) return CCLD_E_KEY_WIDTH;
  if (bits & DS_DUPLICATE) return CCLD_E_DUPLICATE_KEY;
  if (bits & DS_SNAPSHOT_GAP) return CCLD_E_SNAPSHOT_GAP;
  return CCLD_OK;
}

}  // namespace

extern "C" {

ccld_status ccld_default_params(ccld_params* p) {
  if (!p) return CCLD_E_NULL;
  std::memset(p, 0, sizeof(*p));
  p->hang_threshold_ns = 300000000000ll;
  p->tbase_init_ns = INT64_MAX / 4;
  p->tbase_rounds = 100;
  p->repeat_threshold = 2;
  p->tbase_warmup_ns = 120000000000ll;
  p->theta_num = 3; p->theta_den = 1;
  p->alpha_num = 4; p->beta_num = 6; p->ab_den = 10;
  p->barrier_bytes = 4;
  p->kmad_num = 9; p->kmad_den = 2;
  p->lag_floor_ns = 300000;
  p->stall_snapshots = 30;
  p->fifo_depth = 8;
  p->window_batches = 1;
  return CCLD_OK;
}

ccld_status ccld_query_workspace(const ccld_params* params, const ccld_topology* topo, uint64_t max_window_records,
                                 uint64_t max_batch_records, uint64_t max_snapshot_rows, uint64_t* bytes) {
  if (!bytes) return CCLD_E_NULL;
  ccld_status s = check_params(params);
  if (s != CCLD_OK) return s;
  uint64_t n_members = 0;
  s = check_topology(topo, &n_members);
  if (s != CCLD_OK) return s;
  if (max_window_records >= (1ull << 31) || max_batch_records > max_window_records ||
      max_snapshot_rows >= (1ull << 31))
    return CCLD_E_CAPACITY;
  ccld_ctx tmp;
  tmp.p = *params; tmp.cap = max_window_records; tmp.batch_cap = max_batch_records; tmp.snap_cap = max_snapshot_rows;
  tmp.dense_capable = dense_capable(params, topo);
  Carver w{nullptr, 0};
  carve_all(&tmp, w, topo->n_ranks, topo->n_comms, n_members);
  *bytes = w.off + 256;
  return CCLD_OK;
}

ccld_status ccld_create(const ccld_params* params, const ccld_topology* topo, uint64_t max_window_records,
                        uint64_t max_batch_records, uint64_t max_snapshot_rows, void* workspace,
                        uint64_t workspace_bytes, void* hip_stream, ccld_ctx** out) {
  if (!out || !workspace) return CCLD_E_NULL;
  *out = nullptr;
  uint64_t need = 0;
  ccld_status s = ccld_query_workspace(params, topo, max_window_records, max_batch_records, max_snapshot_rows, &need);
  if (s != CCLD_OK) return s;
  if (workspace_bytes < need || ((uintptr_t)workspace & 255) != 0) return CCLD_E_WORKSPACE;
  uint32_t max_size = 1;
  for (uint32_t k = 0; k < topo->n_comms; ++k) max_size = std::max(max_size, topo->size[k]);
  const int mb = bits_for_host(max_size - 1), cb = bits_for_host(topo->n_comms - 1);
  if (mb + cb > 63) return CCLD_E_KEY_WIDTH;
  ccld_ctx* c = new (std::nothrow) ccld_ctx();
  if (!c) return CCLD_E_BAD_ARG;
  c->p = *params;
  c->stream = (hipStream_t)hip_stream;
  c->cap = max_window_records; c->batch_cap = max_batch_records; c->snap_cap = max_snapshot_rows;
  c->kf.mb = mb; c->kf.cb = cb; c->kf.sb = 64 - mb - cb;
  c->dense_capable = dense_capable(params, topo);
  c->last_path = 0;
  c->chain_ready = false;
  c->max_comm_size = max_size;
  c->rank_bits = bits_for_host(topo->n_ranks - 1);
  c->head = 0; c->count = 0; c->next_slot = 0; c->total_ingested = 0;
  // Communicator buckets of the window placement: enough of them that one bucket's payload rows
  // (32 bytes per record) stay within about 100 MB, which the memory-side cache holds while the
  // analysis gathers from that bucket; no more than that, because every further bucket shortens the
  // runs a workgroup writes at ingest (measured at 82M records: 17 buckets 8.46 ms per step, 34
  // buckets 8.60 ms, 9 buckets 8.51 ms, one bucket 9.45 ms).
  {
    int bb = 0;
    while (bb < 6 && ((max_window_records * 32) >> bb) > 100000000ull) ++bb;
    // dense placement partitions every bucket once more: about half a million records per bucket keep the
    // fine buckets of two neighbouring buckets within what a partition workgroup addresses
    if (c->dense_capable) while (bb < 8 && (max_window_records >> bb) > 512 * 1024) ++bb;
    c->bshift = cb > bb ? cb - bb : 0;
  }
  c->n_buckets = ((topo->n_comms - 1) >> c->bshift) + 1;
  c->sorted_buf = 0; c->last_n = 0; c->blame_valid = false; c->sort_passes = 0;
  c->inc_ok = false; c->inc_head = c->inc_count = c->inc_total = 0;
  c->sf.mb = mb; c->sf.ws = 0; c->sf.seq_base = 0;
  uint64_t n_members = 0;
  check_topology(topo, &n_members);
  Carver w{(uint8_t*)workspace, 0};
  carve_all(c, w, topo->n_ranks, topo->n_comms, n_members);
  c->topo.n_ranks = topo->n_ranks; c->topo.n_comms = topo->n_comms;
  c->h_size.assign(topo->size, topo->size + topo->n_comms);
  c->h_pinned = nullptr;
  c->ev_heads = nullptr;
  c->ev_flags = nullptr;

  // derived host tables: sorted member lists, rank -> communicators CSR
  std::vector<uint32_t> sorted(topo->members, topo->members + n_members), sslot(n_members);
  std::vector<uint32_t> rc_off((size_t)topo->n_ranks + 1, 0), rc(n_members), rs_slot(n_members);
  std::vector<int32_t> parent(n_members, -1);
  for (uint32_t k = 0; k < topo->n_comms; ++k) {
    {
      std::vector<uint32_t> ord(topo->size[k]);
      for (uint32_t q = 0; q < topo->size[k]; ++q) ord[q] = q;
      const uint32_t* mem = topo->members + topo->member_off[k];
      std::sort(ord.begin(), ord.end(), [mem](uint32_t a, uint32_t b) { return mem[a] < mem[b]; });
      for (uint32_t q = 0; q < topo->size[k]; ++q) {
        sorted[topo->member_off[k] + q] = mem[ord[q]];
        sslot[topo->member_off[k] + q] = ord[q];
      }
    }
    for (uint32_t q = 0; q < topo->size[k]; ++q) rc_off[topo->members[topo->member_off[k] + q] + 1] += 1;
  }
  for (uint32_t r = 0; r < topo->n_ranks; ++r) rc_off[r + 1] += rc_off[r];
  {
    std::vector<uint32_t> fill(rc_off.begin(), rc_off.end() - 1);
    for (uint32_t k = 0; k < topo->n_comms; ++k)
      for (uint32_t q = 0; q < topo->size[k]; ++q) {
        const uint32_t at = fill[sorted[topo->member_off[k] + q]]++;
        rc[at] = k; rs_slot[at] = q;
      }
  }
  if (topo->tree_parent) parent.assign(topo->tree_parent, topo->tree_parent + n_members);
  std::vector<uint32_t> rc4(4ull * topo->n_ranks, 0xFFFFFFFFu);
  bool fits4 = mb + cb <= 31;       // a padding word then never matches a communicator id
  for (uint32_t r = 0; fits4 && r < topo->n_ranks; ++r) {
    if (rc_off[r + 1] - rc_off[r] > 4) { fits4 = false; break; }
    for (uint32_t q = rc_off[r]; q < rc_off[r + 1]; ++q) rc4[4ull * r + (q - rc_off[r])] = (rc[q] << mb) | rs_slot[q];
  }

  // the same rows with the member index (the row of the snapshot grid) in place of the sorted position: the
  // snapshot placement then needs one lookup per row instead of three
  const int pb = bits_for_host(n_members ? n_members - 1 : 0);
  std::vector<uint32_t> rp4(4ull * topo->n_ranks, 0xFFFFFFFFu);
  const bool fits_cell4 = fits4 && pb + cb <= 31;
  for (uint32_t r = 0; fits_cell4 && r < topo->n_ranks; ++r)
    for (uint32_t q = rc_off[r]; q < rc_off[r + 1]; ++q) {
      const uint32_t k = rc[q], off = topo->member_off[k];
      rp4[4ull * r + (q - rc_off[r])] = (k << pb) | (off + sslot[off + rs_slot[q]]);
    }
  c->topo.pb = pb;

  ccld_status rs = CCLD_OK;
  auto up = [&](const void* dst, const void* src, size_t bytes) {
    if (bytes && hipMemcpyAsync(const_cast<void*>(dst), src, bytes, hipMemcpyHostToDevice, c->stream) != hipSuccess)
      rs = CCLD_E_HIP;
  };
  up(c->topo.algo, topo->algo, topo->n_comms);
  up(c->topo.size, topo->size, 4ull * topo->n_comms);
  up(c->topo.member_off, topo->member_off, 4ull * topo->n_comms);
  up(c->topo.members, topo->members, 4ull * n_members);
  up(c->topo.members_sorted, sorted.data(), 4ull * n_members);
  up(c->topo.sorted_slot, sslot.data(), 4ull * n_members);
  up(c->topo.tree_parent, parent.data(), 4ull * n_members);
  up(c->topo.rank_comm_off, rc_off.data(), 4ull * rc_off.size());
  up(c->topo.rank_comms, rc.data(), 4ull * n_members);
  up(c->topo.rank_slots, rs_slot.data(), 4ull * n_members);
  up(c->topo.rank_memb4, rc4.data(), 4ull * rc4.size());
  if (!fits4) c->topo.rank_memb4 = nullptr;
  std::vector<uint2> cinfo(topo->n_comms);
  for (uint32_t k = 0; k < topo->n_comms; ++k) cinfo[k] = make_uint2(topo->member_off[k], topo->size[k]);
  up(c->comm_info, cinfo.data(), sizeof(uint2) * cinfo.size());
  up(c->topo.rank_cell4, rp4.data(), 4ull * rp4.size());
  if (!fits_cell4) c->topo.rank_cell4 = nullptr;
  if (hipMemsetAsync(c->gstate, 0, sizeof(GroupState) * (uint64_t)topo->n_comms * GROUP_SLOTS, c->stream) != hipSuccess) rs = CCLD_E_HIP;
  if (hipMemsetAsync(c->batch_meta, 0, sizeof(BatchMeta) * ((uint64_t)c->p.window_batches + 2), c->stream) != hipSuccess) rs = CCLD_E_HIP;
  if (hipMemsetAsync(c->counters, 0, sizeof(uint64_t) * CNT_COUNT, c->stream) != hipSuccess) rs = CCLD_E_HIP;
  launch_fill_u64(c->stream, (uint64_t*)c->rate_root, topo->n_comms, (uint64_t)CCLD_NO_RANK);
  if (hipMemsetAsync(c->f_last, 0, sizeof(uint64_t) * 2 * CCLD_FRAME_CHANNELS * n_members, c->stream) != hipSuccess) rs = CCLD_E_HIP;
  if (hipMemsetAsync(c->blame, 0, sizeof(int64_t) * CCLD_BLM_NCOL * (uint64_t)topo->n_ranks, c->stream) != hipSuccess) rs = CCLD_E_HIP;
  {     // pinned readback buffer: the counters, or the headers of every batch slot
    const size_t bytes = std::max<size_t>(4096 * sizeof(uint64_t), sizeof(BatchMeta) * ((size_t)c->p.window_batches + 2));
    if (hipHostMalloc((void**)&c->h_pinned, bytes, hipHostMallocDefault) != hipSuccess) rs = CCLD_E_HIP;
  }
  if (hipEventCreateWithFlags(&c->ev_heads, hipEventDisableTiming) != hipSuccess) { c->ev_heads = nullptr; rs = CCLD_E_HIP; }
  if (hipEventCreateWithFlags(&c->ev_flags, hipEventDisableTiming) != hipSuccess) { c->ev_flags = nullptr; rs = CCLD_E_HIP; }
  if (ccld_static_scratch_init() != CCLD_OK) rs = CCLD_E_HIP;          // address of the static array on this device
  if (hipStreamSynchronize(c->stream) != hipSuccess) rs = CCLD_E_HIP;   // host vectors above die at return
  if (rs != CCLD_OK) {
    (void)hipGetLastError();
    if (c->h_pinned) (void)hipHostFree(c->h_pinned);
    if (c->ev_heads) (void)hipEventDestroy(c->ev_heads);
    if (c->ev_flags) (void)hipEventDestroy(c->ev_flags);
    delete c;
    return rs;
  }
  *out = c;
  return CCLD_OK;
}

ccld_status ccld_destroy(ccld_ctx* c) {
  if (!c) return CCLD_E_NULL;
  (void)hipStreamSynchronize(c->stream);
  if (c->h_pinned) (void)hipHostFree(c->h_pinned);
  if (c->ev_heads) (void)hipEventDestroy(c->ev_heads);
  if (c->ev_flags) (void)hipEventDestroy(c->ev_flags);
  c->prof.destroy();
  delete c;
  return CCLD_OK;
}

ccld_status ccld_reset_window(ccld_ctx* c) {
  if (!c) return CCLD_E_NULL;
  c->head = 0; c->count = 0; c->batch_n.clear(); c->batch_slot.clear(); c->batch_seqno.clear();
  c->inc_ok = false;
  c->chain_ready = false;
  return CCLD_OK;
}

ccld_status ccld_ingest(ccld_ctx* c, const ccld_records* b, uint64_t n) {
  if (!c || !b) return CCLD_E_NULL;
  if (n && (!b->rank || !b->comm || !b->seq || !b->op || !b->bytes || !b->t_enter || !b->t_exit)) return CCLD_E_NULL;
  if (n > c->batch_cap) return CCLD_E_CAPACITY;
  // drop the oldest batch once the window holds window_batches of them
  uint64_t head = c->head, count = c->count;
  size_t drop = 0;
  if (c->batch_n.size() >= c->p.window_batches) {
    drop = c->batch_n.size() - c->p.window_batches + 1;
    for (size_t i = 0; i < drop; ++i) { head = (head + c->batch_n[i]) % std::max<uint64_t>(c->cap, 1); count -= c->batch_n[i]; }
  }
  if (count + n > c->cap) return CCLD_E_CAPACITY;
  c->chain_ready = false;
  IngestArgs a;
  std::memset(&a, 0, sizeof(a));
  const uint32_t slot = c->next_slot;
  a.meta = c->batch_meta + slot;
  if (n == 0) HIP_TRY(hipMemsetAsync(a.meta, 0, sizeof(BatchMeta), c->stream));     // otherwise the counting kernel clears it
  if (b->on_device) {
    a.rank = b->rank; a.comm = b->comm; a.seq = b->seq; a.op = b->op; a.bytes = b->bytes;
    a.t_enter = b->t_enter; a.t_exit = b->t_exit;
  } else if (n) {
    // host batch: copy the seven columns into the staging area, 8-byte columns first
    uint8_t* s = c->stage;
    uint64_t* d_seq = (uint64_t*)s; uint64_t* d_bytes = d_seq + n; int64_t* d_te = (int64_t*)(d_bytes + n);
    int64_t* d_tx = d_te + n; uint32_t* d_rank = (uint32_t*)(d_tx + n); uint32_t* d_comm = d_rank + n;
    uint8_t* d_op = (uint8_t*)(d_comm + n);
    HIP_TRY(hipMemcpyAsync(d_seq, b->seq, 8 * n, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(d_bytes, b->bytes, 8 * n, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(d_te, b->t_enter, 8 * n, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(d_tx, b->t_exit, 8 * n, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(d_rank, b->rank, 4 * n, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(d_comm, b->comm, 4 * n, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(d_op, b->op, n, hipMemcpyHostToDevice, c->stream));
    a.rank = d_rank; a.comm = d_comm; a.seq = d_seq; a.op = d_op; a.bytes = d_bytes; a.t_enter = d_te; a.t_exit = d_tx;
  }
  a.n = n; a.win_key = c->win_key; a.win_row = c->win_row;
  a.tail = (uint32_t)((head + count) % std::max<uint64_t>(c->cap, 1));
  a.cap = (uint32_t)c->cap;
  a.table = c->ing_table; a.bucket_base = c->ing_base; a.scratch_total = &c->counters[CNT_COUNT - 1];
  a.n_buckets = c->n_buckets; a.bshift = c->bshift; a.seqno0 = (uint32_t)c->total_ingested;
  if (c->dense_capable && n) {
    a.range = c->comm_range;
    HIP_TRY(hipMemsetAsync(a.range, 0, 16ull * c->topo.n_comms, c->stream));
  }
  c->prof.begin(CCLD_PROF_INGEST);
  launch_ingest(c->stream, a, c->topo, c->kf);
  c->prof.end(CCLD_PROF_INGEST);
  HIP_TRY(hipGetLastError());
  if (!b->on_device && n) HIP_TRY(hipStreamSynchronize(c->stream));   // the host buffers may go away on return
  c->batch_n.erase(c->batch_n.begin(), c->batch_n.begin() + drop);
  c->batch_slot.erase(c->batch_slot.begin(), c->batch_slot.begin() + drop);
  c->batch_seqno.erase(c->batch_seqno.begin(), c->batch_seqno.begin() + drop);
  c->batch_n.push_back(n);
  c->batch_slot.push_back(slot);
  c->batch_seqno.push_back((uint32_t)c->total_ingested);
  c->total_ingested += n;
  c->next_slot = (slot + 1) % (c->p.window_batches + 2);
  c->head = head; c->count = count + n;
  return CCLD_OK;
}

static void zero_counts(ccld_window_result* o) {
  o->n_records = o->n_seg = o->n_flag = o->n_group = o->n_alert = o->n_cand = 0;
}

// One analysis of the resident window.  dense: bring the collectives together by dense placement instead of
// sorting; *fallback is set (and nothing of the context's detection state has changed) when the window turns
// out not to fill a dense grid, and the caller then sorts.
static ccld_status analyze_window_once(ccld_ctx* c, int64_t now_ns, ccld_window_result* o, bool dense, bool* fallback) {
  zero_counts(o);
  o->status = CCLD_OK;
  o->path = dense ? 1 : 0;
  *fallback = false;
  c->chain_ready = false;
  c->blame_valid = false;
  if (!o->seg || o->seg_cap == 0) return o->status = CCLD_E_NULL;
  if ((o->flag_cap && !o->flag) || (o->group_cap && !o->group) || (o->alert_cap && !o->alert) ||
      (o->cand_cap && !o->cand))
    return o->status = CCLD_E_NULL;
  hipStream_t st = c->stream;
  const uint32_t n = (uint32_t)c->count;
  const uint32_t n_ranks = c->topo.n_ranks;

  // 1. data errors found at ingest, and the widest sequence number in the window
  const size_t nb = c->batch_slot.size();
  uint64_t bits = 0, max_seq = 0, min_seq = ~0ull;
  if (nb) {
    const uint32_t n_meta = c->p.window_batches + 2;
    HIP_TRY(hipMemcpyAsync(c->h_pinned, c->batch_meta, sizeof(BatchMeta) * n_meta, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    const BatchMeta* hm = (const BatchMeta*)c->h_pinned;
    for (size_t i = 0; i < nb; ++i) {
      const BatchMeta& m = hm[c->batch_slot[i]];
      bits |= m.status; max_seq = std::max(max_seq, m.max_seq); min_seq = std::min(min_seq, ~m.max_inv_seq);
    }
  }
  if (bits) { c->inc_ok = false; return o->status = data_status(bits); }     // the kept order does not survive a bad batch
  o->n_records = n;
  {
    const size_t blame_bytes = sizeof(int64_t) * CCLD_BLM_NCOL * (uint64_t)n_ranks;
    uint8_t* c0 = reinterpret_cast<uint8_t*>(c->counters);
    uint8_t* b0 = reinterpret_cast<uint8_t*>(c->blame);
    if (b0 >= c0 && (size_t)(b0 - c0) < 4096) {        // adjacent in the workspace: one fill
      HIP_TRY(hipMemsetAsync(c0, 0, (size_t)(b0 - c0) + blame_bytes, st));
    } else {
      HIP_TRY(hipMemsetAsync(c->counters, 0, sizeof(uint64_t) * CNT_COUNT, st));
      HIP_TRY(hipMemsetAsync(c->blame, 0, blame_bytes, st));
    }
  }
  c->last_n = n;
  if (n == 0) {
    launch_blame_order(st, c->blame, n_ranks, c->blame_list, c->blame_tiles, c->counters, c->blame_order);
    HIP_TRY(hipStreamSynchronize(st));
    c->blame_valid = true;
    return o->status;
  }

  // 2. sort by (communicator, operation counter, rank) on the significant bits only
  // the operation counters of the window relative to its smallest one
  if (min_seq > max_seq) min_seq = max_seq;
  const int mb = c->kf.mb, cb = c->kf.cb, ws = bits_for_host(max_seq - min_seq);
  c->sf.mb = mb; c->sf.ws = ws; c->sf.seq_base = min_seq;
  KeySource src;
  src.key = c->win_key; src.head = (uint32_t)c->head; src.cap = (uint32_t)c->cap;
  src.squeeze = 1;
  src.hi_shift = 64 - cb;                                  // 64 when there is a single communicator
  src.lo_bits = mb + ws;
  src.lo_mask = cb > 0 ? (((uint64_t)1 << (64 - cb)) - 1) : ~0ull;      // everything below the communicator field
  src.lo_sub = min_seq << mb;
  // A window of several batches that still holds at least half of the previously analysed window keeps that
  // window's order: the new records are sorted on their own and merged with the previous order, whose keys are
  // re-based to this window's format and whose entries of the batches that left are dropped on the way.
  const bool was_ok = c->inc_ok && !dense;
  c->inc_ok = false;
  const uint64_t cap = std::max<uint64_t>(c->cap, 1);
  const uint64_t n_new = c->total_ingested - c->inc_total;
  int sorted = -1;
  if (was_ok && n_new > 0 && n_new < n && c->inc_sf.mb == mb && mb + ws + cb <= 64 && mb + ws < 64 &&
      c->inc_sf.mb + c->inc_sf.ws < 64) {
    const uint64_t kept = n - n_new;                                     // records of the previous window still here
    if (kept >= n_new && kept <= c->inc_count) {
      const uint64_t exp_n = c->inc_count - kept;
      const uint64_t old_tail = (c->inc_head + c->inc_count) % cap;
      if ((c->inc_head + exp_n) % cap == c->head && (old_tail + n_new) % cap == (c->head + n) % cap) {
        // the new records end in the third buffer pair (a sort of p passes ends in its buffer (p - 1) % 2), so
        // that the merge can read the previous order where it lies and write beside it
        const int s = c->sorted_buf;
        const int passes = (mb + ws + cb) <= 0 ? 1 : (mb + ws + cb + SORT_RBITS - 1) / SORT_RBITS;
        const int third = (passes - 1) % 2;
        SortBuffers sbn;
        sbn.key[third] = c->keyC; sbn.idx[third] = c->idxC;
        sbn.key[1 - third] = c->sb.key[1 - s]; sbn.idx[1 - third] = c->sb.idx[1 - s];
        sbn.table = c->table2; sbn.totals = c->totals2;
        KeySource fresh = src;
        fresh.head = (uint32_t)old_tail;
        const int rb = radix_sort_pairs(st, fresh, (uint32_t)n_new, sbn, mb + ws + cb, &c->prof, CCLD_PROF_SORT_HIST,
                                        CCLD_PROF_SORT_SCAN, CCLD_PROF_SORT_SCATTER);
        if (rb < 0) return o->status = CCLD_E_HIP;
        if (rb != third) {
          HIP_TRY(hipMemcpyAsync(c->keyC, sbn.key[rb], sizeof(uint64_t) * n_new, hipMemcpyDeviceToDevice, st));
          HIP_TRY(hipMemcpyAsync(c->idxC, sbn.idx[rb], sizeof(uint32_t) * n_new, hipMemcpyDeviceToDevice, st));
        }
        c->prof.begin(CCLD_PROF_SORT_SCATTER);
        RetainArgs ra;
        ra.key = c->sb.key[s]; ra.idx = c->sb.idx[s]; ra.n = (uint32_t)c->inc_count; ra.from = c->inc_sf; ra.to = c->sf;
        ra.exp_lo = (uint32_t)c->inc_head; ra.exp_n = (uint32_t)exp_n; ra.cap = (uint32_t)cap;
        ra.tile_counts = c->tile_flags; ra.total_out = &c->counters[CNT_NRETAINED];
        ra.key_out = c->sb.key[1 - s]; ra.idx_out = c->sb.idx[1 - s];
        launch_merge_kept(st, ra, c->keyC, c->idxC, (uint32_t)n_new, c->tile_heads);
        c->prof.end(CCLD_PROF_SORT_SCATTER);
        sorted = 1 - s;
      }
    }
  }
  DenseArgs da;
  std::memset(&da, 0, sizeof(da));
  uint32_t dense_n_seg = 0, dense_n_fine = 0;
  if (dense) {
    // the grid's layout from the batch's counter ranges; its size comes back while the partition runs
    da.win_key = c->win_key; da.win_row = c->win_row; da.head = (uint32_t)c->head; da.cap = (uint32_t)cap; da.n = n;
    da.kf = c->kf; da.comm_size = c->topo.size; da.n_comms = c->topo.n_comms;
    da.bucket_base = c->ing_base; da.n_buckets = c->n_buckets; da.bshift = c->bshift;
    da.range = c->comm_range; da.lay = (CommLayout*)c->d_lay; da.hdr = c->d_hdr; da.fill = c->d_fill;
    da.rows = c->d_rows; da.fine_cap = c->fine_cap; da.counters = c->counters;
    da.desc = (FineDesc*)c->d_desc; da.seq_base = c->sf.seq_base;
    c->prof.begin(CCLD_PROF_DENSE_PARTITION);
    launch_dense_layout(st, da);
    uint32_t* h_hdr = reinterpret_cast<uint32_t*>(c->h_pinned + 2 * CNT_COUNT);
    HIP_TRY(hipMemcpyAsync(h_hdr, c->d_hdr, sizeof(uint32_t) * DH_COUNT, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipEventRecord(c->ev_heads, st));
    launch_fill_u64(st, reinterpret_cast<uint64_t*>(c->d_fill), ((uint64_t)c->fine_cap + 4) / 2, 0ull);
    launch_dense_partition(st, da);
    launch_scan_tiles(st, c->d_fill, c->fine_cap + 1, &c->counters[CNT_NRETAINED]);
    launch_dense_desc(st, da);
    HIP_TRY(hipEventSynchronize(c->ev_heads));
    if (!h_hdr[DH_FEASIBLE]) {          // far-apart counters or too many fine buckets: the kernels above did nothing
      HIP_TRY(hipStreamSynchronize(st));
      c->prof.end(CCLD_PROF_DENSE_PARTITION);
      c->prof.collect();
      *fallback = true;
      return CCLD_OK;
    }
    dense_n_seg = h_hdr[DH_N_SEG];
    dense_n_fine = h_hdr[DH_N_FINE];
    sorted = 0;
    c->sort_passes = 0;
  } else {
  if (sorted < 0)
    sorted = radix_sort_pairs(st, src, n, c->sb, mb + ws + cb, &c->prof, CCLD_PROF_SORT_HIST,
                              CCLD_PROF_SORT_SCAN, CCLD_PROF_SORT_SCATTER);
  c->sort_passes = (mb + ws + cb) <= 0 ? 1 : (mb + ws + cb + SORT_RBITS - 1) / SORT_RBITS;
  if (sorted < 0) return o->status = CCLD_E_HIP;
  }
  c->sorted_buf = sorted;
  const uint64_t* skey = c->sb.key[sorted];
  const uint32_t* sidx = c->sb.idx[sorted];
  const Row* rows = dense ? c->d_rows : c->win_row;     // payload rows that sidx addresses

  // 3. collectives: heads per tile, their scan, statistics, flags
  SegArgs sa;
  std::memset(&sa, 0, sizeof(sa));
  sa.key = skey; sa.idx = sidx; sa.row = rows; sa.n = n; sa.sf = c->sf; sa.comm_size = c->topo.size;
  sa.member_off = c->topo.member_off; sa.members_sorted = c->topo.members_sorted; sa.comm_info = c->comm_info;
  sa.tile_heads = c->tile_heads; sa.seg = o->seg; sa.seg_cap = o->seg_cap;
  sa.rec_flag = o->rec_flag ? o->rec_flag : c->rec_flag;
  sa.lag_e = o->lag_enter; sa.lag_x = o->lag_exit; sa.flag_lag = c->flag_lag; sa.cap_n = c->cap;
  sa.big_list = c->big_list; sa.big_cap = c->cap / 65 + 2; sa.big_ex = c->big_ex; sa.counters = c->counters;
  sa.lag_floor = c->p.lag_floor_ns; sa.kmad_num = c->p.kmad_num; sa.kmad_den = c->p.kmad_den;
  sa.barrier_bytes = c->p.barrier_bytes; sa.max_size = c->max_comm_size;
  sa.gkey = c->keyC; sa.range_c = c->range_c;
  sa.no_group = (uint64_t)c->topo.n_comms * CCLD_OP_MAX * GROUP_CLS;     // one past every group key
  const uint32_t seg_tiles = (n + SEG_TILE - 1) / SEG_TILE;
  if (dense) {
    // every collective's row of the table is fixed by the layout; a duplicate key or a round without any
    // record shows in the status word at the end (the group stage leaves the detection state alone then)
    c->prof.split(CCLD_PROF_DENSE_PARTITION, CCLD_PROF_SEGMENTS);
    launch_dense_stats(st, sa, da, dense_n_fine, c->sb.key[sorted], c->sb.idx[sorted], c->blame, n_ranks);
    c->prof.split(CCLD_PROF_SEGMENTS, CCLD_PROF_FLAGS);
    o->n_seg = dense_n_seg;
  } else {
  c->prof.begin(CCLD_PROF_SEG_HEADS);
  launch_keys_pass(st, skey, n, c->sf, c->topo, c->blame, c->tile_heads, c->counters);
  launch_scan_tiles(st, c->tile_heads, seg_tiles, &c->counters[CNT_NSEG]);
  // the number of collectives is known here; it comes back while the statistics kernels run
  HIP_TRY(hipMemcpyAsync(c->h_pinned, c->counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipEventRecord(c->ev_heads, st));
  c->prof.split(CCLD_PROF_SEG_HEADS, CCLD_PROF_SEGMENTS);          // one event ends a timed span and begins the next
  launch_seg_analyze(st, sa);
  c->prof.split(CCLD_PROF_SEGMENTS, CCLD_PROF_FLAGS);
  HIP_TRY(hipEventSynchronize(c->ev_heads));
  if (c->h_pinned[CNT_STATUS]) {
    const uint64_t bad = c->h_pinned[CNT_STATUS];
    HIP_TRY(hipStreamSynchronize(st));
    c->prof.collect();
    zero_counts(o);
    return o->status = data_status(bad);
  }
  o->n_seg = c->h_pinned[CNT_NSEG];
  }
  const uint32_t seg_rows = (uint32_t)std::min<uint64_t>(o->n_seg, o->seg_cap);
  FlagArgs fa;
  std::memset(&fa, 0, sizeof(fa));
  fa.key = skey; fa.rec_flag = sa.rec_flag; fa.flag_lag = c->flag_lag; fa.cap_n = c->cap; fa.n = n; fa.sf = c->sf;
  fa.member_off = c->topo.member_off; fa.members_sorted = c->topo.members_sorted;
  fa.tile_flags = c->tile_flags; fa.flag_pos = c->flag_pos; fa.flag = o->flag; fa.flag_cap = o->flag_cap;
  fa.counters = c->counters;
  launch_flag_compact(st, fa);
  // the number of flags comes back while the alert and group kernels run
  uint64_t* h_flags = c->h_pinned + CNT_COUNT;
  HIP_TRY(hipMemcpyAsync(h_flags, c->counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipEventRecord(c->ev_flags, st));
  if (o->perm) launch_perm(st, sidx, rows, n, c->batch_seqno.empty() ? 0u : c->batch_seqno[0], o->perm);

  // 4. hang alerts: which collectives
  AlertArgs aa;
  std::memset(&aa, 0, sizeof(aa));
  aa.seg = o->seg; aa.seg_cap = o->seg_cap; aa.n_seg = seg_rows; aa.now_ns = now_ns;
  aa.hang_threshold_ns = c->p.hang_threshold_ns; aa.key = skey; aa.idx = sidx; aa.row = rows; aa.n = n;
  aa.sf = c->sf; aa.topo = c->topo; aa.tile_counts = c->tile_heads; aa.alert_list = c->alert_list;
  aa.alert_ncand = c->alert_ncand; aa.alert = o->alert; aa.alert_cap = o->alert_cap; aa.cand = o->cand;
  aa.cand_cap = o->cand_cap; aa.counters = c->counters;
  c->prof.split(CCLD_PROF_FLAGS, CCLD_PROF_ALERTS);
  launch_alert_select(st, aa);
  c->prof.split(CCLD_PROF_ALERTS, CCLD_PROF_GROUPS);

  // 5. slow detection and location per detection group (Eq. 1-4): every collective of the table is keyed
  //    (those that take no part sort behind the groups), and the evaluation reads the numbers of groups and of
  //    usable collectives on the device, so nothing here waits for the host
  SortBuffers sb2;
  sb2.key[0] = c->sb.key[1 - sorted]; sb2.idx[0] = c->sb.idx[1 - sorted];
  sb2.key[1] = c->keyC; sb2.idx[1] = c->idxC; sb2.table = c->table2; sb2.totals = c->totals2;
  GroupArgs ga;
  std::memset(&ga, 0, sizeof(ga));
  ga.seg = o->seg; ga.seg_cap = o->seg_cap; ga.n_seg = seg_rows; ga.ws = ws; ga.cb = cb;
  ga.tile_counts = c->tile_flags; ga.counters = c->counters;
  ga.gstate = c->gstate; ga.rate_root = c->rate_root; ga.group = o->group; ga.group_cap = o->group_cap; ga.p = c->p;
  ga.range_c = c->range_c;
  if (seg_rows) {
    const uint64_t no_group = sa.no_group;
    KeySource gs; gs.key = c->keyC; gs.head = 0; gs.cap = seg_rows; gs.squeeze = 0; gs.hi_shift = 0; gs.lo_bits = 0; gs.lo_mask = 0; gs.lo_sub = 0;
    // sort C -> buffers {other main, C}: the first pass reads C and writes buffer 0, so C is free again for pass 2
    const int r3 = radix_sort_pairs(st, gs, seg_rows, sb2, bits_for_host(no_group));
    if (r3 < 0) return o->status = CCLD_E_HIP;
    launch_group_heads(st, sb2.key[r3], seg_rows, no_group, c->tile_flags, c->group_first, c->counters);
    launch_group_eval(st, ga, sb2.key[r3], sb2.idx[r3], c->group_first, c->group_long);
  }
  c->prof.end(CCLD_PROF_GROUPS);
  HIP_TRY(hipGetLastError());
  // 6. blame: flags keyed by rank, sorted, one workgroup per rank sums its run; launched behind the group
  //    kernels, before the host waits for them
  HIP_TRY(hipEventSynchronize(c->ev_flags));
  const uint32_t n_flag = (uint32_t)h_flags[CNT_NFLAG];
  if (n_flag) {
    uint64_t* bk = c->keyC;       // keys are written to C, first pass sorts C -> buffer 0 of sb2
    c->prof.begin(CCLD_PROF_BLAME);
    launch_blame_keys(st, skey, c->flag_pos, n_flag, c->sf, c->topo, bk);
    KeySource bs; bs.key = bk; bs.head = 0; bs.cap = n_flag; bs.squeeze = 0; bs.hi_shift = 0; bs.lo_bits = 0; bs.lo_mask = 0; bs.lo_sub = 0;
    const int r2 = radix_sort_pairs(st, bs, n_flag, sb2, c->rank_bits);
    if (r2 < 0) return o->status = CCLD_E_HIP;
    launch_blame_reduce(st, sb2.key[r2], sb2.idx[r2], n_flag, c->flag_pos, sa.rec_flag, c->flag_lag, c->cap, n_ranks,
                        c->blame_list, c->blame);
    c->prof.end(CCLD_PROF_BLAME);
  }
  // the blame order is ready when ccld_rank_blame asks for it: its kernels are queued here, before the wait
  launch_blame_order(st, c->blame, n_ranks, c->blame_list, c->blame_tiles, c->counters, c->blame_order);
  HIP_TRY(hipMemcpyAsync(c->h_pinned, c->counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (c->h_pinned[CNT_STATUS]) {
    const uint64_t bad = c->h_pinned[CNT_STATUS];
    c->prof.collect();
    zero_counts(o);
    if (dense && (bad & DS_DENSE_FALLBACK)) { *fallback = true; return CCLD_OK; }
    return o->status = data_status(bad);
  }
  o->n_flag = c->h_pinned[CNT_NFLAG];
  o->n_alert = c->h_pinned[CNT_NALERT];
  o->n_group = c->h_pinned[CNT_NGROUP];
  if (o->n_seg > o->seg_cap || o->n_flag > o->flag_cap || o->n_group > o->group_cap) o->status = CCLD_W_TRUNCATED;

  // 7. hang alerts: candidates of every alert
  if (o->n_alert) {
    c->prof.begin(CCLD_PROF_ALERTS);
    launch_alert_candidates(st, aa, (uint32_t)o->n_alert);
    c->prof.end(CCLD_PROF_ALERTS);
    HIP_TRY(hipMemcpyAsync(c->h_pinned, c->counters, sizeof(uint64_t) * CNT_COUNT, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    o->n_cand = c->h_pinned[CNT_NCAND];
    if (o->n_alert > o->alert_cap || o->n_cand > o->cand_cap) o->status = CCLD_W_TRUNCATED;
  }
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(st));
  c->prof.collect();
  c->blame_valid = true;
  // the order of this window serves the next analysis (windows of several batches only)
  c->inc_ok = c->p.window_batches > 1 && !dense;
  c->last_path = dense ? 1 : 0;
  c->chain_ready = true;
  c->last_seg = o->seg; c->last_seg_cap = o->seg_cap; c->last_n_seg = o->n_seg; c->last_n_flag = o->n_flag;
  c->last_rec_flag = sa.rec_flag; c->last_rows = rows;
  c->inc_sf = c->sf; c->inc_head = c->head; c->inc_count = n; c->inc_total = c->total_ingested;
  return o->status;
}

ccld_status ccld_analyze_window(ccld_ctx* c, int64_t now_ns, ccld_window_result* o) {
  if (!c || !o) return CCLD_E_NULL;
  bool fallback = false;
  ccld_status s = CCLD_OK;
  // a window of one batch is first tried by dense placement; one that does not fill a dense grid is sorted
  if (c->dense_capable && c->batch_n.size() == 1 && c->count > 0) s = analyze_window_once(c, now_ns, o, true, &fallback);
  else fallback = true;
  if (fallback) s = analyze_window_once(c, now_ns, o, false, &fallback);
  if (s < 0) {       // an error return may have left work queued and timed spans open
    (void)hipStreamSynchronize(c->stream);
    (void)hipGetLastError();
    c->prof.abandon();
    c->inc_ok = false;
  }
  return s;
}

ccld_status ccld_rank_blame(ccld_ctx* c, int64_t* blame, uint32_t* order) {
  if (!c) return CCLD_E_NULL;
  if (!c->blame_valid) return CCLD_E_BAD_ARG;
  const uint32_t n_ranks = c->topo.n_ranks;
  launch_blame_out(c->stream, c->blame, c->blame_order, n_ranks, blame, order);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(c->stream));
  return CCLD_OK;
}

ccld_status ccld_profile_enable(ccld_ctx* c, int32_t on) {
  if (!c) return CCLD_E_NULL;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (on < 0 || on >= 2 + CCLD_PROF_NCLASS) return CCLD_E_BAD_ARG;
  return c->prof.enable(c->stream, on != 0, on >= 2 ? on - 2 : -1) ? CCLD_OK : CCLD_E_HIP;
}

ccld_status ccld_profile_read(ccld_ctx* c, double* ms, uint64_t* launches, uint64_t* sort_passes) {
  if (!c) return CCLD_E_NULL;
  HIP_TRY(hipStreamSynchronize(c->stream));
  c->prof.collect();
  for (int i = 0; i < CCLD_PROF_NCLASS; ++i) {
    if (ms) ms[i] = c->prof.ms[i];
    if (launches) launches[i] = c->prof.cnt[i];
  }
  if (sort_passes) *sort_passes = (uint64_t)c->sort_passes;
  return CCLD_OK;
}

const char* ccld_status_str(ccld_status s) {
  switch (s) {
    case CCLD_OK: return "OK";
    case CCLD_E_UNKNOWN_COMM: return "E_UNKNOWN_COMM";
    case CCLD_E_RANK_NOT_MEMBER: return "E_RANK_NOT_MEMBER";
    case CCLD_E_RANGE: return "E_RANGE";
    case CCLD_E_DUPLICATE_KEY: return "E_DUPLICATE_KEY";
    case CCLD_E_SNAPSHOT_GAP: return "E_SNAPSHOT_GAP";
    case CCLD_E_BAD_ARG: return "E_BAD_ARG";
    case CCLD_E_NULL: return "E_NULL";
    case CCLD_E_CAPACITY: return "E_CAPACITY";
    case CCLD_E_KEY_WIDTH: return "E_KEY_WIDTH";
    case CCLD_E_BAD_TOPOLOGY: return "E_BAD_TOPOLOGY";
    case CCLD_E_HIP: return "E_HIP";
    case CCLD_E_WORKSPACE: return "E_WORKSPACE";
    case CCLD_W_TRUNCATED: return "W_TRUNCATED";
    default: return "E_UNKNOWN";
  }
}

}  // extern "C"
