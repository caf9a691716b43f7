// Host-callable launchers of the window-analysis kernels (defined in window.hip).
#pragma once
#include "ccld_internal.h"

namespace ccld {

struct IngestArgs {
  const uint32_t *rank, *comm;
  const uint64_t* seq;
  const uint8_t* op;
  const uint64_t* bytes;
  const int64_t *t_enter, *t_exit;
  uint64_t n;
  uint64_t* win_key;
  Row* win_row;
  uint32_t tail, cap;
  BatchMeta* meta;
  uint32_t* table;           // [n_buckets][workgroups] records per communicator bucket and workgroup
  uint32_t* bucket_base;     // [n_buckets + 1]
  uint64_t* scratch_total;
  uint32_t n_buckets;
  int bshift;                // bucket = comm >> bshift
  uint32_t seqno0;           // arrival number of the batch's first record
  uint64_t* range;           // [n_comms][2] per communicator: largest operation counter, largest complement of one
                             // (zeroed by the caller); null: not wanted.  At most INGEST_RANGE_COMMS communicators.
  uint64_t chunk;            // records per placement workgroup (a multiple of 256 * hist_split)
  uint32_t hist_split;       // counting workgroups per placement workgroup
};
constexpr uint32_t INGEST_BLOCKS = 1024;
constexpr uint32_t INGEST_MAX_BUCKETS = 4096;
constexpr uint32_t INGEST_STAGED_BUCKETS = 256;   // most buckets the LDS-regrouped placement kernel handles
constexpr uint32_t INGEST_RANGE_COMMS = 3584;     // most communicators whose counter ranges fit the counting kernel's LDS
void launch_ingest(hipStream_t st, const IngestArgs& a, const DeviceTopology& T, const KeyFormat& kf);
void launch_fill_u64(hipStream_t st, uint64_t* p, uint64_t n, uint64_t v);

struct SegArgs {
  const uint64_t* key;       // sorted squeezed keys
  const uint32_t* idx;       // window slot of each sorted record
  const Row* row;
  uint32_t n;
  SqueezedFormat sf;
  const uint32_t* comm_size;
  const uint32_t *member_off, *members_sorted;   // key slot -> rank
  const uint2* comm_info;    // [n_comms] (member_off, comm_size) side by side
  uint32_t* tile_heads;      // [tiles + 1] head counts, then (after the scan) first segment ordinal of each tile
  int64_t* seg;
  uint64_t seg_cap;
  uint8_t* rec_flag;
  int64_t *lag_e, *lag_x;    // optional per-record outputs
  int64_t* flag_lag;         // [2][cap_n] lags of flagged records by sorted position
  uint64_t cap_n;
  uint32_t* big_list;
  uint64_t big_cap;          // entries the list holds
  int64_t* big_ex;           // [2][cap_n]
  uint64_t* counters;
  int64_t lag_floor;
  uint32_t kmad_num, kmad_den, barrier_bytes;
  uint32_t max_size;         // members of the largest communicator (host-side: which size classes can occur)
  // detection-group key (communicator, op, size class) and T_max - T_min of every collective, for the
  // group stage; a collective that takes no part gets no_group, one value past every real key
  uint64_t* gkey;
  int64_t* range_c;
  uint64_t no_group;
};
void launch_scan_tiles(hipStream_t st, uint32_t* counts, uint32_t n_tiles, uint64_t* total_out);
void launch_seg_analyze(hipStream_t st, const SegArgs& a);        // small collectives, then the oversized ones

struct FlagArgs {
  const uint64_t* key;
  const uint8_t* rec_flag;
  const int64_t* flag_lag;
  uint64_t cap_n;
  uint32_t n;
  SqueezedFormat sf;
  const uint32_t *member_off, *members_sorted;
  uint32_t* tile_flags;      // [tiles + 1]
  uint32_t* flag_pos;
  int64_t* flag;             // caller's table (may be NULL)
  uint64_t flag_cap;
  uint64_t* counters;
};
void launch_flag_compact(hipStream_t st, const FlagArgs& a);

// one pass over the sorted keys: collective heads per tile (tile_heads), duplicates (status counter),
// records per rank (added into the zeroed records column of blame)
void launch_keys_pass(hipStream_t st, const uint64_t* key, uint32_t n, const SqueezedFormat& sf,
                      const DeviceTopology& T, int64_t* blame, uint32_t* tile_heads, uint64_t* counters);
void launch_blame_keys(hipStream_t st, const uint64_t* key, const uint32_t* flag_pos, uint32_t n_flag,
                       const SqueezedFormat& sf, const DeviceTopology& T, uint64_t* out_key);
void launch_blame_reduce(hipStream_t st, const uint64_t* skey, const uint32_t* sidx, uint32_t n_flag,
                         const uint32_t* flag_pos, const uint8_t* rec_flag, const int64_t* flag_lag,
                         uint64_t cap_n, uint32_t n_ranks, uint32_t* run /* [2 n_ranks] scratch */, int64_t* blame);
void launch_blame_order(hipStream_t st, const int64_t* blame, uint32_t n_ranks, uint32_t* lists,
                        uint32_t* tile_counts, uint64_t* counters, uint32_t* order);

struct GroupArgs {
  const int64_t* seg;
  uint64_t seg_cap;
  uint32_t n_seg;            // rows present in the table
  int ws, cb;
  uint32_t* tile_counts;
  uint64_t* counters;
  const int64_t* range_c;    // [n_seg] T_max - T_min of each usable collective (written with the collectives' statistics)
  GroupState* gstate;
  const int64_t* rate_root;  // [n_comms] minimal-rate member per communicator (CCLD_NO_RANK before any rate pass)
  int64_t* group;
  uint64_t group_cap;
  ccld_params p;
};
void launch_blame_out(hipStream_t st, const int64_t* blame, const uint32_t* order_in, uint32_t n_ranks, int64_t* table_out,
                      uint32_t* order_out);
void launch_group_heads(hipStream_t st, const uint64_t* skey, uint32_t n_rows, uint64_t no_group, uint32_t* tile_counts,
                        uint32_t* group_first, uint64_t* counters);
void launch_group_eval(hipStream_t st, const GroupArgs& a, const uint64_t* skey, const uint32_t* sidx,
                       const uint32_t* group_first, uint32_t* long_list);

struct AlertArgs {
  const int64_t* seg;
  uint64_t seg_cap;
  uint32_t n_seg;
  int64_t now_ns, hang_threshold_ns;
  const uint64_t* key;
  const uint32_t* idx;
  const Row* row;
  uint32_t n;
  SqueezedFormat sf;
  DeviceTopology topo;
  uint32_t* tile_counts;
  uint32_t* alert_list;
  uint32_t* alert_ncand;
  int64_t* alert;
  uint64_t alert_cap;
  int64_t* cand;
  uint64_t cand_cap;
  uint64_t* counters;
};
void launch_alert_select(hipStream_t st, const AlertArgs& a);
void launch_alert_candidates(hipStream_t st, const AlertArgs& a, uint32_t n_alert);

void launch_perm(hipStream_t st, const uint32_t* idx, const Row* row, uint32_t n, uint32_t seqno_head, uint32_t* perm);

}  // namespace ccld
