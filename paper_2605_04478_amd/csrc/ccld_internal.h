// Context layout and kernel-launcher declarations shared by the translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

#include "ccld.h"
#include "radix_sort.h"
#include "profiler.h"

namespace ccld {

// One stored record: the payload the analysis gathers by sorted position (32 bytes, one
// aligned access); communicator, sequence number and member slot live in the key.
struct __attribute__((aligned(32))) Row {
  int64_t t_enter, t_exit;
  uint64_t bytes;
  uint32_t op, pad;
};

// Key layout at ingest: comm << (64 - cb) | seq << mb | slot.  slot is the record's rank counted
// among its communicator's members in ascending rank order, so keys order like (comm, seq, rank)
// while the field needs only as many bits as the largest communicator has members; mb / cb are
// the bit widths of the largest slot / communicator id.  The sort squeezes the unused middle bits out.
struct KeyFormat {
  int mb, cb;          // member-slot bits, communicator bits
  int sb;              // bits available to the sequence number: 64 - mb - cb
};

// Squeezed key used from the sort onwards: comm << (mb + ws) | (seq - seq_base) << mb | slot, with
// seq_base the window's smallest operation counter: a long-running job's large counters do not
// widen the key.
struct SqueezedFormat {
  int mb, ws;          // member-slot bits, bits of (largest - smallest operation counter) in this window
  uint64_t seq_base;   // the window's smallest operation counter
};

struct DeviceTopology {
  uint32_t n_ranks, n_comms;
  const uint8_t* algo;
  const uint32_t* size;
  const uint32_t* member_off;
  const uint32_t* members;
  const uint32_t* members_sorted;   // each communicator's members in ascending rank order
  const uint32_t* sorted_slot;      // slot (position in members[]) of each entry of members_sorted
  const int32_t* tree_parent;
  const uint32_t* rank_comm_off;    // [n_ranks + 1] CSR: communicators each rank belongs to
  const uint32_t* rank_comms;
  const uint32_t* rank_slots;       // parallel to rank_comms: the rank's position in members_sorted of that communicator
  const uint32_t* rank_memb4;       // [n_ranks][4] words comm << mb | position (padded with 0xFFFFFFFF); null if a rank is in more than four communicators or cb + mb > 31
  const uint32_t* rank_cell4;       // [n_ranks][4] words comm << pb | member index (member_off[comm] + slot in members[]), padded alike; null if a rank is in more than four communicators or cb + pb > 31
  int pb;                           // bits of the largest member index
};

// rank of the record whose key carries (comm, slot)
__device__ __forceinline__ uint32_t rank_of_slot(const uint32_t* __restrict__ member_off,
                                                 const uint32_t* __restrict__ members_sorted, uint32_t comm,
                                                 uint32_t slot) {
  return members_sorted[member_off[comm] + slot];
}

// Eq. 1 state and repetition counter of one detection group (communicator, op, size class).
struct GroupState {
  uint32_t cnt, frozen, repeats, pad;
  int64_t sum, t0, tbase_dyn;
  uint64_t baselined_wm, baseline_last_seq, detected_wm;
};
constexpr int GROUP_CLS = 64;
constexpr int GROUP_SLOTS = CCLD_OP_MAX * GROUP_CLS;

// status bits accumulated on the device
enum { DS_UNKNOWN_COMM = 1, DS_NOT_MEMBER = 2, DS_RANGE = 4, DS_KEY_WIDTH = 8, DS_DUPLICATE = 16,
       DS_SNAPSHOT_GAP = 32,
       DS_SUSPECT = 64,     // snapshot grid placed without the presence bitmap: a cell still holds the fill pattern
       DS_DENSE_FALLBACK = 128 };   // the window does not fill a dense grid (far-apart counters, a round without any record): sort instead

struct BatchSlot { uint64_t n; };

// device-side header of per-batch results: status bits, largest operation counter, and the largest
// complement of one (i.e. ~smallest counter), so that a zeroed header means "no record yet"
struct BatchMeta { uint64_t status; uint64_t max_seq; uint64_t max_inv_seq; uint64_t pad; };

constexpr int SEG_TILE = 1024;       // sorted records owned by one workgroup of the segment kernels
constexpr int SEG_THREADS = 256;
constexpr int SEL_TILE = 2048;       // records per workgroup of the compaction kernels
constexpr int RANKCOUNT_BLOCKS = 2048;

// device counters written by kernels and read back by the host
enum { CNT_NSEG, CNT_NFLAG, CNT_NBIG, CNT_NUSABLE, CNT_NGROUP, CNT_NALERT, CNT_NCAND, CNT_STATUS, CNT_NBLAMED, CNT_NCLEAN, CNT_NLONG,
       CNT_NRETAINED, CNT_COUNT = 16 };
constexpr uint32_t GROUP_LONG_MIN = 4096;   // a detection group of more rounds than this gets a whole workgroup

}  // namespace ccld

struct ccld_ctx {
  ccld_params p;
  hipStream_t stream;
  uint64_t cap, batch_cap, snap_cap;
  ccld::KeyFormat kf;
  int rank_bits;                      // bit width of the largest rank
  // topology
  std::vector<uint32_t> h_size;
  ccld::DeviceTopology topo;
  // window (circular)
  uint64_t head, count;
  std::vector<uint64_t> batch_n;      // sizes of the resident batches, oldest first
  std::vector<uint32_t> batch_slot;   // meta slot of each resident batch
  uint32_t next_slot;
  uint64_t* win_key;
  ccld::Row* win_row;
  ccld::BatchMeta* batch_meta;        // [window_batches + 1]
  std::vector<uint32_t> batch_seqno;  // arrival number of each resident batch's first record
  uint64_t total_ingested;
  uint32_t* ing_table;                // [n_buckets][INGEST_BLOCKS]
  uint32_t* ing_base;                 // [n_buckets + 1]
  uint32_t n_buckets; int bshift;
  // sort
  ccld::SortBuffers sb;               // main sort
  uint64_t* keyC; uint32_t* idxC;     // third pair for the small sorts
  uint32_t* table2; uint32_t* totals2;
  // analysis scratch
  uint32_t* tile_heads;               // [seg tiles + 1]
  uint32_t* tile_flags;               // [sel tiles + 1]
  uint8_t* rec_flag;                  // [cap]
  uint32_t* flag_pos;                 // [cap] sorted position of the k-th flagged record
  int64_t* flag_lag;                  // [2][cap]
  uint32_t* big_list;                 // [cap / 65 + 2][3]  (segment ordinal, first position, length) of the collectives over 64 records
  int64_t* big_ex;                    // [2][cap]
  int64_t* range_c;                   // [cap] T_max - T_min of every usable collective
  int64_t* blame;                     // [CCLD_BLM_NCOL][n_ranks]
  uint32_t* blame_list;               // [2][n_ranks] flagged ranks, then the others, each ascending
  uint32_t* blame_tiles;              // [n_ranks / SEL_TILE + 3]
  uint32_t* blame_order;              // [n_ranks] ranks by (flags, summed lag, rank), written at the end of every analysis
  uint32_t* group_long;               // [cap / GROUP_LONG_MIN + 2] detection groups left to the workgroup-per-group pass
  uint32_t* group_first;              // [cap + 1]
  uint32_t* alert_list;               // [cap]
  uint32_t* alert_ncand;              // [cap + 1]
  uint2* comm_info;                   // [n_comms] (first member index, members) of every communicator: one load for both
  ccld::GroupState* gstate;           // [n_comms][GROUP_SLOTS]
  uint64_t* counters;                 // [CNT_COUNT] device
  uint32_t max_comm_size;             // members of the largest communicator
  uint64_t sort_cap;                  // items the sort buffers hold: max(window records, communicator members)
  uint64_t* h_pinned;                 // pinned host staging
  hipEvent_t ev_heads;                // marks the early readback of the collective count
  hipEvent_t ev_flags;                // marks the early readback of the flag count
  // staging for host-resident batches
  uint8_t* stage;                     // [batch_cap * 41] device
  // hang location
  uint64_t n_members;                 // member slots over all communicators
  uint64_t* h_cell;                   // [snap_cap][2]  (operation counter, sent | recv << 32)
  uint32_t* h_cnt;                    // [snap_cap / 32 + 1] presence bitmap of the grid cells
  int64_t* h_pair;                    // [CCLD_HPAIR_NCOL][n_members]
  int64_t* h_comm;                    // [CCLD_HCOMM_NCOL][n_comms]
  int32_t* h_wait_slot;               // [n_members] slot waited on, -1 = none
  uint8_t* h_cand;                    // [n_members]
  uint64_t* h_layer_max;              // [n_members]
  uint32_t* h_root_list;              // [n_members]
  int64_t* rate_root;                 // [n_comms] member of minimal SendRate / RecvRate from the latest rate pass, or CCLD_NO_RANK
  uint64_t* f_last;                   // [n_members][CCLD_FRAME_CHANNELS][2] remembered (operation counter, sent | recv << 32) per member and channel
  uint32_t* f_seen;                   // [n_ranks / 32 + 1] ranks that delivered a frame in the current call
  uint8_t* h_stage;                   // [snap_cap * 32] device staging for host-resident snapshots
  // dense placement (single-batch windows)
  bool dense_capable;                 // window_batches == 1, every communicator fits a fine bucket, few enough communicators
  uint64_t* comm_range;               // [n_comms][2] per communicator of the latest batch: largest counter, largest complement
  void* d_lay;                        // [n_comms + 1] CommLayout
  uint32_t* d_hdr;                    // [DH_COUNT]
  uint32_t* d_fill;                   // [fine_cap + 2]
  ccld::Row* d_rows;                  // [fine_cap * DENSE_STRIDE]
  void* d_desc;                       // [fine_cap] FineDesc
  uint32_t fine_cap;
  int last_path;                      // 1: the last analysis used the dense placement
  // what ccld_flag_chains needs of the most recent analysis
  bool chain_ready;                   // the sorted order, flag positions and lags of that analysis are still in the workspace
  const int64_t* last_seg; uint64_t last_seg_cap, last_n_seg, last_n_flag;
  const uint8_t* last_rec_flag;
  const ccld::Row* last_rows;         // payload rows that the sorted row indices address
  uint32_t* chain_first;              // [n_comms + 2] first table row of each communicator
  // last analysis
  int sorted_buf;                     // which ping-pong buffer holds the sorted window
  // the order of the last analysed window, kept for the next analysis of a window of several batches
  bool inc_ok;                        // sb.key/idx[sorted_buf] hold it, in format inc_sf
  ccld::SqueezedFormat inc_sf;
  uint64_t inc_head, inc_count, inc_total;   // that window's first slot, records, and total_ingested at the time
  uint64_t last_n;
  ccld::SqueezedFormat sf;
  bool blame_valid;
  ccld::Profiler prof;
  int sort_passes;                    // passes of the last main sort
};

// looks up the device address of the library's static scratch array on the current device (hang.hip)
ccld_status ccld_static_scratch_init();
