// Sort-free analysis of a single-batch window: every rank bumps the same operation counter per
// communicator (the Trace ID of Section 5.1), so (communicator, counter - smallest counter, member
// slot) is a dense grid whose cell of every record is known without sorting.  The grid is cut into
// fine buckets of whole collectives that fit LDS; one partition pass moves every payload row into
// its fine bucket with coalesced writes, and the statistics kernel places a bucket's rows in LDS by
// cell and streams the collectives in (communicator, counter, rank) order.
#pragma once
#include "ccld_internal.h"
#include "window_kernels.h"

namespace ccld {

constexpr uint32_t DENSE_B = 2048;          // grid cells (= LDS cells of the statistics kernel) per fine bucket
constexpr uint32_t DENSE_STRIDE = 2048;     // rows reserved per fine bucket in the partitioned row array
constexpr uint32_t DENSE_SPAN = 4096;       // fine buckets one partition workgroup can address
constexpr uint32_t DENSE_PART_BLOCKS = 256; // partition workgroups (one per compute unit)
constexpr uint32_t DENSE_MAX_COMMS = INGEST_RANGE_COMMS;

// Per communicator: where its part of the grid lies.  Rounds are numbered from the window's smallest
// operation counter of the communicator; rpb rounds make one fine bucket.
struct CommLayout {
  uint64_t seq_min;        // smallest operation counter in the window
  uint32_t fb_base;        // first fine bucket
  uint32_t rpb;            // rounds per fine bucket: DENSE_B / members
  uint32_t rounds;         // largest - smallest operation counter + 1 (0: no record)
  uint32_t seg_base;       // row of the collective table of the first round
};

// What the statistics kernel needs to know about one fine bucket (written once the records per bucket are
// known): its communicator, the collectives it holds and where their records and table rows go.
struct FineDesc {
  uint32_t comm, size;     // communicator and its members
  uint32_t K;              // collectives (rounds) in the bucket
  uint32_t rec0, cnt;      // first record of the bucket in (communicator, counter, rank) order; records placed
  uint32_t srow0;          // row of the collective table of the bucket's first round
  uint64_t rel0;           // operation counter of the first round minus the window's smallest counter
};

// device-side header of the layout
enum { DH_FEASIBLE, DH_N_FINE, DH_N_SEG, DH_COUNT = 8 };

struct DenseArgs {
  // window (one batch, circular addressing)
  const uint64_t* win_key;
  const Row* win_row;
  uint32_t head, cap, n;
  KeyFormat kf;
  // topology and the batch's coarse buckets (communicator >> bshift) as ingest placed them
  const uint32_t* comm_size;
  uint32_t n_comms;
  const uint32_t* bucket_base;   // [n_buckets + 1] first record of each coarse bucket in the batch
  uint32_t n_buckets;
  int bshift;
  // layout
  const uint64_t* range;         // [n_comms][2] largest counter, largest complement (zero pair: no record)
  CommLayout* lay;               // [n_comms + 1]
  uint32_t* hdr;                 // [DH_COUNT]
  // fine buckets
  uint32_t* fill;                // [fine_cap + 1] records per fine bucket, later their exclusive scan
  FineDesc* desc;                // [fine_cap]
  uint64_t seq_base;             // the window's smallest operation counter
  Row* rows;                     // [fine_cap * DENSE_STRIDE]
  uint32_t fine_cap;
  uint64_t* counters;
};

void launch_dense_layout(hipStream_t st, const DenseArgs& d);
void launch_dense_partition(hipStream_t st, const DenseArgs& d);
void launch_dense_desc(hipStream_t st, const DenseArgs& d);      // after the scan of fill
// statistics of every collective from the partitioned rows (segments.hip); also writes the sorted keys
// and row indices that the flag, blame, group and alert stages read; n_fine: the fine buckets of the layout
// (one workgroup each)
void launch_dense_stats(hipStream_t st, const SegArgs& a, const DenseArgs& d, uint32_t n_fine, uint64_t* skey,
                        uint32_t* sidx, int64_t* blame, uint32_t n_ranks);

}  // namespace ccld
