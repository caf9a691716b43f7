// Keeping the window's order from one analysis to the next (windows of several batches): the sorted
// (key, window slot) arrays of the previous analysis lose the records of the batches that left the
// window, are re-based to the new window's key format, and are merged with the sorted new records.
#pragma once
#include "ccld_internal.h"

namespace ccld {

struct RetainArgs {
  const uint64_t* key;       // previous order, n entries
  const uint32_t* idx;
  uint32_t n;
  SqueezedFormat from, to;   // key formats of the previous and of the new window (same mb)
  uint32_t exp_lo, exp_n;    // window slots [exp_lo, exp_lo + exp_n) modulo cap left the window
  uint32_t cap;
  uint32_t* tile_counts;     // [tiles + 1] scratch
  uint64_t* total_out;       // device counter that receives the number of entries kept
  uint64_t* key_out;
  uint32_t* idx_out;
};
// entries whose slot is still in the window, in order, with keys in the new format
void launch_retain(hipStream_t st, const RetainArgs& a);
// two sorted sequences -> one (at equal keys the first sequence's entry comes first)
// split: scratch of (na + nb) / 2048 + 2 words
void launch_merge(hipStream_t st, const uint64_t* ka, const uint32_t* ia, uint32_t na, const uint64_t* kb,
                  const uint32_t* ib, uint32_t nb, uint32_t* split, uint64_t* ko, uint32_t* io);

}  // namespace ccld
