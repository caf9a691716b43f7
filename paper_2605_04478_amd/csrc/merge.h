// Keeping the window's order from one analysis to the next (windows of several batches): the sorted
// (key, window slot) arrays of the previous analysis lose the records of the batches that left the
// window and are re-based to the new window's key format while they are merged with the sorted new records.
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
// The previous order (a.key, a.idx: a.n entries, those that left included) merged with the sorted new records
// (kb, ib: nb entries) into a.key_out / a.idx_out, which must not overlap the inputs: the entries that left are
// dropped, keys are written in the new format, and at equal keys the previous order's entry comes first.
// a.tile_counts: a.n / 2048 + 2 words; split: (a.n + nb) / 2048 + 2 words.
void launch_merge_kept(hipStream_t st, const RetainArgs& a, const uint64_t* kb, const uint32_t* ib, uint32_t nb,
                       uint32_t* split);

}  // namespace ccld
