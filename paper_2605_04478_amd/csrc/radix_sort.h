// LSD radix sort of (u64 key, u32 index) pairs on one GPU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ccld {

constexpr int SORT_RBITS = 8;                    // widest digit of one pass
constexpr int SORT_RADIX = 1 << SORT_RBITS;
constexpr int SORT_THREADS = 512;
constexpr int SORT_ITEMS = 8;                    // keys per thread
constexpr int SORT_TILE = SORT_THREADS * SORT_ITEMS;
// arrays of at least this many tiles (268 MB of keys) exceed the memory-side cache: eight tiles per
// histogram workgroup, loads with the non-temporal hint
constexpr uint32_t SORT_STREAM_TILES = 8192;

// Where the first pass reads its keys.  The window keeps records in a circular buffer and
// keys with a gap between the (sequence, rank) field and the communicator field; the first
// pass reads element (head + j) mod cap, squeezes the gap out, and pairs it with that index.
struct KeySource {
  const uint64_t* key;
  uint32_t head, cap;        // circular: element j lives at (head + j) mod cap
  int squeeze;               // 1: key' = ((key >> hi_shift) << lo_bits) | ((key & lo_mask) - lo_sub); hi_shift 64 = no high field
  int hi_shift, lo_bits;
  uint64_t lo_mask, lo_sub;
};

struct SortBuffers {
  uint64_t* key[2];          // ping-pong, n elements each
  uint32_t* idx[2];
  uint32_t* table;           // [SORT_RADIX][n_tiles] per-tile digit counts / offsets
  uint32_t* totals;          // [SORT_RADIX]
};

inline uint32_t sort_tiles(uint64_t n) { return (uint32_t)((n + SORT_TILE - 1) / SORT_TILE); }
inline uint64_t sort_table_words(uint64_t n_max) { return (uint64_t)SORT_RADIX * (sort_tiles(n_max) + 1); }

// Sorts n pairs stably by the low `bits` bits of the (squeezed) key.  The first pass reads
// src; the result lands in buf.key[r], buf.idx[r] where r is the return value (0 or 1), or
// a negative value if a launch failed.  bits == 0 still performs one copying pass.
// prof (optional) times the launches: class ids for the histogram, scan and scatter kernels.
struct Profiler;
int radix_sort_pairs(hipStream_t stream, const KeySource& src, uint32_t n, const SortBuffers& buf, int bits,
                     Profiler* prof = nullptr, int cls_hist = 0, int cls_scan = 0, int cls_scatter = 0);

}  // namespace ccld
