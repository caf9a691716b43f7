// LSD radix sort of (u64 key, u32 index) pairs for gfx950.
//
// One pass = three kernels: per-tile digit histograms in LDS, an exclusive scan of
// every digit's row of tile counts, and a scatter that ranks the tile's keys with
// wavefront ballots (stable), regroups them by digit in LDS and writes each digit's
// run to its place with consecutive lanes on consecutive addresses.
//
// When the significant key bits and the index bits fit one 64-bit word together, the
// passes move a single packed word (key << index_bits | index) instead of the pair and
// only the last pass writes the pair out again.
#include "radix_sort.h"
#include "device_utils.h"
#include "profiler.h"

namespace ccld {

enum SortIn { IN_SOURCE, IN_PAIR, IN_PACKED };
enum SortOut { OUT_PAIR, OUT_PACKED };

// Arrays larger than the memory-side cache are read once per kernel and gone before the next one
// reads them again: their loads carry the non-temporal hint so that they do not displace the lines
// the scatter's partial writes are merged in.  Smaller arrays are read plainly (the scatter finds
// in the cache what the histogram just read).
template <bool STREAM, class T> __device__ __forceinline__ T load_once(const T* p) {
  return STREAM ? __builtin_nontemporal_load(p) : *p;
}

__device__ __forceinline__ u64 squeeze_key(const KeySource& s, u64 k) {
  if (s.squeeze) k = (s.hi_shift < 64 ? (k >> s.hi_shift) << s.lo_bits : 0ull) | ((k & s.lo_mask) - s.lo_sub);
  return k;
}
template <bool STREAM>
__device__ __forceinline__ u64 load_key(const KeySource& s, u32 j, u32* phys) {
  u32 p = s.head + j;                       // head < cap and j < cap <= 2^31: no wrap below 2^32
  if (p >= s.cap) p -= s.cap;
  *phys = p;
  return squeeze_key(s, load_once<STREAM>(s.key + p));
}

// ---- per-tile digit histogram --------------------------------------------------------------
// A workgroup counts HIST_TILES consecutive tiles, so that each digit's counts leave as one
// contiguous 32-byte piece of the digit-major table instead of eight scattered words.
// Small inputs take fewer tiles per workgroup so that there are still several workgroups per compute unit.
template <bool FIRST, int HIST_TILES>
__global__ __launch_bounds__(SORT_THREADS) void k_radix_hist(KeySource src, const u64* __restrict__ key_in,
                                                             u32* __restrict__ table, u32 n, u32 n_tiles,
                                                             int shift, u32 dmask) {
  constexpr bool STREAM = HIST_TILES == 8;      // the many-tile variant serves the arrays beyond the cache size
  __shared__ u32 s_hist[HIST_TILES][SORT_RADIX];
  const u32 tid = threadIdx.x, tile0 = blockIdx.x * HIST_TILES;
  for (u32 i = tid; i < HIST_TILES * SORT_RADIX; i += SORT_THREADS) (&s_hist[0][0])[i] = 0;
  __syncthreads();
#pragma unroll 4
  for (int t = 0; t < HIST_TILES; ++t) {
    const u32 base = (tile0 + t) * SORT_TILE;
    if (tile0 + t >= n_tiles) continue;
    // full tile of consecutive, 16-byte aligned keys (a plain array, or a stretch of the circular
    // window that does not wrap): 16-byte loads, two keys per lane
    u32 p0 = base;
    bool plain = base + SORT_TILE <= n;
    if (FIRST) {
      p0 = src.head + base;
      if (p0 >= src.cap) p0 -= src.cap;
      plain = plain && p0 + SORT_TILE <= src.cap && (p0 & 1) == 0;
    }
    if (plain) {
      const ulonglong2* __restrict__ in2 = reinterpret_cast<const ulonglong2*>((FIRST ? src.key : key_in) + p0);
      ulonglong2 kk[SORT_ITEMS / 2];
#pragma unroll
      for (int it = 0; it < SORT_ITEMS / 2; ++it) {
        typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
        const u64x2 t2 = load_once<STREAM>(reinterpret_cast<const u64x2*>(in2 + it * SORT_THREADS + tid));
        kk[it].x = t2.x; kk[it].y = t2.y;
        if (FIRST) { kk[it].x = squeeze_key(src, kk[it].x); kk[it].y = squeeze_key(src, kk[it].y); }
      }
#pragma unroll
      for (int it = 0; it < SORT_ITEMS / 2; ++it) {
        atomicAdd(&s_hist[t][(u32)(kk[it].x >> shift) & dmask], 1u);
        atomicAdd(&s_hist[t][(u32)(kk[it].y >> shift) & dmask], 1u);
      }
      continue;
    }
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
      u32 j = base + it * SORT_THREADS + tid;
      if (j < n) {
        u64 k;
        if (FIRST) { u32 ph; k = load_key<STREAM>(src, j, &ph); } else k = key_in[j];
        atomicAdd(&s_hist[t][(u32)(k >> shift) & dmask], 1u);
      }
    }
  }
  __syncthreads();
  const u32 nt = (n_tiles - tile0) < (u32)HIST_TILES ? (n_tiles - tile0) : (u32)HIST_TILES;
  for (u32 d = tid; d <= dmask; d += SORT_THREADS)
    for (u32 t = 0; t < nt; ++t) table[(u64)d * n_tiles + tile0 + t] = s_hist[t][d];
}

// ---- exclusive scan of each digit's row of tile counts ------------------------------------
// one workgroup per digit; every thread scans SCAN_PER consecutive tiles serially
constexpr int SCAN_PER = 8;
__device__ __forceinline__ void scan_row_load(const u32* row, u32 i0, u32 n, bool vec, u32 (&v)[SCAN_PER]) {
  if (vec && i0 + SCAN_PER <= n) {
    const uint4 a = *reinterpret_cast<const uint4*>(row + i0), b = *reinterpret_cast<const uint4*>(row + i0 + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) v[k] = (i0 + k) < n ? row[i0 + k] : 0u;
  }
}
__global__ __launch_bounds__(SORT_THREADS) void k_radix_scan(u32* __restrict__ table, u32* __restrict__ totals,
                                                             u32 n_tiles) {
  static_assert(SCAN_PER == 8, "two 16-byte pieces per thread");
  __shared__ u32 s_wave[SORT_THREADS / CCLD_WAVE];
  u32* row = table + (u64)blockIdx.x * n_tiles;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
  u32 carry = 0;
  u32 v[SCAN_PER], nv[SCAN_PER];
  scan_row_load(row, threadIdx.x * SCAN_PER, n_tiles, vec, v);
  for (u32 base = 0; base < n_tiles; base += SORT_THREADS * SCAN_PER) {
    const u32 i0 = base + threadIdx.x * SCAN_PER;
    // the next round's counts are on their way while this round is scanned and stored
    scan_row_load(row, i0 + SORT_THREADS * SCAN_PER, n_tiles, vec, nv);
    u32 sum = 0;
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) sum += v[k];
    u32 tot;
    u32 ex = carry + block_exclusive_sum<SORT_THREADS>(sum, s_wave, &tot);
    if (vec && i0 + SCAN_PER <= n_tiles) {
      u32 o[SCAN_PER];
#pragma unroll
      for (int k = 0; k < SCAN_PER; ++k) { o[k] = ex; ex += v[k]; }
      *reinterpret_cast<uint4*>(row + i0) = make_uint4(o[0], o[1], o[2], o[3]);
      *reinterpret_cast<uint4*>(row + i0 + 4) = make_uint4(o[4], o[5], o[6], o[7]);
    } else {
#pragma unroll
      for (int k = 0; k < SCAN_PER; ++k) { if ((i0 + k) < n_tiles) row[i0 + k] = ex; ex += v[k]; }
    }
    carry += tot;
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) v[k] = nv[k];
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

// ---- rank, regroup in LDS, scatter --------------------------------------------------------------
// shift addresses the digit inside the word the kernel ranks: the key itself, or the packed word
// (key << ibits | index) when either side is packed.
template <int IN, int OUT, bool STREAM>
__global__ __launch_bounds__(SORT_THREADS)
__attribute__((amdgpu_waves_per_eu(((IN == IN_PACKED) || (OUT == OUT_PACKED)) ? 8 : 4))) void k_radix_scatter(KeySource src, const u64* __restrict__ key_in,
                                                                const u32* __restrict__ idx_in,
                                                                u64* __restrict__ key_out, u32* __restrict__ idx_out,
                                                                const u32* __restrict__ table,
                                                                const u32* __restrict__ totals, u32 n, u32 n_tiles,
                                                                int shift, int nbits, int ibits) {
  constexpr int NW = SORT_THREADS / CCLD_WAVE;
  constexpr bool PACKED = (IN == IN_PACKED) || (OUT == OUT_PACKED);   // one word per element inside the kernel
  // per-wavefront digit counters, then each wavefront's base inside the digit (at most 4,096: 16 bits, which
  // keeps the packed variants within 40 KB of LDS, four workgroups per compute unit)
  __shared__ unsigned short s_cnt[NW][SORT_RADIX];
  __shared__ u32 s_dstart[SORT_RADIX];    // first tile-local position of each digit
  __shared__ u32 s_gbase[SORT_RADIX];     // global position of tile-local position 0 of each digit (minus dstart)
  __shared__ u32 s_wave[NW];
  __shared__ u64 s_key[SORT_TILE];
  __shared__ u32 s_idx[PACKED ? 1 : SORT_TILE];

  const u32 tid = threadIdx.x, lane = lane_id(), wave = tid / CCLD_WAVE;
  // Workgroups are dealt to the eight XCDs in turn.  Neighbouring tiles write neighbouring runs of
  // every digit, so each XCD takes one contiguous eighth of the tiles: the two halves of an output
  // line then meet in one L2 instead of leaving two L2s as partial lines.
  const u32 per_xcd = (n_tiles + 7) / 8;
  const u32 tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= n_tiles) return;
  const u32 dmask = (1u << nbits) - 1u;
  const u32 base = tile * SORT_TILE;
  const u32 valid = (n - base) < (u32)SORT_TILE ? (n - base) : (u32)SORT_TILE;

  for (u32 i = tid; i < NW * SORT_RADIX; i += SORT_THREADS) (&s_cnt[0][0])[i] = 0;

  // wavefront w owns tile elements [w*64*ITEMS, (w+1)*64*ITEMS); item `it` of lane l is element
  // w*64*ITEMS + it*64 + l, so (wavefront, item, lane) order is input order
  u64 k[SORT_ITEMS];
  u32 v[SORT_ITEMS], pre[SORT_ITEMS];
  u32 src_p0 = 0;
  bool src_plain = false;
  if (IN == IN_SOURCE) {
    src_p0 = src.head + base;
    if (src_p0 >= src.cap) src_p0 -= src.cap;
    src_plain = src_p0 + SORT_TILE <= src.cap;
  }
  // the digit is recomputed from the key where it is needed (eight registers fewer)
  auto digit_of = [&](u64 key) -> u32 { return (u32)(key >> shift) & dmask; };
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; ++it) {
    u32 e = wave * (CCLD_WAVE * SORT_ITEMS) + it * CCLD_WAVE + lane;
    v[it] = 0;
    if (e < valid) {
      if (IN == IN_SOURCE) {
        if (src_plain) {      // the tile does not cross the end of the circular window
          v[it] = src_p0 + e;
          k[it] = squeeze_key(src, load_once<STREAM>(src.key + src_p0 + e));
        } else {
          k[it] = load_key<STREAM>(src, base + e, &v[it]);
        }
        if (PACKED) k[it] = (k[it] << ibits) | v[it];
      } else if (IN == IN_PAIR) {
        k[it] = load_once<STREAM>(key_in + base + e); v[it] = load_once<STREAM>(idx_in + base + e);
      } else {
        k[it] = load_once<STREAM>(key_in + base + e);
      }
    } else {
      k[it] = ~0ull;                // padding: the last digit, after every real key of it
    }
  }
  __syncthreads();

#pragma unroll
  for (int it = 0; it < SORT_ITEMS; ++it) {
    const u32 d = digit_of(k[it]);
    u64 same = ~0ull;                      // lanes of this wavefront holding the same digit
#pragma unroll
    for (int b = 0; b < SORT_RBITS; ++b) {
      if (b < nbits) {
        const bool bit = (d >> b) & 1u;
        const u64 bal = ballot64(bit);
        same &= bit ? bal : ~bal;
      }
    }
    const u32 below = mbcnt64(same), cnt = (u32)__popcll(same);
    const u32 old = s_cnt[wave][d];
    __builtin_amdgcn_wave_barrier();
    if (below == cnt - 1) s_cnt[wave][d] = (unsigned short)(old + cnt);
    __builtin_amdgcn_wave_barrier();
    pre[it] = old + below;
  }
  __syncthreads();

  // per digit: base of each wavefront inside the digit, tile total; then digit starts
  {
    u32 tot = 0;
    u32 gtot = 0;
    if (tid < SORT_RADIX) {
#pragma unroll
      for (int w = 0; w < NW; ++w) { u32 c = s_cnt[w][tid]; s_cnt[w][tid] = (unsigned short)tot; tot += c; }
      gtot = tid <= dmask ? totals[tid] : 0u;
    }
    u32 t0, t1;
    u32 dstart = block_exclusive_sum<SORT_THREADS>(tot, s_wave, &t0);
    u32 gbase = block_exclusive_sum<SORT_THREADS>(gtot, s_wave, &t1);
    if (tid < SORT_RADIX) {
      s_dstart[tid] = dstart;
      u32 toff = tid <= dmask ? table[(u64)tid * n_tiles + tile] : 0u;
      s_gbase[tid] = gbase + toff - dstart;
    }
  }
  __syncthreads();

#pragma unroll
  for (int it = 0; it < SORT_ITEMS; ++it) {
    const u32 d = digit_of(k[it]);
    const u32 pos = s_dstart[d] + s_cnt[wave][d] + pre[it];
    s_key[pos] = k[it];
    if (!PACKED) s_idx[pos] = v[it];
  }
  __syncthreads();

  const u64 imask = ibits >= 64 ? ~0ull : (((u64)1 << ibits) - 1);
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; ++it) {
    const u32 pos = it * SORT_THREADS + tid;
    if (pos < valid) {
      const u64 kk = s_key[pos];
      const u32 g = s_gbase[(u32)(kk >> shift) & dmask] + pos;
      if (OUT == OUT_PACKED) {
        key_out[g] = kk;
      } else if (PACKED) {
        key_out[g] = kk >> ibits;
        idx_out[g] = (u32)(kk & imask);
      } else {
        key_out[g] = kk;
        idx_out[g] = s_idx[pos];
      }
    }
  }
}

static_assert(SORT_RADIX <= SORT_THREADS, "one thread per digit in the scatter prologue");

template <int IN, int OUT>
static void launch_scatter(hipStream_t stream, const KeySource& src, const u64* key_in, const u32* idx_in,
                           u64* key_out, u32* idx_out, const SortBuffers& buf, u32 n, u32 n_tiles, int shift,
                           int nbits, int ibits) {
  if (n_tiles >= SORT_STREAM_TILES)
    hipLaunchKernelGGL((k_radix_scatter<IN, OUT, true>), dim3((n_tiles + 7) / 8 * 8), dim3(SORT_THREADS), 0, stream, src, key_in, idx_in,
                       key_out, idx_out, (const u32*)buf.table, (const u32*)buf.totals, n, n_tiles, shift, nbits, ibits);
  else
    hipLaunchKernelGGL((k_radix_scatter<IN, OUT, false>), dim3((n_tiles + 7) / 8 * 8), dim3(SORT_THREADS), 0, stream, src, key_in, idx_in,
                       key_out, idx_out, (const u32*)buf.table, (const u32*)buf.totals, n, n_tiles, shift, nbits, ibits);
}

static int host_bits(uint64_t v) { int b = 0; while (v) { ++b; v >>= 1; } return b; }

// ---- sorts of at most SMALL_SORT_MAX pairs: one launch ------------------------------------------------------
// One workgroup sorts composite words (key bits << 12 | position in the source) with a bitonic network in
// LDS: equal keys keep their source order, as in the radix passes.  For key widths of at most 52 bits.
constexpr u32 SMALL_SORT_MAX = 4096;
constexpr int SMALL_SORT_BITS = 52;
__global__ __launch_bounds__(1024) void k_small_sort(KeySource src, u32 n, int bits, u64* __restrict__ key_out,
                                                     u32* __restrict__ idx_out) {
  __shared__ u64 s_c[SMALL_SORT_MAX];
  const u32 t = threadIdx.x;
  u32 P = 2;
  while (P < n) P <<= 1;
  const u64 kmask = bits <= 0 ? 0ull : (((u64)1 << bits) - 1);
  auto phys = [&](u32 j) -> u32 { u32 p = src.head + j; if (p >= src.cap) p -= src.cap; return p; };
  for (u32 j = t; j < P; j += 1024)
    s_c[j] = j < n ? (((squeeze_key(src, src.key[phys(j)]) & kmask) << 12) | (u64)j) : ~0ull;
  __syncthreads();
  for (u32 k = 2; k <= P; k <<= 1) {
    for (u32 jj = k >> 1, first = 1; jj; jj >>= 1, first = 0) {
      const u32 M = first ? k - 1 : jj;               // the merge's first step mirrors, the others halve the stride
      for (u32 q = t; q < P / 2; q += 1024) {
        const u32 lo = q & (jj - 1), ia = ((q - lo) << 1) | lo, ib = ia ^ M;
        const u64 va = s_c[ia], vb = s_c[ib];
        if (vb < va) { s_c[ia] = vb; s_c[ib] = va; }
      }
      __syncthreads();
    }
  }
  for (u32 i = t; i < n; i += 1024) {
    const u32 p = phys((u32)(s_c[i] & (SMALL_SORT_MAX - 1)));
    key_out[i] = squeeze_key(src, src.key[p]);
    idx_out[i] = p;
  }
}

int radix_sort_pairs(hipStream_t stream, const KeySource& src_in, uint32_t n, const SortBuffers& buf, int bits,
                     Profiler* prof, int cls_hist, int cls_scan, int cls_scatter) {
  if (n == 0) return 0;
  if (n <= SMALL_SORT_MAX && bits <= SMALL_SORT_BITS && src_in.key != buf.key[0]) {
    if (prof) prof->begin(cls_scatter);
    hipLaunchKernelGGL(k_small_sort, dim3(1), dim3(1024), 0, stream, src_in, n, bits, buf.key[0], buf.idx[0]);
    if (prof) prof->end(cls_scatter);
    return hipGetLastError() == hipSuccess ? 0 : -1;
  }
  const KeySource& src = src_in;
  const u32 n_tiles = sort_tiles(n);
  const int passes = bits <= 0 ? 1 : (bits + SORT_RBITS - 1) / SORT_RBITS;
  const int ibits = host_bits(src.cap ? src.cap - 1 : 0);
  const bool packed = passes >= 2 && bits + ibits <= 64;
  int done_bits = 0, cur = -1;
  for (int p = 0; p < passes; ++p) {
    // spread the bits evenly over the passes, the narrower digits first (the first pass also squeezes the
    // keys and is the slowest: fewer digit values mean longer runs in its scatter)
    int left = bits - done_bits, nb = bits <= 0 ? 1 : left / (passes - p);
    if (nb < 1) nb = 1;
    const u32 dmask = (1u << nb) - 1u;
    const int out = cur < 0 ? 0 : 1 - cur;
    const bool first = p == 0, last = p == passes - 1;
    // digit position inside the word each kernel looks at
    const int hist_shift = done_bits + ((packed && !first) ? ibits : 0);
    const int scat_shift = done_bits + (packed ? ibits : 0);
    if (prof && first) prof->begin(cls_hist);
    const u64* hin = first ? nullptr : buf.key[cur];
    if (n_tiles >= SORT_STREAM_TILES) {
      if (first) hipLaunchKernelGGL((k_radix_hist<true, 8>), dim3((n_tiles + 7) / 8), dim3(SORT_THREADS), 0, stream, src, hin, buf.table, n, n_tiles, hist_shift, dmask);
      else hipLaunchKernelGGL((k_radix_hist<false, 8>), dim3((n_tiles + 7) / 8), dim3(SORT_THREADS), 0, stream, src, hin, buf.table, n, n_tiles, hist_shift, dmask);
    } else {
      if (first) hipLaunchKernelGGL((k_radix_hist<true, 1>), dim3(n_tiles), dim3(SORT_THREADS), 0, stream, src, hin, buf.table, n, n_tiles, hist_shift, dmask);
      else hipLaunchKernelGGL((k_radix_hist<false, 1>), dim3(n_tiles), dim3(SORT_THREADS), 0, stream, src, hin, buf.table, n, n_tiles, hist_shift, dmask);
    }
    if (prof) prof->split(cls_hist, cls_scan);
    hipLaunchKernelGGL(k_radix_scan, dim3(dmask + 1), dim3(SORT_THREADS), 0, stream, buf.table, buf.totals, n_tiles);
    if (prof) prof->split(cls_scan, cls_scatter);
    const u64* kin = first ? nullptr : buf.key[cur];
    const u32* iin = first ? nullptr : buf.idx[cur];
    if (!packed) {
      if (first) launch_scatter<IN_SOURCE, OUT_PAIR>(stream, src, kin, iin, buf.key[out], buf.idx[out], buf, n, n_tiles, scat_shift, nb, ibits);
      else launch_scatter<IN_PAIR, OUT_PAIR>(stream, src, kin, iin, buf.key[out], buf.idx[out], buf, n, n_tiles, scat_shift, nb, ibits);
    } else {
      if (first) launch_scatter<IN_SOURCE, OUT_PACKED>(stream, src, kin, iin, buf.key[out], buf.idx[out], buf, n, n_tiles, scat_shift, nb, ibits);
      else if (!last) launch_scatter<IN_PACKED, OUT_PACKED>(stream, src, kin, iin, buf.key[out], buf.idx[out], buf, n, n_tiles, scat_shift, nb, ibits);
      else launch_scatter<IN_PACKED, OUT_PAIR>(stream, src, kin, iin, buf.key[out], buf.idx[out], buf, n, n_tiles, scat_shift, nb, ibits);
    }
    if (prof) { if (last) prof->end(cls_scatter); else prof->split(cls_scatter, cls_hist); }
    if (hipGetLastError() != hipSuccess) return -1;
    done_bits += nb;
    cur = out;
  }
  return cur;
}

}  // namespace ccld
