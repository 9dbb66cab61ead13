// Shared device-side definitions of the gfx950 gradient compressor: tile geometry,
// per-segment control block, wave64 helpers.  Wave size is 64 everywhere.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparsify.h"

namespace sp {

constexpr int kBlock = 256;                       // threads per workgroup (4 waves)
constexpr int kWaves = kBlock / 64;
constexpr int kSlots = 4;                         // float4 loads per thread per tile
constexpr int kPerThread = 4 * kSlots;            // 16 elements per thread
constexpr int kChunk = kBlock * kPerThread;       // 4096 elements = 16 KiB per array
// A workgroup's unit of work, a "tile", is `tile_chunks` (odd) consecutive chunks (chosen per call so
// that a vector has at most about four thousand tiles: the per-tile partial results that the
// small per-segment kernels must combine then stay few, whatever d is).
constexpr int kNumThres = 10;                     // thresholds reachable by <= 3 nudges

// Thresholds reachable from thres0 by `a` multiplications by 1.5 and `b` halvings, a+b <= 3
// (Alg. 1 steps 8-11).  Halving is exact, so the value depends only on (a, b).
__host__ __device__ inline int thres_index(int a, int b) { return (a + b) * (a + b + 1) / 2 + a; }
// Position of threshold (a, b) when the ten are sorted by their ratio to thres0:
// 1/8, 1/4, 3/8, 1/2, 3/4, 1, 9/8, 3/2, 9/4, 27/8.
__host__ __device__ inline int thres_pos(int a, int b) {
  // indexed by thres_index(a, b); packed 4 bits each: {5,3,7,1,4,8,0,2,6,9}
  return (int)((0x9620841735ull >> (4 * thres_index(a, b))) & 0xF);
}

constexpr uint32_t kNoListKey = 0x7FFFFFFFu;  // a listing key that no key exceeds: nothing is listed

// One per segment, lives in the workspace; written by kernels, read by later kernels.
struct SegCtrl {
  // layout
  int64_t start, end;       // [start, end) in the flat buffer
  int64_t k, cap, out_base; // target survivors, output capacity, first output slot
  uint32_t tile0, ntiles;   // first tile id and number of tiles of this segment
  uint32_t bad;             // layout invalid: produce nothing
  uint32_t group0;          // first of this segment's groups of 64 tiles (layer-wise calls)
  // Gaussian_k
  double z;                 // upper-tail normal quantile of k / (tail_div * d)
  double t64[kNumThres];    // ascending order of nominal ratio (see thres_pos)
  float t32[kNumThres];
  float t_final;            // fp32 threshold of the mask-producing evaluation
  uint32_t select_none;     // overflow / bad: select nothing
  uint32_t sorted_ok;       // the ten thresholds are in non-decreasing order (thres0 > 0)
  uint32_t flags;           // result flags raised so far (Gaussian_k)
  // Top_k
  uint32_t prefix;          // digits of the k-th key decided so far (high bits)
  uint32_t k_rem;           // survivors still to take among keys matching the prefix
  uint32_t n_eq;            // number of keys equal to the k-th key
  uint32_t rank_ties;       // 1 if only some of the equal keys are kept (needs index order)
  uint32_t sel_prefix[8];   // fused flat paths: prefix and rank left after each digit choice
  uint32_t sel_krem[8];     //   (one slot per choice: a kernel reads one slot and writes the next)
  uint32_t topk_key;        // fused flat paths: the k-th key and the ties to keep
  uint32_t topk_take;
  uint32_t tau_key;         // short-list form (topk_list.h): entries with a larger key are listed
  uint32_t list_mode;       //   1 once the kernel after the accumulate kernel found the lists usable
                            //   (layer-wise calls: 1 when a stretch of this segment's lists ran out)
  uint32_t list_count;      // layer-wise Top_k with lists: entries of this segment listed
};

struct Args {
  int32_t L;          // segments (1 for the flat calls)
  int32_t inplace;    // acc == residual
  int32_t norms;      // also reduce ||acc||^2 and ||residual'||^2
  int64_t d_total;
  int64_t flat_k, flat_cap;
  const int64_t* seg_off;
  const int64_t* seg_k;
  const int64_t* out_off;
  int64_t out_cap;
  const float* grad;
  float* resid;
  float* acc;
  uint32_t* out_idx;
  float* out_val;
  sparsify_result* result;
  SegCtrl* ctrl;
  uint32_t* tile_start;   // [L+1], segmented only
  double* partial;        // [3][max_tiles]: n, mean, M2
  double* folded;         // [3][1024]: the same after a fold of the per-chunk partials (long vectors)
  uint32_t use_folded;    // the count kernel reads `folded` (stride 1024) instead of `partial`
  uint32_t* tile_counts;  // [kNumThres][max_tiles]
  uint32_t* tile_base;    // [max_tiles]
  uint32_t* group_counts; // [64][kNumThres]: totals of groups of 64 tiles (fused flat path)
  uint32_t* seg_groups;   // [max_groups][kNumThres]: the same per segment (layer-wise calls)
  uint32_t max_groups;
  double* norm_partial;   // [2][max_tiles]: per-tile sum of acc^2 and of residual'^2
  uint32_t* hist;         // [L][hist_copies][256]
  uint32_t* tie_base;     // [max_tiles] (layer-wise Top_k with lists: one listing key per segment instead)
  uint32_t* tile_hist;    // [up to 4096 tiles][128]: per-tile histogram of the last digit (Top_k in place)
  uint32_t hist_copies;   // replicas of each segment's histogram (spreads the atomics)
  uint32_t max_tiles;
  uint32_t tile_chunks;   // chunks per tile
  uint32_t moment_parts;  // flat calls: number of moment partials (accumulate workgroups)
  int32_t ddof;
  double tail_div;
  // DGC_k
  int64_t sample_stride;  // stratum length S
  int64_t sample_m;       // number of strata = sample size
  int64_t sample_k;       // rank of the threshold inside the sample
  uint64_t sample_seed;
  // Top_k, short-list form (topk_list.h); `list` is null when the call does not use it
  uint2* list;            // (index, bits of acc): every wave appends to its own stretch
  uint2* run_table;       // [chunks * 16]: (first entry, entries) of each 256-element run
  uint32_t* list_stats;   // [2][kListStatCopies]: entries listed (replicated sums), stretches that ran out
  uint32_t compact_tiles; // Gaussian_k, flat: consecutive tiles per workgroup of the compact kernel
  uint32_t flat_tiles;    //   and the number of tiles of the vector
  uint32_t list_cap;      // entries per wave of the kernel that writes the lists
  uint32_t run_cap;       // records the run table holds (host-side check only)
  uint32_t list_last;     // index of the buffer's last entry
};

// Tile j of a segment covers the absolute range [base + j*E, base + (j+1)*E) cut to
// [start, end), E = tile_chunks * kChunk, with base = start rounded down to a multiple of 4 so
// that full float4 slots are 16-byte aligned whatever the segment's start.
__host__ __device__ inline int64_t seg_base(int64_t start) { return start & ~int64_t(3); }
__host__ __device__ inline uint32_t seg_ntiles(int64_t start, int64_t end, uint32_t tile_chunks) {
  const int64_t e = (int64_t)tile_chunks * kChunk;
  return (uint32_t)((end - seg_base(start) + e - 1) / e);
}

// One chunk: what the tile_io loads and stores address.
struct Tile {
  int seg;
  int64_t tbase;   // absolute index of the chunk's first slot (multiple of 4)
  int64_t lo, hi;  // valid absolute range of this chunk
  bool full;       // every slot of the chunk is inside [lo, hi)
};

// One workgroup's tile: `nchunks` chunks starting at `base`, valid range [lo, hi).
struct Span {
  int seg;
  int64_t base, lo, hi;
  uint32_t nchunks;
};

__device__ inline Tile chunk_of(const Span& s, uint32_t u) {
  Tile t;
  t.seg = s.seg;
  t.tbase = s.base + (int64_t)u * kChunk;
  t.lo = t.tbase > s.lo ? t.tbase : s.lo;
  t.hi = (t.tbase + kChunk < s.hi) ? t.tbase + kChunk : s.hi;
  t.full = (t.tbase >= s.lo) && (t.tbase + kChunk <= s.hi);
  return t;
}

__device__ inline void make_span(Span* out, int seg, int64_t start, int64_t end, int64_t tb,
                                 uint32_t tile_chunks) {
  const int64_t te = tb + (int64_t)tile_chunks * kChunk;
  out->seg = seg;
  out->base = tb;
  out->lo = tb > start ? tb : start;
  out->hi = te < end ? te : end;
  out->nchunks = (uint32_t)((out->hi - tb + kChunk - 1) / kChunk);
}

// Maps a tile id to its segment and range.  Flat calls: one segment starting at 0.
template <bool SEG>
__device__ inline bool locate_span(const Args& a, uint32_t t, Span* out) {
  const int64_t e = (int64_t)a.tile_chunks * kChunk;
  if (!SEG) {
    const int64_t tb = (int64_t)t * e;
    if (tb >= a.d_total) return false;
    make_span(out, 0, 0, a.d_total, tb, a.tile_chunks);
    return true;
  }
  // Largest s with tile_start[s] <= t, found by the whole wave at once: 64 evenly spaced
  // entries per round (one load latency per round instead of one per bisection step).
  const uint32_t* ts = a.tile_start;
  const uint32_t total = ts[a.L];
  const uint32_t lane = threadIdx.x & 63u;
  uint32_t lo = 0, n = (uint32_t)a.L;
  while (n > 1) {
    const uint32_t stride = (n + 63u) / 64u;
    const uint32_t off = lane * stride;
    const uint32_t v = off < n ? ts[lo + off] : 0xFFFFFFFFu;
    const uint32_t below = (uint32_t)__builtin_popcountll(__ballot(v <= t));  // >= 1: ts[lo] <= t
    const uint32_t first = (below - 1u) * stride;
    lo += first;
    n = (n - first < stride) ? n - first : stride;
  }
  if (t >= total) return false;
  const SegCtrl& c = a.ctrl[lo];
  make_span(out, (int)lo, c.start, c.end, seg_base(c.start) + (int64_t)(t - c.tile0) * e,
            a.tile_chunks);
  return true;
}

__device__ inline uint32_t mag_key(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

__device__ inline int lane_id() { return (int)(threadIdx.x & 63); }
__device__ inline int wave_id() { return (int)(threadIdx.x >> 6); }

// number of set bits of `mask` in lanes below the calling lane
__device__ inline uint32_t lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ inline uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// inclusive prefix sum across the 64 lanes
__device__ inline uint32_t wave_inclusive_scan(uint32_t v) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(v, off, 64);
    if (lane_id() >= off) v += o;
  }
  return v;
}

// Exclusive prefix sum over a workgroup of NW waves in thread order; *total gets the block
// sum.  `lds` must hold NW words.  Contains two barriers.
template <int NW = kWaves>
__device__ inline uint32_t block_exclusive_scan(uint32_t v, uint32_t* lds, uint32_t* total) {
  const uint32_t inc = wave_inclusive_scan(v);
  if (lane_id() == 63) lds[wave_id()] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t s = lds[w];
    if (w < wave_id()) before += s;
    all += s;
  }
  __syncthreads();
  *total = all;
  return before + inc - v;
}

// Histogram increments in LDS.  Atomics of one wave instruction that name the same LDS address
// are performed one after the other, so data that puts every element into one bin (an all-zero
// or constant vector: a frozen layer, say) would make the digit passes several times slower.
// When all active lanes name the same bin, one lane adds the lot.
__device__ inline void wave_hist_add(uint32_t* h, uint32_t bin, bool active) {
  const uint64_t act = __ballot(active);
  if (act == 0) return;
  const int first = (int)__builtin_ctzll(act);
  const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)bin, first);
  if (__ballot(active && bin == b0) == act) {
    if (lane_id() == first) atomicAdd(&h[b0], (uint32_t)__builtin_popcountll(act));
  } else if (active) {
    atomicAdd(&h[bin], 1u);
  }
}
// Cheap guess, once per chunk, whether the careful forms above are worth their instructions:
// true when the 64 lanes' first elements all fall into one bin (practically never on
// bell-shaped data, always on constant data).
__device__ inline bool wave_bins_look_uniform(uint32_t bin) {
  return __ballot(bin == (uint32_t)__builtin_amdgcn_readfirstlane((int)bin)) == ~0ull;
}

// Workgroups of the per-segment finalising kernels: one block per segment reads thousands of
// per-tile partials that other XCDs wrote, so every load pays a full trip to memory; they use
// 1024 threads and issue their loads in unrolled batches to pay that latency once.
constexpr int kFinBlock = 1024;
constexpr int kFinWaves = kFinBlock / 64;

// Ranks in index order (slots, then lanes, then the four components) of the elements of a tile
// flagged in `sel` (bit e = element e of this thread).  first[j] receives the rank of this
// thread's first flagged element of slot j; returns the number flagged in the whole tile.
// One barrier; `lds` must hold kSlots * kWaves words and may be reused after the next barrier.
__device__ inline uint32_t tile_rank(uint32_t sel, uint32_t* lds, uint32_t (&first)[kSlots]) {
  if (__ballot(sel != 0) == 0) {  // wave-uniform: nothing flagged in this wave's 1024 elements
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      first[j] = 0;
      if (lane_id() == 0) lds[j * kWaves + wave_id()] = 0;
    }
  } else {
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      uint32_t tot = 0, mine = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint64_t m = __ballot((sel >> (4 * j + q)) & 1u);
        tot += (uint32_t)__builtin_popcountll(m);
        mine += lanes_below(m);
      }
      first[j] = mine;
      if (lane_id() == 0) lds[j * kWaves + wave_id()] = tot;
    }
  }
  __syncthreads();
  uint32_t run = 0;
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      if (w == wave_id()) first[j] += run;
      run += lds[j * kWaves + w];
    }
  }
  return run;
}

// Squared norms that ride on the compaction pass: sum of x^2 over the valid elements of a tile,
// and over those not selected (the residual).
struct NormAcc {
  double all, rest;
};
__device__ inline void norm_accumulate(NormAcc& n, const float (&v)[kPerThread], uint32_t valid,
                                       uint32_t sel) {
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    if ((valid >> i) & 1u) {
      const double x = (double)v[i];
      n.all = fma(x, x, n.all);
      if (!((sel >> i) & 1u)) n.rest = fma(x, x, n.rest);
    }
  }
}
// One barrier; `lds` holds 2 * kWaves doubles.
__device__ inline void store_norm_partial(const Args& a, const NormAcc& n, uint32_t tile,
                                          double* lds) {
  const double x = wave_sum(n.all), y = wave_sum(n.rest);
  if (lane_id() == 0) {
    lds[2 * wave_id()] = x;
    lds[2 * wave_id() + 1] = y;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double sx = 0.0, sy = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      sx += lds[2 * w];
      sy += lds[2 * w + 1];
    }
    a.norm_partial[tile] = sx;
    a.norm_partial[(size_t)a.max_tiles + tile] = sy;
  }
}

// Running (count, mean, sum of squared deviations) and its pairwise merge.
struct Moments {
  double n, mean, m2;
};
__device__ inline Moments merge(const Moments& a, const Moments& b) {
  if (b.n == 0.0) return a;
  if (a.n == 0.0) return b;
  Moments r;
  r.n = a.n + b.n;
  const double delta = b.mean - a.mean;
  r.mean = a.mean + delta * (b.n / r.n);
  r.m2 = a.m2 + b.m2 + delta * delta * (a.n * b.n / r.n);
  return r;
}

}  // namespace sp
