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
constexpr int kTile = kBlock * kPerThread;        // 4096 elements = 16 KiB per array
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

// One per segment, lives in the workspace; written by kernels, read by later kernels.
struct SegCtrl {
  // layout
  int64_t start, end;       // [start, end) in the flat buffer
  int64_t k, cap, out_base; // target survivors, output capacity, first output slot
  uint32_t tile0, ntiles;   // first tile id and number of tiles of this segment
  uint32_t bad;             // layout invalid: produce nothing
  uint32_t pad0;
  // Gaussian_k
  double z;                 // upper-tail normal quantile of k / (tail_div * d)
  double t64[kNumThres];    // ascending order of nominal ratio (see thres_pos)
  float t32[kNumThres];
  float t_final;            // fp32 threshold of the mask-producing evaluation
  uint32_t select_none;     // overflow / bad: select nothing
  uint32_t sorted_ok;       // the ten thresholds are in non-decreasing order (thres0 > 0)
  uint32_t pad2;
  // Top_k
  uint32_t prefix;          // digits of the k-th key decided so far (high bits)
  uint32_t k_rem;           // survivors still to take among keys matching the prefix
  uint32_t n_eq;            // number of keys equal to the k-th key
  uint32_t rank_ties;       // 1 if only some of the equal keys are kept (needs index order)
  uint32_t cursor;          // output slots handed out so far (starts after the ordered part)
  uint32_t pad1;
};

struct Args {
  int32_t L;          // segments (1 for the flat calls)
  int32_t inplace;    // acc == residual
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
  uint32_t* tile_counts;  // [kNumThres][max_tiles]
  uint32_t* tile_base;    // [max_tiles]
  uint32_t* hist;         // [L][hist_copies][256]
  uint32_t* tie_base;     // [max_tiles]
  uint32_t hist_copies;   // replicas of each segment's histogram (spreads the atomics)
  uint32_t max_tiles;
  int32_t ddof;
  double tail_div;
};

// Tile j of a segment covers the absolute range [base + j*kTile, base + (j+1)*kTile) cut to
// [start, end), with base = start rounded down to a multiple of 4 so that full float4 slots
// are 16-byte aligned whatever the segment's start.
__host__ __device__ inline int64_t seg_base(int64_t start) { return start & ~int64_t(3); }
__host__ __device__ inline uint32_t seg_ntiles(int64_t start, int64_t end) {
  return (uint32_t)((end - seg_base(start) + kTile - 1) / kTile);
}

struct Tile {
  int seg;
  int64_t tbase;   // absolute index of the tile's first slot (multiple of 4)
  int64_t lo, hi;  // valid absolute range of this tile
  bool full;       // every slot of the tile is inside [lo, hi)
};

// Maps a tile id to its segment and range.  Flat calls: one segment starting at 0.
template <bool SEG>
__device__ inline bool locate_tile(const Args& a, uint32_t t, Tile* out) {
  if (!SEG) {
    const int64_t tb = (int64_t)t * kTile;
    if (tb >= a.d_total) return false;
    out->seg = 0;
    out->tbase = tb;
    out->lo = tb;
    out->hi = (tb + kTile < a.d_total) ? tb + kTile : a.d_total;
    out->full = (tb + kTile <= a.d_total);
    return true;
  }
  const uint32_t* ts = a.tile_start;
  if (t >= ts[a.L]) return false;
  int lo = 0, hi = a.L;  // largest s with ts[s] <= t
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (ts[mid] <= t) lo = mid; else hi = mid;
  }
  const SegCtrl& c = a.ctrl[lo];
  const int64_t tb = seg_base(c.start) + (int64_t)(t - c.tile0) * kTile;
  out->seg = lo;
  out->tbase = tb;
  out->lo = tb > c.start ? tb : c.start;
  out->hi = (tb + kTile < c.end) ? tb + kTile : c.end;
  out->full = (tb >= c.start) && (tb + kTile <= c.end);
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
