// Exact Top_k (Sec. 1 definition) by radix select over the bit pattern of |acc|: four digit
// passes (8, 8, 8, 7 bits, most significant first) with per-wave histograms in LDS, a digit
// choice after each pass, then compaction of {key > T} plus the lowest-index ties.  This file
// holds the building blocks (digit layout, histogram flush, the accumulate kernel with the first
// digit's histogram, one chunk of the ordered compaction) and the eleven-launch form of the
// layer-wise calls in place: one single-workgroup "select" kernel per segment after each pass,
// one more pass over acc that counts every tile's survivors and ties once the k-th key T is
// known, and a per-segment scan of those counts.  The other forms are in topk_filter.h (flat),
// topk_seg.h (layer-wise, separate acc) and topk_flat.h (flat, in place).
// Global atomics on one address cost tens of nanoseconds each on this chip, so the global
// histogram is replicated, and every survivor's output slot comes from counts (per-tile counts,
// scanned or totalled per group): no output cursor anywhere, so the pairs of every form come
// out in ascending index order, the same from run to run.
#pragma once
#include "common.h"
#include "gaussiank.h"
#include "tile_io.h"

namespace sp {

constexpr int kDigits = 4;
__device__ __host__ inline int digit_shift(int pass) { return pass == 0 ? 23 : pass == 1 ? 15 : pass == 2 ? 7 : 0; }
__device__ __host__ inline int digit_bits(int pass) { return pass == 3 ? 7 : 8; }

// Adds this block's per-wave LDS histograms into one replica of segment s's global histogram
// and clears them.
__device__ inline void flush_hist(const Args& a, int s, uint32_t (*h)[256]) {
  __syncthreads();
  const int bin = threadIdx.x;  // kBlock == 256 bins
  uint32_t v = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    v += h[w][bin];
    h[w][bin] = 0;
  }
  const uint32_t copy = blockIdx.x % a.hist_copies;
  if (v) atomicAdd(&a.hist[((size_t)s * a.hist_copies + copy) * 256 + bin], v);
  __syncthreads();
}

// ---- T1: acc = grad + residual, histogram of the top digit (the exponent byte) ---------------
template <bool FULL>
__device__ inline void accum_hist_tile(const Args& a, const Tile& t, uint32_t* h) {
  float g[kPerThread], e[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.grad, t, g);
  load_tile<FULL>(a.resid, t, e);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) g[i] = g[i] + e[i];
  store_tile<FULL>(a.acc, t, g, valid);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i)
    if (FULL || ((valid >> i) & 1u)) atomicAdd(&h[mag_key(g[i]) >> 23], 1u);
}

__global__ __launch_bounds__(kBlock) void k_topk_accum_hist(const Args a) {
  __shared__ uint32_t h[kWaves][256];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  __syncthreads();
  Span sp_;
  if (!locate_span<true>(a, blockIdx.x, &sp_)) return;
  if (a.ctrl[sp_.seg].bad) return;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) accum_hist_tile<true>(a, t, h[wave_id()]);
    else accum_hist_tile<false>(a, t, h[wave_id()]);
  }
  flush_hist(a, sp_.seg, h);
}

// ---- T3: histogram of digit `pass` over the keys whose higher digits equal the prefix --------
// The last pass also counts, per tile, the keys whose leading 24 bits already exceed the
// prefix: they are survivors whatever the last digit turns out to be.
template <bool FULL, bool LAST>
__device__ inline uint32_t hist_tile(const Args& a, const Tile& t, int pass, uint32_t prefix,
                                     uint32_t* h) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  const int hi_shift = digit_shift(pass - 1);
  const int shift = digit_shift(pass);
  const uint32_t mask = (1u << digit_bits(pass)) - 1u;
  uint32_t sure = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const uint32_t key = mag_key(v[i]);
    const bool ok = FULL || ((valid >> i) & 1u);
    if (ok && (key >> hi_shift) == prefix) atomicAdd(&h[(key >> shift) & mask], 1u);
    if (LAST) sure += (ok && (key >> hi_shift) > prefix) ? 1u : 0u;
  }
  return sure;
}

template <bool LAST>
__global__ __launch_bounds__(kBlock) void k_topk_hist(const Args a, int pass) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sure[kWaves];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  __syncthreads();
  Span sp_;
  // odd passes walk the tiles backwards: each pass starts where the previous one ended, on the
  // part of acc most likely still to sit in the last-level cache
  const uint32_t tile = (pass & 1) ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  if (!locate_span<true>(a, tile, &sp_)) return;
  const SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad || c.select_none) return;
  const uint32_t prefix = c.prefix;
  uint32_t sure = 0;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) sure += hist_tile<true, LAST>(a, t, pass, prefix, h[wave_id()]);
    else sure += hist_tile<false, LAST>(a, t, pass, prefix, h[wave_id()]);
  }
  if (LAST) {
    sure = wave_sum(sure);
    if (lane_id() == 0) lds_sure[wave_id()] = sure;
  }
  flush_hist(a, sp_.seg, h);  // starts with a barrier
  if (LAST && threadIdx.x == 0) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds_sure[w];
    a.tile_counts[tile] = s;
  }
}

// ---- T2: per segment, pick the digit holding the k_rem-th largest key ------------------------
// One workgroup of kFinBlock threads per segment; the first 256 threads own one bin each, in
// descending digit order.
__global__ __launch_bounds__(kFinBlock) void k_topk_select(const Args a, int pass) {
  __shared__ uint32_t lds_scan[kFinWaves];
  const int s = blockIdx.x;
  SegCtrl& c = a.ctrl[s];
  if (c.bad || c.select_none) return;
  const uint32_t nbins = 1u << digit_bits(pass);
  const bool owner = threadIdx.x < 256;
  const uint32_t bin = 255u - (threadIdx.x & 255u);
  uint32_t v = 0;
  if (owner) {
    uint32_t* hp = a.hist + (size_t)s * a.hist_copies * 256 + bin;
    for (uint32_t r0 = 0; r0 < a.hist_copies; r0 += 16) {
      uint32_t x[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) x[u] = (r0 + u < a.hist_copies) ? hp[(size_t)(r0 + u) * 256] : 0u;
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        v += x[u];
        if (r0 + u < a.hist_copies) hp[(size_t)(r0 + u) * 256] = 0;  // ready for the next pass
      }
    }
    if (bin >= nbins) v = 0;
  }
  const uint32_t k_rem = c.k_rem;
  const uint32_t prefix = c.prefix;
  uint32_t total;
  const uint32_t above = block_exclusive_scan<kFinWaves>(v, lds_scan, &total);  // keys in higher digits
  if (owner && above < k_rem && k_rem <= above + v) {
    const uint32_t np = (prefix << digit_bits(pass)) | bin;
    const uint32_t nk = k_rem - above;
    c.prefix = np;
    c.k_rem = nk;
    if (pass == kDigits - 1) {
      c.n_eq = v;
      c.rank_ties = v > nk ? 1u : 0u;
      sparsify_result& r = a.result[s];
      r.topk_key = np;
      r.topk_ties_taken = nk;
    }
  }
}

// ---- once T is known: every tile's survivors and keys equal to T ------------------------------
// One more pass over acc.  A tile's count of survivors (row 0) is what the last digit pass left
// there (keys whose leading 24 bits exceed T's) plus the keys above T that share those bits, plus
// the keys equal to T when all of those are kept; when only some are kept (ties are ranked by
// index) the tile's number of keys equal to T goes to row 1.
template <bool FULL>
__device__ inline void near_count_chunk(const Args& a, const Tile& t, uint32_t T, uint32_t& gt,
                                        uint32_t& eq) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const uint32_t key = mag_key(v[i]);
    const bool ok = FULL || ((valid >> i) & 1u);
    gt += (ok && (key >> 7) == (T >> 7) && key > T) ? 1u : 0u;
    eq += (ok && key == T) ? 1u : 0u;
  }
}

__global__ __launch_bounds__(kBlock) void k_topk_tie_count(const Args a) {
  __shared__ uint32_t lds[2 * kWaves];
  Span sp_;
  if (!locate_span<true>(a, blockIdx.x, &sp_)) return;
  const SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad || c.select_none) return;
  const uint32_t T = c.prefix;
  const bool rank_ties = c.rank_ties != 0;
  uint32_t gt = 0, eq = 0;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) near_count_chunk<true>(a, t, T, gt, eq);
    else near_count_chunk<false>(a, t, T, gt, eq);
  }
  gt = wave_sum(gt);
  eq = wave_sum(eq);
  if (lane_id() == 0) {
    lds[2 * wave_id()] = gt;
    lds[2 * wave_id() + 1] = eq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t g = 0, e = 0;
    for (int w = 0; w < kWaves; ++w) {
      g += lds[2 * w];
      e += lds[2 * w + 1];
    }
    a.tile_counts[blockIdx.x] += g + (rank_ties ? 0u : e);
    if (rank_ties) a.tile_counts[(size_t)a.max_tiles + blockIdx.x] = e;
  }
}

// Per segment: the tiles' first output slots (and, when ties are ranked, the number of keys equal
// to T before each tile) by a scan of the counts above.
__global__ __launch_bounds__(kFinBlock) void k_topk_tie_scan(const Args a) {
  __shared__ uint32_t lds_scan[kFinWaves];
  __shared__ uint32_t stage[kFinBlock * (kScanPer + 1)];
  const int s = blockIdx.x;
  const SegCtrl& c = a.ctrl[s];
  if (c.bad || c.select_none) return;
  const uint32_t tile0 = c.tile0, ntiles = c.ntiles;
  scan_tiles(a.tile_counts + tile0, ntiles, a.tile_base + tile0, stage, lds_scan);
  if (c.rank_ties)
    scan_tiles(a.tile_counts + (size_t)a.max_tiles + tile0, ntiles, a.tie_base + tile0, stage, lds_scan);
}

// ---- compaction in index order, residual write -------------------------------------------------
// `out0`, `cap`: first slot and capacity of the output range; `none`: select nothing.
struct OrderedSel {
  uint32_t T, take;
  bool rank_ties, none;
  int64_t out0, cap;
};
template <bool FULL, bool NORMS, bool STREAM = false>  // STREAM: see compact_chunk
__device__ inline void ordered_compact_chunk(const Args& a, const Tile& t, const OrderedSel& o,
                                             uint32_t& out_run, uint32_t& tie_run,
                                             uint32_t* lds, NormAcc& norms) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL, STREAM>(a.acc, t, v);
  const uint32_t T = o.T, take = o.take;
  const bool rank_ties = o.rank_ties;
  uint32_t sel = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    if ((FULL || ((valid >> i) & 1u)) && !o.none) {
      const uint32_t key = mag_key(v[i]);
      sel |= ((key > T || (!rank_ties && key == T)) ? 1u : 0u) << i;
      eq |= ((rank_ties && key == T) ? 1u : 0u) << i;
    }
  }
  uint32_t first[kSlots];
  if (rank_ties && __syncthreads_or(eq != 0)) {
    // keep a tie only if fewer than `take` ties precede it in index order
    const uint32_t n_eq = tile_rank(eq, lds, first);
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      uint32_t r = tie_run + first[j];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if ((eq >> (4 * j + q)) & 1u) {
          if (r < take) sel |= 1u << (4 * j + q);
          ++r;
        }
      }
    }
    tie_run += n_eq;
    __syncthreads();  // lds is reused below
  }
  const uint32_t n_sel = tile_rank(sel, lds, first);
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    uint32_t r = out_run + first[j];
    const int64_t i0 = slot_index(t, j);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if ((sel >> (4 * j + q)) & 1u) {
        if ((int64_t)r < o.cap) {
          a.out_idx[o.out0 + r] = (uint32_t)(i0 + q);
          a.out_val[o.out0 + r] = v[4 * j + q];
        }
        ++r;
      }
    }
  }
  out_run += n_sel;
  if (NORMS) norm_accumulate(norms, v, valid, sel);
  if (a.inplace) {  // acc is the residual: only the selected entries change
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if ((sel >> i) & 1u) a.resid[slot_index(t, i >> 2) + (i & 3)] = 0.0f;
  } else {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if ((sel >> i) & 1u) v[i] = 0.0f;
    store_tile<FULL>(a.resid, t, v, valid);
  }
  __syncthreads();  // lds is reused by the next chunk
}

template <bool NORMS>
__global__ __launch_bounds__(kBlock) void k_topk_compact(const Args a) {
  __shared__ uint32_t lds[kSlots * kWaves];
  __shared__ double lds_n[2 * kWaves];
  Span sp_;
  if (!locate_span<true>(a, blockIdx.x, &sp_)) return;
  const SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad) return;
  const OrderedSel o = {c.prefix, c.k_rem, c.rank_ties != 0, c.select_none != 0, c.out_base, c.cap};
  // ties before the tile are capped at the number kept: the lowest indices win
  uint32_t tie_run = o.rank_ties ? a.tie_base[blockIdx.x] : 0u;
  uint32_t out_run = a.tile_base[blockIdx.x] + (tie_run < o.take ? tie_run : o.take);
  NormAcc norms = {0.0, 0.0};
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) ordered_compact_chunk<true, NORMS>(a, t, o, out_run, tie_run, lds, norms);
    else ordered_compact_chunk<false, NORMS>(a, t, o, out_run, tie_run, lds, norms);
  }
  if (NORMS) store_norm_partial(a, norms, blockIdx.x, lds_n);
}

}  // namespace sp
