// Exact Top_k (Sec. 1 definition) by radix select over the bit pattern of |acc|: four digit
// passes (8, 8, 8, 7 bits, most significant first) with per-wave histograms in LDS, a digit
// choice after each pass, then compaction of {key > T} plus the lowest-index ties.  This file
// holds the building blocks (digit layout, histogram flush, the accumulate kernel with the first
// digit's histogram, tie counting, one chunk of the cursor-based compaction) and the general
// twelve-launch form with one single-workgroup "select" kernel per segment after each pass; it
// serves layer-wise calls in place and flat calls whose forced tiling exceeds the fused forms'
// tables.  The forms normally used are in topk_filter.h (flat), topk_seg.h (layer-wise) and
// topk_flat.h (flat, in place).
// Global atomics on one address cost tens of nanoseconds each on this chip, so the global
// histogram is replicated and the output slots of the bulk of the survivors come from a scan of
// per-tile counts; only the few survivors that share the k-th key's leading 24 bits take their
// slots from an atomic cursor.
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

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_topk_accum_hist(const Args a) {
  __shared__ uint32_t h[kWaves][256];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  __syncthreads();
  Span sp_;
  if (!locate_span<SEG>(a, blockIdx.x, &sp_)) return;
  if (SEG && a.ctrl[sp_.seg].bad) return;
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

template <bool SEG, bool LAST>
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
  if (!locate_span<SEG>(a, tile, &sp_)) return;
  const SegCtrl& c = a.ctrl[sp_.seg];
  if (SEG && (c.bad || c.select_none)) return;
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
// descending digit order.  After the last pass the same block turns the per-tile counts of
// sure survivors into their first output slots.
template <bool SEG>
__global__ __launch_bounds__(kFinBlock) void k_topk_select(const Args a, int pass) {
  __shared__ uint32_t lds_scan[kFinWaves];
  __shared__ uint32_t stage[kFinBlock * (kScanPer + 1)];
  const int s = blockIdx.x;
  SegCtrl& c = a.ctrl[s];
  if (SEG && (c.bad || c.select_none)) return;
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
  if (pass == kDigits - 1) {
    const uint32_t tile0 = SEG ? c.tile0 : 0u;
    const uint32_t ntiles = SEG ? c.ntiles : seg_ntiles(0, a.d_total, a.tile_chunks);
    const uint32_t sure = scan_tiles(a.tile_counts + tile0, ntiles, a.tile_base + tile0, stage, lds_scan);
    if (threadIdx.x == 0) c.cursor = sure;  // the other survivors take slots from here on
  }
}

// ---- ties: when only some of the keys equal to T are kept, rank them by index ----------------
template <bool FULL>
__device__ inline uint32_t tie_count_chunk(const Args& a, const Tile& t, uint32_t T) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  uint32_t n = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i)
    n += ((FULL || ((valid >> i) & 1u)) && mag_key(v[i]) == T) ? 1u : 0u;
  return n;
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_topk_tie_count(const Args a) {
  __shared__ uint32_t lds[kWaves];
  Span sp_;
  if (!locate_span<SEG>(a, blockIdx.x, &sp_)) return;
  const SegCtrl& c = a.ctrl[sp_.seg];
  if ((SEG && (c.bad || c.select_none)) || !c.rank_ties) return;
  uint32_t n = 0;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    n += t.full ? tie_count_chunk<true>(a, t, c.prefix) : tie_count_chunk<false>(a, t, c.prefix);
  }
  n = wave_sum(n);
  if (lane_id() == 0) lds[wave_id()] = n;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t s = 0;
    for (int w = 0; w < kWaves; ++w) s += lds[w];
    a.tile_counts[(size_t)a.max_tiles + blockIdx.x] = s;
  }
}

template <bool SEG>
__global__ __launch_bounds__(kFinBlock) void k_topk_tie_scan(const Args a) {
  __shared__ uint32_t lds_scan[kFinWaves];
  __shared__ uint32_t stage[kFinBlock * (kScanPer + 1)];
  const int s = blockIdx.x;
  const SegCtrl& c = a.ctrl[s];
  if ((SEG && (c.bad || c.select_none)) || !c.rank_ties) return;
  const uint32_t tile0 = SEG ? c.tile0 : 0u;
  const uint32_t ntiles = SEG ? c.ntiles : seg_ntiles(0, a.d_total, a.tile_chunks);
  scan_tiles(a.tile_counts + (size_t)a.max_tiles + tile0, ntiles, a.tie_base + tile0, stage, lds_scan);
}

// ---- T5: compaction of {key > T} and the kept ties, residual write ---------------------------
// Survivors whose leading 24 bits exceed T's go, in index order, to the slots the scan assigned
// to their tile.  Survivors that share T's leading 24 bits (normally a handful in the whole
// vector) take theirs from the segment's cursor, one reservation per chunk that has any.
struct TopkSel {
  uint32_t T, take;       // the k-th key; ties to keep
  bool rank_ties, none;
  int64_t out0, cap;
  uint32_t sure_run;      // sure survivors of this tile's earlier chunks
  uint32_t tie_run;       // ties met so far in index order (this tile's base + earlier chunks)
  uint32_t tile_sure0;    // first output slot of this tile's sure survivors
};

template <bool FULL, bool NORMS>
__device__ inline void topk_compact_chunk(const Args& a, const Tile& t, SegCtrl& c, TopkSel& k,
                                          uint32_t* lds, uint32_t* lds_base, NormAcc& norms) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  const uint32_t T = k.T;
  uint32_t sure = 0, near = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    if ((FULL || ((valid >> i) & 1u)) && !k.none) {
      const uint32_t key = mag_key(v[i]);
      sure |= ((key >> 7) > (T >> 7) ? 1u : 0u) << i;
      near |= (((key >> 7) == (T >> 7)) && key > T ? 1u : 0u) << i;
      eq |= (key == T ? 1u : 0u) << i;
    }
  }
  uint32_t first[kSlots];
  const uint32_t n_sure = tile_rank(sure, lds, first);
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    uint32_t r = k.tile_sure0 + k.sure_run + first[j];
    const int64_t i0 = slot_index(t, j);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if ((sure >> (4 * j + q)) & 1u) {
        if ((int64_t)r < k.cap) {
          a.out_idx[k.out0 + r] = (uint32_t)(i0 + q);
          a.out_val[k.out0 + r] = v[4 * j + q];
        }
        ++r;
      }
    }
  }
  k.sure_run += n_sure;
  // the rest: same leading bits as T.  Block-uniform early out when the chunk has none.
  if (__syncthreads_or((near | eq) != 0)) {
    if (k.rank_ties) {
      // keep a tie only if fewer than `take` ties precede it in index order
      const uint32_t n_eq = tile_rank(eq, lds, first);
      uint32_t kept = 0;
#pragma unroll
      for (int j = 0; j < kSlots; ++j) {
        uint32_t r = k.tie_run + first[j];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if ((eq >> (4 * j + q)) & 1u) {
            if (r < k.take) kept |= 1u << (4 * j + q);
            ++r;
          }
        }
      }
      eq = kept;
      k.tie_run += n_eq;
      __syncthreads();
    }
    near |= eq;
    const uint32_t n_near = tile_rank(near, lds, first);
    if (n_near != 0) {
      if (threadIdx.x == 0) *lds_base = atomicAdd(&c.cursor, n_near);
      __syncthreads();
      const uint32_t base = *lds_base;
#pragma unroll
      for (int j = 0; j < kSlots; ++j) {
        uint32_t r = base + first[j];
        const int64_t i0 = slot_index(t, j);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if ((near >> (4 * j + q)) & 1u) {
            if ((int64_t)r < k.cap) {
              a.out_idx[k.out0 + r] = (uint32_t)(i0 + q);
              a.out_val[k.out0 + r] = v[4 * j + q];
            }
            ++r;
          }
        }
      }
    }
  } else {
    near = 0;
  }
  const uint32_t sel = sure | near;
  if (NORMS) norm_accumulate(norms, v, valid, sel);
  if (a.inplace) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if ((sel >> i) & 1u) a.resid[slot_index(t, i >> 2) + (i & 3)] = 0.0f;
  } else {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if ((sel >> i) & 1u) v[i] = 0.0f;
    store_tile<FULL>(a.resid, t, v, valid);
  }
  __syncthreads();  // lds and lds_base are reused by the next chunk
}

template <bool SEG, bool NORMS>
__global__ __launch_bounds__(kBlock) void k_topk_compact(const Args a) {
  __shared__ uint32_t lds[kSlots * kWaves];
  __shared__ double lds_n[2 * kWaves];
  __shared__ uint32_t lds_base;
  Span sp_;
  if (!locate_span<SEG>(a, blockIdx.x, &sp_)) return;
  SegCtrl& c = a.ctrl[sp_.seg];
  if (SEG && c.bad) return;
  TopkSel k;
  k.T = c.prefix;
  k.take = c.k_rem;
  k.rank_ties = c.rank_ties != 0;
  k.none = SEG && c.select_none != 0;
  k.out0 = SEG ? c.out_base : 0;
  k.cap = SEG ? c.cap : a.flat_cap;
  k.sure_run = 0;
  k.tie_run = k.rank_ties ? a.tie_base[blockIdx.x] : 0u;
  k.tile_sure0 = a.tile_base[blockIdx.x];
  NormAcc norms = {0.0, 0.0};
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) topk_compact_chunk<true, NORMS>(a, t, c, k, lds, &lds_base, norms);
    else topk_compact_chunk<false, NORMS>(a, t, c, k, lds, &lds_base, norms);
  }
  if (NORMS) store_norm_partial(a, norms, blockIdx.x, lds_n);
}

}  // namespace sp
