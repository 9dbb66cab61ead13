// Exact Top_k (Sec. 1 definition) by radix select over the bit pattern of |acc|: four digit
// passes (8, 8, 8, 7 bits, most significant first) with per-wave histograms in LDS, a
// per-segment digit choice, then compaction of {key > T} plus the lowest-index ties.
#pragma once
#include "common.h"
#include "tile_io.h"

namespace sp {

constexpr int kDigits = 4;
__device__ __host__ inline int digit_shift(int pass) { return pass == 0 ? 23 : pass == 1 ? 15 : pass == 2 ? 7 : 0; }
__device__ __host__ inline int digit_bits(int pass) { return pass == 3 ? 7 : 8; }

constexpr int kStage = 2048;  // pairs a block buffers in LDS between output reservations

// Adds this block's per-wave LDS histograms into segment s's global histogram and clears them.
__device__ inline void flush_hist(const Args& a, int s, uint32_t (*h)[256]) {
  __syncthreads();
  const int bin = threadIdx.x;  // kBlock == 256 bins
  uint32_t v = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    v += h[w][bin];
    h[w][bin] = 0;
  }
  if (v) atomicAdd(&a.hist[(size_t)s * 256 + bin], v);
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
  int cur = -1;
  for (uint32_t tid = blockIdx.x;; tid += gridDim.x) {
    Tile t;
    if (!locate_tile<SEG>(a, tid, &t)) break;
    if (SEG && a.ctrl[t.seg].bad) continue;
    if (t.seg != cur) {
      if (cur >= 0) flush_hist(a, cur, h);
      cur = t.seg;
    }
    if (t.full) accum_hist_tile<true>(a, t, h[wave_id()]);
    else accum_hist_tile<false>(a, t, h[wave_id()]);
  }
  if (cur >= 0) flush_hist(a, cur, h);
}

// ---- T3: histogram of digit `pass` over the keys whose higher digits equal the prefix --------
template <bool FULL>
__device__ inline void hist_tile(const Args& a, const Tile& t, int pass, uint32_t prefix,
                                 uint32_t* h) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  const int hi_shift = digit_shift(pass - 1);
  const int shift = digit_shift(pass);
  const uint32_t mask = (1u << digit_bits(pass)) - 1u;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const uint32_t key = mag_key(v[i]);
    if ((FULL || ((valid >> i) & 1u)) && (key >> hi_shift) == prefix)
      atomicAdd(&h[(key >> shift) & mask], 1u);
  }
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_topk_hist(const Args a, int pass) {
  __shared__ uint32_t h[kWaves][256];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  __syncthreads();
  int cur = -1;
  uint32_t prefix = 0;
  for (uint32_t tid = blockIdx.x;; tid += gridDim.x) {
    Tile t;
    if (!locate_tile<SEG>(a, tid, &t)) break;
    if (SEG && (a.ctrl[t.seg].bad || a.ctrl[t.seg].select_none)) continue;
    if (t.seg != cur) {
      if (cur >= 0) flush_hist(a, cur, h);
      cur = t.seg;
      prefix = a.ctrl[cur].prefix;
    }
    if (t.full) hist_tile<true>(a, t, pass, prefix, h[wave_id()]);
    else hist_tile<false>(a, t, pass, prefix, h[wave_id()]);
  }
  if (cur >= 0) flush_hist(a, cur, h);
}

// ---- T2: per segment, pick the digit holding the k_rem-th largest key ------------------------
template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_topk_select(const Args a, int pass) {
  __shared__ uint32_t lds_scan[kWaves + 1];
  const int s = blockIdx.x;
  SegCtrl& c = a.ctrl[s];
  if (SEG && (c.bad || c.select_none)) return;
  const uint32_t nbins = 1u << digit_bits(pass);
  const uint32_t bin = 255u - threadIdx.x;  // thread order = descending digit
  uint32_t* hp = a.hist + (size_t)s * 256 + bin;
  const uint32_t v = bin < nbins ? *hp : 0u;
  const uint32_t k_rem = c.k_rem;
  const uint32_t prefix = c.prefix;
  uint32_t total;
  const uint32_t above = block_exclusive_scan(v, lds_scan, &total);  // keys in higher digits
  *hp = 0;  // ready for the next pass
  if (above < k_rem && k_rem <= above + v) {
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

// ---- ties: when only some of the keys equal to T are kept, rank them by index ----------------
template <bool FULL>
__device__ inline void tie_count_tile(const Args& a, const Tile& t, uint32_t tile_id, uint32_t T,
                                      uint32_t* lds) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  uint32_t n = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i)
    n += ((FULL || ((valid >> i) & 1u)) && mag_key(v[i]) == T) ? 1u : 0u;
  n = wave_sum(n);
  if (lane_id() == 0) lds[wave_id()] = n;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t s = 0;
    for (int w = 0; w < kWaves; ++w) s += lds[w];
    a.tile_counts[(size_t)tile_id * kNumThres] = s;
  }
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_topk_tie_count(const Args a) {
  __shared__ uint32_t lds[kWaves];
  Tile t;
  if (!locate_tile<SEG>(a, blockIdx.x, &t)) return;
  const SegCtrl& c = a.ctrl[t.seg];
  if ((SEG && (c.bad || c.select_none)) || !c.rank_ties) return;
  if (t.full) tie_count_tile<true>(a, t, blockIdx.x, c.prefix, lds);
  else tie_count_tile<false>(a, t, blockIdx.x, c.prefix, lds);
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_topk_tie_scan(const Args a) {
  __shared__ uint32_t lds_scan[kWaves + 1];
  const int s = blockIdx.x;
  const SegCtrl& c = a.ctrl[s];
  if ((SEG && (c.bad || c.select_none)) || !c.rank_ties) return;
  const uint32_t tile0 = SEG ? c.tile0 : 0u;
  const uint32_t ntiles = SEG ? c.ntiles : seg_ntiles(0, a.d_total);
  const uint32_t per = (ntiles + kBlock - 1) / kBlock;
  const uint32_t b = threadIdx.x * per;
  const uint32_t e = (b + per < ntiles) ? b + per : ntiles;
  uint32_t sum = 0;
  for (uint32_t i = b; i < e; ++i) sum += a.tile_counts[(size_t)(tile0 + i) * kNumThres];
  uint32_t total;
  uint32_t run = block_exclusive_scan(sum, lds_scan, &total);
  for (uint32_t i = b; i < e; ++i) {
    a.tile_base[tile0 + i] = run;
    run += a.tile_counts[(size_t)(tile0 + i) * kNumThres];
  }
}

// ---- T5: compaction of {key > T} and the kept ties, residual write ---------------------------
struct Stage {
  uint32_t idx[kStage];
  float val[kStage];
  uint32_t scan[kWaves + 1];
  uint32_t tie[kSlots * kWaves];
  uint32_t base;
};

// Hands the staged pairs to segment s's output range: one atomic reservation per flush.
template <bool SEG>
__device__ inline void flush_stage(const Args& a, int s, Stage& st, uint32_t staged) {
  __syncthreads();
  if (staged == 0) return;
  SegCtrl& c = a.ctrl[s];
  if (threadIdx.x == 0) st.base = atomicAdd(&c.cursor, staged);
  __syncthreads();
  const uint32_t base = st.base;
  const int64_t out0 = SEG ? c.out_base : 0;
  const int64_t cap = SEG ? c.cap : a.flat_cap;
  for (uint32_t i = threadIdx.x; i < staged; i += kBlock) {
    if ((int64_t)(base + i) < cap) {
      a.out_idx[out0 + base + i] = st.idx[i];
      a.out_val[out0 + base + i] = st.val[i];
    }
  }
  __syncthreads();
}

template <bool SEG, bool FULL>
__device__ inline uint32_t topk_compact_tile(const Args& a, const Tile& t, uint32_t tile_id,
                                             Stage& st, uint32_t staged) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  SegCtrl& c = a.ctrl[t.seg];
  const uint32_t T = c.prefix;
  const uint32_t take = c.k_rem;  // ties to keep
  const bool rank_ties = c.rank_ties != 0;
  const bool none = SEG && c.select_none != 0;
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    if ((FULL || ((valid >> i) & 1u)) && !none) {
      const uint32_t key = mag_key(v[i]);
      gt |= (key > T ? 1u : 0u) << i;
      eq |= (key == T ? 1u : 0u) << i;
    }
  }
  if (rank_ties) {
    // keep a tie only if fewer than `take` ties precede it in index order
    uint32_t below[kSlots];
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      uint32_t tot = 0, mine = 0;
#pragma unroll
      for (int cpt = 0; cpt < 4; ++cpt) {
        const uint64_t m = __ballot((eq >> (4 * j + cpt)) & 1u);
        tot += (uint32_t)__builtin_popcountll(m);
        mine += lanes_below(m);
      }
      below[j] = mine;
      if (lane_id() == 0) st.tie[j * kWaves + wave_id()] = tot;
    }
    __syncthreads();
    uint32_t run = a.tile_base[tile_id];
    uint32_t kept = 0;
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        if (w == wave_id()) {
          uint32_t r = run + below[j];
#pragma unroll
          for (int cpt = 0; cpt < 4; ++cpt) {
            if ((eq >> (4 * j + cpt)) & 1u) {
              if (r < take) kept |= 1u << (4 * j + cpt);
              ++r;
            }
          }
        }
        run += st.tie[j * kWaves + w];
      }
    }
    eq = kept;
    __syncthreads();
  }
  const uint32_t sel = gt | eq;
  uint32_t total;
  uint32_t pos = block_exclusive_scan((uint32_t)__popc(sel), st.scan, &total);
  if (total != 0) {
    if (staged + total > (uint32_t)kStage) {
      flush_stage<SEG>(a, t.seg, st, staged);
      staged = 0;
    }
    if (total > (uint32_t)kStage) {  // dense tile: reserve and write straight to the output
      if (threadIdx.x == 0) st.base = atomicAdd(&c.cursor, total);
      __syncthreads();
      const uint32_t base = st.base;
      const int64_t out0 = SEG ? c.out_base : 0;
      const int64_t cap = SEG ? c.cap : a.flat_cap;
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) {
        if ((sel >> i) & 1u) {
          if ((int64_t)(base + pos) < cap) {
            a.out_idx[out0 + base + pos] = (uint32_t)(slot_index(t, i >> 2) + (i & 3));
            a.out_val[out0 + base + pos] = v[i];
          }
          ++pos;
        }
      }
      __syncthreads();
    } else {
      pos += staged;
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) {
        if ((sel >> i) & 1u) {
          st.idx[pos] = (uint32_t)(slot_index(t, i >> 2) + (i & 3));
          st.val[pos] = v[i];
          ++pos;
        }
      }
      staged += total;
    }
  }
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
  return staged;
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_topk_compact(const Args a) {
  __shared__ Stage st;
  int cur = -1;
  uint32_t staged = 0;
  for (uint32_t tid = blockIdx.x;; tid += gridDim.x) {
    Tile t;
    if (!locate_tile<SEG>(a, tid, &t)) break;
    if (SEG && a.ctrl[t.seg].bad) continue;
    if (t.seg != cur) {
      if (cur >= 0) flush_stage<SEG>(a, cur, st, staged);
      staged = 0;
      cur = t.seg;
    }
    if (t.full) staged = topk_compact_tile<SEG, true>(a, t, tid, st, staged);
    else staged = topk_compact_tile<SEG, false>(a, t, tid, st, staged);
  }
  if (cur >= 0) flush_stage<SEG>(a, cur, st, staged);
}

}  // namespace sp
