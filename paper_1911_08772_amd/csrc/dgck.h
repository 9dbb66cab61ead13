// DGC_k, the hierarchical-sampling selection the paper compares Gaussian_k with (Sec. 3.3;
// Sec. 4.3 uses a 1 % sample): a top-k on a sample of |acc| gives a threshold, every entry that
// reaches it is kept, and a second top-k runs on the kept entries when they are more than k.
// The paper states no more than that; the sampling rule (one hashed position per stratum of
// `sample_stride` elements), the rank inside the sample (ceil(k m / d)) and ">=" are readings.
//
// Both selections are radix selects over short per-tile key lists, with the machinery of
// topk_filter.h: the accumulate kernel leaves the sampled keys of each tile in the tile's stretch
// of the (idle) residual buffer; three list passes and the prologue of the filter kernel find
// the sample's threshold Ts; the filter kernel, the one further pass over acc, replaces the lists
// by the keys >= Ts; three more list passes and the final kernel find the k-th key among those
// (when they are more than k); the ordered compaction of topk_filter.h writes pairs and residual.
// Eight histogram buffers: 0-3 for the sample's digits, 4-7 for the kept keys'.
//
// From 6 M elements (where the workspace holds the list buffers of topk_list.h) the sample is
// drawn first, straight from g and eps, so that Ts is known when the accumulate pass runs: that
// pass then also writes the residual and lists every entry that reaches Ts, and what follows
// (the digits of the kept keys, the per-tile counts, the compaction) reads those lists, about k
// entries, instead of acc: twelve launches, one pass over the vector.  Should a list run out of
// room (Ts = 0, a sample that sat on the small entries) the later kernels take the bodies
// described above; the launches are the same either way.
#pragma once
#include "common.h"
#include "topk_filter.h"

namespace sp {

constexpr int kDgcHistWords = 2 * kTopkHistWords;
constexpr int kColCand = 2;  // column of group_counts: keys that reach the sample threshold

// Position sampled in stratum j: a 64-bit finaliser of (seed, j) (xor-shift-multiply rounds with
// the SplitMix64 constants), high 32 bits scaled to the stratum's length by a multiply-shift.
__device__ inline int64_t sample_position(const Args& a, int64_t j) {
  uint64_t x = a.sample_seed + (uint64_t)(j + 1) * 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  x ^= x >> 31;
  const int64_t lo = j * a.sample_stride;
  const int64_t rest = a.d_total - lo;
  const uint64_t len = (uint64_t)(rest < a.sample_stride ? rest : a.sample_stride);
  return lo + (int64_t)(((x >> 32) * len) >> 32);
}

// ---- accumulate + sample -----------------------------------------------------------------------
template <bool FULL>
__device__ inline void accum_plain_chunk(const Args& a, const Tile& t) {
  float g[kPerThread], e[kPerThread];
  const uint32_t valid = load_tile<FULL, true>(a.grad, t, g);
  load_tile<FULL>(a.resid, t, e);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) g[i] = g[i] + e[i];
  store_tile<FULL>(a.acc, t, g, valid);
}

__global__ __launch_bounds__(kBlock) void k_dgck_accum_sample(const Args a) {
  __shared__ uint32_t h[256];
  __shared__ uint32_t lds_cursor;
  h[threadIdx.x] = 0;
  if (threadIdx.x == 0) lds_cursor = 0;
  const uint32_t tile = blockIdx.x;
  Span sp_;
  if (!locate_span<false>(a, tile, &sp_)) return;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) accum_plain_chunk<true>(a, t);
    else accum_plain_chunk<false>(a, t);
  }
  // From here on nobody reads this tile's stretch of the residual again, and the tile's acc is
  // visible to the whole workgroup.
  __syncthreads();
  uint32_t* list = tile_candidates(a, tile);
  const int64_t j0 = sp_.lo / a.sample_stride, j1 = (sp_.hi - 1) / a.sample_stride;
  for (int64_t j = j0 + threadIdx.x; j <= j1; j += kBlock) {
    const int64_t p = sample_position(a, j);
    if (p >= sp_.lo && p < sp_.hi) {
      const uint32_t key = mag_key(a.acc[p]);
      list[atomicAdd(&lds_cursor, 1u)] = key;
      atomicAdd(&h[key >> 23], 1u);
    }
  }
  __syncthreads();
  const uint32_t v = h[threadIdx.x];
  if (v) atomicAdd(&pass_hist(a, 0)[(blockIdx.x % kTopkCopies) * 256 + threadIdx.x], v);
  if (threadIdx.x == 0) tile_row(a, kRowCand)[tile] = lds_cursor;
}

// ---- the sample on its own (the form with lists) ------------------------------------------------
// acc[p] = g[p] + eps[p] at the sampled positions (the accumulate pass makes the same fp32 add),
// keys to the head of the list buffer, which is idle until that pass, in stratum order.
constexpr int kSampleBatch = 2;
__device__ inline uint32_t* sample_keys(const Args& a) { return reinterpret_cast<uint32_t*>(a.list); }

__global__ __launch_bounds__(kBlock) void k_dgck_sample(const Args a) {
  __shared__ uint32_t h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int64_t j0 = (int64_t)blockIdx.x * (kBlock * kSampleBatch) + threadIdx.x;
  int64_t p[kSampleBatch];
  float g[kSampleBatch], e[kSampleBatch];
#pragma unroll
  for (int u = 0; u < kSampleBatch; ++u) {
    const int64_t j = j0 + u * kBlock;
    p[u] = sample_position(a, j < a.sample_m ? j : a.sample_m - 1);  // (no load behind a branch)
  }
#pragma unroll
  for (int u = 0; u < kSampleBatch; ++u) g[u] = a.grad[p[u]];
#pragma unroll
  for (int u = 0; u < kSampleBatch; ++u) e[u] = a.resid[p[u]];
  uint32_t* keys = sample_keys(a);
#pragma unroll
  for (int u = 0; u < kSampleBatch; ++u) {
    const int64_t j = j0 + u * kBlock;
    if (j < a.sample_m) {
      const uint32_t key = mag_key(g[u] + e[u]);  // Eq. (2): one fp32 add
      keys[j] = key;
      atomicAdd(&h[key >> 23], 1u);
    }
  }
  __syncthreads();
  const uint32_t v = h[threadIdx.x];
  if (v) atomicAdd(&pass_hist(a, 0)[(blockIdx.x % kTopkCopies) * 256 + threadIdx.x], v);
}

// ---- one digit pass over the per-tile lists ----------------------------------------------------
// stage 1..3: digits 1..3 of the sample (rank sample_k); stage 5..7: digits 1..3 of the kept keys
// (rank k).  Prologue: the previous digit, from histogram buffer stage-1; the choice goes to
// control slot stage-1.  One wave per list.
__global__ __launch_bounds__(kBlock) void k_dgck_lists_hist(const Args a, int stage) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sel[kWaves + 3];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  SegCtrl& c = a.ctrl[0];
  // (the kept keys are all taken, from the lists: there is no k-th key to find among them)
  if ((stage & 4) && a.list && c.list_mode == 2) return;
  const int pass = stage & 3;
  const uint32_t k0 = (uint32_t)((stage & 4) ? a.flat_k : a.sample_k);
  const uint32_t prefix_in = pass == 1 ? 0u : c.sel_prefix[stage - 2];
  const uint32_t k_in = pass == 1 ? k0 : c.sel_krem[stage - 2];
  const Digit dg = choose_digit(pass_hist(a, stage - 1), pass - 1, prefix_in, k_in, lds_sel);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    c.sel_prefix[stage - 1] = dg.prefix;
    c.sel_krem[stage - 1] = dg.k_rem;
  }
  const uint32_t ntiles = seg_ntiles(0, a.d_total, a.tile_chunks);
  const int hi_shift = digit_shift(pass - 1);
  const int shift = digit_shift(pass);
  const uint32_t mask = (1u << digit_bits(pass)) - 1u;
  uint32_t* hw = h[wave_id()];
  if (a.list && !(stage & 4)) {
    // the sample as one array (k_dgck_sample): every workgroup takes stretches of it
    const uint32_t* keys = sample_keys(a);
    const int64_t span = (int64_t)kBlock * kCandBatch;
    for (int64_t b = (int64_t)blockIdx.x * span; b < a.sample_m; b += (int64_t)gridDim.x * span) {
      uint32_t key[kCandBatch];
#pragma unroll
      for (int u = 0; u < kCandBatch; ++u) {
        const int64_t i = b + u * kBlock + threadIdx.x;
        key[u] = keys[i < a.sample_m ? i : a.sample_m - 1];
      }
#pragma unroll
      for (int u = 0; u < kCandBatch; ++u) {
        const bool valid = b + u * kBlock + threadIdx.x < a.sample_m;
        wave_hist_add(hw, (key[u] >> shift) & mask, valid && (key[u] >> hi_shift) == dg.prefix);
      }
    }
  } else if (a.list && c.list_mode) {
    // the kept keys from the accumulate pass's lists; nothing to find when all of them are taken
    if (c.list_mode == 1) list_digit_pass(a, pass, dg.prefix, hw);
  } else {
    for_each_candidate(a, blockIdx.x * kWaves + wave_id(), ntiles, [&](uint32_t key, bool valid) {
      wave_hist_add(hw, (key >> shift) & mask, valid && (key >> hi_shift) == dg.prefix);
    });
  }
  __syncthreads();
  const int bin = threadIdx.x;
  uint32_t v = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) v += h[w][bin];
  if (v) atomicAdd(&pass_hist(a, stage)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
}

// ---- the pass over acc that keeps what reaches the sample's threshold --------------------------
template <bool FULL>
__device__ inline void dgck_filter_chunk(const Args& a, const Tile& t, uint32_t Ts, uint32_t* list,
                                         uint32_t* h, uint32_t* lds_cursor) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  uint32_t cmask = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i)
    cmask |= (((FULL || ((valid >> i) & 1u)) && mag_key(v[i]) >= Ts) ? 1u : 0u) << i;
  if (__ballot(cmask != 0) == 0) return;  // wave-uniform
  const uint32_t n = (uint32_t)__builtin_popcount(cmask);
  const uint32_t inc = wave_inclusive_scan(n);
  uint32_t base = 0;
  if (lane_id() == 63) base = atomicAdd(lds_cursor, inc);
  base = __shfl(base, 63, 64);
  uint32_t pos = base + inc - n;
  if (wave_bins_look_uniform(cmask == 0xFFFFu ? mag_key(v[0]) >> 23 : 256u + lane_id())) {
    // everything kept and the first elements share a bin: constant data, aggregate
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const uint32_t key = mag_key(v[i]);
      list[pos++] = key;
      wave_hist_add(h, key >> 23, true);
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    if ((cmask >> i) & 1u) {
      const uint32_t key = mag_key(v[i]);
      list[pos++] = key;
      atomicAdd(&h[key >> 23], 1u);
    }
  }
}

__global__ __launch_bounds__(kBlock) void k_dgck_filter(const Args a) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sel[kWaves + 3];
  __shared__ uint32_t lds_cursor;
  __shared__ uint32_t lds_lists[2];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  if (threadIdx.x == 0) lds_cursor = 0;
  const uint32_t tile = gridDim.x - 1u - blockIdx.x;
  Span sp_;
  if (!locate_span<false>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[0];
  if (a.list) {
    // the accumulate pass listed the keys that reach Ts (and published Ts).  If no stretch ran
    // out the lists are the kept entries: more than k of them, a second selection follows (way
    // 1: the first digit's histogram from the lists, one wave per tile); otherwise all of them
    // are the result (way 2).
    list_totals(a, lds_lists);
    const uint32_t way = lds_lists[1] != 0 ? 0u : (int64_t)lds_lists[0] > a.flat_k ? 1u : 2u;
    if (tile == 0 && threadIdx.x == 0) c.list_mode = way;
    if (way == 1 && blockIdx.x * kWaves < gridDim.x) {
      list_digit_pass(a, 0, 0u, h[wave_id()]);
      __syncthreads();
      uint32_t v = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) v += h[w][threadIdx.x];
      if (v) atomicAdd(&pass_hist(a, 4)[(blockIdx.x % kTopkCopies) * 256 + threadIdx.x], v);
    }
    if (way != 0) return;
  }
  const Digit dg = choose_digit(pass_hist(a, 3), 3, c.sel_prefix[2], c.sel_krem[2], lds_sel);
  const uint32_t Ts = dg.prefix;  // the sample's threshold: a whole 31-bit key
  if (tile == 0 && threadIdx.x == 0) {
    c.sel_prefix[3] = Ts;
    c.sel_krem[3] = dg.k_rem;
  }
  uint32_t* list = tile_candidates(a, tile);
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) dgck_filter_chunk<true>(a, t, Ts, list, h[wave_id()], &lds_cursor);
    else dgck_filter_chunk<false>(a, t, Ts, list, h[wave_id()], &lds_cursor);
  }
  __syncthreads();
  {
    const int bin = threadIdx.x;
    uint32_t v = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) v += h[w][bin];
    if (v) atomicAdd(&pass_hist(a, 4)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
  }
  if (threadIdx.x == 0) {
    const uint32_t n = lds_cursor;
    tile_row(a, kRowCand)[tile] = n;
    if (n) atomicAdd(&a.group_counts[(tile / kGroupTiles) * kNumThres + kColCand], n);
  }
}

// ---- after the last list pass ------------------------------------------------------------------
// n = number of kept keys.  n <= k: all of them are the result.  Otherwise the last digit of the
// k-th key among them, the ties to keep, and the per-tile counts the compaction needs.
__global__ __launch_bounds__(kBlock) void k_dgck_final(const Args a) {
  __shared__ uint32_t lds_sel[kWaves + 3];
  __shared__ uint32_t lds_n;
  __shared__ uint32_t lds_lists[2];
  SegCtrl& c = a.ctrl[0];
  const uint32_t ntiles = seg_ntiles(0, a.d_total, a.tile_chunks);
  const bool listed = a.list && c.list_mode != 0;
  if (listed) {
    list_totals(a, lds_lists);  // barrier
    if (threadIdx.x == 0) lds_n = lds_lists[0];
  } else if (wave_id() == 0) {
    const uint32_t ngroups = (ntiles + kGroupTiles - 1) / kGroupTiles;
    uint32_t g = (uint32_t)lane_id() < ngroups ? a.group_counts[lane_id() * kNumThres + kColCand] : 0u;
    g = wave_sum(g);
    if (lane_id() == 0) lds_n = g;
  }
  const Digit dg = choose_digit(pass_hist(a, 7), 3, c.sel_prefix[6], c.sel_krem[6], lds_sel);  // barriers
  const uint32_t n = lds_n;
  const uint32_t Ts = c.sel_prefix[3];
  const bool second = n > (uint32_t)a.flat_k;
  const uint32_t T = second ? dg.prefix : Ts;
  const bool rank_ties = second && dg.count > dg.k_rem;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    c.topk_key = T;
    c.topk_take = second ? dg.k_rem : 0u;
    c.n_eq = second ? dg.count : 0u;
    c.rank_ties = rank_ties ? 1u : 0u;
    sparsify_result& r = a.result[0];
    r.nnz = second ? (uint32_t)a.flat_k : n;
    r.rounds = second ? 2u : 1u;
    r.count[0] = n;
    r.count[1] = (uint32_t)a.sample_m;
    r.count[2] = (uint32_t)a.sample_k;
    r.thres_f32 = __uint_as_float(Ts);
    r.thres = (double)__uint_as_float(Ts);
    r.topk_key = T;
    r.topk_ties_taken = second ? dg.k_rem : 0u;
    if (a.list) r.flags = listed ? SPARSIFY_F_SHORTLIST : SPARSIFY_F_SHORTLIST_MISS;  // which way, no result
  }
  if (listed) {
    list_tile_counts<kGroupTiles>(a, T, rank_ties);
    return;
  }
  const uint32_t tile = blockIdx.x * kWaves + wave_id();
  uint32_t gt = 0, eq = 0;
  for_each_candidate(a, tile, ntiles, [&](uint32_t key, bool valid) {
    gt += (valid && key > T) ? 1u : 0u;
    eq += (valid && key == T) ? 1u : 0u;
  });
  gt = wave_sum(gt);
  eq = wave_sum(eq);
  if (tile < ntiles && lane_id() == 0) {
    const uint32_t taken = gt + (rank_ties ? 0u : eq);
    tile_row(a, kRowTake)[tile] = taken;
    uint32_t* grp = a.group_counts + (tile / kGroupTiles) * kNumThres;
    if (taken) atomicAdd(&grp[kColTake], taken);
    if (rank_ties) {
      tile_row(a, kRowTies)[tile] = eq;
      if (eq) atomicAdd(&grp[kColTies], eq);
    }
  }
}

}  // namespace sp
