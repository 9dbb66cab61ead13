// Exact Top_k, flat vectors with a separate accumulator: radix select with candidate filtering.
// Once the exponent byte of the k-th key is known, only the keys that share it (a few per cent
// of a bell-shaped vector) can still be the k-th key.  The one remaining pass over the whole of
// acc writes those keys out, tile by tile, and the three later digit passes read them instead
// of acc: 12 + 4 + 8 bytes per element instead of 12 + 3 * 4 + 8.
//
// The candidate keys of a tile go to the residual buffer, at the tile's own offset: the old
// residual has been consumed by the accumulate kernel and the new one is not written before
// the compaction kernel, so in between the buffer is free and a tile's stretch of it can hold
// every key of the tile if it must.  (With acc == residual there is no such room; that case
// keeps the unfiltered passes of topk_flat.h.)
//
// From 6 M elements the accumulate pass also builds short lists (topk_list.h); when they hold at
// least k entries, which the workgroups of k_topk_filter find out, the kernels of this file take
// their list bodies instead of the ones described here.  Same launches, same results.
//
// Every survivor's output slot is fixed by counts: per tile, the keys above the k-th key T and
// the keys equal to it are counted from the candidates, the compaction kernel turns group and
// tile totals into its first slot, and ties are kept lowest index first.  The pairs come out in
// ascending index order; no output cursor is needed.
#pragma once
#include "common.h"
#include "gaussiank_flat.h"
#include "topk.h"
#include "topk_flat.h"

namespace sp {

__device__ inline uint32_t* tile_candidates(const Args& a, uint32_t tile) {
  return reinterpret_cast<uint32_t*>(a.resid) + (int64_t)tile * a.tile_chunks * kChunk;
}

// ---- accumulate, flat vectors -------------------------------------------------------------------
// A resident grid (one workgroup per compute unit) walks the chunks with a grid stride and
// flushes its histogram once: the same shape as the Gaussian_k accumulate kernel.
__global__ __launch_bounds__(kBlock) void k_topk_accum_hist_resident(const Args a) {
  __shared__ uint32_t h[kWaves][256];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  __syncthreads();
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  for (uint32_t ch = blockIdx.x; ch < nchunks; ch += gridDim.x) {
    Tile t;
    t.seg = 0;
    t.tbase = (int64_t)ch * kChunk;
    t.lo = t.tbase;
    t.hi = (t.tbase + kChunk < a.d_total) ? t.tbase + kChunk : a.d_total;
    t.full = t.tbase + kChunk <= a.d_total;
    if (t.full) accum_hist_tile<true>(a, t, h[wave_id()]);
    else accum_hist_tile<false>(a, t, h[wave_id()]);
  }
  __syncthreads();
  const int bin = threadIdx.x;
  uint32_t v = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) v += h[w][bin];
  if (v) atomicAdd(&pass_hist(a, 0)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
}

// ---- accumulate for long vectors ---------------------------------------------------------------
// One chunk per workgroup in dispatch order (see k_accum_moments_chunks): beyond the last-level
// cache this streams faster than one multi-chunk tile per workgroup.  The histogram flush then
// puts a few thousand atomics on each hot bin of each replica; they need no reply and drain
// under the stream.
__global__ __launch_bounds__(kBlock) void k_topk_accum_hist_chunks(const Args a) {
  __shared__ uint32_t h[kWaves][256];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  __syncthreads();
  Tile t;
  t.seg = 0;
  t.tbase = (int64_t)blockIdx.x * kChunk;
  t.lo = t.tbase;
  t.hi = (t.tbase + kChunk < a.d_total) ? t.tbase + kChunk : a.d_total;
  t.full = t.tbase + kChunk <= a.d_total;
  if (t.full) accum_hist_tile<true>(a, t, h[wave_id()]);
  else accum_hist_tile<false>(a, t, h[wave_id()]);
  __syncthreads();
  const int bin = threadIdx.x;
  uint32_t v = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) v += h[w][bin];
  if (v) atomicAdd(&pass_hist(a, 0)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
}

// ---- the one pass over acc after the accumulate kernel ----------------------------------------
// Prologue: the exponent byte E of the k-th key.  Then, per tile: the keys with exponent E are
// appended (in no particular order) to the tile's candidate list and enter the histogram of the
// second digit; the keys with a larger exponent are counted.
template <bool FULL>
__device__ inline uint32_t filter_chunk(const Args& a, const Tile& t, uint32_t E, uint32_t* cand,
                                        uint32_t* h, uint32_t* lds_cursor) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  uint32_t above = 0, cmask = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const uint32_t key = mag_key(v[i]);
    const bool ok = FULL || ((valid >> i) & 1u);
    above += (ok && (key >> 23) > E) ? 1u : 0u;
    cmask |= ((ok && (key >> 23) == E) ? 1u : 0u) << i;
  }
  const uint32_t n = (uint32_t)__builtin_popcount(cmask);
  const uint32_t inc = wave_inclusive_scan(n);
  const uint32_t wave_total = __shfl(inc, 63, 64);
  if (wave_total != 0) {  // wave-uniform
    uint32_t base = 0;
    if (lane_id() == 63) base = atomicAdd(lds_cursor, wave_total);  // LDS: one per wave and chunk
    base = __shfl(base, 63, 64);
    uint32_t pos = base + inc - n;
    if (wave_bins_look_uniform(cmask == 0xFFFFu ? (mag_key(v[0]) >> 15) & 255u : 256u + lane_id())) {
      // every element of the wave's chunk is a candidate and the first ones share a bin:
      // constant data, aggregate the histogram increments
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) {
        const uint32_t key = mag_key(v[i]);
        cand[pos++] = key;
        wave_hist_add(h, (key >> 15) & 255u, true);
      }
    } else {
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) {
        if ((cmask >> i) & 1u) {
          const uint32_t key = mag_key(v[i]);
          cand[pos++] = key;
          atomicAdd(&h[(key >> 15) & 255u], 1u);
        }
      }
    }
  }
  return above;
}

__global__ __launch_bounds__(kBlock) void k_topk_filter(const Args a) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sel[kWaves + 3];
  __shared__ uint32_t lds_above[kWaves];
  __shared__ uint32_t lds_lists[2];
  __shared__ uint32_t lds_cursor;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  if (threadIdx.x == 0) lds_cursor = 0;
  const uint32_t tile = gridDim.x - 1u - blockIdx.x;  // starts where the accumulate kernel ended
  Span sp_;
  if (!locate_span<false>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[0];
  bool usable = false;
  if (a.list) {  // short-list form (topk_list.h): do the lists serve?
    usable = lists_usable(a, lds_lists);
    if (tile == 0 && threadIdx.x == 0) c.list_mode = usable ? 1u : 0u;
    // one wave per tile reads the lists: the workgroups beyond a quarter of the grid have nothing
    // to do (but the first tile's, which publishes the digit)
    if (usable && tile != 0 && blockIdx.x * kWaves >= gridDim.x) return;
  }
  const Digit dg = choose_digit(pass_hist(a, 0), 0, 0u, (uint32_t)a.flat_k, lds_sel);  // barriers
  if (tile == 0 && threadIdx.x == 0) {
    c.sel_prefix[0] = dg.prefix;
    c.sel_krem[0] = dg.k_rem;
  }
  if (a.list) {  // if the lists serve, the second digit's histogram from them
    if (usable) {
      list_digit_pass(a, 1, dg.prefix, h[wave_id()]);
      __syncthreads();
      uint32_t v = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) v += h[w][threadIdx.x];
      if (v) atomicAdd(&pass_hist(a, 1)[(blockIdx.x % kTopkCopies) * 256 + threadIdx.x], v);
      return;
    }
  }
  uint32_t* cand = tile_candidates(a, tile);
  uint32_t above = 0;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) above += filter_chunk<true>(a, t, dg.prefix, cand, h[wave_id()], &lds_cursor);
    else above += filter_chunk<false>(a, t, dg.prefix, cand, h[wave_id()], &lds_cursor);
  }
  above = wave_sum(above);
  if (lane_id() == 0) lds_above[wave_id()] = above;
  __syncthreads();
  {
    const int bin = threadIdx.x;
    uint32_t v = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) v += h[w][bin];
    if (v) atomicAdd(&pass_hist(a, 1)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
  }
  if (threadIdx.x == 0) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds_above[w];
    tile_row(a, kRowAbove)[tile] = s;
    tile_row(a, kRowCand)[tile] = lds_cursor;
  }
}

// ---- digit passes 2 and 3 over the candidates -------------------------------------------------
// One wave per tile's candidate list (a few hundred keys as a rule), four lists per workgroup.
// `fn(key, valid)` is called by the whole wave for every 64 candidates of its tile (`valid` false in
// the lanes past the end of the list).
constexpr int kCandBatch = 4;
template <typename F>
__device__ inline void for_each_candidate(const Args& a, uint32_t tile, uint32_t ntiles, F fn) {
  if (tile >= ntiles) return;
  const uint32_t n = tile_row(a, kRowCand)[tile];
  const uint32_t* cand = tile_candidates(a, tile);
  for (uint32_t i0 = 0; i0 < n; i0 += 64 * kCandBatch) {
    uint32_t key[kCandBatch];
#pragma unroll
    for (int u = 0; u < kCandBatch; ++u) {
      const uint32_t i = i0 + u * 64 + lane_id();
      key[u] = i < n ? cand[i] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kCandBatch; ++u)
      if (i0 + u * 64 < n) fn(key[u], i0 + u * 64 + lane_id() < n);  // wave-uniform condition
  }
}

__global__ __launch_bounds__(kBlock) void k_topk_cand_hist(const Args a, int pass) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sel[kWaves + 3];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  SegCtrl& c = a.ctrl[0];
  const Digit dg = choose_digit(pass_hist(a, pass - 1), pass - 1, c.sel_prefix[pass - 2],
                                c.sel_krem[pass - 2], lds_sel);  // barriers
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    c.sel_prefix[pass - 1] = dg.prefix;
    c.sel_krem[pass - 1] = dg.k_rem;
  }
  const uint32_t ntiles = seg_ntiles(0, a.d_total, a.tile_chunks);
  const int hi_shift = digit_shift(pass - 1);
  const int shift = digit_shift(pass);
  const uint32_t mask = (1u << digit_bits(pass)) - 1u;
  uint32_t* hw = h[wave_id()];
  if (c.list_mode) {  // short-list form: the accumulate kernel's lists instead of the filter's
    list_digit_pass(a, pass, dg.prefix, hw);
  } else {
    // one wave per list; with more lists than waves in the grid a wave takes several
    for (uint32_t tile = blockIdx.x * kWaves + wave_id(); tile < ntiles; tile += gridDim.x * kWaves) {
      for_each_candidate(a, tile, ntiles, [&](uint32_t key, bool valid) {
        wave_hist_add(hw, (key >> shift) & mask, valid && (key >> hi_shift) == dg.prefix);
      });
    }
  }
  __syncthreads();
  const int bin = threadIdx.x;
  uint32_t v = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) v += h[w][bin];
  if (v) atomicAdd(&pass_hist(a, pass)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
}

// After the last digit: T, the ties to keep, whether they must be ranked; per tile, the number of
// survivors (keys above T; keys equal to T as well when all of them are kept) and, when ties are
// ranked, the number of keys equal to T.
template <int GT>  // tiles per group
__global__ __launch_bounds__(kBlock) void k_topk_cand_final(const Args a) {
  __shared__ uint32_t lds_sel[kWaves + 3];
  SegCtrl& c = a.ctrl[0];
  const Digit dg = choose_digit(pass_hist(a, 3), 3, c.sel_prefix[2], c.sel_krem[2], lds_sel);
  const uint32_t T = dg.prefix;
  const bool rank_ties = dg.count > dg.k_rem;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    c.topk_key = T;
    c.topk_take = dg.k_rem;
    c.n_eq = dg.count;
    c.rank_ties = rank_ties ? 1u : 0u;
    sparsify_result& r = a.result[0];
    r.topk_key = T;
    r.topk_ties_taken = dg.k_rem;
    if (a.list) r.flags = c.list_mode ? SPARSIFY_F_SHORTLIST : SPARSIFY_F_SHORTLIST_MISS;  // which way, no result
  }
  if (c.list_mode) {  // short-list form
    list_tile_counts<GT>(a, T, rank_ties);
    return;
  }
  const uint32_t ntiles = seg_ntiles(0, a.d_total, a.tile_chunks);
  for (uint32_t tile = blockIdx.x * kWaves + wave_id(); tile < ntiles; tile += gridDim.x * kWaves) {
    uint32_t gt = 0, eq = 0;
    for_each_candidate(a, tile, ntiles, [&](uint32_t key, bool valid) {
      gt += (valid && key > T) ? 1u : 0u;
      eq += (valid && key == T) ? 1u : 0u;
    });
    gt = wave_sum(gt);
    eq = wave_sum(eq);
    if (lane_id() == 0) {
      const uint32_t taken = tile_row(a, kRowAbove)[tile] + gt + (rank_ties ? 0u : eq);
      tile_row(a, kRowTake)[tile] = taken;
      uint32_t* grp = a.group_counts + (tile / GT) * kNumThres;
      if (taken) atomicAdd(&grp[kColTake], taken);
      if (rank_ties) {
        tile_row(a, kRowTies)[tile] = eq;
        if (eq) atomicAdd(&grp[kColTies], eq);
      }
    }
  }
}

// ---- compaction in index order (ordered_compact_chunk of topk.h), residual write ------------------
template <bool NORMS, int GT, int MG, bool STREAM>  // tiles per group, groups at most, non-temporal reads
__global__ __launch_bounds__(kBlock) void k_topk_compact_ordered(const Args a) {
  __shared__ uint32_t lds[kSlots * kWaves];
  __shared__ uint32_t lds_base[2];
  __shared__ double lds_n[2 * kWaves];
  const uint32_t tile = blockIdx.x;
  Span sp_;
  if (!locate_span<false>(a, tile, &sp_)) return;
  const SegCtrl& c = a.ctrl[0];
  const OrderedSel o = {c.topk_key, c.topk_take, c.rank_ties != 0, false, 0, a.flat_cap};
  const uint32_t take = o.take;
  const bool rank_ties = o.rank_ties;
  const uint32_t g = tile / GT, g0 = g * GT, within = tile - g0;
  if (wave_id() == 0) {  // survivors and ties before this tile: whole groups, then tiles of its own
    uint32_t x = 0, y = 0;
    // (no load behind a branch, so that all of them are on their way before the first is
    // waited for: a lane with nothing to add re-reads entry 0 and drops the value)
#pragma unroll
    for (int j0 = 0; j0 < MG; j0 += 64) {
      const uint32_t j = j0 + lane_id(), jc = j < g ? j : 0u;
      const uint32_t vx = a.group_counts[jc * kNumThres + kColTake];
      const uint32_t vy = a.group_counts[jc * kNumThres + kColTies];
      x += j < g ? vx : 0u;
      y += (j < g && rank_ties) ? vy : 0u;
    }
#pragma unroll
    for (int j0 = 0; j0 < GT; j0 += 64) {
      const uint32_t j = j0 + lane_id(), jc = j < within ? j : 0u;
      const uint32_t vx = tile_row(a, kRowTake)[g0 + jc];
      const uint32_t vy = tile_row(a, kRowTies)[g0 + jc];
      x += j < within ? vx : 0u;
      y += (j < within && rank_ties) ? vy : 0u;
    }
    x = wave_sum(x);
    y = wave_sum(y);
    if (lane_id() == 0) {
      lds_base[0] = x;
      lds_base[1] = y;
    }
  }
  __syncthreads();
  uint32_t tie_run = lds_base[1];
  uint32_t out_run = lds_base[0] + (tie_run < take ? tie_run : take);
  if (c.list_mode) {  // short-list form: the tile's pairs from the lists, by one wave
    if (wave_id() == 0) list_compact_tile(a, tile, o.T, take, rank_ties, out_run, tie_run);
    return;
  }
  NormAcc norms = {0.0, 0.0};
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) ordered_compact_chunk<true, NORMS, STREAM>(a, t, o, out_run, tie_run, lds, norms);
    else ordered_compact_chunk<false, NORMS, STREAM>(a, t, o, out_run, tie_run, lds, norms);
  }
  if (NORMS) store_norm_partial(a, norms, tile, lds_n);
}

}  // namespace sp
