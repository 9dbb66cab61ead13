// Exact Top_k, layer-wise calls with a separate accumulator: the candidate-filtering radix
// select of topk_filter.h applied per segment.  Every segment has its own four per-pass
// histograms ([pass][segment][replica][256]) and its own groups of 64 tiles (numbered by
// k_seg_setup); a tile's candidate keys live in the tile's stretch of the idle residual buffer.
// Each workgroup works for one tile and chooses its segment's digits itself; the workgroup of a
// segment's first tile publishes them.  Launches: setup, histogram clear, accumulate, filter,
// two list passes, final, ordered compaction.
#pragma once
#include "common.h"
#include "gaussiank_seg.h"
#include "topk_filter.h"

namespace sp {

__device__ inline uint32_t* seg_pass_hist(const Args& a, int pass, int seg) {
  return a.hist + ((size_t)pass * a.L + seg) * a.hist_copies * 256;
}
__device__ inline uint32_t* span_candidates(const Args& a, const Span& s) {
  return reinterpret_cast<uint32_t*>(a.resid) + s.lo;
}
__device__ inline void flush_seg_hist(const Args& a, int pass, int seg, uint32_t (*h)[256]) {
  const int bin = threadIdx.x;
  uint32_t v = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) v += h[w][bin];
  if (v) atomicAdd(&seg_pass_hist(a, pass, seg)[(blockIdx.x % a.hist_copies) * 256 + bin], v);
}

__global__ __launch_bounds__(kBlock) void k_topk_filter_seg(const Args a) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sel[kWaves + 3];
  __shared__ uint32_t lds_above[kWaves];
  __shared__ uint32_t lds_cursor;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  if (threadIdx.x == 0) lds_cursor = 0;
  const uint32_t tile = gridDim.x - 1u - blockIdx.x;
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad || c.select_none) return;
  const Digit dg = choose_digit_n(seg_pass_hist(a, 0, sp_.seg), a.hist_copies, 0, 0u, (uint32_t)c.k,
                                  lds_sel);  // barriers
  if (tile == c.tile0 && threadIdx.x == 0) {
    c.sel_prefix[0] = dg.prefix;
    c.sel_krem[0] = dg.k_rem;
  }
  uint32_t* cand = span_candidates(a, sp_);
  uint32_t above = 0;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) above += filter_chunk<true>(a, t, dg.prefix, cand, h[wave_id()], &lds_cursor);
    else above += filter_chunk<false>(a, t, dg.prefix, cand, h[wave_id()], &lds_cursor);
  }
  above = wave_sum(above);
  if (lane_id() == 0) lds_above[wave_id()] = above;
  __syncthreads();
  flush_seg_hist(a, 1, sp_.seg, h);
  if (threadIdx.x == 0) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds_above[w];
    tile_row(a, kRowAbove)[tile] = s;
    tile_row(a, kRowCand)[tile] = lds_cursor;
  }
}

// Digit passes 2 and 3: one workgroup per tile's candidate list.
__global__ __launch_bounds__(kBlock) void k_topk_cand_hist_seg(const Args a, int pass) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sel[kWaves + 3];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  const uint32_t tile = blockIdx.x;
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad || c.select_none) return;
  const Digit dg = choose_digit_n(seg_pass_hist(a, pass - 1, sp_.seg), a.hist_copies, pass - 1,
                                  c.sel_prefix[pass - 2], c.sel_krem[pass - 2], lds_sel);  // barriers
  if (tile == c.tile0 && threadIdx.x == 0) {
    c.sel_prefix[pass - 1] = dg.prefix;
    c.sel_krem[pass - 1] = dg.k_rem;
  }
  const int hi_shift = digit_shift(pass - 1);
  const int shift = digit_shift(pass);
  const uint32_t mask = (1u << digit_bits(pass)) - 1u;
  const uint32_t n = tile_row(a, kRowCand)[tile];
  const uint32_t* cand = span_candidates(a, sp_);
  uint32_t* hw = h[wave_id()];
  for (uint32_t i0 = 0; i0 < n; i0 += kBlock) {  // block-uniform trip count
    const uint32_t i = i0 + threadIdx.x;
    const uint32_t key = i < n ? cand[i] : 0u;
    wave_hist_add(hw, (key >> shift) & mask, i < n && (key >> hi_shift) == dg.prefix);
  }
  __syncthreads();
  flush_seg_hist(a, pass, sp_.seg, h);
}

// After the last digit: the segment's T and ties; per tile, survivors and (ranked) ties, added
// into the segment's group totals.
__global__ __launch_bounds__(kBlock) void k_topk_cand_final_seg(const Args a) {
  __shared__ uint32_t lds_sel[kWaves + 3];
  __shared__ uint32_t lds_c[2 * kWaves];
  const uint32_t tile = blockIdx.x;
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad || c.select_none) return;
  const Digit dg = choose_digit_n(seg_pass_hist(a, 3, sp_.seg), a.hist_copies, 3, c.sel_prefix[2],
                                  c.sel_krem[2], lds_sel);
  const uint32_t T = dg.prefix;
  const bool rank_ties = dg.count > dg.k_rem;
  if (tile == c.tile0 && threadIdx.x == 0) {
    c.topk_key = T;
    c.topk_take = dg.k_rem;
    c.n_eq = dg.count;
    c.rank_ties = rank_ties ? 1u : 0u;
    sparsify_result& r = a.result[sp_.seg];
    r.topk_key = T;
    r.topk_ties_taken = dg.k_rem;
  }
  const uint32_t n = tile_row(a, kRowCand)[tile];
  const uint32_t* cand = span_candidates(a, sp_);
  uint32_t gt = 0, eq = 0;
  for (uint32_t i = threadIdx.x; i < n; i += kBlock) {
    const uint32_t key = cand[i];
    gt += key > T ? 1u : 0u;
    eq += key == T ? 1u : 0u;
  }
  gt = wave_sum(gt);
  eq = wave_sum(eq);
  if (lane_id() == 0) {
    lds_c[2 * wave_id()] = gt;
    lds_c[2 * wave_id() + 1] = eq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    gt = 0;
    eq = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      gt += lds_c[2 * w];
      eq += lds_c[2 * w + 1];
    }
    const uint32_t taken = tile_row(a, kRowAbove)[tile] + gt + (rank_ties ? 0u : eq);
    tile_row(a, kRowTake)[tile] = taken;
    tile_row(a, kRowTies)[tile] = rank_ties ? eq : 0u;
    uint32_t* grp = a.seg_groups + (size_t)(c.group0 + (tile - c.tile0) / kSegGroupTiles) * kNumThres;
    if (taken) atomicAdd(&grp[kColTake], taken);
    if (rank_ties && eq) atomicAdd(&grp[kColTies], eq);
  }
}

// Ordered compaction per segment.  Segments that select nothing (output range smaller than k)
// still get residual' = acc.
template <bool NORMS>
__global__ __launch_bounds__(kBlock) void k_topk_compact_ordered_seg(const Args a) {
  __shared__ uint32_t lds_tot[kNumThres];
  __shared__ uint32_t lds_pre[kNumThres];
  __shared__ uint32_t lds[kSlots * kWaves];
  __shared__ double lds_n[2 * kWaves];
  const uint32_t tile = blockIdx.x;
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  const SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad) return;
  const bool none = c.select_none != 0;
  const OrderedSel o = {c.topk_key, c.topk_take, c.rank_ties != 0, none, c.out_base, c.cap};
  uint32_t tie_run = 0, out_run = 0;
  if (!none) {  // block-uniform
    segment_totals(a, c, tile, lds_tot, lds_pre);
    tie_run = o.rank_ties ? lds_pre[kColTies] : 0u;
    out_run = lds_pre[kColTake] + (tie_run < o.take ? tie_run : o.take);
  }
  NormAcc norms = {0.0, 0.0};
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) ordered_compact_chunk<true, NORMS>(a, t, o, out_run, tie_run, lds, norms);
    else ordered_compact_chunk<false, NORMS>(a, t, o, out_run, tie_run, lds, norms);
  }
  if (NORMS) store_norm_partial(a, norms, tile, lds_n);
}

}  // namespace sp
