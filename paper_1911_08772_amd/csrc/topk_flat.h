// Exact Top_k, flat vectors, accumulator aliased to the residual (in-place mode): seven launches
// with three full digit passes.  (With a separate accumulator the candidate-filtering form of
// topk_filter.h is used instead; it shares this file's initialisation and digit choice, and this
// form ends in that file's ordered compaction.)
// The per-segment "select" kernels of topk.h are latency-bound single workgroups that each cost a
// launch; here every workgroup of the next pass chooses the digit itself from the replicated
// histogram of the previous pass (same arithmetic, same inputs: all agree), and each pass has its
// own histogram buffer (cleared once by the init kernel).  The last pass leaves, per tile, the
// number of keys whose leading 24 bits already exceed the prefix and the histogram of the last
// digit among the keys that share the prefix; once the last digit is chosen these give every
// tile's number of survivors and of keys equal to the k-th key without another look at acc, so
// every output slot is fixed by counts and the pairs come out in ascending index order.
//
// From 6 M elements the accumulate pass also builds short lists (topk_list.h); when they hold at
// least k entries, which the workgroups of the first k_topk_hist_fused find out, the kernels of
// this file take their list bodies instead of the ones described here.
#pragma once
#include "common.h"
#include "gaussiank_flat.h"
#include "topk.h"
#include "topk_select.h"
#include "topk_list.h"

namespace sp {

// Passes 1..3.  Prologue: the digit of the previous pass.  The last pass also counts, per tile,
// the keys whose leading 24 bits already exceed the prefix (survivors whatever the last digit
// is) and adds them into the per-group totals.
template <bool LAST>
__global__ __launch_bounds__(kBlock) void k_topk_hist_fused(const Args a, int pass) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_sel[kWaves + 3];
  __shared__ uint32_t lds_sure[kWaves];
  __shared__ uint32_t lds_lists[2];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  // odd passes walk the tiles backwards (see k_topk_hist)
  const uint32_t tile = (pass & 1) ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  Span sp_;
  if (!locate_span<false>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[0];
  const uint32_t prefix_in = pass == 1 ? 0u : c.sel_prefix[pass - 2];
  const uint32_t k_in = pass == 1 ? (uint32_t)a.flat_k : c.sel_krem[pass - 2];
  const Digit dg = choose_digit(pass_hist(a, pass - 1), pass - 1, prefix_in, k_in, lds_sel);
  if (tile == 0 && threadIdx.x == 0) {  // published for the next kernel's prologue (own slot:
    c.sel_prefix[pass - 1] = dg.prefix;  // other workgroups of this kernel still read the last)
    c.sel_krem[pass - 1] = dg.k_rem;
  }
  if (a.list) {  // short-list form (topk_list.h): this digit's histogram from the lists, if they serve
    bool usable;
    if (pass == 1) {  // the kernel after the accumulate kernel decides, for the whole call
      usable = lists_usable(a, lds_lists);
      if (tile == 0 && threadIdx.x == 0) c.list_mode = usable ? 1u : 0u;
    } else {
      usable = c.list_mode != 0;
    }
    if (usable) {
      list_digit_pass(a, pass, dg.prefix, h[wave_id()]);
      __syncthreads();
      uint32_t v = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) v += h[w][threadIdx.x];
      if (v) atomicAdd(&pass_hist(a, pass)[(blockIdx.x % kTopkCopies) * 256 + threadIdx.x], v);
      return;
    }
  }
  uint32_t sure = 0;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) sure += hist_tile<true, LAST>(a, t, pass, dg.prefix, h[wave_id()]);
    else sure += hist_tile<false, LAST>(a, t, pass, dg.prefix, h[wave_id()]);
  }
  if (LAST) {
    sure = wave_sum(sure);
    if (lane_id() == 0) lds_sure[wave_id()] = sure;
  }
  __syncthreads();
  {
    const int bin = threadIdx.x;
    uint32_t v = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) v += h[w][bin];
    if (v) atomicAdd(&pass_hist(a, pass)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
    if (LAST && bin < kLastDigitBins) a.tile_hist[(size_t)tile * kLastDigitBins + bin] = v;
  }
  if (LAST && threadIdx.x == 0) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds_sure[w];
    tile_row(a, kRowAbove)[tile] = s;
  }
}

// After the last pass: every workgroup chooses the last digit (so T, the ties to keep and whether
// they must be ranked are known; workgroup 0 publishes them); then one wave per tile turns the
// tile's last-digit histogram into its number of survivors (keys above T, and keys equal to T
// when all of those are kept) and, when ties are ranked, its number of keys equal to T; both go
// to the per-group totals the ordered compaction reads.
__global__ __launch_bounds__(kBlock) void k_topk_ties_fused(const Args a) {
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
    list_tile_counts<kGroupTiles>(a, T, rank_ties);
    return;
  }
  const uint32_t ntiles = seg_ntiles(0, a.d_total, a.tile_chunks);
  const uint32_t digit = T & (uint32_t)(kLastDigitBins - 1);
  for (uint32_t tile = blockIdx.x * kWaves + wave_id(); tile < ntiles; tile += gridDim.x * kWaves) {
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < kLastDigitBins; j += 64) {
      const uint32_t bin = j + lane_id();
      const uint32_t v = a.tile_hist[(size_t)tile * kLastDigitBins + bin];
      gt += bin > digit ? v : 0u;
      eq += bin == digit ? v : 0u;
    }
    gt = wave_sum(gt);
    eq = wave_sum(eq);
    if (lane_id() == 0) {
      const uint32_t taken = tile_row(a, kRowAbove)[tile] + gt + (rank_ties ? 0u : eq);
      tile_row(a, kRowTake)[tile] = taken;
      uint32_t* grp = a.group_counts + (tile / kGroupTiles) * kNumThres;
      if (taken) atomicAdd(&grp[kColTake], taken);
      if (rank_ties) {
        tile_row(a, kRowTies)[tile] = eq;
        if (eq) atomicAdd(&grp[kColTies], eq);
      }
    }
  }
}

}  // namespace sp
