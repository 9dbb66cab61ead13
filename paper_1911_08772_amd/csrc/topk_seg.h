// Exact Top_k, layer-wise calls with a separate accumulator: the candidate-filtering radix
// select of topk_filter.h applied per segment.  Every segment has its own four per-pass
// histograms ([pass][segment][replica][256]) and its own groups of 64 tiles (numbered by
// k_seg_setup); a tile's candidate keys live in the tile's stretch of the idle residual buffer.
// Each workgroup works for one tile and chooses its segment's digits itself; the workgroup of a
// segment's first tile publishes them.  Launches: setup (which also clears the histograms),
// accumulate, filter, two list passes, final, ordered compaction.
//
// With short lists (topk_list.h, per segment; vectors of 6 M elements and more where the
// workspace has room): beside the workgroup that numbers the tiles, the setup kernel has one
// workgroup per segment that takes a sample of it and sets its listing key; the accumulate kernel
// also writes the residual (as if nothing were selected) and lists the entries above their
// segment's key, a stretch of the list buffer per wave of a tile's workgroup.  A segment whose
// lists hold at least its k entries, none of its stretches having run out, is served from them
// by the five kernels that follow (one wave per tile reads the tile's lists); every other
// segment of the same call takes the bodies without lists, which overwrite whatever the
// accumulate kernel left in its stretch of the residual.  Same launches, same results.
#pragma once
#include "common.h"
#include "gaussiank_seg.h"
#include "topk_filter.h"
#include "topk_list.h"

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

// ---- short lists per segment ------------------------------------------------------------------------
constexpr int64_t kSegListFrom = 4 * kListSample;      // shorter segments are sampled entry by entry

// The sample of topk_list.h over one segment (single loads: a segment may start anywhere).  From
// kSegListFrom elements: 4096 entries of acc, four consecutive ones every n/1024 elements.  Shorter
// segments: min(n, 4096) entries evenly spaced, so that a segment of up to 4096 elements is its
// own sample.
__device__ inline uint32_t sample_listing_key_seg(const Args& a, int64_t start, int64_t n, int64_t k,
                                                  uint32_t* lds_h, uint32_t* lds_sel) {
  uint32_t key[16];
  int64_t m = kListSample;
  if (n >= kSegListFrom) {  // block-uniform
    const int64_t stride4 = (n / 4) / (kListSample / 4);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = start + (int64_t)(u * kBlock + (int)threadIdx.x) * stride4 * 4;
#pragma unroll
      for (int q = 0; q < 4; ++q) key[4 * u + q] = mag_key(a.grad[i + q] + a.resid[i + q]);
    }
  } else {
    static_assert(kListSample == 4096, "the spacing below is a shift");
    const uint32_t n32 = (uint32_t)n;
    const uint32_t m32 = n32 < (uint32_t)kListSample ? n32 : (uint32_t)kListSample;
    m = m32;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const uint32_t j = (uint32_t)(u * kBlock) + threadIdx.x;
      const uint32_t jc = j < m32 ? j : m32 - 1u;  // (a lane beyond the sample re-reads its last entry)
      const int64_t i = start + (n32 < (uint32_t)kListSample ? jc : (jc * n32) >> 12);
      const float x = a.grad[i] + a.resid[i];
      key[u] = j < m32 ? mag_key(x) : 0u;
    }
  }
  return listing_key_from_sample(key, k, n, m, lds_h, lds_sel);
}

// The listing keys live in a table that the layer-wise form with a separate acc does not use
// otherwise (the in-place form's tie offsets: one word per tile, and there are more tiles than
// segments).
__device__ inline uint32_t* seg_listing_keys(const Args& a) { return a.tie_base; }

// The setup kernel of the layer-wise Top_k call: workgroup 0 numbers the tiles (setup.h); with
// lists, workgroup 1 + s sets the listing key of segment s from the layout arrays themselves
// (it looks at the segment's own bounds only, which is all its loads need; what else makes a
// segment invalid is workgroup 0's business, and an invalid segment's key is never read); the
// remaining workgroups clear the histograms.
__global__ __launch_bounds__(kBlock) void k_topk_seg_setup(const Args a, uint32_t hist_words, uint32_t samplers) {
  __shared__ uint32_t lds_h[256];
  __shared__ uint32_t lds_sel[kWaves + 3];
  if (blockIdx.x == 0) {
    seg_setup_body(a, 0);
    return;
  }
  if (blockIdx.x > samplers) {
    const uint32_t nb = gridDim.x - 1u - samplers;
    for (uint32_t i = (blockIdx.x - 1u - samplers) * kBlock + threadIdx.x; i < hist_words; i += nb * kBlock)
      a.hist[i] = 0;
    return;
  }
  const uint32_t s = blockIdx.x - 1u;
  const int64_t start = a.seg_off[s], end = a.seg_off[s + 1], k = a.seg_k[s];
  const int64_t n = end - start;
  uint32_t tau = kNoListKey;
  // as the flat call: lists of about 8 k entries at most are to stay within a tenth of n (a
  // segment that fits a wave's stretch of the list buffer whole cannot make one run out)
  const bool sample = start >= 0 && end > start && end <= a.d_total && k >= 1 && k <= n &&
                      !(2 * kListAim * k * 10 > n && n > (int64_t)a.list_cap);
  if (sample) tau = sample_listing_key_seg(a, start, n, k, lds_h, lds_sel);  // block-uniform; barriers
  if (threadIdx.x == 0) seg_listing_keys(a)[s] = tau;
}

// The accumulate kernel with lists: k_topk_accum_hist plus the residual write and the lists of
// the tile's entries above its segment's key.  The runs are numbered by tile and chunk
// (gaussiank_seg.h); the segment's control block collects how many entries its tiles listed and
// whether a stretch ran out.
__global__ __launch_bounds__(kBlock) void k_topk_accum_list_seg(const Args a) {
  __shared__ uint32_t h[kWaves][256];
  __shared__ uint32_t lds_stat[2 * kWaves];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
  __syncthreads();
  const uint32_t tile = blockIdx.x;
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad) return;
  const uint32_t tau = seg_listing_keys(a)[sp_.seg];
  const uint32_t worker = tile * kWaves + wave_id();
  ListCursor lc;
  lc.cur = worker * a.list_cap;
  lc.end = lc.cur + a.list_cap;
  lc.over = false;
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    const uint32_t run0 = (tile * a.tile_chunks + u) * kRunsPerChunk;
    if (t.full) accum_hist_list_chunk<true, true>(a, t, run0, h[wave_id()], tau, lc);
    else accum_hist_list_chunk<false, true>(a, t, run0, h[wave_id()], tau, lc);
  }
  if (lane_id() == 0) {
    lds_stat[2 * wave_id()] = lc.cur - worker * a.list_cap;
    lds_stat[2 * wave_id() + 1] = lc.over ? 1u : 0u;
  }
  flush_hist(a, sp_.seg, h);  // starts with a barrier
  if (threadIdx.x == 0) {
    uint32_t n = 0, over = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      n += lds_stat[2 * w];
      over |= lds_stat[2 * w + 1];
    }
    if (n) atomicAdd(&c.list_count, n);
    if (over) atomicOr(&c.list_mode, 1u);
  }
}

// Whether a segment's lists serve it: none of its stretches ran out and they hold at least k
// entries (then they hold the k largest: every key >= the k-th key exceeds the listing key).
// Every workgroup of the kernels after the accumulate kernel reads the same final words.
__device__ inline bool seg_lists_usable(const Args& a, const SegCtrl& c) {
  return a.list && c.list_mode == 0 && (int64_t)c.list_count >= c.k;
}
// the runs of a layer-wise tile
__device__ inline void seg_tile_runs(const Args& a, uint32_t tile, const Span& s, uint32_t* r0, uint32_t* r1) {
  *r0 = tile * a.tile_chunks * kRunsPerChunk;
  *r1 = *r0 + s.nchunks * kRunsPerChunk;
}
// The five kernels after the accumulate kernel make two or three dependent trips to memory before
// they know whether their tile's lists serve; the first wave of each workgroup has the head of
// the tile's lists (lists.h) fetched meanwhile: the records before the tile is located (its run
// slots follow from the tile number), the entries while the segment's control block and
// histogram are on their way.
__device__ inline bool seg_list_head_records(const Args& a, uint32_t tile, ListHead& head) {
  if (!a.list || wave_id() != 0) return false;
  list_head_records(a, tile * a.tile_chunks * kRunsPerChunk, a.tile_chunks * kRunsPerChunk, head);
  return true;
}
// A digit pass over a tile's lists by the workgroup's first wave (list_digit_pass of topk_list.h).
__device__ inline void seg_list_digit_pass(const Args& a, uint32_t r0, uint32_t r1, const ListHead& head,
                                           int pass, uint32_t prefix, uint32_t* hw) {
  if (wave_id() != 0) return;
  const int hi_shift = pass == 0 ? 31 : digit_shift(pass - 1);
  const int shift = digit_shift(pass);
  const uint32_t mask = (1u << digit_bits(pass)) - 1u;
  for_each_list_entry_of_runs(a, r0, r1, &head, [&](uint2 e, bool valid) {
    const uint32_t key = e.y & 0x7FFFFFFFu;
    wave_hist_add(hw, (key >> shift) & mask, valid && (key >> hi_shift) == prefix);
  });
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
  ListHead head;
  const bool heads = seg_list_head_records(a, tile, head);
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  if (heads) list_head_entries(a, head);
  SegCtrl& c = a.ctrl[sp_.seg];
  const uint32_t bins = load_digit_bins(seg_pass_hist(a, 0, sp_.seg), a.hist_copies);
  const bool usable = seg_lists_usable(a, c);
  if (c.bad || c.select_none) return;
  const Digit dg = digit_from_bins(bins, 0, 0u, (uint32_t)c.k, lds_sel);  // barriers
  if (tile == c.tile0 && threadIdx.x == 0) {
    c.sel_prefix[0] = dg.prefix;
    c.sel_krem[0] = dg.k_rem;
  }
  if (usable) {  // the second digit's histogram from the tile's lists
    uint32_t r0, r1;
    seg_tile_runs(a, tile, sp_, &r0, &r1);
    seg_list_digit_pass(a, r0, r1, head, 1, dg.prefix, h[0]);
    __syncthreads();
    flush_seg_hist(a, 1, sp_.seg, h);
    return;
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
  ListHead head;
  const bool heads = seg_list_head_records(a, tile, head);
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  if (heads) list_head_entries(a, head);
  SegCtrl& c = a.ctrl[sp_.seg];
  const uint32_t bins = load_digit_bins(seg_pass_hist(a, pass - 1, sp_.seg), a.hist_copies);
  const bool usable = seg_lists_usable(a, c);
  if (c.bad || c.select_none) return;
  const Digit dg = digit_from_bins(bins, pass - 1, c.sel_prefix[pass - 2], c.sel_krem[pass - 2],
                                   lds_sel);  // barriers
  if (tile == c.tile0 && threadIdx.x == 0) {
    c.sel_prefix[pass - 1] = dg.prefix;
    c.sel_krem[pass - 1] = dg.k_rem;
  }
  if (usable) {
    uint32_t r0, r1;
    seg_tile_runs(a, tile, sp_, &r0, &r1);
    seg_list_digit_pass(a, r0, r1, head, pass, dg.prefix, h[0]);
    __syncthreads();
    flush_seg_hist(a, pass, sp_.seg, h);
    return;
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
  ListHead head;
  const bool heads = seg_list_head_records(a, tile, head);
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  if (heads) list_head_entries(a, head);
  SegCtrl& c = a.ctrl[sp_.seg];
  const uint32_t bins = load_digit_bins(seg_pass_hist(a, 3, sp_.seg), a.hist_copies);
  const bool usable = seg_lists_usable(a, c);
  if (c.bad || c.select_none) return;
  const Digit dg = digit_from_bins(bins, 3, c.sel_prefix[2], c.sel_krem[2], lds_sel);
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
    if (a.list) r.flags |= usable ? SPARSIFY_F_SHORTLIST : SPARSIFY_F_SHORTLIST_MISS;  // which way, no result
  }
  uint32_t gt = 0, eq = 0;
  if (usable) {  // the tile's counts from its lists, by one wave
    if (wave_id() != 0) return;
    uint32_t r0, r1;
    seg_tile_runs(a, tile, sp_, &r0, &r1);
    for_each_list_entry_of_runs(a, r0, r1, &head, [&](uint2 e, bool valid) {
      const uint32_t key = e.y & 0x7FFFFFFFu;
      gt += (valid && key > T) ? 1u : 0u;
      eq += (valid && key == T) ? 1u : 0u;
    });
    gt = wave_sum(gt);
    eq = wave_sum(eq);
    if (lane_id() == 0) {
      const uint32_t taken = gt + (rank_ties ? 0u : eq);
      tile_row(a, kRowTake)[tile] = taken;
      tile_row(a, kRowTies)[tile] = rank_ties ? eq : 0u;
      uint32_t* grp = a.seg_groups + (size_t)(c.group0 + (tile - c.tile0) / kSegGroupTiles) * kNumThres;
      if (taken) atomicAdd(&grp[kColTake], taken);
      if (rank_ties && eq) atomicAdd(&grp[kColTies], eq);
    }
    return;
  }
  const uint32_t n = tile_row(a, kRowCand)[tile];
  const uint32_t* cand = span_candidates(a, sp_);
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
  ListHead head;
  const bool heads = seg_list_head_records(a, tile, head);
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  if (heads) list_head_entries(a, head);
  const SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad) return;
  const bool none = c.select_none != 0;
  if (a.list && none) return;  // the accumulate kernel has written residual' = acc
  const OrderedSel o = {c.topk_key, c.topk_take, c.rank_ties != 0, none, c.out_base, c.cap};
  uint32_t tie_run = 0, out_run = 0;
  if (!none) {  // block-uniform
    segment_totals(a, c, tile, lds_tot, lds_pre);
    tie_run = o.rank_ties ? lds_pre[kColTies] : 0u;
    out_run = lds_pre[kColTake] + (tie_run < o.take ? tie_run : o.take);
  }
  if (seg_lists_usable(a, c)) {  // the tile's pairs from its lists, by one wave; the residual is in place
    if (wave_id() != 0) return;
    uint32_t r0, r1;
    seg_tile_runs(a, tile, sp_, &r0, &r1);
    list_compact_runs(a, r0, r1, o.T, o.take, o.rank_ties, out_run, tie_run, o.out0, o.cap, &head);
    return;
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
