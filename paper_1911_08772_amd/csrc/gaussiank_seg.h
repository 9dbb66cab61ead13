// Gaussian_k, layer-wise calls: three launches for up to 256 segments (the accumulate kernel has
// the setup in it), setup + three beyond.  The same idea as gaussiank_flat.h, per
// segment: every workgroup of the count kernel merges the moment partials of its own segment's
// tiles and derives the ten thresholds; every workgroup of the compact kernel totals its
// segment's groups of 64 tiles, walks Algorithm 1 and finds its first output slot.  A segment's
// groups are its own (numbered by k_seg_setup), so no total mixes two segments' thresholds.
// All workgroups of a segment run the same arithmetic on the same inputs in the same order.
//
// With short lists (gaussiank_list.h; vectors of 6 M elements and more, where the workspace has
// room): the count kernel also writes the residual and lists each tile's entries above its
// segment's thres0, and the tiles of a segment whose walk ended at thres0 or above take their
// pairs from the lists.  Segments decide for themselves (a stretch of the list buffer that ran
// out leaves its own segment with the streaming compaction, no other).  A tile's runs are
// numbered (tile * tile_chunks + chunk) * 16 + run.
#pragma once
#include "common.h"
#include "gaussiank.h"
#include "gaussiank_list.h"
#include "setup.h"
#include "tile_io.h"

namespace sp {

// Layer-wise calls of up to kBlock segments need no setup launch before the accumulate kernel:
// every workgroup runs the one round of the setup walk itself (seg_setup_round of setup.h: the
// layout arrays, two scans) and finds its tile's segment in what the round leaves; one more
// workgroup, which streams nothing, is the setup kernel: it writes the control blocks, the tile
// numbering, the cleared records and the group totals that the kernels after this one read.
// (The quantile goes into a field of the control block that the setup does not write.)
__global__ __launch_bounds__(kBlock) void k_accum_moments_seg_setup(const Args a) {
  __shared__ double lds[4 * kWaves];
  __shared__ uint32_t lds_scan[kWaves + 1];
  __shared__ int64_t lds_max[kWaves];
  __shared__ int64_t lds_seg[3];  // start, end, k of the tile's segment
  __shared__ uint32_t lds_found[2];  // the segment, its first tile
  if (blockIdx.x == gridDim.x - 1u) {
    seg_setup_body(a, 1);
    return;
  }
  const uint32_t tile = blockIdx.x;
  if (threadIdx.x == 0) lds_found[0] = 0xFFFFFFFFu;
  int64_t off_max = 0;
  const SegRound r = seg_setup_round(a, 0, 0u, 0u, off_max, lds_scan, lds_max);  // barriers
  if (r.s < a.L && tile >= r.tile0 && tile - r.tile0 < r.nt) {  // one thread at most: the tiles of valid segments are disjoint
    lds_found[0] = (uint32_t)r.s;
    lds_found[1] = r.tile0;
    lds_seg[0] = r.start;
    lds_seg[1] = r.end;
    lds_seg[2] = r.k;
  }
  __syncthreads();
  const uint32_t seg = lds_found[0];
  if (seg == 0xFFFFFFFFu) return;  // a surplus workgroup, or a tile number an invalid segment left unused
  const uint32_t tile0 = lds_found[1];
  const int64_t start = lds_seg[0], end = lds_seg[1];
  Span sp_;
  make_span(&sp_, (int)seg, start, end,
            seg_base(start) + (int64_t)(tile - tile0) * a.tile_chunks * kChunk, a.tile_chunks);
  MomAcc m = {0.0, 0.0, 0.0, 0.0, false};
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) accum_moments_chunk<true>(a, t, m);
    else accum_moments_chunk<false>(a, t, m);
  }
  store_moment_partial(a, m, tile, lds);
  if (threadIdx.x == 0 && tile == tile0)
    a.ctrl[seg].z = norm_isf((double)lds_seg[2] / (a.tail_div * (double)(end - start)));
}

// Counts: thresholds of the tile's segment from that segment's moment partials (one pass
// around the provisional centre P = mean of the segment's first partial, as in
// k_gk_count_fused), then the ten counts of the tile.
__global__ __launch_bounds__(kBlock) void k_gk_count_seg(const Args a) {
  __shared__ double lds_m[2 * kWaves];
  __shared__ uint32_t lds[kWaves * kNumThres];
  const uint32_t tile = gridDim.x - 1u - blockIdx.x;
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad) return;
  const uint32_t parts = c.ntiles;
  const double* pn = a.partial + c.tile0;
  const double* pm = pn + a.max_tiles;
  const double* pq = pm + a.max_tiles;
  const double z = c.z;
  const int64_t n_seg = c.end - c.start;
  const double P = pm[0];
  double A = 0.0, B = 0.0;
  for (uint32_t b0 = 0; b0 < parts; b0 += 4 * kBlock) {
    double n[4], mu[4], q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = b0 + u * kBlock + threadIdx.x;
      const bool ok = i < parts;
      n[u] = ok ? pn[i] : 0.0;
      mu[u] = ok ? pm[i] : P;
      q[u] = ok ? pq[i] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const double dm = mu[u] - P;
      A = fma(n[u], dm, A);
      B += fma(n[u] * dm, dm, q[u]);
    }
  }
  A = wave_sum(A);
  B = wave_sum(B);
  if (lane_id() == 0) {
    lds_m[2 * wave_id()] = A;
    lds_m[2 * wave_id() + 1] = B;
  }
  __syncthreads();
  A = 0.0;
  B = 0.0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    A += lds_m[2 * w];
    B += lds_m[2 * w + 1];
  }
  const double N = (double)n_seg;
  const double mean = P + A / N;
  double m2 = B - A * (A / N);
  m2 = m2 < 0.0 ? 0.0 : m2;
  const double sd = (n_seg - a.ddof < 1) ? 0.0 : sqrt(m2 / (double)(n_seg - a.ddof));
  const double thres0 = mean + sd * z;
  double t64[kNumThres];
  candidate_thresholds(thres0, t64);
  float thr[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) thr[p] = (float)t64[p];
  const bool can_skip = thres0 > 0.0;
  if (tile == c.tile0 && threadIdx.x == 0) {  // the segment's first tile publishes
#pragma unroll
    for (int p = 0; p < kNumThres; ++p) {
      c.t64[p] = t64[p];
      c.t32[p] = thr[p];
    }
    uint32_t flags = 0;
    if (!isfinite(mean) || !isfinite(sd) || !isfinite(thres0)) flags |= SPARSIFY_F_NONFINITE;
    c.flags = flags;
    sparsify_result& r = a.result[sp_.seg];
    r.mean = mean;
    r.std = sd;
    r.z = z;
    r.thres0 = thres0;
  }

  uint32_t cnt[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) cnt[p] = 0;
  if (a.list && can_skip) {
    // with lists: the entries above thres0, and the residual as if nothing were selected; each
    // wave has a stretch of the list buffer for this tile
    const uint32_t worker = tile * kWaves + wave_id();
    ListCursor lc;
    lc.cur = worker * a.list_cap;
    lc.end = lc.cur + a.list_cap;
    lc.over = false;
    for (uint32_t u = 0; u < sp_.nchunks; ++u) {
      const Tile t = chunk_of(sp_, u);
      const uint32_t run0 = (tile * a.tile_chunks + u) * kRunsPerChunk;
      if (t.full) count_list_chunk<true, false>(a, t, run0, thr, cnt, lc);
      else count_list_chunk<false, false>(a, t, run0, thr, cnt, lc);
    }
    if (lc.over && lane_id() == 0) atomicOr(&c.list_mode, 1u);  // this segment's lists are incomplete
  } else {
    for (uint32_t u = 0; u < sp_.nchunks; ++u) {
      const Tile t = chunk_of(sp_, u);
      if (t.full) count_chunk<true>(a, t, thr, can_skip, cnt);
      else count_chunk<false>(a, t, thr, can_skip, cnt);
    }
  }
  if (lane_id() == 0) {
#pragma unroll
    for (int p = 0; p < kNumThres; ++p) lds[wave_id() * kNumThres + p] = cnt[p];
  }
  __syncthreads();
  if (threadIdx.x < kNumThres) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds[w * kNumThres + threadIdx.x];
    a.tile_counts[(size_t)threadIdx.x * a.max_tiles + tile] = s;  // [threshold][tile]
    const uint32_t g = c.group0 + (tile - c.tile0) / kSegGroupTiles;
    if (s) atomicAdd(&a.seg_groups[(size_t)g * kNumThres + threadIdx.x], s);
  }
}

// Totals of the segment's groups (all ten thresholds) and, of the same, what lies before `tile`:
// the groups before its own plus the tiles before it inside its group.  Results in
// lds_tot[kNumThres] and lds_pre[kNumThres] (integer adds in LDS: order does not matter).
// Two barriers.
__device__ inline void segment_totals(const Args& a, const SegCtrl& c, uint32_t tile,
                                      uint32_t* lds_tot, uint32_t* lds_pre) {
  if (threadIdx.x < kNumThres) {
    lds_tot[threadIdx.x] = 0;
    lds_pre[threadIdx.x] = 0;
  }
  __syncthreads();
  const uint32_t rel = tile - c.tile0;
  const uint32_t g_own = rel / kSegGroupTiles, within = rel % kSegGroupTiles;
  const uint32_t ng = (c.ntiles + kSegGroupTiles - 1) / kSegGroupTiles;
  const uint32_t* grp = a.seg_groups + (size_t)c.group0 * kNumThres;  // the segment's groups are contiguous
  for (uint32_t i0 = 0; i0 < ng * kNumThres; i0 += 4 * kBlock) {
    uint32_t x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * kBlock + threadIdx.x;
      x[u] = i < ng * kNumThres ? grp[i] : 0u;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * kBlock + threadIdx.x;
      if (i < ng * kNumThres && x[u] != 0) {
        atomicAdd(&lds_tot[i % kNumThres], x[u]);
        if (i / kNumThres < g_own) atomicAdd(&lds_pre[i % kNumThres], x[u]);
      }
    }
  }
  const uint32_t first = c.tile0 + g_own * kSegGroupTiles;  // first tile of this tile's group
  for (uint32_t i = threadIdx.x; i < within * kNumThres; i += kBlock) {
    const uint32_t p = i / within, j = i % within;
    const uint32_t x = a.tile_counts[(size_t)p * a.max_tiles + first + j];
    if (x) atomicAdd(&lds_pre[p], x);
  }
  __syncthreads();
}

template <bool NORMS>
__global__ __launch_bounds__(kBlock) void k_gk_compact_seg(const Args a) {
  __shared__ uint32_t lds_tot[kNumThres];
  __shared__ uint32_t lds_pre[kNumThres];
  __shared__ uint32_t lds[kSlots * kWaves];
  __shared__ double lds_n[2 * kWaves];
  const uint32_t tile = blockIdx.x;
  Span sp_;
  if (!locate_span<true>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[sp_.seg];
  if (c.bad) return;
  // with lists: the runs of this tile, and their records fetched before the tables
  const uint32_t r0 = tile * a.tile_chunks * kRunsPerChunk, r1 = r0 + sp_.nchunks * kRunsPerChunk;
  uint2 first_rec = make_uint2(0u, 0u);
  if (a.list) first_rec = gk_list_first_records(a, r0, r1);
  const uint32_t list_over = c.list_mode;
  double t64[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) t64[p] = c.t64[p];
  const uint32_t flags0 = c.flags;
  segment_totals(a, c, tile, lds_tot, lds_pre);
  uint32_t tot[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) tot[p] = lds_tot[p];
  const Walk w = walk_thresholds(tot, c.k);
  const bool overflow = (int64_t)tot[w.pos] > c.cap;
  const double tf = t64[w.pos];
  const float thr = (float)tf;
  // With lists: they hold the segment's survivors when none of its stretches ran out, its
  // thres0 is positive and its walk ended at thres0 or above it.
  const bool listed = a.list && list_over == 0 && w.pos >= kGkListPos && t64[kGkListPos] > 0.0;
  if (tile == c.tile0 && threadIdx.x == 0) {
    uint32_t flags = flags0;
    if (!w.in_band) flags |= SPARSIFY_F_EXHAUSTED;
    if (overflow) flags |= SPARSIFY_F_OVERFLOW;
    if (a.list) flags |= listed ? SPARSIFY_F_SHORTLIST : SPARSIFY_F_SHORTLIST_MISS;  // which way, no result
    sparsify_result& r = a.result[sp_.seg];
    r.nnz = overflow ? 0u : tot[w.pos];
    r.rounds = w.rounds;
    r.count[0] = w.counts[0];
    r.count[1] = w.counts[1];
    r.count[2] = w.counts[2];
    r.count[3] = w.counts[3];
    r.flags = flags;
    r.thres = tf;
    r.thres_f32 = thr;
    r.topk_key = 0;
    r.topk_ties_taken = 0;
    r.acc_sqnorm = 0.0;
    r.residual_sqnorm = 0.0;
  }
  const int64_t out0 = c.out_base + (int64_t)lds_pre[w.pos];
  if (listed) {  // the residual is in place (the count kernel wrote it); one wave writes the tile's pairs
    if (!overflow && wave_id() == 0) gk_list_compact_tile(a, r0, r1, thr, out0, c.out_base + c.cap, first_rec);
    return;
  }
  uint32_t run = 0;
  NormAcc norms = {0.0, 0.0};
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) run = compact_chunk<true, NORMS>(a, t, thr, overflow, out0, run, lds, norms);
    else run = compact_chunk<false, NORMS>(a, t, thr, overflow, out0, run, lds, norms);
  }
  if (NORMS) store_norm_partial(a, norms, tile, lds_n);
}

}  // namespace sp
