// Gaussian_k, flat vectors: three launches.  A launch costs 3-4 us on the stream even when the
// kernel does nothing, and a single workgroup that combines per-tile partials is latency-bound;
// here every workgroup of the count kernel derives the thresholds from the (few) moment partials
// itself, and every workgroup of the compact kernel walks Algorithm 1 and finds its own output
// base from per-group totals.  All workgroups run the same arithmetic on the same inputs in the
// same order, so they agree bit for bit.
//
// The group tables hold kFusedMaxTiles tiles (kBigMaxTiles for long vectors); the host chooses
// the tile length accordingly and refuses a forced tile length that would need more.
//
// From 6 M elements the count kernel also writes the residual and lists the entries above
// thres0, and the compact kernel writes the pairs from those lists when the walk ended at
// thres0 or above (gaussiank_list.h): two passes over the vector instead of three.
#pragma once
#include "common.h"
#include "gaussiank.h"
#include "gaussiank_list.h"
#include "tile_io.h"

namespace sp {

constexpr int kGroupTiles = 64;                                   // tiles per group
constexpr int kFusedMaxTiles = 4096;
constexpr int kMaxGroups = kFusedMaxTiles / kGroupTiles;          // 64
// Long vectors (Gaussian_k): groups of kBigGroupTiles tiles, up to kBigMaxTiles tiles, so that a
// tile can stay three chunks long (with tiles of tens of chunks, thousands of workgroups stream
// from places hundreds of kilobytes apart and the memory system slows down).
constexpr int kBigGroupTiles = 256;
constexpr int kBigMaxGroups = 256;
constexpr int kBigMaxTiles = kBigGroupTiles * kBigMaxGroups;     // 65536
constexpr int kMaxMomentParts = 1024;                             // accumulate workgroups at most

// K1: a resident grid of `moment_parts` workgroups walks the chunks with a grid stride and leaves
// one moment partial per workgroup (the moments need no particular partition of the vector),
// plus one more workgroup that streams nothing: it clears the group totals the count kernel adds
// into and computes the normal quantile (a few microseconds of dependent fp64 arithmetic in one
// thread, which would otherwise stick out at the end of a workgroup that also streams).
template <bool STREAM>  // acc is stored with the non-temporal hint (the host picks by the vector length)
__global__ __launch_bounds__(kBlock) void k_accum_moments_fused(const Args a) {
  __shared__ double lds[4 * kWaves];
  if (blockIdx.x == a.moment_parts) {
    for (uint32_t i = threadIdx.x; i < (uint32_t)(kMaxGroups * kNumThres); i += kBlock)
      a.group_counts[i] = 0;
    if (a.list && threadIdx.x < 2 * kListStatCopies) a.list_stats[threadIdx.x] = 0;
    if (threadIdx.x == 0)
      a.ctrl[0].z = norm_isf((double)a.flat_k / (a.tail_div * (double)a.d_total));
    return;
  }
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  const uint32_t nfull = (uint32_t)(a.d_total / kChunk);
  const uint32_t step = a.moment_parts;
  MomAcc m = {0.0, 0.0, 0.0, 0.0, false};
  // Full chunks, two register sets in turn: the loads of the workgroup's next chunk are issued
  // before this chunk's additions, stores and fp64 sums, so that with one workgroup per compute
  // unit the memory pipes still have the next 32 KiB on order while this one is worked on.
  // (No load sits behind a branch inside the loop: where two paths meet, the wait for the
  // oldest loads is placed for the path with the fewest in flight, and that would drain the
  // other path's prefetch.)
  const uint32_t n = blockIdx.x < nfull ? (nfull - blockIdx.x + step - 1) / step : 0u;  // my full chunks
  auto at = [&](uint32_t k) { return (int64_t)(blockIdx.x + k * step) * kChunk; };
  if (n > 0) {
    AccIn x, y;
    uint32_t k = 0;
    accum_issue(a, at(0), x);
    while (k + 2 < n) {
      accum_issue(a, at(k + 1), y);
      __builtin_amdgcn_sched_barrier(0);  // nothing of the work below moves above the loads
      accum_finish<STREAM>(a, at(k), x, m);
      accum_issue(a, at(k + 2), x);
      __builtin_amdgcn_sched_barrier(0);
      accum_finish<STREAM>(a, at(k + 1), y, m);
      k += 2;
    }
    if (n - k == 2) {
      accum_issue(a, at(k + 1), y);
      __builtin_amdgcn_sched_barrier(0);
      accum_finish<STREAM>(a, at(k), x, m);
      accum_finish<STREAM>(a, at(k + 1), y, m);
    } else {
      accum_finish<STREAM>(a, at(k), x, m);
    }
  }
  // the ragged last chunk, if there is one, belongs to the workgroup whose turn it is
  if (nfull < nchunks && nfull % step == blockIdx.x) {
    Tile t;
    t.seg = 0;
    t.tbase = (int64_t)nfull * kChunk;
    t.lo = t.tbase;
    t.hi = a.d_total;
    t.full = false;
    accum_moments_chunk<false>(a, t, m);
  }
  store_moment_partial(a, m, blockIdx.x, lds);
}

// K1 for long vectors: one chunk per workgroup, in dispatch order.  Beyond what the last-level
// cache holds, the hardware's in-order dispatch of many small workgroups keeps the addresses in
// flight inside a narrow window and streams faster than a resident grid walking the vector with
// a stride (measured at 537 M elements: 6.0 against 5.1 TB/s); the price is one moment partial
// per chunk, folded to at most kMaxMomentParts by k_fold_moments before the count kernel.
__global__ __launch_bounds__(kBlock) void k_accum_moments_chunks(const Args a) {
  __shared__ double lds[4 * kWaves];
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  if (blockIdx.x == nchunks) {  // the extra workgroup: see k_accum_moments_fused
    for (uint32_t i = threadIdx.x; i < (uint32_t)(kBigMaxGroups * kNumThres); i += kBlock)
      a.group_counts[i] = 0;
    if (a.list && threadIdx.x < 2 * kListStatCopies) a.list_stats[threadIdx.x] = 0;
    if (threadIdx.x == 0)
      a.ctrl[0].z = norm_isf((double)a.flat_k / (a.tail_div * (double)a.d_total));
    return;
  }
  Tile t;
  t.seg = 0;
  t.tbase = (int64_t)blockIdx.x * kChunk;
  t.lo = t.tbase;
  t.hi = (t.tbase + kChunk < a.d_total) ? t.tbase + kChunk : a.d_total;
  t.full = t.tbase + kChunk <= a.d_total;
  MomAcc m = {0.0, 0.0, 0.0, 0.0, false};
  if (t.full) accum_moments_chunk<true>(a, t, m);
  else accum_moments_chunk<false>(a, t, m);
  store_moment_partial(a, m, blockIdx.x, lds);
}

// Folds the per-chunk partials into `moment_parts` partials: workgroup j merges a contiguous run
// (one pass around the mean of the run's first partial, fixed order).
__global__ __launch_bounds__(kBlock) void k_fold_moments(const Args a) {
  __shared__ double lds_m[3 * kWaves];
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  const uint32_t per = (nchunks + a.moment_parts - 1) / a.moment_parts;
  const uint32_t lo = blockIdx.x * per;
  const uint32_t hi = lo + per < nchunks ? lo + per : nchunks;
  const double* pn = a.partial;
  const double* pm = pn + a.max_tiles;
  const double* pq = pm + a.max_tiles;
  double N = 0.0, A = 0.0, B = 0.0;
  const double P = lo < hi ? pm[lo] : 0.0;
  for (uint32_t i = lo + threadIdx.x; i < hi; i += kBlock) {
    const double n = pn[i], dm = pm[i] - P;
    N += n;
    A = fma(n, dm, A);
    B += fma(n * dm, dm, pq[i]);
  }
  N = wave_sum(N);
  A = wave_sum(A);
  B = wave_sum(B);
  if (lane_id() == 0) {
    lds_m[3 * wave_id()] = N;
    lds_m[3 * wave_id() + 1] = A;
    lds_m[3 * wave_id() + 2] = B;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    N = 0.0;
    A = 0.0;
    B = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      N += lds_m[3 * w];
      A += lds_m[3 * w + 1];
      B += lds_m[3 * w + 2];
    }
    const double mean = N > 0.0 ? P + A / N : 0.0;
    const double m2 = N > 0.0 ? B - A * (A / N) : 0.0;
    a.folded[blockIdx.x] = N;
    a.folded[kMaxMomentParts + blockIdx.x] = mean;
    a.folded[2 * kMaxMomentParts + blockIdx.x] = m2 < 0.0 ? 0.0 : m2;
  }
}

// K3: thresholds from the moment partials (every workgroup), then the ten counts of its tile.
// One pass over the partials around the provisional centre P = mean of partial 0:
//   A = sum n_i (mean_i - P), B = sum M2_i + n_i (mean_i - P)^2, mean = P + A/N, M2 = B - A^2/N.
template <int GT, bool STREAM = false>  // tiles per group; non-temporal reads of acc (with lists only)
__global__ __launch_bounds__(kBlock) void k_gk_count_fused(const Args a) {
  __shared__ double lds_m[2 * kWaves];
  __shared__ uint32_t lds[kWaves * kNumThres];
  __shared__ uint32_t lds_over[kWaves];
  // The tiles are visited from the last to the first: the end of acc is what the accumulate
  // kernel wrote most recently, so it is the part most likely still to sit in the last-level cache.
  const uint32_t tile = gridDim.x - 1u - blockIdx.x;
  Span sp_;
  if (!locate_span<false>(a, tile, &sp_)) return;
  SegCtrl& c = a.ctrl[0];
  const uint32_t parts = a.moment_parts;
  const double* pn = a.use_folded ? a.folded : a.partial;
  const double* pm = pn + (a.use_folded ? (uint32_t)kMaxMomentParts : a.max_tiles);
  const double* pq = pm + (a.use_folded ? (uint32_t)kMaxMomentParts : a.max_tiles);
  const double z = c.z;
  const double P = pm[0];
  double A = 0.0, B = 0.0;
  for (uint32_t b0 = 0; b0 < parts; b0 += 4 * kBlock) {  // four partials per thread per round
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
  const double N = (double)a.d_total;
  const double mean = P + A / N;
  double m2 = B - A * (A / N);
  m2 = m2 < 0.0 ? 0.0 : m2;
  const double sd = (a.d_total - a.ddof < 1) ? 0.0 : sqrt(m2 / (double)(a.d_total - a.ddof));
  const double thres0 = mean + sd * z;
  double t64[kNumThres];
  candidate_thresholds(thres0, t64);
  float thr[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) thr[p] = (float)t64[p];
  const bool can_skip = thres0 > 0.0;
  if (tile == 0 && threadIdx.x == 0) {  // one workgroup publishes what every workgroup computed
#pragma unroll
    for (int p = 0; p < kNumThres; ++p) {
      c.t64[p] = t64[p];
      c.t32[p] = thr[p];
    }
    uint32_t flags = 0;
    if (!isfinite(mean) || !isfinite(sd) || !isfinite(thres0)) flags |= SPARSIFY_F_NONFINITE;
    c.flags = flags;
    sparsify_result& r = a.result[0];
    r.mean = mean;
    r.std = sd;
    r.z = z;
    r.thres0 = thres0;
  }

  uint32_t cnt[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) cnt[p] = 0;
  bool over = true;  // whether this tile's lists are incomplete (no lists at all: as good as that)
  if (a.list && can_skip) {
    // with lists (gaussiank_list.h): the entries above thres0, and the residual as if nothing
    // were selected; each wave has a stretch of the list buffer for this tile
    const uint32_t worker = tile * kWaves + wave_id();
    ListCursor lc;
    lc.cur = worker * a.list_cap;
    lc.end = lc.cur + a.list_cap;
    lc.over = false;
    for (uint32_t u = 0; u < sp_.nchunks; ++u) {
      const Tile t = chunk_of(sp_, u);
      const uint32_t run0 = (uint32_t)(t.tbase / kRun);
      if (t.full) count_list_chunk<true, STREAM>(a, t, run0, thr, cnt, lc);
      else count_list_chunk<false, STREAM>(a, t, run0, thr, cnt, lc);
    }
    over = lc.over;
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
    lds_over[wave_id()] = over ? 1u : 0u;
  }
  __syncthreads();
  if (threadIdx.x < kNumThres) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds[w * kNumThres + threadIdx.x];
    a.tile_counts[(size_t)threadIdx.x * a.max_tiles + tile] = s;  // [threshold][tile]
    if (s) atomicAdd(&a.group_counts[(tile / GT) * kNumThres + threadIdx.x], s);
  }
  if (a.list && threadIdx.x == 0) {
    // the compact kernel streams a tile whose lists are incomplete; the call's record says
    // whether there was one
    uint32_t any = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) any |= lds_over[w];
    a.tile_base[tile] = any;
    if (any) atomicOr(&a.list_stats[kListStatCopies + tile % kListStatCopies], 1u);
  }
}

// K5: every workgroup totals the group counts, walks Alg. 1 steps 5-13, finds the first output
// slot of its tile (groups before its own + tiles before it inside its group), then compacts.
// A workgroup takes a.compact_tiles consecutive tiles of one group (one tile without lists;
// with lists several, so that the tables are read a fraction as often: a wave then writes a
// tile's pairs from its lists, and if the lists do not serve the workgroup streams its tiles one
// after the other).
template <bool NORMS, int GT, int MG, bool STREAM>  // tiles per group, groups at most, non-temporal reads
__global__ __launch_bounds__(kBlock) void k_gk_compact_fused(const Args a) {
  __shared__ uint32_t lds_g[MG * kNumThres];    // group totals [group][threshold]
  __shared__ uint32_t lds_t[GT * kNumThres];    // counts of my group's tiles [threshold][tile]
  __shared__ uint32_t lds_tot[kNumThres];
  __shared__ uint32_t lds_base[2];              // survivors in the groups before mine; before the tile
  __shared__ uint32_t lds_lists[2];
  __shared__ uint32_t lds[kSlots * kWaves];
  __shared__ double lds_n[2 * kWaves];
  const uint32_t ntiles = a.flat_tiles;
  const uint32_t tile0 = blockIdx.x * a.compact_tiles;
  if (tile0 >= ntiles) return;
  const uint32_t tile1 = tile0 + a.compact_tiles < ntiles ? tile0 + a.compact_tiles : ntiles;
  SegCtrl& c = a.ctrl[0];
  const uint32_t ngroups = (ntiles + GT - 1) / GT;
  const uint32_t g = tile0 / GT, g0 = g * GT;                // (GT is a multiple of a.compact_tiles)
  // with lists: what the end of this kernel reads first is fetched before the tables (the lists'
  // statistics words, the records of the runs of this wave's first tile), so that those trips to
  // memory overlap the prologue
  uint32_t list_word = 0, over_mask = 0;  // bit j: the lists of tile0 + j are incomplete
  uint2 first_rec = make_uint2(0u, 0u);
  if (a.list) {
    list_word = a.list_stats[lane_id()];
    for (uint32_t j = 0; j < tile1 - tile0; ++j) over_mask |= (a.tile_base[tile0 + j] != 0 ? 1u : 0u) << j;
    const uint32_t t = tile0 + wave_id();
    uint32_t r0, r1;
    tile_runs(a, t < tile1 ? t : tile1 - 1u, &r0, &r1);
    first_rec = gk_list_first_records(a, r0, r1);
  }

  // Both tables go to LDS in rounds of four loads per thread, every load issued before the first
  // is waited for and none behind a branch (an index beyond the table re-reads a valid entry).
  for (uint32_t i0 = 0; i0 < ngroups * kNumThres; i0 += 4 * kBlock) {
    uint32_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * kBlock + threadIdx.x;
      v[u] = a.group_counts[i < ngroups * kNumThres ? i : 0u];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * kBlock + threadIdx.x;
      if (i < ngroups * kNumThres) lds_g[i] = v[u];
    }
  }
  const uint32_t upto = tile1 - 1u - g0;  // tiles of the group before my last tile: all I need
  for (uint32_t i0 = 0; i0 < (uint32_t)(GT * kNumThres); i0 += 4 * kBlock) {
    uint32_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * kBlock + threadIdx.x;
      const uint32_t p = i < (uint32_t)(GT * kNumThres) ? i / GT : 0u, j = i % GT;
      v[u] = a.tile_counts[(size_t)p * a.max_tiles + g0 + (j < upto ? j : upto)];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * kBlock + threadIdx.x;
      if (i < (uint32_t)(GT * kNumThres)) lds_t[i] = (i % GT < upto) ? v[u] : 0u;
    }
  }
  double t64[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) t64[p] = c.t64[p];
  const uint32_t flags0 = c.flags;
  __syncthreads();
  if (threadIdx.x < kNumThres) {
    uint32_t s = 0;
    for (uint32_t j = 0; j < ngroups; ++j) s += lds_g[j * kNumThres + threadIdx.x];
    lds_tot[threadIdx.x] = s;
  }
  __syncthreads();
  uint32_t tot[kNumThres];
#pragma unroll
  for (int p = 0; p < kNumThres; ++p) tot[p] = lds_tot[p];
  const Walk w = walk_thresholds(tot, a.flat_k);
  const bool overflow = (int64_t)tot[w.pos] > a.flat_cap;
  if (wave_id() == 0) {
    uint32_t x = 0, y = 0;
#pragma unroll
    for (int j = 0; j < MG; j += 64)
      if ((uint32_t)(j + lane_id()) < g) x += lds_g[(j + lane_id()) * kNumThres + w.pos];
#pragma unroll
    for (int j = 0; j < GT; j += 64)
      if ((uint32_t)(j + lane_id()) < tile0 - g0) y += lds_t[w.pos * GT + j + lane_id()];
    x = wave_sum(x);
    y = wave_sum(y);
    if (lane_id() == 0) {
      lds_base[0] = x;
      lds_base[1] = x + y;  // survivors before my first tile
    }
  }
  const double tf = t64[w.pos];
  const float thr = (float)tf;
  // With lists (gaussiank_list.h): a tile's lists hold its survivors when none of its stretches
  // ran out, thres0 is positive and the walk ended at thres0 or above it; a tile whose lists
  // are incomplete is streamed.  The record says "from the lists" when every tile's were.
  const bool lists_ok = a.list && w.pos >= kGkListPos && t64[kGkListPos] > 0.0;
  bool listed = false;
  if (a.list) {
    if (wave_id() == 0) {  // (list_totals of lists.h on the word fetched above)
      const uint64_t over = __ballot(lane_id() >= kListStatCopies && list_word != 0);
      if (lane_id() == 0) lds_lists[1] = over != 0 ? 1u : 0u;
    }
    __syncthreads();
    listed = lists_ok && lds_lists[1] == 0;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t flags = flags0;
    if (!w.in_band) flags |= SPARSIFY_F_EXHAUSTED;
    if (overflow) flags |= SPARSIFY_F_OVERFLOW;
    if (a.list) flags |= listed ? SPARSIFY_F_SHORTLIST : SPARSIFY_F_SHORTLIST_MISS;  // which way, no result
    sparsify_result& r = a.result[0];
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
    r.acc_sqnorm = 0.0;  // filled by k_norms_finalize when asked for
    r.residual_sqnorm = 0.0;
  }
  __syncthreads();
  const uint32_t groups_before = lds_base[0];
  // survivors of my group's tiles before `tile` (lds_t holds zeros from my last tile on)
  auto before_in_group = [&](uint32_t tile) {
    uint32_t x = 0;
#pragma unroll
    for (int j = 0; j < GT; j += 64)
      if ((uint32_t)(j + lane_id()) < tile - g0) x += lds_t[w.pos * GT + j + lane_id()];
    return wave_sum(x);
  };
  if (lists_ok && !overflow) {
    // the residual is in place (the count kernel wrote it); a wave writes a tile's pairs
    for (uint32_t tile = tile0 + wave_id(); tile < tile1; tile += kWaves) {
      if ((over_mask >> (tile - tile0)) & 1u) continue;
      uint32_t r0, r1;
      tile_runs(a, tile, &r0, &r1);
      const uint2 rec = tile == tile0 + wave_id() ? first_rec : gk_list_first_records(a, r0, r1);
      gk_list_compact_tile(a, r0, r1, thr, (int64_t)(groups_before + before_in_group(tile)), a.flat_cap, rec);
    }
    if (over_mask == 0) return;
    __syncthreads();
  } else if (lists_ok) {
    return;  // more survivors than cap: nothing is selected, and the residual is acc already
  }
  // the streaming compaction: every tile without lists, or the tiles whose lists are incomplete
  for (uint32_t tile = tile0; tile < tile1; ++tile) {
    if (lists_ok && !((over_mask >> (tile - tile0)) & 1u)) continue;
    Span sp_;
    if (!locate_span<false>(a, tile, &sp_)) return;
    if (tile != tile0 || lists_ok) {  // (without lists the first tile's slot is there already)
      __syncthreads();
      if (wave_id() == 0) {
        const uint32_t x = before_in_group(tile);
        if (lane_id() == 0) lds_base[1] = groups_before + x;
      }
      __syncthreads();
    }
    const int64_t out0 = (int64_t)lds_base[1];
    uint32_t run = 0;
    NormAcc norms = {0.0, 0.0};
    for (uint32_t u = 0; u < sp_.nchunks; ++u) {
      const Tile t = chunk_of(sp_, u);
      if (t.full) run = compact_chunk<true, NORMS, STREAM>(a, t, thr, overflow, out0, run, lds, norms);
      else run = compact_chunk<false, NORMS, STREAM>(a, t, thr, overflow, out0, run, lds, norms);
    }
    if (NORMS) store_norm_partial(a, norms, tile, lds_n);
  }
}

static_assert(kMaxGroups % 64 == 0 && kGroupTiles % 64 == 0 && kBigMaxGroups % 64 == 0 &&
              kBigGroupTiles % 64 == 0, "whole waves of lanes walk the groups and a group's tiles");

}  // namespace sp
