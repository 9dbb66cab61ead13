// Gaussian_k with short lists (vectors of 6 M elements and more, where the workspace has room
// for them; flat calls: gaussiank_flat.h, layer-wise calls, per segment: gaussiank_seg.h).
// The count kernel knows thres0 when it streams acc, and in every walk of Alg. 1
// steps 5-13 that ends at thres0 or above it (1, 1.125, 1.5, 2.25 or 3.375 times thres0: what
// error feedback produces, since the accumulated vector has lost its tail) the survivors are
// among the entries above thres0, about k of them.  So the count kernel also lists those
// entries (lists.h) and writes the residual as if nothing were selected, and the compact kernel,
// once it has walked the ten totals, writes the pairs from the lists and clears the selected
// entries of the residual instead of streaming acc and the residual once more: 12 + 8 bytes per
// element instead of 12 + 4 + 8 (12 + 4 instead of 12 + 4 + 4 in place).
//
// A walk that ends below thres0 or a thres0 that is not positive (the ten thresholds are then
// not in ascending order) leave the lists unused: the compact kernel takes its streaming body,
// which rewrites the whole residual.  A tile whose lists ran out of room (a flag per tile) is
// streamed in the same way, alone; in a layer-wise call its whole segment is.  Same launches,
// same results.
#pragma once
#include "common.h"
#include "gaussiank.h"
#include "lists.h"
#include "tile_io.h"

namespace sp {

constexpr int kGkListPos = 5;  // position of thres0 among the ten thresholds in ascending order

// count_values of gaussiank.h for thresholds known to ascend, plus the list of the slot's
// entries above thr[kGkListPos] (the ballots are those of the count).
template <bool FULL>
__device__ inline void count_list_values(const Args& a, int64_t tbase, uint32_t run0,
                                         const float (&v)[kPerThread], uint32_t valid,
                                         const float (&thr)[kNumThres], uint32_t (&cnt)[kNumThres],
                                         ListCursor& lc) {
  uint32_t off[kSlots], len[kSlots];
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    float x[4], m[4];
    bool ok[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      x[q] = v[4 * j + q];
      m[q] = fabsf(x[q]);
      ok[q] = FULL || ((valid >> (4 * j + q)) & 1u);
    }
    uint64_t any = 0;
#pragma unroll
    for (int p = 0; p < kGkListPos; ++p) {
      any = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint64_t b = __ballot(ok[q] && (m[q] > thr[p]));
        cnt[p] += (uint32_t)__builtin_popcountll(b);
        any |= b;
      }
    }
    off[j] = lc.cur;
    len[j] = 0;
    if (any != 0) {  // wave-uniform
      bool in[4];
      any = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        in[q] = ok[q] && (m[q] > thr[kGkListPos]);
        const uint64_t b = __ballot(in[q]);
        cnt[kGkListPos] += (uint32_t)__builtin_popcountll(b);
        any |= b;
      }
      if (any != 0) {
#pragma unroll
        for (int p = kGkListPos + 1; p < kNumThres; ++p) {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            cnt[p] += (uint32_t)__builtin_popcountll(__ballot(ok[q] && (m[q] > thr[p])));
        }
        const uint32_t i0 = (uint32_t)(tbase + (int64_t)(j * kBlock + (int)threadIdx.x) * 4);
        list_append_run(a, i0, x, in, lc, &off[j], &len[j]);
      }
    }
  }
  list_record_runs(a, run0, off, len);
}

// One chunk of the count kernel with lists: counts, the residual as if nothing were selected
// (nothing to write when acc is the residual), the list.
template <bool FULL, bool STREAM>  // STREAM: acc is read with the non-temporal hint (its last use if the lists serve)
__device__ inline void count_list_chunk(const Args& a, const Tile& t, uint32_t run0,
                                        const float (&thr)[kNumThres], uint32_t (&cnt)[kNumThres],
                                        ListCursor& lc) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL, STREAM>(a.acc, t, v);
  count_list_values<FULL>(a, t.tbase, run0, v, valid, thr, cnt, lc);
  if (!a.inplace) store_tile<FULL>(a.resid, t, v, valid);
}

// The records of the first 64 runs of a tile (runs r0 .. r1 - 1), one per lane: fetched before
// the compact kernel's prologue so that they are there when the walk is done.
__device__ inline uint2 gk_list_first_records(const Args& a, uint32_t r0, uint32_t r1) {
  const uint32_t r = r0 + lane_id();
  return a.run_table[r < r1 ? r : r1 - 1u];
}

// The pairs of one tile (runs r0 .. r1 - 1) from its lists, in index order, by one wave: the
// tile's first pair goes to slot `out0`; nothing is written at or beyond slot `cap`.  A lane owns a run; the lanes' counts are scanned across the wave, then every lane
// writes its run's survivors one after the other and clears them in the residual.  `first` holds
// the records of the tile's first 64 runs (gk_list_first_records).  Runs of up to kListBatch
// entries, the rule, are read once and kept in registers between the count and the write.
__device__ inline void gk_list_compact_tile(const Args& a, uint32_t r0, uint32_t r1, float thr,
                                            int64_t out0, int64_t cap, uint2 first) {
  int64_t out_run = out0;
  for (uint32_t rb = r0; rb < r1; rb += 64) {
    const uint32_t r = rb + lane_id();
    const uint2 rec = rb == r0 ? first : a.run_table[r < r1 ? r : r1 - 1u];
    const uint32_t n = r < r1 ? rec.y : 0u, off = rec.x;
    const uint32_t last = n ? n - 1u : 0u;
    const uint32_t nmax = wave_max(n);
    if (nmax == 0) continue;
    auto fetch = [&](uint32_t i0, uint2 (&e)[kListBatch]) {
#pragma unroll
      for (int u = 0; u < kListBatch; ++u) {
        uint32_t i = off + (i0 + u < last ? i0 + u : last);
        i = i < a.list_last ? i : a.list_last;
        e[u] = a.list[i];
      }
    };
    auto emit = [&](uint32_t i0, const uint2 (&e)[kListBatch], int64_t& pos) {
#pragma unroll
      for (int u = 0; u < kListBatch; ++u) {
        const float val = __uint_as_float(e[u].y);
        if (i0 + u < n && fabsf(val) > thr) {
          if (pos < cap) {
            a.out_idx[pos] = e[u].x;
            a.out_val[pos] = val;
          }
          a.resid[e[u].x] = 0.0f;
          ++pos;
        }
      }
    };
    uint2 e[kListBatch];
    uint32_t csel = 0;
    for (uint32_t i0 = 0; i0 < nmax; i0 += kListBatch) {
      fetch(i0, e);
#pragma unroll
      for (int u = 0; u < kListBatch; ++u)
        csel += (i0 + u < n && fabsf(__uint_as_float(e[u].y)) > thr) ? 1u : 0u;
    }
    const uint32_t inc = wave_inclusive_scan(csel);
    int64_t pos = out_run + (int64_t)(inc - csel);
    if (nmax <= (uint32_t)kListBatch) {
      emit(0, e, pos);  // (the one batch is still in registers)
    } else {
      for (uint32_t i0 = 0; i0 < nmax; i0 += kListBatch) {
        fetch(i0, e);
        emit(i0, e, pos);
      }
    }
    out_run += (int64_t)__shfl(inc, 63, 64);
  }
}

}  // namespace sp
