// Short lists of (index, value) entries written by a kernel that streams the vector, read back by
// the kernels after it (Top_k and DGC_k: topk_list.h, dgck.h; Gaussian_k: gaussiank_list.h).
//
// Lists are kept per wave of the writing kernel: a wave appends the entries of each 256-element
// run it streams (one wave instruction's worth of a chunk, in index order) to its own stretch of
// the list buffer and records (first entry, entries) per run, so that later kernels find the
// entries of a tile in index order.  A stretch that runs out of room is reported in the lists'
// statistics words, and the kernels after it then do not use the lists at all.
#pragma once
#include "common.h"
#include "tile_io.h"

namespace sp {

constexpr int kRun = 256;                         // elements per run: 64 lanes x 4
constexpr int kRunsPerChunk = kChunk / kRun;      // 16
constexpr int kListStatCopies = 32;               // replicas of the lists' length and overflow words

// A wave's position in its stretch of the list buffer (wave-uniform).
struct ListCursor {
  uint32_t cur, end;
  bool over;
};

// Appends this wave's entries of one run: the lanes' elements i0 .. i0 + 3 (values x[0..3]) for
// which in[q] holds, lane after lane.  Returns the run's record (first entry, entries) in
// *off, *cnt; a run that does not fit makes the stretch run out (sticky: nothing more is appended).
__device__ inline void list_append_run(const Args& a, uint32_t i0, const float (&x)[4],
                                       const bool (&in)[4], ListCursor& lc, uint32_t* off,
                                       uint32_t* cnt) {
  uint32_t tot = 0, mine = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint64_t m = __ballot(in[q]);
    tot += (uint32_t)__builtin_popcountll(m);
    mine += lanes_below(m);
  }
  if (tot > lc.end - lc.cur) lc.over = true;
  *off = lc.cur;
  *cnt = lc.over ? 0u : tot;
  if (!lc.over && tot != 0) {
    uint32_t pos = lc.cur + mine;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (in[q]) {
        a.list[pos] = make_uint2(i0 + q, __float_as_uint(x[q]));
        ++pos;
      }
    }
    lc.cur += tot;
  }
}

// The records of this wave's four runs of a chunk whose first run is run0: run (chunk, slot j,
// wave w) is run0 + 4 j + w.  (Flat vectors: run0 = tbase / 256, run r covers elements
// [256 r, 256 r + 256); layer-wise calls number the runs by tile and chunk.)
__device__ inline void list_record_runs(const Args& a, uint32_t run0, const uint32_t (&off)[kSlots],
                                        const uint32_t (&cnt)[kSlots]) {
  if (lane_id() < kSlots) {
    const int j = lane_id();
    const uint32_t o = j == 0 ? off[0] : j == 1 ? off[1] : j == 2 ? off[2] : off[3];
    const uint32_t c = j == 0 ? cnt[0] : j == 1 ? cnt[1] : j == 2 ? cnt[2] : cnt[3];
    a.run_table[run0 + j * kWaves + wave_id()] = make_uint2(o, c);
  }
}

// lds[0] = entries listed, lds[1] = whether a stretch ran out (then lds[0] is not all of them).
// `lds` holds 2 words; one barrier.
__device__ inline void list_totals(const Args& a, uint32_t* lds) {
  if (wave_id() == 0) {
    static_assert(2 * kListStatCopies == 64, "one lane per word");
    const uint32_t w = a.list_stats[lane_id()];
    const uint32_t total = wave_sum(lane_id() < kListStatCopies ? w : 0u);
    const uint64_t over = __ballot(lane_id() >= kListStatCopies && w != 0);
    if (lane_id() == 0) {
      lds[0] = total;
      lds[1] = over != 0 ? 1u : 0u;
    }
  }
  __syncthreads();
}

// the runs of a tile (every chunk has kRunsPerChunk records, empty ones beyond the vector's end)
__device__ inline void tile_runs(const Args& a, uint32_t tile, uint32_t* r0, uint32_t* r1) {
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  const uint32_t c0 = tile * a.tile_chunks;
  const uint32_t c1 = c0 + a.tile_chunks < nchunks ? c0 + a.tile_chunks : nchunks;
  *r0 = c0 * kRunsPerChunk;
  *r1 = c1 * kRunsPerChunk;
}

__device__ inline uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = __shfl_xor(v, off, 64);
    v = o > v ? o : v;
  }
  return v;
}

// One lane per run of the tile (runs r0 .. r1 - 1), 64 runs at a time: the lanes fetch their runs' records, then
// their runs' entries four at a time.  No load sits behind a branch (a wave would wait for each
// before it issues the next): a lane past the end of its run re-reads the run's last entry (an
// empty run the entry at its offset), kept inside the buffer, and reports it as not valid.
// fn(entry, valid) is called by the whole wave; the order of the calls is not the index order.
constexpr int kListBatch = 4;

// The head of a tile's lists, which a wave can have on order before it knows the tile's extent
// or whether it will read the lists at all (a kernel whose prologue makes several dependent
// trips to memory of its own): the records of the tile's first 64 run slots, then the first
// kListBatch entries at each record's offset.  A slot beyond the tile's chunks was never written
// and may hold anything: every index is kept inside the buffers, and the reader drops what lies
// beyond the tile's runs and the runs' lengths.
struct ListHead {
  uint2 rec;
  uint2 e[kListBatch];
};
__device__ inline void list_head_records(const Args& a, uint32_t r0, uint32_t nslots, ListHead& h) {
  const uint32_t l = (uint32_t)lane_id();
  h.rec = a.run_table[r0 + (l < nslots ? l : nslots - 1u)];
}
__device__ inline void list_head_entries(const Args& a, ListHead& h) {
#pragma unroll
  for (int u = 0; u < kListBatch; ++u) {
    const uint32_t i = h.rec.x + (uint32_t)u;
    h.e[u] = a.list[i < a.list_last ? i : a.list_last];
  }
}

// `head`: the head of these runs if the caller has fetched it (then r0 is its first slot), else null.
template <typename F>
__device__ inline void for_each_list_entry_of_runs(const Args& a, uint32_t r0, uint32_t r1,
                                                   const ListHead* head, F fn) {
  for (uint32_t rb = r0; rb < r1; rb += 64) {
    const uint32_t r = rb + lane_id();
    const bool first = head != nullptr && rb == r0;  // wave-uniform
    const uint2 rec = first ? head->rec : a.run_table[r < r1 ? r : r1 - 1u];
    const uint32_t n = r < r1 ? rec.y : 0u, off = rec.x;
    const uint32_t last = n ? n - 1u : 0u;
    const uint32_t nmax = wave_max(n);
    for (uint32_t i0 = 0; i0 < nmax; i0 += kListBatch) {
      uint2 e[kListBatch];
      if (first && i0 == 0) {
#pragma unroll
        for (int u = 0; u < kListBatch; ++u) e[u] = head->e[u];
      } else {
#pragma unroll
        for (int u = 0; u < kListBatch; ++u) {
          uint32_t i = off + (i0 + u < last ? i0 + u : last);
          i = i < a.list_last ? i : a.list_last;
          e[u] = a.list[i];
        }
      }
#pragma unroll
      for (int u = 0; u < kListBatch; ++u)
        if (i0 + u < nmax) fn(e[u], i0 + u < n);  // wave-uniform condition
    }
  }
}
template <typename F>
__device__ inline void for_each_list_entry(const Args& a, uint32_t tile, F fn) {
  uint32_t r0, r1;
  tile_runs(a, tile, &r0, &r1);
  for_each_list_entry_of_runs(a, r0, r1, nullptr, fn);
}

}  // namespace sp
