// Exact Top_k, flat vectors, the short-list form.  Before the accumulate pass one workgroup
// takes a sample of acc and sets a listing key tau a little below where the k-th key is expected
// (the sample's quantile for about four times k entries).  The accumulate kernel then, besides
// acc and the first digit's histogram, writes the residual (as if nothing were selected) and a
// list of every entry whose key exceeds tau.  If the lists hold at least k entries they hold the
// k largest (every key >= the k-th key exceeds tau), and everything that follows reads the lists,
// a fraction of a per cent of the vector, instead of acc: the three remaining digit passes, the
// per-tile counts, and the compaction, which only clears the selected entries of the residual.
// 16 bytes per element instead of 24 (12 instead of 28 in place).
//
// The guess cannot make the result wrong.  Whether the lists are used is decided from their
// exact length; if they are too short (a sample that misleads: a constant vector, say) or a
// list ran out of room, every later kernel of the call takes its other body, the form without
// lists (topk_filter.h, or topk_flat.h in place), which overwrites whatever the accumulate
// kernel put into the residual.  The launch sequence is the same either way.
//
// The lists themselves (per-wave stretches, one record per 256-element run): lists.h.
#pragma once
#include "common.h"
#include "tile_io.h"
#include "gaussiank.h"
#include "lists.h"
#include "topk.h"
#include "topk_select.h"

namespace sp {

constexpr int kListSample = 16 * kBlock;          // entries of acc the init kernel looks at
constexpr int kListAim = 4;                       // the lists should hold about this many times k

// ---- the listing key (one workgroup, inside the init kernel) -------------------------------------
// 4096 entries of acc, four consecutive ones every d/1024 elements; tau is the lower edge of the
// 16-bit key bin (sign dropped: exponent and eight mantissa bits) that holds the sample's r-th
// largest key, r = the sample's share of kListAim * k entries, at least 16.  `lds_h` holds 256
// words, `lds_sel` kWaves + 3.
__device__ inline uint32_t listing_key_from_sample(const uint32_t (&key)[16], int64_t k, int64_t n,
                                                   int64_t m, uint32_t* lds_h, uint32_t* lds_sel);
__device__ inline uint32_t sample_listing_key(const Args& a, uint32_t* lds_h, uint32_t* lds_sel) {
  const int64_t stride4 = (a.d_total / 4) / (kListSample / 4);  // >= 1: the host asks for d >= 4 * kListSample
  uint32_t key[16];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = (int64_t)(u * kBlock + (int)threadIdx.x) * stride4 * 4;
    const f32x4 g = *reinterpret_cast<const f32x4*>(a.grad + i);
    const f32x4 e = *reinterpret_cast<const f32x4*>(a.resid + i);
    key[4 * u + 0] = mag_key(g.x + e.x);
    key[4 * u + 1] = mag_key(g.y + e.y);
    key[4 * u + 2] = mag_key(g.z + e.z);
    key[4 * u + 3] = mag_key(g.w + e.w);
  }
  return listing_key_from_sample(key, a.flat_k, a.d_total, kListSample, lds_h, lds_sel);
}

// The sample holds m of the n entries (keys beyond the sample are zero) and k entries are asked for.
__device__ inline uint32_t listing_key_from_sample(const uint32_t (&key)[16], int64_t k, int64_t n,
                                                   int64_t m, uint32_t* lds_h, uint32_t* lds_sel) {
  uint64_t want = ((uint64_t)kListAim * (uint64_t)k * (uint64_t)m + (uint64_t)n - 1) / (uint64_t)n;
  if (want < 16) want = 16;
  if (want > (uint64_t)m) want = (uint64_t)m;
  {
    // As a rule the key asked for lies within a factor of two of the sample's largest: then one
    // histogram of the distance to it, in steps of the 16-bit key, finds it, and only the few
    // keys that close to the largest are added (an exponent histogram of the whole sample puts
    // half of its 4096 increments on one LDS address, one after the other).
    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = (key[i] >> 15) > mx ? (key[i] >> 15) : mx;
    mx = wave_max(mx);
    lds_h[threadIdx.x] = 0;
    if (lane_id() == 0) lds_sel[wave_id()] = mx;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mx = lds_sel[w] > mx ? lds_sel[w] : mx;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t dist = mx - (key[i] >> 15);
      if (dist < 255u) atomicAdd(&lds_h[dist], 1u);
    }
    __syncthreads();
    const uint32_t v = threadIdx.x < 255u ? lds_h[threadIdx.x] : 0u;
    if (threadIdx.x == 0) lds_sel[kWaves] = 0xFFFFFFFFu;
    uint32_t total;
    const uint32_t closer = block_exclusive_scan<kWaves>(v, lds_sel, &total);  // keys nearer to the largest
    if (v != 0 && closer < (uint32_t)want && (uint32_t)want <= closer + v) lds_sel[kWaves] = threadIdx.x;
    __syncthreads();
    const uint32_t dist = lds_sel[kWaves];
    __syncthreads();  // lds_h and lds_sel are used again below
    if (dist != 0xFFFFFFFFu) return (mx - dist) << 15;  // block-uniform
  }
  uint32_t prefix = 0, rank = (uint32_t)want;
#pragma unroll 1
  for (int pass = 0; pass < 2; ++pass) {
    lds_h[threadIdx.x] = 0;
    __syncthreads();
    const int shift = digit_shift(pass), hi_shift = digit_shift(pass - 1);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (pass == 0 || (key[i] >> hi_shift) == prefix) atomicAdd(&lds_h[(key[i] >> shift) & 255u], 1u);
    __syncthreads();
    const Digit dg = digit_from_bins(lds_h[255u - threadIdx.x], pass, prefix, rank, lds_sel);  // barriers
    prefix = dg.prefix;
    rank = dg.k_rem;
  }
  return prefix << digit_shift(1);
}

// Clears the histograms and the group totals, resets the selection state (k_topk_init_fused) and
// sets the listing key.
__global__ __launch_bounds__(kBlock) void k_topk_init_list(const Args a, uint32_t hist_words) {
  __shared__ uint32_t lds_h[256];
  __shared__ uint32_t lds_sel[kWaves + 3];
  for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < hist_words; i += gridDim.x * kBlock)
    a.hist[i] = 0;
  if (blockIdx.x != 0) return;
  for (uint32_t i = threadIdx.x; i < (uint32_t)(kBigMaxGroups * kNumThres); i += kBlock)
    a.group_counts[i] = 0;
  if (threadIdx.x < 2 * kListStatCopies) a.list_stats[threadIdx.x] = 0;
  const uint32_t tau = sample_listing_key(a, lds_h, lds_sel);
  if (threadIdx.x == 0) {
    SegCtrl& c = a.ctrl[0];
    c.prefix = 0;
    c.k_rem = (uint32_t)a.flat_k;
    c.n_eq = 0;
    c.rank_ties = 0;
    c.select_none = 0;
    c.bad = 0;
    c.tau_key = tau;
    c.list_mode = 0;
    sparsify_result& r = a.result[0];
    clear_result(r);
    r.nnz = (uint32_t)a.flat_k;
  }
}

// ---- the accumulate kernel with lists -------------------------------------------------------------
// Appends the entries of this wave's four runs of a chunk (keys above tau) and records the runs.
// `v` holds acc.
template <bool FULL>
__device__ inline void list_chunk(const Args& a, int64_t tbase, uint32_t run0,
                                  const float (&v)[kPerThread], uint32_t valid, uint32_t tau,
                                  ListCursor& lc) {
  uint32_t off[kSlots], cnt[kSlots];
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    bool in[4];
    float x[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bool ok = FULL || ((valid >> (4 * j + q)) & 1u);
      x[q] = v[4 * j + q];
      in[q] = ok && (mag_key(x[q]) > tau);
    }
    const uint32_t i0 = (uint32_t)(tbase + (int64_t)(j * kBlock + (int)threadIdx.x) * 4);
    list_append_run(a, i0, x, in, lc, &off[j], &cnt[j]);
  }
  list_record_runs(a, run0, off, cnt);
}

template <bool FULL, bool HIST>
__device__ inline void accum_hist_list_chunk(const Args& a, const Tile& t, uint32_t run0, uint32_t* h,
                                             uint32_t tau, ListCursor& lc) {
  float g[kPerThread], e[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.grad, t, g);
  load_tile<FULL>(a.resid, t, e);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) g[i] = g[i] + e[i];  // Eq. (2): one fp32 add
  if (!a.inplace) store_tile<FULL>(a.acc, t, g, valid);
  store_tile<FULL>(a.resid, t, g, valid);  // the residual if nothing of this chunk is selected
  if (HIST) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if (FULL || ((valid >> i) & 1u)) atomicAdd(&h[mag_key(g[i]) >> 23], 1u);
  }
  list_chunk<FULL>(a, t.tbase, run0, g, valid, tau, lc);
}

// A full chunk whose loads were issued earlier (accum_issue of gaussiank.h).
template <bool HIST>
__device__ inline void accum_hist_list_finish(const Args& a, int64_t tbase, AccIn& in, uint32_t* h,
                                              uint32_t tau, ListCursor& lc) {
  const Tile t = full_chunk_at(tbase);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) in.g[i] = in.g[i] + in.e[i];  // Eq. (2): one fp32 add
  // (acc is not read again by this call when the lists serve, nor by the next call: its
  // stores are marked non-temporal so that it does not displace the residual, which the next
  // call reads first)
  if (!a.inplace) store_tile<true, true>(a.acc, t, in.g, 0xFFFFu);
  store_tile<true>(a.resid, t, in.g, 0xFFFFu);
  if (HIST) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) atomicAdd(&h[mag_key(in.g[i]) >> 23], 1u);
  }
  list_chunk<true>(a, tbase, (uint32_t)(tbase / kRun), in.g, 0xFFFFu, tau, lc);
}

// End of an accumulate kernel with lists: the workgroup's histogram into one replica of the
// global one, the entries its waves listed (and whether a stretch ran out) into one replica of
// the lists' statistics.  `lds_stat` holds 2 * kWaves words.
template <bool HIST>
__device__ inline void finish_accum_list(const Args& a, uint32_t (*h)[256], const ListCursor& lc,
                                         uint32_t worker, uint32_t* lds_stat) {
  if (lane_id() == 0) {
    lds_stat[2 * wave_id()] = lc.cur - worker * a.list_cap;
    lds_stat[2 * wave_id() + 1] = lc.over ? 1u : 0u;
  }
  __syncthreads();
  if (HIST) {
    const int bin = threadIdx.x;
    uint32_t v = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) v += h[w][bin];
    if (v) atomicAdd(&pass_hist(a, 0)[(blockIdx.x % kTopkCopies) * 256 + bin], v);
  }
  if (threadIdx.x == 0) {
    uint32_t n = 0, over = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      n += lds_stat[2 * w];
      over |= lds_stat[2 * w + 1];
    }
    const uint32_t copy = blockIdx.x % kListStatCopies;
    if (n) atomicAdd(&a.list_stats[copy], n);
    if (over) atomicOr(&a.list_stats[kListStatCopies + copy], 1u);
  }
}

// The resident accumulate kernel of topk_filter.h plus the residual write and the lists, with
// the next chunk's loads in flight while this one is worked on (two register sets in turn, no
// load behind a branch inside the loop: see k_accum_moments_fused).
//
// DGC: the same pass for DGC_k (dgck.h).  The listing key is then the sample's threshold Ts
// itself, chosen in the prologue from the last digit pass over the sample: every entry whose key
// reaches Ts is listed (key >= Ts is key > Ts - 1; with Ts = 0 everything is kept, which no list
// holds: the stretches are reported as run out at once).  No histogram is taken.
template <bool DGC>
__global__ __launch_bounds__(kBlock) void k_topk_accum_list(const Args a) {
  __shared__ uint32_t h[DGC ? 1 : kWaves][256];
  __shared__ uint32_t lds_stat[2 * kWaves];
  __shared__ uint32_t lds_sel[kWaves + 3];
  uint32_t tau;
  bool none = false;
  if (DGC) {
    SegCtrl& c = a.ctrl[0];
    const Digit dg = choose_digit(pass_hist(a, 3), 3, c.sel_prefix[2], c.sel_krem[2], lds_sel);  // barriers
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      c.sel_prefix[3] = dg.prefix;  // Ts: a whole 31-bit key
      c.sel_krem[3] = dg.k_rem;
    }
    none = dg.prefix == 0;
    tau = none ? 0u : dg.prefix - 1u;
  } else {
#pragma unroll
    for (int w = 0; w < kWaves; ++w) h[w][threadIdx.x] = 0;
    __syncthreads();
    tau = a.ctrl[0].tau_key;
  }
  const uint32_t worker = blockIdx.x * kWaves + wave_id();
  ListCursor lc;
  lc.cur = worker * a.list_cap;
  lc.end = lc.cur + a.list_cap;
  lc.over = none;
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  const uint32_t nfull = (uint32_t)(a.d_total / kChunk);
  const uint32_t step = gridDim.x;
  const uint32_t n = blockIdx.x < nfull ? (nfull - blockIdx.x + step - 1) / step : 0u;  // my full chunks
  auto at = [&](uint32_t k) { return (int64_t)(blockIdx.x + k * step) * kChunk; };
  uint32_t* hw = h[DGC ? 0 : wave_id()];
  constexpr bool HIST = !DGC;
  if (n > 0) {
    AccIn x, y;
    uint32_t k = 0;
    accum_issue(a, at(0), x);
    while (k + 2 < n) {
      accum_issue(a, at(k + 1), y);
      __builtin_amdgcn_sched_barrier(0);
      accum_hist_list_finish<HIST>(a, at(k), x, hw, tau, lc);
      accum_issue(a, at(k + 2), x);
      __builtin_amdgcn_sched_barrier(0);
      accum_hist_list_finish<HIST>(a, at(k + 1), y, hw, tau, lc);
      k += 2;
    }
    if (n - k == 2) {
      accum_issue(a, at(k + 1), y);
      __builtin_amdgcn_sched_barrier(0);
      accum_hist_list_finish<HIST>(a, at(k), x, hw, tau, lc);
      accum_hist_list_finish<HIST>(a, at(k + 1), y, hw, tau, lc);
    } else {
      accum_hist_list_finish<HIST>(a, at(k), x, hw, tau, lc);
    }
  }
  if (nfull < nchunks && nfull % step == blockIdx.x) {  // the ragged last chunk
    Tile t;
    t.seg = 0;
    t.tbase = (int64_t)nfull * kChunk;
    t.lo = t.tbase;
    t.hi = a.d_total;
    t.full = false;
    accum_hist_list_chunk<false, HIST>(a, t, (uint32_t)(t.tbase / kRun), hw, tau, lc);
  }
  finish_accum_list<HIST>(a, h, lc, worker, lds_stat);
}

// ---- reading the lists -----------------------------------------------------------------------------
// Whether the lists can serve the call: no stretch ran out and they hold at least k entries.
// Computed the same way by every workgroup of the kernel that follows the accumulate kernel
// (`lds` holds 2 words; one barrier); the first tile's workgroup publishes it.
__device__ inline bool lists_usable(const Args& a, uint32_t* lds) {
  list_totals(a, lds);
  return lds[1] == 0 && (int64_t)lds[0] >= a.flat_k;
}

// A digit pass over the lists: the histogram of digit `pass` among the listed keys whose higher
// digits equal `prefix` (pass 0: among all of them), one wave per tile (any grid), into the
// wave's LDS histogram `hw`.
__device__ inline void list_digit_pass(const Args& a, int pass, uint32_t prefix, uint32_t* hw) {
  const uint32_t ntiles = seg_ntiles(0, a.d_total, a.tile_chunks);
  const int hi_shift = pass == 0 ? 31 : digit_shift(pass - 1);  // keys have 31 bits: prefix 0 matches all
  const int shift = digit_shift(pass);
  const uint32_t mask = (1u << digit_bits(pass)) - 1u;
  for (uint32_t tile = blockIdx.x * kWaves + wave_id(); tile < ntiles; tile += gridDim.x * kWaves) {
    for_each_list_entry(a, tile, [&](uint2 e, bool valid) {
      const uint32_t key = e.y & 0x7FFFFFFFu;
      wave_hist_add(hw, (key >> shift) & mask, valid && (key >> hi_shift) == prefix);
    });
  }
}

// Per tile, from the lists: the survivors (keys above T, plus the keys equal to T when all of
// those are kept) and, when ties are ranked, the keys equal to T; per-group totals by atomics.
// One wave per tile (any grid).
template <int GT>
__device__ inline void list_tile_counts(const Args& a, uint32_t T, bool rank_ties) {
  const uint32_t ntiles = seg_ntiles(0, a.d_total, a.tile_chunks);
  for (uint32_t tile = blockIdx.x * kWaves + wave_id(); tile < ntiles; tile += gridDim.x * kWaves) {
    uint32_t gt = 0, eq = 0;
    for_each_list_entry(a, tile, [&](uint2 e, bool valid) {
      const uint32_t key = e.y & 0x7FFFFFFFu;
      gt += (valid && key > T) ? 1u : 0u;
      eq += (valid && key == T) ? 1u : 0u;
    });
    gt = wave_sum(gt);
    eq = wave_sum(eq);
    if (lane_id() == 0) {
      const uint32_t taken = gt + (rank_ties ? 0u : eq);
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

// The pairs of one tile (runs r0 .. r1 - 1) from its lists, in index order, by one wave: `out_run` survivors and
// `tie_run` keys equal to T precede the tile (ties before it capped by the caller).  A lane owns
// a run; the lanes' counts are scanned across the wave, then every lane writes its run's
// survivors one after the other and clears them in the residual.
// The output range starts at slot `out0` and holds `cap` pairs (flat calls: 0 and the call's cap).
// `head`: the head of these runs (lists.h) if the caller has fetched it, else null.
__device__ inline void list_compact_runs(const Args& a, uint32_t r0, uint32_t r1, uint32_t T,
                                         uint32_t take, bool rank_ties, uint32_t out_run,
                                         uint32_t tie_run, int64_t out0, int64_t cap,
                                         const ListHead* head = nullptr) {
  for (uint32_t rb = r0; rb < r1; rb += 64) {
    const uint32_t r = rb + lane_id();
    const bool first = head != nullptr && rb == r0;  // wave-uniform
    const uint2 rec = first ? head->rec : a.run_table[r < r1 ? r : r1 - 1u];
    const uint32_t n = r < r1 ? rec.y : 0u, off = rec.x;
    const uint32_t last = n ? n - 1u : 0u;
    const uint32_t nmax = wave_max(n);
    uint32_t csel = 0, ceq = 0;
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
      for (int u = 0; u < kListBatch; ++u) {
        const uint32_t key = e[u].y & 0x7FFFFFFFu;
        const bool valid = i0 + u < n;
        csel += (valid && (key > T || (!rank_ties && key == T))) ? 1u : 0u;
        ceq += (valid && rank_ties && key == T) ? 1u : 0u;
      }
    }
    // ties in index order: this lane's come after those of the lanes below
    const uint32_t ties_inc = wave_inclusive_scan(ceq);
    const uint32_t ties_before = tie_run + ties_inc - ceq;
    const uint32_t room = take > ties_before ? take - ties_before : 0u;
    const uint32_t kept_ties = ceq < room ? ceq : room;
    const uint32_t mine = csel + kept_ties;
    const uint32_t inc = wave_inclusive_scan(mine);
    uint32_t pos = out_run + inc - mine;
    uint32_t tie_pos = ties_before;
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
      for (int u = 0; u < kListBatch; ++u) {
        const uint32_t key = e[u].y & 0x7FFFFFFFu;
        const bool valid = i0 + u < n;
        bool sel = valid && (key > T || (!rank_ties && key == T));
        if (valid && rank_ties && key == T) {
          sel = tie_pos < take;
          ++tie_pos;
        }
        if (sel) {
          if ((int64_t)pos < cap) {
            a.out_idx[out0 + pos] = e[u].x;
            a.out_val[out0 + pos] = __uint_as_float(e[u].y);
          }
          a.resid[e[u].x] = 0.0f;
          ++pos;
        }
      }
    }
    out_run += __shfl(inc, 63, 64);
    tie_run += __shfl(ties_inc, 63, 64);
  }
}
__device__ inline void list_compact_tile(const Args& a, uint32_t tile, uint32_t T, uint32_t take,
                                         bool rank_ties, uint32_t out_run, uint32_t tie_run) {
  uint32_t r0, r1;
  tile_runs(a, tile, &r0, &r1);
  list_compact_runs(a, r0, r1, T, take, rank_ties, out_run, tie_run, 0, a.flat_cap);
}

}  // namespace sp
