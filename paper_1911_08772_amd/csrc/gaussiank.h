// Gaussian_k (Algorithm 1) on gfx950: fused accumulate + fp64 moments, on-device normal
// quantile, one multi-threshold count pass, on-device threshold walk, ordered compaction with
// the residual write.  This file holds the building blocks shared by the forms (quantile,
// moment accumulation, threshold candidates, the walk, count and compact of one chunk, sums and
// prefix sums by one large workgroup).  The flat form is in gaussiank_flat.h, the layer-wise form
// in gaussiank_seg.h.
#pragma once
#include "common.h"
#include "tile_io.h"

namespace sp {

// ---- upper-tail standard normal quantile (Alg. 1 steps 3-4) ---------------------------------
// Rational starting value (Hastings' approximation, |error| < 5e-4) polished by Halley steps on
// f(z) = erfc(z/sqrt 2)/2 - q, f' = -pdf(z), f'' = z pdf(z); cubic convergence, so three steps
// reach fp64 accuracy from that start.
__device__ inline double norm_isf(double q) {
  if (!(q > 0.0)) return __longlong_as_double(0x7FF0000000000000ll);
  if (q >= 1.0) return -__longlong_as_double(0x7FF0000000000000ll);
  const bool flip = q > 0.5;
  const double p = flip ? 1.0 - q : q;
  if (p == 0.5) return 0.0;
  const double t = sqrt(-2.0 * log(p));
  double z = t - (2.515517 + t * (0.802853 + t * 0.010328)) /
                     (1.0 + t * (1.432788 + t * (0.189269 + t * 0.001308)));
  if (z < 0.0) z = 0.0;
  for (int it = 0; it < 4; ++it) {
    const double pdf = exp(-0.5 * z * z) * 0.3989422804014326779399461;
    if (!(pdf > 0.0)) break;
    const double f = 0.5 * erfc(z * 0.7071067811865475244008444) - p;
    const double dz = 2.0 * f / (2.0 * pdf - f * z);
    z += dz;
    if (fabs(dz) <= 1e-16 * fabs(z)) break;
  }
  return flip ? -z : z;
}

// ---- K1: acc = grad + residual, per-tile (n, mean, M2) --------------------------------------
// Per-thread shifted sums sum(x-p), sum((x-p)^2) in fp64 around a wave-uniform pivot p taken
// from a register (the first valid element the wave meets), so nothing is lost to cancellation
// whatever the mean is.
struct MomAcc {
  double n, s1, s2, pivot;
  bool have_pivot;
};

template <bool FULL>
__device__ inline void accum_moments_chunk(const Args& a, const Tile& t, MomAcc& m) {
  float g[kPerThread], e[kPerThread];
  const uint32_t valid = load_tile<FULL, true>(a.grad, t, g);
  load_tile<FULL>(a.resid, t, e);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) g[i] = g[i] + e[i];  // Eq. (2): one fp32 add
  store_tile<FULL>(a.acc, t, g, valid);

  if (!m.have_pivot) {  // wave-uniform
    float first = g[0];
    bool has = true;
    if (!FULL) {
      has = valid != 0;
      first = 0.0f;
#pragma unroll
      for (int i = kPerThread - 1; i >= 0; --i)
        if ((valid >> i) & 1u) first = g[i];
    }
    const uint64_t owners = __ballot(has);
    if (owners != 0) {
      m.pivot = (double)__shfl(first, __builtin_ctzll(owners), 64);
      m.have_pivot = true;
    }
  }
  if (m.have_pivot) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      if (FULL || ((valid >> i) & 1u)) {
        const double c = (double)g[i] - m.pivot;
        m.s1 += c;
        m.s2 = fma(c, c, m.s2);
      }
    }
    m.n += FULL ? (double)kPerThread : (double)__popc(valid);
  }
}

// The same for a full chunk in two halves, so that a caller can have the next chunk's loads in
// flight while it works on this one: `accum_issue` only issues the eight 16-byte loads.
struct AccIn {
  float g[kPerThread], e[kPerThread];
};
__device__ inline Tile full_chunk_at(int64_t tbase) {
  Tile t;
  t.seg = 0;
  t.tbase = tbase;
  t.lo = tbase;
  t.hi = tbase + kChunk;
  t.full = true;
  return t;
}
__device__ inline void accum_issue(const Args& a, int64_t tbase, AccIn& in) {
  const Tile t = full_chunk_at(tbase);
  load_tile<true, true>(a.grad, t, in.g);
  load_tile<true>(a.resid, t, in.e);
}
template <bool STREAM = false>
__device__ inline void accum_finish(const Args& a, int64_t tbase, AccIn& in, MomAcc& m) {
  const Tile t = full_chunk_at(tbase);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) in.g[i] = in.g[i] + in.e[i];  // Eq. (2): one fp32 add
  store_tile<true, STREAM>(a.acc, t, in.g, 0xFFFFu);
  if (!m.have_pivot) {  // wave-uniform: the first element the wave meets
    m.pivot = (double)__shfl(in.g[0], 0, 64);
    m.have_pivot = true;
  }
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const double c = (double)in.g[i] - m.pivot;
    m.s1 += c;
    m.s2 = fma(c, c, m.s2);
  }
  m.n += (double)kPerThread;
}

// Combines the four waves' shifted sums around the first wave's pivot (no merge divisions) and
// stores the workgroup's (n, mean, M2) as partial `slot`.
__device__ inline void store_moment_partial(const Args& a, const MomAcc& m, uint32_t slot,
                                            double* lds) {
  const double n = wave_sum(m.n), s1 = wave_sum(m.s1), s2 = wave_sum(m.s2);
  if (lane_id() == 0) {
    double* w = lds + 4 * wave_id();
    w[0] = n;
    w[1] = s1;
    w[2] = s2;
    w[3] = m.pivot;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double N = 0.0, S1 = 0.0, S2 = 0.0, P = 0.0;
    bool have = false;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const double nw = lds[4 * w], s1w = lds[4 * w + 1], s2w = lds[4 * w + 2], pw = lds[4 * w + 3];
      if (nw > 0.0) {
        if (!have) {
          P = pw;
          have = true;
        }
        const double dp = pw - P;  // sum (x-P) = s1 + n dp ; sum (x-P)^2 = s2 + 2 dp s1 + n dp^2
        N += nw;
        S1 += fma(nw, dp, s1w);
        S2 += s2w + dp * fma(nw, dp, 2.0 * s1w);
      }
    }
    const double mean = N > 0.0 ? P + S1 / N : 0.0;
    const double m2 = N > 0.0 ? S2 - S1 * (S1 / N) : 0.0;
    a.partial[slot] = N;
    a.partial[(size_t)a.max_tiles + slot] = mean;
    a.partial[2 * (size_t)a.max_tiles + slot] = m2 < 0.0 ? 0.0 : m2;  // rounding only; NaN stays
  }
}

// Layer-wise calls: one workgroup and one partial per tile.
__global__ __launch_bounds__(kBlock) void k_accum_moments_seg(const Args a) {
  __shared__ double lds[4 * kWaves];
  Span sp_;
  if (!locate_span<true>(a, blockIdx.x, &sp_)) return;
  if (a.ctrl[sp_.seg].bad) return;
  MomAcc m = {0.0, 0.0, 0.0, 0.0, false};
  for (uint32_t u = 0; u < sp_.nchunks; ++u) {
    const Tile t = chunk_of(sp_, u);
    if (t.full) accum_moments_chunk<true>(a, t, m);
    else accum_moments_chunk<false>(a, t, m);
  }
  store_moment_partial(a, m, blockIdx.x, lds);
  // The quantile depends on the arguments only; the workgroup of a segment's first tile
  // computes it here, hidden under the stream.
  if (threadIdx.x == 0) {
    SegCtrl& c = a.ctrl[sp_.seg];
    if (blockIdx.x == c.tile0)
      c.z = norm_isf((double)c.k / (a.tail_div * (double)(c.end - c.start)));
  }
}

// The ten thresholds reachable from thres0 (Alg. 1 steps 8-11): `na` multiplications by 1.5 in
// sequence, then halvings (exact), stored in ascending order of their nominal ratio to thres0.
__device__ inline void candidate_thresholds(double thres0, double (&t64)[kNumThres]) {
  double up = thres0;
#pragma unroll
  for (int na = 0; na <= 3; ++na) {
    double v = up;
#pragma unroll
    for (int nb = 0; nb <= 3 - na; ++nb) {
      t64[thres_pos(na, nb)] = v;
      v = 0.5 * v;
    }
    up = 1.5 * up;
  }
}

// Alg. 1 steps 5-13 on the ten totals: at most four evaluations ("for i = 0 -> 3"); the mask
// is the one of the last evaluated threshold.  Returns its position.
struct Walk {
  int pos;
  uint32_t rounds;
  uint32_t counts[4];
  bool in_band;
};
__device__ inline Walk walk_thresholds(const uint32_t (&tot)[kNumThres], int64_t k) {
  Walk w = {0, 0, {0, 0, 0, 0}, false};
  int na = 0, nb = 0;
  for (int round = 0; round <= 3; ++round) {
    w.pos = thres_pos(na, nb);
    const int64_t est = tot[w.pos];
    w.counts[round] = tot[w.pos];
    w.rounds = round + 1;
    if (3 * est < 2 * k) {          // estimated_k < 2k/3: halve the threshold
      if (round < 3) ++nb;
    } else if (3 * est > 4 * k) {   // estimated_k > 4k/3: threshold x 1.5
      if (round < 3) ++na;
    } else {
      w.in_band = true;
      break;
    }
  }
  return w;
}

// ---- sums over a workgroup of kFinBlock threads (the per-segment finalising kernels) ----------
__device__ inline double fin_block_sum(double v, double* lds) {
  v = wave_sum(v);
  __syncthreads();
  if (lane_id() == 0) lds[wave_id()] = v;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int w = 0; w < kFinWaves; ++w) s += lds[w];
  return s;
}

constexpr int kFinBatch = 4;  // partials per thread per round: 4096 tiles per round

// ---- K3: per tile, count |acc| > t for all ten candidate thresholds --------------------------
// The thresholds sit in ascending order, so once no element of a wave's slot exceeds one of them
// the larger ones need not be tested (only when the ordering is known to hold).
template <bool FULL>
__device__ inline void count_values(const float (&v)[kPerThread], uint32_t valid,
                                    const float (&thr)[kNumThres], bool can_skip,
                                    uint32_t (&cnt)[kNumThres]) {
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    float m[4];
    bool ok[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      m[q] = fabsf(v[4 * j + q]);
      ok[q] = FULL || ((valid >> (4 * j + q)) & 1u);
    }
    uint64_t any = 0;
#pragma unroll
    for (int p = 0; p < 5; ++p) {
      any = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint64_t b = __ballot(ok[q] && (m[q] > thr[p]));
        cnt[p] += (uint32_t)__builtin_popcountll(b);
        any |= b;
      }
    }
    if (!can_skip || any != 0) {
      any = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint64_t b = __ballot(ok[q] && (m[q] > thr[5]));
        cnt[5] += (uint32_t)__builtin_popcountll(b);
        any |= b;
      }
      if (!can_skip || any != 0) {
#pragma unroll
        for (int p = 6; p < kNumThres; ++p) {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            cnt[p] += (uint32_t)__builtin_popcountll(__ballot(ok[q] && (m[q] > thr[p])));
        }
      }
    }
  }
}

template <bool FULL>
__device__ inline void count_chunk(const Args& a, const Tile& t, const float (&thr)[kNumThres],
                                   bool can_skip, uint32_t (&cnt)[kNumThres]) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  count_values<FULL>(v, valid, thr, can_skip, cnt);
}

// ---- prefix sums of per-tile counts by one workgroup -------------------------------------------
constexpr int kScanPer = 4;                        // consecutive tiles per thread per scan round
constexpr int kScanChunk = kFinBlock * kScanPer;   // 4096 tiles staged in LDS per round

// Exclusive prefix sum of col[0..n) into base[0..n) by one workgroup of kFinBlock threads;
// returns the total.  `stage` holds kFinBlock*(kScanPer+1) words, `lds_scan` kFinWaves words.
__device__ inline uint32_t scan_tiles(const uint32_t* col, uint32_t ntiles, uint32_t* base,
                                      uint32_t* stage, uint32_t* lds_scan) {
  uint32_t carry = 0;
  for (uint32_t c0 = 0; c0 < ntiles; c0 += kScanChunk) {
    const uint32_t n = (ntiles - c0 < (uint32_t)kScanChunk) ? ntiles - c0 : (uint32_t)kScanChunk;
    uint32_t x[kScanPer];
#pragma unroll
    for (int u = 0; u < kScanPer; ++u) {  // coalesced loads, all in flight at once
      const uint32_t i = u * kFinBlock + threadIdx.x;
      x[u] = (i < n) ? col[c0 + i] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kScanPer; ++u) {  // +1 word per thread row: no bank conflicts
      const uint32_t i = u * kFinBlock + threadIdx.x;
      stage[(i / kScanPer) * (kScanPer + 1) + (i % kScanPer)] = x[u];
    }
    __syncthreads();
    const uint32_t b = threadIdx.x * kScanPer;
    const uint32_t* mine = stage + threadIdx.x * (kScanPer + 1);
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kScanPer; ++i) sum += mine[i];
    uint32_t total;
    uint32_t run = carry + block_exclusive_scan<kFinWaves>(sum, lds_scan, &total);
#pragma unroll
    for (int i = 0; i < kScanPer; ++i) {
      if (b + i < n) base[c0 + b + i] = run;
      run += mine[i];
    }
    carry += total;
    __syncthreads();
  }
  return carry;
}

// ---- K5: compaction in index order + residual (Alg. 1 step 14, Eq. (2)) ----------------------
// `run` is the number of survivors of this tile's earlier chunks (block-uniform).
template <bool FULL, bool NORMS>
__device__ inline uint32_t compact_values(const Args& a, const Tile& t, float (&v)[kPerThread],
                                          uint32_t valid, float thr, bool none, int64_t out0,
                                          uint32_t run, uint32_t* lds, NormAcc& norms) {
  uint32_t sel = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const bool ok = FULL || ((valid >> i) & 1u);
    if (ok && !none && (fabsf(v[i]) > thr)) sel |= 1u << i;
  }
  if (NORMS) norm_accumulate(norms, v, valid, sel);
  uint32_t first[kSlots];
  const uint32_t total = tile_rank(sel, lds, first);
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    uint32_t r = run + first[j];
    const int64_t i0 = slot_index(t, j);
#pragma unroll
    for (int cpt = 0; cpt < 4; ++cpt) {
      if ((sel >> (4 * j + cpt)) & 1u) {
        a.out_idx[out0 + r] = (uint32_t)(i0 + cpt);
        a.out_val[out0 + r] = v[4 * j + cpt];
        ++r;
      }
    }
  }
  if (a.inplace) {
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      const int64_t i0 = slot_index(t, j);
#pragma unroll
      for (int cpt = 0; cpt < 4; ++cpt)
        if ((sel >> (4 * j + cpt)) & 1u) a.resid[i0 + cpt] = 0.0f;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if ((sel >> i) & 1u) v[i] = 0.0f;
    store_tile<FULL>(a.resid, t, v, valid);
  }
  __syncthreads();  // lds is reused by the next chunk
  return run + total;
}

// STREAM: acc is read with the non-temporal hint (its last use in the call); the host picks by
// the vector length.
template <bool FULL, bool NORMS, bool STREAM = false>
__device__ inline uint32_t compact_chunk(const Args& a, const Tile& t, float thr, bool none,
                                         int64_t out0, uint32_t run, uint32_t* lds,
                                         NormAcc& norms) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL, STREAM>(a.acc, t, v);
  return compact_values<FULL, NORMS>(a, t, v, valid, thr, none, out0, run, lds, norms);
}

// ---- optional: ||acc||^2 and ||residual'||^2 from the per-tile sums of the compact kernel ----
template <bool SEG>
__global__ __launch_bounds__(kFinBlock) void k_norms_finalize(const Args a) {
  __shared__ double lds[kFinWaves];
  const int s = blockIdx.x;
  const SegCtrl& c = a.ctrl[s];
  if (SEG && c.bad) return;
  const uint32_t tile0 = SEG ? c.tile0 : 0u;
  const uint32_t ntiles = SEG ? c.ntiles : seg_ntiles(0, a.d_total, a.tile_chunks);
  double out[2];
  for (int which = 0; which < 2; ++which) {
    const double* p = a.norm_partial + (size_t)which * a.max_tiles + tile0;
    double acc = 0.0;
    for (uint32_t base = 0; base < ntiles; base += kFinBlock * kFinBatch) {
      double x[kFinBatch];
#pragma unroll
      for (int u = 0; u < kFinBatch; ++u) {
        const uint32_t i = base + u * kFinBlock + threadIdx.x;
        x[u] = (i < ntiles) ? p[i] : 0.0;
      }
#pragma unroll
      for (int u = 0; u < kFinBatch; ++u) acc += x[u];
    }
    out[which] = fin_block_sum(acc, lds);
  }
  if (threadIdx.x == 0) {
    a.result[s].acc_sqnorm = out[0];
    a.result[s].residual_sqnorm = out[1];
  }
}

}  // namespace sp
