// Gaussian_k (Algorithm 1) on gfx950: fused accumulate + fp64 moments, on-device normal
// quantile, one multi-threshold count pass, on-device threshold walk, ordered compaction with
// the residual write.  All inter-block results go through per-tile partials that a small
// per-segment kernel combines in a fixed order: no atomics, bit-reproducible output.
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
template <bool FULL>
__device__ inline void accum_moments_tile(const Args& a, const Tile& t, uint32_t tile_id,
                                          double* lds) {
  float g[kPerThread], e[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.grad, t, g);
  load_tile<FULL>(a.resid, t, e);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) g[i] = g[i] + e[i];  // Eq. (2): one fp32 add
  store_tile<FULL>(a.acc, t, g, valid);

  // Wave-uniform pivot taken from a register (the first valid element held by the wave), so the
  // shifted sums sum((x-p)), sum((x-p)^2) lose nothing to cancellation whatever the mean is.
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
  double n = 0.0, s1 = 0.0, s2 = 0.0, pivot = 0.0;
  if (owners != 0) {
    const int src = __builtin_ctzll(owners);
    pivot = (double)__shfl(first, src, 64);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      if (FULL || ((valid >> i) & 1u)) {
        const double c = (double)g[i] - pivot;
        s1 += c;
        s2 = fma(c, c, s2);
      }
    }
    n = FULL ? (double)kPerThread : (double)__popc(valid);
  }
  n = wave_sum(n);
  s1 = wave_sum(s1);
  s2 = wave_sum(s2);
  if (lane_id() == 0) {
    double* w = lds + 3 * wave_id();
    const double mean = n > 0.0 ? pivot + s1 / n : 0.0;
    const double m2 = n > 0.0 ? s2 - s1 * (s1 / n) : 0.0;
    w[0] = n;
    w[1] = mean;
    w[2] = m2 > 0.0 ? m2 : 0.0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    Moments m = {lds[0], lds[1], lds[2]};
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = merge(m, Moments{lds[3 * w], lds[3 * w + 1], lds[3 * w + 2]});
    double* out = a.partial + 3 * (size_t)tile_id;
    out[0] = m.n;
    out[1] = m.mean;
    out[2] = m.m2;
  }
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_accum_moments(const Args a) {
  __shared__ double lds[3 * kWaves];
  Tile t;
  if (!locate_tile<SEG>(a, blockIdx.x, &t)) return;
  if (SEG && a.ctrl[t.seg].bad) return;
  if (t.full) accum_moments_tile<true>(a, t, blockIdx.x, lds);
  else accum_moments_tile<false>(a, t, blockIdx.x, lds);
  if (!SEG && blockIdx.x == 0 && threadIdx.x == 0) {
    // The quantile depends on the arguments only; compute it here, hidden under the stream.
    a.ctrl[0].z = norm_isf((double)a.flat_k / (a.tail_div * (double)a.d_total));
  }
}

// ---- K2: per segment, combine partials -> mean, std, threshold candidates -------------------
template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_gk_threshold(const Args a) {
  __shared__ double lds[3 * kWaves];
  const int s = blockIdx.x;
  SegCtrl& c = a.ctrl[s];
  uint32_t tile0 = 0, ntiles = seg_ntiles(0, a.d_total);
  int64_t n_seg = a.d_total;
  if (SEG) {
    if (c.bad) return;
    tile0 = c.tile0;
    ntiles = c.ntiles;
    n_seg = c.end - c.start;
  }
  Moments m = {0.0, 0.0, 0.0};
  for (uint32_t i = threadIdx.x; i < ntiles; i += kBlock) {
    const double* p = a.partial + 3 * (size_t)(tile0 + i);
    m = merge(m, Moments{p[0], p[1], p[2]});
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {  // fixed-shape tree: lane i absorbs lane i+off
    Moments o = {__shfl_down(m.n, off, 64), __shfl_down(m.mean, off, 64),
                 __shfl_down(m.m2, off, 64)};
    if ((lane_id() & (2 * off - 1)) == 0) m = merge(m, o);
  }
  if (lane_id() == 0) {
    lds[3 * wave_id()] = m.n;
    lds[3 * wave_id() + 1] = m.mean;
    lds[3 * wave_id() + 2] = m.m2;
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  m = Moments{lds[0], lds[1], lds[2]};
  for (int w = 1; w < kWaves; ++w) m = merge(m, Moments{lds[3 * w], lds[3 * w + 1], lds[3 * w + 2]});

  const double denom = (double)(n_seg - a.ddof);
  const double sd = (n_seg - a.ddof < 1) ? 0.0 : sqrt(m.m2 / denom);
  const double z = c.z;
  const double thres0 = m.mean + sd * z;
  // candidate thresholds: `na` multiplications by 1.5 in sequence, then halvings (exact)
  double up = thres0;
  for (int na = 0; na <= 3; ++na) {
    double v = up;
    for (int nb = 0; na + nb <= 3; ++nb) {
      const int j = thres_index(na, nb);
      c.t64[j] = v;
      c.t32[j] = (float)v;
      v = 0.5 * v;
    }
    up = 1.5 * up;
  }
  sparsify_result& r = a.result[s];
  r.mean = m.mean;
  r.std = sd;
  r.z = z;
  r.thres0 = thres0;
  uint32_t flags = 0;
  if (!isfinite(m.mean) || !isfinite(sd) || !isfinite(thres0)) flags |= SPARSIFY_F_NONFINITE;
  r.flags = flags;
}

// ---- K3: per tile, count |acc| > t for all ten candidate thresholds --------------------------
template <bool FULL>
__device__ inline void count_tile(const Args& a, const Tile& t, uint32_t tile_id, uint32_t* lds) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  const SegCtrl& c = a.ctrl[t.seg];
  float thr[kNumThres];
#pragma unroll
  for (int j = 0; j < kNumThres; ++j) thr[j] = c.t32[j];
  uint32_t cnt[kNumThres];
#pragma unroll
  for (int j = 0; j < kNumThres; ++j) cnt[j] = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const float m = fabsf(v[i]);
    const bool ok = FULL || ((valid >> i) & 1u);
#pragma unroll
    for (int j = 0; j < kNumThres; ++j)
      cnt[j] += (uint32_t)__builtin_popcountll(__ballot(ok && (m > thr[j])));
  }
  if (lane_id() == 0) {
#pragma unroll
    for (int j = 0; j < kNumThres; ++j) lds[wave_id() * kNumThres + j] = cnt[j];
  }
  __syncthreads();
  if (threadIdx.x < kNumThres) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds[w * kNumThres + threadIdx.x];
    a.tile_counts[(size_t)tile_id * kNumThres + threadIdx.x] = s;
  }
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_gk_count(const Args a) {
  __shared__ uint32_t lds[kWaves * kNumThres];
  Tile t;
  if (!locate_tile<SEG>(a, blockIdx.x, &t)) return;
  if (SEG && a.ctrl[t.seg].bad) return;
  if (t.full) count_tile<true>(a, t, blockIdx.x, lds);
  else count_tile<false>(a, t, blockIdx.x, lds);
}

// ---- K4: per segment, total the counts, walk Alg. 1 steps 5-13, scan the chosen column -------
template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_gk_decide(const Args a) {
  __shared__ uint32_t lds_cnt[kWaves * kNumThres];
  __shared__ uint32_t lds_scan[kWaves + 1];
  __shared__ uint32_t lds_final;
  const int s = blockIdx.x;
  SegCtrl& c = a.ctrl[s];
  uint32_t tile0 = 0, ntiles = seg_ntiles(0, a.d_total);
  int64_t k = a.flat_k, cap = a.flat_cap;
  if (SEG) {
    if (c.bad) return;
    tile0 = c.tile0;
    ntiles = c.ntiles;
    k = c.k;
    cap = c.cap;
  }
  uint32_t cnt[kNumThres];
#pragma unroll
  for (int j = 0; j < kNumThres; ++j) cnt[j] = 0;
  for (uint32_t i = threadIdx.x; i < ntiles; i += kBlock) {
    const uint32_t* p = a.tile_counts + (size_t)(tile0 + i) * kNumThres;
#pragma unroll
    for (int j = 0; j < kNumThres; ++j) cnt[j] += p[j];
  }
#pragma unroll
  for (int j = 0; j < kNumThres; ++j) cnt[j] = wave_sum(cnt[j]);
  if (lane_id() == 0) {
#pragma unroll
    for (int j = 0; j < kNumThres; ++j) lds_cnt[wave_id() * kNumThres + j] = cnt[j];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t tot[kNumThres];
    for (int j = 0; j < kNumThres; ++j) {
      tot[j] = 0;
      for (int w = 0; w < kWaves; ++w) tot[j] += lds_cnt[w * kNumThres + j];
    }
    sparsify_result& r = a.result[s];
    int na = 0, nb = 0, j = 0;
    bool in_band = false;
    uint32_t rounds = 0;
    for (int round = 0; round <= 3; ++round) {
      j = thres_index(na, nb);
      const int64_t est = tot[j];
      r.count[round] = tot[j];
      rounds = round + 1;
      if (3 * est < 2 * k) {
        if (round < 3) ++nb;
      } else if (3 * est > 4 * k) {
        if (round < 3) ++na;
      } else {
        in_band = true;
        break;
      }
    }
    for (uint32_t q = rounds; q < 4; ++q) r.count[q] = 0;
    uint32_t flags = r.flags;  // NONFINITE bit from the threshold kernel
    if (!in_band) flags |= SPARSIFY_F_EXHAUSTED;
    const bool overflow = (int64_t)tot[j] > cap;
    if (overflow) flags |= SPARSIFY_F_OVERFLOW;
    r.rounds = rounds;
    r.flags = flags;
    r.thres = c.t64[j];
    r.thres_f32 = c.t32[j];
    r.nnz = overflow ? 0u : tot[j];
    r.topk_key = 0;
    r.topk_ties_taken = 0;
    c.t_final = c.t32[j];
    c.select_none = overflow ? 1u : 0u;
    lds_final = (uint32_t)j;
  }
  __syncthreads();
  const uint32_t jf = lds_final;
  // exclusive scan of column jf over this segment's tiles -> first output slot of each tile
  const uint32_t per = (ntiles + kBlock - 1) / kBlock;
  const uint32_t b = threadIdx.x * per;
  const uint32_t e = (b + per < ntiles) ? b + per : ntiles;
  uint32_t sum = 0;
  for (uint32_t i = b; i < e; ++i) sum += a.tile_counts[(size_t)(tile0 + i) * kNumThres + jf];
  uint32_t total;
  uint32_t run = block_exclusive_scan(sum, lds_scan, &total);
  for (uint32_t i = b; i < e; ++i) {
    a.tile_base[tile0 + i] = run;
    run += a.tile_counts[(size_t)(tile0 + i) * kNumThres + jf];
  }
}

// ---- K5: compaction in index order + residual (Alg. 1 step 14, Eq. (2)) ----------------------
template <bool SEG, bool FULL>
__device__ inline void compact_tile(const Args& a, const Tile& t, uint32_t tile_id,
                                    uint32_t* lds) {
  float v[kPerThread];
  const uint32_t valid = load_tile<FULL>(a.acc, t, v);
  const SegCtrl& c = a.ctrl[t.seg];
  const float thr = c.t_final;
  const bool none = c.select_none != 0;
  uint32_t sel = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const bool ok = FULL || ((valid >> i) & 1u);
    if (ok && !none && (fabsf(v[i]) > thr)) sel |= 1u << i;
  }
  // rank of each survivor in index order: slots, then lanes, then the 4 components
  uint32_t below[kSlots];
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    uint32_t tot = 0, mine = 0;
#pragma unroll
    for (int cpt = 0; cpt < 4; ++cpt) {
      const uint64_t m = __ballot((sel >> (4 * j + cpt)) & 1u);
      tot += (uint32_t)__builtin_popcountll(m);
      mine += lanes_below(m);
    }
    below[j] = mine;
    if (lane_id() == 0) lds[j * kWaves + wave_id()] = tot;
  }
  __syncthreads();
  const int64_t out0 = (SEG ? c.out_base : 0) + (int64_t)a.tile_base[tile_id];
  uint32_t run = 0;
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t x = lds[j * kWaves + w];
      if (w == wave_id()) {
        uint32_t r = run + below[j];
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
      run += x;
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
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) void k_gk_compact(const Args a) {
  __shared__ uint32_t lds[kSlots * kWaves];
  Tile t;
  if (!locate_tile<SEG>(a, blockIdx.x, &t)) return;
  if (SEG && a.ctrl[t.seg].bad) return;
  if (t.full) compact_tile<SEG, true>(a, t, blockIdx.x, lds);
  else compact_tile<SEG, false>(a, t, blockIdx.x, lds);
}

}  // namespace sp
