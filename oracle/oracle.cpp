// CPU oracle: see oracle.h.  TEST INFRASTRUCTURE ONLY -- never part of the product path.
// Build: g++ -std=c++17 -O2 -ffp-contract=off (no fast-math, denormals kept).
#include "oracle.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <limits>
#include <vector>

namespace {

inline uint32_t bits_of(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  return u;
}

// Bit pattern of |x|: monotone in |x| over all non-NaN floats; NaN sorts above +Inf.
inline uint32_t mag_key(float x) { return bits_of(x) & 0x7FFFFFFFu; }

inline double upper_tail(double z) { return 0.5 * std::erfc(z / std::sqrt(2.0)); }

void clear_result(oracle_result* r) { std::memset(r, 0, sizeof(*r)); }

}  // namespace

extern "C" {

void oracle_accumulate(int64_t d, const float* g, const float* eps, float* acc) {
  for (int64_t i = 0; i < d; ++i) acc[i] = g[i] + eps[i];
}

void oracle_moments(int64_t d, const float* acc, int32_t ddof, double* mean, double* std_) {
  double s = 0.0;
  for (int64_t i = 0; i < d; ++i) s += (double)acc[i];
  const double mu = s / (double)d;
  double m2 = 0.0;
  for (int64_t i = 0; i < d; ++i) {
    const double c = (double)acc[i] - mu;
    m2 += c * c;
  }
  *mean = mu;
  *std_ = (d - ddof < 1) ? 0.0 : std::sqrt(m2 / (double)(d - ddof));
}

double oracle_norm_isf(double q) {
  if (!(q > 0.0)) return std::numeric_limits<double>::infinity();
  if (q >= 1.0) return -std::numeric_limits<double>::infinity();
  if (q > 0.5) return -oracle_norm_isf(1.0 - q);
  if (q == 0.5) return 0.0;
  // upper_tail is strictly decreasing on [0, 40] from 0.5 to (numerically) 0: bisect.
  double lo = 0.0, hi = 40.0;
  for (int it = 0; it < 200; ++it) {
    const double mid = 0.5 * (lo + hi);
    if (upper_tail(mid) > q) lo = mid; else hi = mid;
  }
  double z = 0.5 * (lo + hi);
  // Newton polish on f(z) = upper_tail(z) - q, f'(z) = -pdf(z).
  for (int it = 0; it < 8; ++it) {
    const double pdf = std::exp(-0.5 * z * z) / std::sqrt(2.0 * M_PI);
    if (!(pdf > 0.0)) break;
    const double dz = (upper_tail(z) - q) / pdf;
    z += dz;
    if (std::fabs(dz) < 1e-15 * std::fabs(z)) break;
  }
  return z;
}

double oracle_sqnorm(int64_t d, const float* x) {
  double s = 0.0;
  for (int64_t i = 0; i < d; ++i) s += (double)x[i] * (double)x[i];
  return s;
}

int oracle_topk(int64_t d, int64_t k, const float* acc, uint32_t* idx, float* val,
                float* eps_out, oracle_result* res) {
  if (d < 1 || d >= (int64_t(1) << 31) || k < 1 || k > d) return 1;
  clear_result(res);
  // Total order: larger |acc| first; among equal magnitudes the lower index first.
  // Encoded as one descending 64-bit order: (key, ~index).
  static thread_local std::vector<uint64_t> order;  // scratch kept between calls
  order.resize((size_t)d);
  for (int64_t i = 0; i < d; ++i)
    order[(size_t)i] = ((uint64_t)mag_key(acc[i]) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)i);
  std::nth_element(order.begin(), order.begin() + (k - 1), order.end(), std::greater<uint64_t>());
  const uint64_t kth = order[(size_t)(k - 1)];
  const uint32_t T = (uint32_t)(kth >> 32);
  std::vector<uint32_t> chosen((size_t)k);
  uint32_t ties = 0;
  for (int64_t j = 0; j < k; ++j) {
    chosen[(size_t)j] = 0xFFFFFFFFu - (uint32_t)(order[(size_t)j] & 0xFFFFFFFFu);
    if ((uint32_t)(order[(size_t)j] >> 32) == T) ++ties;
  }
  std::sort(chosen.begin(), chosen.end());
  for (int64_t i = 0; i < d; ++i) eps_out[i] = acc[i];
  for (int64_t j = 0; j < k; ++j) {
    const uint32_t i = chosen[(size_t)j];
    idx[j] = i;
    val[j] = acc[i];
    eps_out[i] = 0.0f;
  }
  res->nnz = (uint32_t)k;
  res->topk_key = T;
  res->topk_ties_taken = ties;
  return 0;
}

int oracle_gaussiank(int64_t d, int64_t k, const float* acc, int64_t cap, double tail_div,
                     int32_t ddof, uint32_t* idx, float* val, float* eps_out,
                     oracle_result* res) {
  if (d < 1 || d >= (int64_t(1) << 31) || k < 1 || k > d || cap < 0 || !(tail_div >= 1.0) ||
      (ddof != 0 && ddof != 1))
    return 1;
  clear_result(res);
  // step 2: mean and std of the vector
  oracle_moments(d, acc, ddof, &res->mean, &res->std);
  // steps 3-4: threshold from the normal quantile; the upper-tail mass is k/(tail_div*d)
  const double q = (double)k / (tail_div * (double)d);
  res->z = oracle_norm_isf(q);
  res->thres0 = res->mean + res->std * res->z;
  if (!std::isfinite(res->mean) || !std::isfinite(res->std) || !std::isfinite(res->thres0))
    res->flags |= ORACLE_F_NONFINITE;

  // steps 5-13: at most four evaluations of the count, nudging the threshold
  double thres = res->thres0;
  float t32 = 0.0f;
  int64_t est = 0;
  bool in_band = false;
  for (int round = 0; round <= 3; ++round) {
    t32 = (float)thres;
    est = 0;
    for (int64_t i = 0; i < d; ++i) est += (std::fabs(acc[i]) > t32) ? 1 : 0;
    res->count[round] = (uint32_t)est;
    res->rounds = (uint32_t)(round + 1);
    res->thres = thres;
    res->thres_f32 = t32;
    if (3 * est < 2 * k) {
      if (round < 3) thres = 0.5 * thres;
    } else if (3 * est > 4 * k) {
      if (round < 3) thres = 1.5 * thres;
    } else {
      in_band = true;
      break;
    }
  }
  if (!in_band) res->flags |= ORACLE_F_EXHAUSTED;

  // step 14 with the mask of the last evaluation; residual of Eq. (2)
  for (int64_t i = 0; i < d; ++i) eps_out[i] = acc[i];
  if (est > cap) {
    res->flags |= ORACLE_F_OVERFLOW;
    res->nnz = 0;
    return 0;
  }
  int64_t n = 0;
  for (int64_t i = 0; i < d; ++i) {
    if (std::fabs(acc[i]) > t32) {
      idx[n] = (uint32_t)i;
      val[n] = acc[i];
      eps_out[i] = 0.0f;
      ++n;
    }
  }
  res->nnz = (uint32_t)n;
  return 0;
}

// Counter-based choice of the sample position inside stratum j: a 64-bit finaliser of the
// (seed, j) pair (xor-shift-multiply rounds with the constants of the SplitMix64 generator,
// Steele, Lea & Flood 2014), whose high 32 bits are scaled to [0, len) by a multiply-shift.
static uint64_t stratum_hash(uint64_t seed, uint64_t j) {
  uint64_t x = seed + (j + 1) * 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

int oracle_dgck(int64_t d, int64_t k, const float* acc, int32_t sample_stride, uint64_t seed,
                uint32_t* idx, float* val, float* eps_out, oracle_result* res,
                uint32_t* sample_pos) {
  if (d < 1 || d >= (int64_t(1) << 31) || k < 1 || k > d || sample_stride < 1) return 1;
  clear_result(res);
  const int64_t S = sample_stride;
  const int64_t m = (d + S - 1) / S;
  // the sample: one position per stratum
  std::vector<uint32_t> skey((size_t)m);
  for (int64_t j = 0; j < m; ++j) {
    const int64_t lo = j * S;
    const uint64_t len = (uint64_t)std::min<int64_t>(S, d - lo);
    const uint64_t hi32 = stratum_hash(seed, (uint64_t)j) >> 32;
    const int64_t p = lo + (int64_t)((hi32 * len) >> 32);
    if (sample_pos) sample_pos[j] = (uint32_t)p;
    skey[(size_t)j] = mag_key(acc[p]);
  }
  // first selection: the k_s-th largest magnitude of the sample is the threshold
  const int64_t ks = (k * m + d - 1) / d;
  std::nth_element(skey.begin(), skey.begin() + (ks - 1), skey.end(), std::greater<uint32_t>());
  const uint32_t Ts = skey[(size_t)(ks - 1)];
  // keep what reaches the threshold
  std::vector<uint32_t> kept;
  for (int64_t i = 0; i < d; ++i)
    if (mag_key(acc[i]) >= Ts) kept.push_back((uint32_t)i);
  const int64_t n = (int64_t)kept.size();
  res->rounds = 1;
  res->count[0] = (uint32_t)n;
  res->count[1] = (uint32_t)m;
  res->count[2] = (uint32_t)ks;
  std::memcpy(&res->thres_f32, &Ts, 4);
  res->thres = (double)res->thres_f32;
  res->topk_key = Ts;
  if (n > k) {
    // second selection, on the kept entries only: larger magnitude first, lower index first
    std::stable_sort(kept.begin(), kept.end(), [&](uint32_t a, uint32_t b) {
      return mag_key(acc[a]) > mag_key(acc[b]);  // kept is in index order: stable = lower index
    });
    const uint32_t T = mag_key(acc[kept[(size_t)(k - 1)]]);
    kept.resize((size_t)k);
    uint32_t ties = 0;
    for (uint32_t i : kept) ties += mag_key(acc[i]) == T ? 1u : 0u;
    std::sort(kept.begin(), kept.end());
    res->rounds = 2;
    res->topk_key = T;
    res->topk_ties_taken = ties;
  }
  for (int64_t i = 0; i < d; ++i) eps_out[i] = acc[i];
  for (size_t j = 0; j < kept.size(); ++j) {
    idx[j] = kept[j];
    val[j] = acc[kept[j]];
    eps_out[kept[j]] = 0.0f;
  }
  res->nnz = (uint32_t)kept.size();
  return 0;
}

int oracle_randk_dense(int64_t d, int64_t k, const float* acc, const uint32_t* chosen,
                       float* dense_out) {
  if (d < 1 || k < 1 || k > d) return 1;
  for (int64_t i = 0; i < d; ++i) dense_out[i] = 0.0f;
  for (int64_t j = 0; j < k; ++j) {
    if (chosen[j] >= (uint64_t)d) return 1;
    dense_out[chosen[j]] = acc[chosen[j]];
  }
  return 0;
}

int oracle_scatter_add(int64_t d, int32_t num_lists, const uint32_t* idx, const float* val,
                       int64_t list_stride, const uint32_t* nnz, float scale, float* dense) {
  if (d < 1 || d >= (int64_t(1) << 31) || num_lists < 1 || list_stride < 0) return 1;
  for (int32_t p = 0; p < num_lists; ++p) {
    if ((int64_t)nnz[p] > list_stride) return 1;
    for (uint32_t j = 0; j < nnz[p]; ++j)
      if ((int64_t)idx[(int64_t)p * list_stride + j] >= d) return 1;
  }
  for (int64_t i = 0; i < d; ++i) dense[i] = 0.0f;
  // the sum over the workers of Eq. (2): worker after worker, each list from its first pair on
  for (int32_t p = 0; p < num_lists; ++p) {
    const uint32_t* pi = idx + (int64_t)p * list_stride;
    const float* pv = val + (int64_t)p * list_stride;
    for (uint32_t j = 0; j < nnz[p]; ++j) dense[pi[j]] = dense[pi[j]] + pv[j];
  }
  for (int64_t i = 0; i < d; ++i) dense[i] = dense[i] * scale;  // 1/P for the average of Eq. (2)
  return 0;
}

int oracle_segmented(int32_t num_segments, const int64_t* seg_off, const int64_t* seg_k,
                     int32_t mode, const float* acc, const int64_t* out_off, double tail_div,
                     int32_t ddof, uint32_t* idx, float* val, float* eps_out,
                     oracle_result* res) {
  if (num_segments < 1 || (mode != 0 && mode != 1)) return 1;
  for (int32_t l = 0; l < num_segments; ++l) {
    const int64_t a = seg_off[l], b = seg_off[l + 1];
    if (a < 0 || b <= a || out_off[l + 1] < out_off[l]) return 1;
    if (seg_k[l] < 1 || seg_k[l] > b - a) return 1;
  }
  for (int32_t l = 0; l < num_segments; ++l) {
    const int64_t a = seg_off[l], n = seg_off[l + 1] - a;
    const int64_t cap = out_off[l + 1] - out_off[l];
    uint32_t* sidx = idx + out_off[l];
    float* sval = val + out_off[l];
    int rc;
    if (mode == 0) {
      if (cap < seg_k[l]) {  // cannot hold k pairs: nothing selected
        std::memset(&res[l], 0, sizeof(res[l]));
        res[l].flags = ORACLE_F_OVERFLOW;
        for (int64_t i = 0; i < n; ++i) eps_out[a + i] = acc[a + i];
        continue;
      }
      rc = oracle_topk(n, seg_k[l], acc + a, sidx, sval, eps_out + a, &res[l]);
    } else {
      rc = oracle_gaussiank(n, seg_k[l], acc + a, cap, tail_div, ddof, sidx, sval, eps_out + a,
                            &res[l]);
    }
    if (rc != 0) return rc;
    for (uint32_t j = 0; j < res[l].nnz; ++j) sidx[j] += (uint32_t)a;  // flat positions
  }
  return 0;
}

}  // extern "C"
