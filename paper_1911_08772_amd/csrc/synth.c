/* Seeded synthetic gradient vectors (test and benchmark INPUT only).
 *
 * Counter-based: element i of stream s under a seed is a pure function of
 * (seed, s, i), so any slice can be produced independently and in parallel and
 * the CPU checker and the GPU path are fed byte-identical host arrays.  This
 * file holds no arithmetic of the compression method itself.
 *
 * Distributions stand in for the bell-shaped, near-zero-centred gradient
 * histograms the paper reports (Sec. 3.1, Fig. 2) at the sizes of its Table 1.
 */
#include <math.h>
#include <stdint.h>

static inline uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

/* j-th 64-bit word of element i in stream `stream`. */
static inline uint64_t word(uint64_t seed, uint64_t stream, uint64_t i, uint64_t j) {
  uint64_t h = mix64(seed ^ mix64(stream * 0xD1342543DE82EF95ull + 0x632BE59BD9B4E019ull));
  return mix64(h ^ mix64(i * 8u + j));
}

/* uniform in (0,1] and [0,1) from 53 random bits */
static inline double u_open0(uint64_t w) { return ((double)(w >> 11) + 1.0) * 0x1.0p-53; }
static inline double u_half(uint64_t w) { return (double)(w >> 11) * 0x1.0p-53; }

/* one standard normal from two words (Box-Muller, cosine branch) */
static inline double normal01(uint64_t w0, uint64_t w1) {
  const double two_pi = 6.283185307179586476925286766559;
  return sqrt(-2.0 * log(u_open0(w0))) * cos(two_pi * u_half(w1));
}

/* two independent standard normals from two words (both Box-Muller branches) */
static inline void normal01_pair(uint64_t w0, uint64_t w1, double* a, double* b) {
  const double two_pi = 6.283185307179586476925286766559;
  const double r = sqrt(-2.0 * log(u_open0(w0))), t = two_pi * u_half(w1);
  *a = r * cos(t);
  *b = r * sin(t);
}

/* out[i] = sigma * N(0,1), i = 0..n-1, counters index0+i */
void synth_normal(float* out, int64_t n, uint64_t seed, uint64_t stream, int64_t index0,
                  double sigma) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint64_t c = (uint64_t)(index0 + i);
    out[i] = (float)(sigma * normal01(word(seed, stream, c, 0), word(seed, stream, c, 1)));
  }
}

/* per element: sigma_b with probability p_b, else sigma_a */
void synth_mixture(float* out, int64_t n, uint64_t seed, uint64_t stream, int64_t index0,
                   double sigma_a, double sigma_b, double p_b) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint64_t c = (uint64_t)(index0 + i);
    double s = u_half(word(seed, stream, c, 2)) < p_b ? sigma_b : sigma_a;
    out[i] = (float)(s * normal01(word(seed, stream, c, 0), word(seed, stream, c, 1)));
  }
}

/* scale * Z / sqrt((Z1^2+Z2^2+Z3^2)/3): Student-t with 3 degrees of freedom */
void synth_student_t3(float* out, int64_t n, uint64_t seed, uint64_t stream, int64_t index0,
                      double scale) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint64_t c = (uint64_t)(index0 + i);
    double z, a, b, e;
    normal01_pair(word(seed, stream, c, 0), word(seed, stream, c, 1), &z, &a);
    normal01_pair(word(seed, stream, c, 2), word(seed, stream, c, 3), &b, &e);
    out[i] = (float)(scale * z / sqrt((a * a + b * b + e * e) / 3.0));
  }
}

/* uniform doubles in [0,1): used for segment sizes / scales and random index draws */
void synth_uniform(double* out, int64_t n, uint64_t seed, uint64_t stream, int64_t index0) {
  for (int64_t i = 0; i < n; ++i)
    out[i] = u_half(word(seed, stream, (uint64_t)(index0 + i), 0));
}
