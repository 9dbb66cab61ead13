/* CPU oracle for the per-worker gradient compressor of "Understanding Top-k
 * Sparsification in Distributed Deep Learning" (Eq. (2), the Top_k / Rand_k
 * definitions of Sec. 1, Algorithm 1).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, single-threaded, deliberately slow C++ that
 * a reader can check against the paper by eye.  It shares no code with the HIP
 * library and must never be reached from the product path: only the tests, the
 * smoke check and the benchmark's CPU-baseline leg may load it.
 *
 * Pins (see tests, all CPU-only): Top_k against a brute-force stable sort on tiny
 * vectors; exactly-k survivors; acc == Comp_k(acc) + eps' bit for bit; the
 * Top_k <= Rand_k error inequality and the Rand_k expectation of Eq. (4); the
 * Gaussian closed form of the Top_k error ratio and the (1-k/d)^2 bound of
 * Theorem 1; the normal quantile against tabulated values and a library
 * routine; moments against closed forms; Algorithm 1's count-and-nudge walk
 * against counts known in closed form on constructed vectors; DGC_k against Top_k when the
 * sample is the whole vector, against planted vectors whose outcome is known, and against the
 * exact Top_k whenever its second selection runs; the aggregation of sparse lists against
 * a numpy scatter (one worker, disjoint workers), exact integer sums in any order, a planted
 * collision whose fp32 sum depends on the order of the workers, and a sequential library sum.
 * Parity unpinned (conventions the paper does not fix; both sides implement the
 * same reading): the two-sided tail 1-k/(2d) default, the sample (n-1) standard
 * deviation, the fp32 rounding of the threshold before comparing, and the use of
 * the last evaluated mask when the four evaluations run out.
 *
 * All pointers are host pointers.  Functions return 0 on success, 1 on invalid
 * arguments (nothing written).
 */
#ifndef ORACLE_H_
#define ORACLE_H_
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_F_OVERFLOW = 1u, ORACLE_F_NONFINITE = 2u, ORACLE_F_EXHAUSTED = 4u };

typedef struct {
  uint32_t nnz;       /* pairs written */
  uint32_t rounds;    /* Gaussian_k: count evaluations done (1..4); Top_k: 0 */
  uint32_t count[4];  /* Gaussian_k: estimated_k of each evaluation */
  uint32_t flags;
  float thres_f32;    /* fp32 value the final mask compared against */
  double mean, std, z, thres0, thres;
  uint32_t topk_key;        /* Top_k: bit pattern of the k-th largest |acc| */
  uint32_t topk_ties_taken; /* Top_k: entries equal to that magnitude that were kept */
} oracle_result;

/* Eq. (2): acc[i] = g[i] + eps[i], one fp32 round-to-nearest add. */
void oracle_accumulate(int64_t d, const float* g, const float* eps, float* acc);

/* Algorithm 1, step 2: two-pass fp64 mean and standard deviation (divisor d-ddof). */
void oracle_moments(int64_t d, const float* acc, int32_t ddof, double* mean, double* std_);

/* Upper-tail standard normal quantile: the z with P(Z > z) = q (Algorithm 1, steps 3-4). */
double oracle_norm_isf(double q);

/* sum of squares in fp64 (for the contraction-property checks of Eq. (3)-(4), Theorem 1) */
double oracle_sqnorm(int64_t d, const float* x);

/* Top_k (Sec. 1): the k entries largest in |.|, lower index wins ties.  Pairs come out
 * in ascending index order; eps_out[i] = selected ? +0 : acc[i]. */
int oracle_topk(int64_t d, int64_t k, const float* acc, uint32_t* idx, float* val,
                float* eps_out, oracle_result* res);

/* Gaussian_k (Algorithm 1).  tail_div = 2 gives the quantile 1-k/(2d), 1 the printed 1-k/d.
 * If the final count exceeds cap nothing is selected (flag OVERFLOW, eps_out = acc). */
int oracle_gaussiank(int64_t d, int64_t k, const float* acc, int64_t cap, double tail_div,
                     int32_t ddof, uint32_t* idx, float* val, float* eps_out,
                     oracle_result* res);

/* DGC_k, the hierarchical-sampling selection the paper compares against (Sec. 3.3; Sec. 4.3
 * uses a 1 % sample): a top-k on a sample gives a threshold, the entries at or above it are
 * kept, and if that is more than k a second top-k runs on those.  The paper gives no more
 * than that; the rest is this build's reading, shared by both sides (parity unpinned):
 *   sample   one position per stratum [j*S, min((j+1)*S, d)), S = sample_stride, chosen by a
 *            counter-based hash of (seed, j): m = ceil(d/S) positions (written to
 *            sample_pos if it is not null);
 *   first    k_s = ceil(k*m/d); the threshold is the k_s-th largest |acc| of the sample;
 *   keep     every i with |acc[i]| >= threshold (n of them);
 *   second   only if n > k: the k largest of the kept, lower index wins ties.
 * res: nnz; rounds = top-k selections run (1 or 2); count[0] = n, count[1] = m,
 * count[2] = k_s; thres_f32 / thres = the sample threshold; topk_key = bit pattern of the
 * smallest kept magnitude bound (the k-th key when the second selection ran, else the
 * threshold's); topk_ties_taken = entries equal to the k-th key kept by the second selection
 * (0 when it did not run).  Pairs ascending in index, eps_out as for Top_k. */
int oracle_dgck(int64_t d, int64_t k, const float* acc, int32_t sample_stride, uint64_t seed,
                uint32_t* idx, float* val, float* eps_out, oracle_result* res,
                uint32_t* sample_pos);

/* Rand_k (Sec. 1) with the random choice passed in: dense out[i] = acc[i] on the k given
 * (distinct) indices, 0 elsewhere. */
int oracle_randk_dense(int64_t d, int64_t k, const float* acc, const uint32_t* chosen,
                       float* dense_out);

/* Decompression and aggregation, the sum over the P workers in Eq. (2):
 *   dense = scale * sum_p Comp_k(acc_p),   Comp_k(acc_p) given as worker p's (index, value) pairs.
 * Worker p's pairs are idx/val[p*list_stride + j], j < nnz[p].  Every element starts at +0 and
 * receives its contributions one fp32 addition at a time, worker 0 first, each worker's pairs in
 * list order; at the end every element is multiplied once by `scale` in fp32 (1 gives the plain
 * sum, 1/P the average that Eq. (2) applies).  Invalid (index >= d, nnz[p] > list_stride): 1. */
int oracle_scatter_add(int64_t d, int32_t num_lists, const uint32_t* idx, const float* val,
                       int64_t list_stride, const uint32_t* nnz, float scale, float* dense);

/* Layer-wise form: the flat routine applied to each [seg_off[l], seg_off[l+1]) with
 * seg_k[l]; indices are positions in the flat buffer; segment l's pairs start at
 * out_off[l] and its capacity is out_off[l+1]-out_off[l].  mode 0 = Top_k, 1 = Gaussian_k. */
int oracle_segmented(int32_t num_segments, const int64_t* seg_off, const int64_t* seg_k,
                     int32_t mode, const float* acc, const int64_t* out_off, double tail_div,
                     int32_t ddof, uint32_t* idx, float* val, float* eps_out,
                     oracle_result* res);

#ifdef __cplusplus
}
#endif
#endif
