/* sparsify.h -- C ABI of the MI355X (gfx950) gradient compressor.
 *
 * One call performs, for one worker and one iteration, the per-worker half of the
 * error-compensated sparsified update (paper Eq. (2)):
 *
 *     acc  = grad + residual                    (accumulate, one fp32 add per element)
 *     S    = Comp_k(acc)                        (Top_k of Sec. 1, or Gaussian_k of Algorithm 1)
 *     out  = {(i, acc[i]) : i in S}             (compacted (index, value) pairs)
 *     residual' = acc with the entries in S set to +0
 *
 * Every step runs in HIP kernels enqueued on the caller's stream; the calls return
 * without synchronising and copy nothing to the host.
 *
 * Pointers.  Unless marked HOST, every pointer is a DEVICE pointer owned by the caller and
 *   must be 16-byte aligned (`workspace` 256-byte).  The library allocates no device memory
 *   and keeps no state between calls.  `grad` is only read.  `residual` holds eps on entry
 *   and eps' on exit.  `acc` receives grad+residual; `acc == residual` is allowed (in-place
 *   mode: the buffer then ends as eps').  Any other overlap between buffers is an error.
 *   Between its first and its last kernel a call may use `residual` (when it is not `acc`)
 *   as scratch: its contents are defined again only when the call's work has completed.
 * Sizes.  1 <= k <= d < 2^31.  Indices are uint32 positions in the flat buffer.
 * Output order.  Every selector writes its pairs in ascending index order (per segment in the
 *   layer-wise call), the same from run to run.  Entries beyond `nnz` are not written.
 * Errors.  Argument errors that the host can see return a non-zero sparsify_status before
 *   anything is launched and touch no buffer.  Data-dependent conditions are reported in
 *   sparsify_result.flags, never by the return code.
 * Overlap.  Calls that share a workspace must be ordered on one stream.
 */
#ifndef SPARSIFY_H_
#define SPARSIFY_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPARSIFY_OK = 0,
  SPARSIFY_E_INVALID = 1,   /* bad d/k/cap, null or misaligned pointer, forbidden overlap */
  SPARSIFY_E_WORKSPACE = 2, /* workspace too small or misaligned */
  SPARSIFY_E_LAUNCH = 3     /* the HIP runtime refused a launch */
} sparsify_status;

enum {
  SPARSIFY_F_OVERFLOW = 1u,  /* more survivors than `cap`: nothing selected, residual' = acc */
  SPARSIFY_F_NONFINITE = 2u, /* mean, std or threshold not finite */
  SPARSIFY_F_EXHAUSTED = 4u, /* four count evaluations used, last one still outside the band */
  SPARSIFY_F_BADSEGMENT = 8u, /* segmented call: this segment's offsets, k or output range are
                                invalid (or its start lies before an earlier offset); no kernel
                                touches its stretch of acc, residual or the output */
  /* The next two say which way a flat call (or a segment of a layer-wise call) took,
     not what it computed (the results are the same either way); neither is set when the call
     built no short lists to begin with. */
  SPARSIFY_F_SHORTLIST = 16u,     /* the pairs (Top_k, DGC_k: and the digit passes) were taken from
                                     the short lists */
  SPARSIFY_F_SHORTLIST_MISS = 32u /* the lists were built but held fewer than k entries (Top_k),
                                     ran out of room, or do not hold the survivors (Gaussian_k: the
                                     walk ended below thres0, or thres0 is not positive): the
                                     passes over acc ran after all (Gaussian_k with lists that ran
                                     out of room: over the tiles, or the segment, concerned) */
};

/* Written on the stream; valid once the stream has been synchronised. */
typedef struct {
  uint32_t nnz;       /* pairs written */
  uint32_t rounds;    /* Gaussian_k: count evaluations performed, 1..4.  Top_k: 0.  DGC_k: top-k
                         selections performed, 1 or 2 */
  uint32_t count[4];  /* Gaussian_k: estimated_k of each evaluation (Alg. 1, step 7).  DGC_k: entries
                         that reach the sample's threshold, sample size, rank used in the sample */
  uint32_t flags;     /* SPARSIFY_F_* */
  float thres_f32;    /* fp32 value the final mask compared against (DGC_k: the sample's threshold) */
  double mean, std;   /* Alg. 1 step 2 (std with divisor d - ddof) */
  double z;           /* upper-tail normal quantile of k / (tail_div * d) */
  double thres0;      /* mean + std * z (Alg. 1 step 4) */
  double thres;       /* fp64 threshold of the evaluation that produced the mask */
  uint32_t topk_key;        /* Top_k: bit pattern of the k-th largest |acc| */
  uint32_t topk_ties_taken; /* Top_k: selected entries whose magnitude equals that one */
  double acc_sqnorm;        /* ||acc||^2 and ||acc - Comp_k(acc)||^2 = ||residual'||^2 in fp64: the */
  double residual_sqnorm;   /* two sides of the contraction property (Eq. (3)-(5), Theorem 1).
                               Filled only when sparsify_opts.error_norms is set, else 0. */
} sparsify_result;

/* HOST struct; pass NULL for the defaults. */
typedef struct {
  double tail_div; /* 2.0 (default): quantile 1 - k/(2d), consistent with the two-sided mask
                      |acc| > thres of Alg. 1 step 6.  1.0: the quantile 1 - k/d as printed in
                      Alg. 1 step 3.  Must be >= 1. */
  int32_t ddof;    /* 1 (default): sample standard deviation; 0: population */
  int32_t tile_chunks; /* 0 (default): automatic.  Otherwise the number of 4096-element chunks one
                      workgroup processes; a tuning knob, results do not depend on it.  The flat
                      calls refuse (SPARSIFY_E_INVALID) a value that leaves more than 4096 tiles
                      (65536 beyond 123 M elements for Gaussian_k and for Top_k with a separate
                      acc) */
  void* trace;     /* NULL, or a sparsify_trace* to record per-kernel timings of this call */
  int32_t error_norms; /* 0 (default).  1: also reduce ||acc||^2 and ||residual'||^2 (fp64) into the
                      result record; the sums ride on the compaction pass, one small launch more */
  int32_t sample_stride; /* DGC_k only.  0 (default): 100, a 1 % sample (Sec. 4.3).  Otherwise the
                      stratum length S >= 1: one sampled position per S consecutive elements */
  uint64_t sample_seed;  /* DGC_k only: seed of the counter-based choice of those positions */
  int32_t short_list;    /* 0 (default): the library
                      decides.  -1: never build the short lists (below).  Results do not depend
                      on it. */
} sparsify_opts;

/* Bytes of `workspace` for a vector of d_total elements in num_segments segments (1 for the
 * flat calls).  Returns 0 for invalid arguments.
 *   sparsify_workspace_bytes      the size to allocate.  For vectors of 6 M elements and more (in
 *                                 up to 1024 segments) it includes room for short lists (0.8
 *                                 bytes per element).  Top_k, flat call:
 *                                 the accumulate pass then also writes the residual and
 *                                 lists the entries above a key guessed from a sample of acc,
 *                                 a fraction of a per cent of the vector; if the lists turn out
 *                                 to hold at least k entries, the digit passes and the compaction
 *                                 read them instead of acc (16 bytes per element instead of 24,
 *                                 12 instead of 28 in place); if not, or if k > d / 80, the
 *                                 passes over acc run as they do without the lists.  DGC_k uses
 *                                 the same room: it draws its sample first (where the sample is
 *                                 no longer than the list buffer: strides from about 10), and
 *                                 the accumulate pass lists the entries that reach the sample's
 *                                 threshold.  So does Gaussian_k: its count pass writes the
 *                                 residual and lists the entries above thres0, and when the
 *                                 refinement ends at thres0 or above, the pairs are written from
 *                                 those lists (20 bytes per element instead of 24, 16 instead of
 *                                 20 in place).  In the layer-wise calls (Gaussian_k; Top_k with a
 *                                 separate acc, where every segment is sampled for a key of its
 *                                 own) every segment decides for itself.
 *   sparsify_workspace_bytes_min  the smallest size any call accepts; with less than the size
 *                                 above, no call builds the lists. */
size_t sparsify_workspace_bytes(int64_t d_total, int32_t num_segments);
size_t sparsify_workspace_bytes_min(int64_t d_total, int32_t num_segments);

/* Gaussian_k compressor (Algorithm 1; accumulate and residual of Eq. (2)).
 *   d, k      vector length and target number of survivors
 *   grad      fp32[d], read only
 *   residual  fp32[d], eps in / eps' out
 *   acc       fp32[d], out (may equal residual)
 *   out_idx   uint32[cap], out_val fp32[cap]; cap >= 1.  The method may select more or fewer
 *             than k entries (Appendix A.5); if the final count exceeds cap nothing is selected
 *             and SPARSIFY_F_OVERFLOW is set.
 *   result    one sparsify_result
 *   opts      HOST, may be NULL
 *   stream    hipStream_t passed as void* (NULL = the default stream)                         */
int sparsify_gaussiank(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                       uint32_t* out_idx, float* out_val, int64_t cap, sparsify_result* result,
                       void* workspace, size_t workspace_bytes, const sparsify_opts* opts,
                       void* stream);

/* sparsify_gaussiank for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as sparsify_gaussiank except that there is no workspace
 * argument: the partial results live in a 6 MiB array built into the library (one copy per GPU,
 * held until the process ends), which limits d to 2^27 = 134,217,728 elements; a larger d returns
 * SPARSIFY_E_WORKSPACE before anything is launched.  The call allocates nothing and frees
 * nothing.  The array keeps the previous call's contents (the kernels rewrite what they read) and
 * every call on one GPU shares it: calls that overlap on one GPU, on whatever streams, race;
 * order them on one stream or with events.  The first call on a device looks up the array's
 * device address (once per device, with that device current). */
int sparsify_gaussiank_static(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                              uint32_t* out_idx, float* out_val, int64_t cap,
                              sparsify_result* result, const sparsify_opts* opts, void* stream);

/* Exact Top_k compressor (definition in Sec. 1: the k entries largest in absolute value;
 * among equal magnitudes the lower index wins).  Same arguments; cap >= k is required; exactly
 * k pairs are written.  opts: tail_div and ddof are checked but not used. */
int sparsify_topk(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                  uint32_t* out_idx, float* out_val, int64_t cap, sparsify_result* result,
                  void* workspace, size_t workspace_bytes, const sparsify_opts* opts,
                  void* stream);

/* DGC_k, the hierarchical-sampling selection the paper compares Gaussian_k with (Sec. 3.3; a
 * 1 % sample in Sec. 4.3): an exact top-k on a sample of |acc| gives a threshold, every entry
 * whose magnitude reaches it is kept, and if those are more than k an exact top-k (lower index
 * wins ties) is run on them.  The paper gives only this outline; the sample (one position per
 * stratum of opts->sample_stride elements, chosen by a hash of opts->sample_seed and the
 * stratum's number), the rank ceil(k m / d) inside a sample of m, and ">=" are this library's
 * reading.  Same arguments as sparsify_topk; cap >= k is required; at most k pairs are written,
 * in ascending index order (fewer than k when the sample's threshold is too high: nothing is
 * added then).  acc == residual is not supported, nor an opts->tile_chunks that leaves more than
 * 4096 tiles (both SPARSIFY_E_INVALID).  result: see the fields'
 * comments; topk_key is the smallest magnitude that could be kept (bit pattern). */
int sparsify_dgck(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                  uint32_t* out_idx, float* out_val, int64_t cap, sparsify_result* result,
                  void* workspace, size_t workspace_bytes, const sparsify_opts* opts,
                  void* stream);

/* Layer-wise form: the flat compressor applied independently to each of num_segments
 * contiguous segments of one flat buffer, all in one call.
 *   d_total   length of grad/residual/acc; must equal seg_off[num_segments]
 *   seg_off   int64[num_segments+1], DEVICE: segment l is [seg_off[l], seg_off[l+1]), seg_off[0]=0,
 *             strictly increasing
 *   seg_k     int64[num_segments], DEVICE: 1 <= seg_k[l] <= length of segment l
 *   mode      0 = Top_k, 1 = Gaussian_k
 *   out_off   int64[num_segments+1], DEVICE, non-decreasing: segment l's pairs are written from
 *             out_idx[out_off[l]] and its capacity is out_off[l+1]-out_off[l]
 *   out_cap   number of elements in out_idx / out_val (>= out_off[num_segments])
 *   results   sparsify_result[num_segments]
 * Indices are positions in the flat buffer.  The three layout arrays are read on the device
 * only; a segment whose entries are invalid, or that starts before an earlier entry of seg_off
 * (so that it could overlap an earlier segment), gets SPARSIFY_F_BADSEGMENT and produces nothing. */
int sparsify_segmented(int32_t num_segments, int64_t d_total, const int64_t* seg_off,
                       const int64_t* seg_k, int32_t mode, const float* grad, float* residual,
                       float* acc, uint32_t* out_idx, float* out_val, const int64_t* out_off,
                       int64_t out_cap, sparsify_result* results, void* workspace,
                       size_t workspace_bytes, const sparsify_opts* opts, void* stream);

/* Decompression and aggregation: the sum over the P workers in Eq. (2),
 *     dense = scale * sum_p Comp_k(acc_p),
 * from the workers' compacted lists (as they sit in one buffer after an all-gather).
 *   d            length of dense, 1 <= d < 2^31
 *   num_lists    P, 1 <= P <= 1024
 *   idx, val     uint32 / fp32 [P][list_stride], DEVICE: worker p's pairs are entries
 *                p*list_stride + j, j < nnz of worker p.  Every list must be strictly ascending
 *                in index (every compressor of this library writes its pairs that way) with
 *                indices below d.
 *   nnz          DEVICE: worker p's pair count is the uint32 at byte offset p*nnz_stride_bytes
 *                (4 for a plain array; sizeof(sparsify_result) to read the counts straight from an
 *                array of result records, whose first field is nnz)
 *   scale        every element is multiplied by it once at the end: 1 for the sum, 1/P for the
 *                average that Eq. (2) applies
 *   dense        fp32[d], out, 16-byte aligned: every element is written.  Element i starts at +0
 *                and receives its contributions one fp32 addition at a time in worker order
 *                (worker 0 first), so the result is reproducible bit for bit; no workspace, no
 *                floating-point atomics
 *   status       one uint32, DEVICE, sticky: the call ORs bits into it and never clears it (the
 *                caller zeroes it once, and again after reading a set bit).  Bit 0 = some list is
 *                not strictly ascending or holds an index >= d, bit 1 = some count exceeds
 *                list_stride (it is cut to list_stride).  A call that sets a bit leaves the
 *                contents of dense unspecified; nothing outside dense is written whatever the
 *                lists hold.
 * Argument errors (sizes, null or misaligned pointers, dense overlapping an input) return
 * SPARSIFY_E_INVALID before anything is launched.  The call enqueues one kernel and returns. */
int sparsify_scatter_add(int64_t d, int32_t num_lists, const uint32_t* idx, const float* val,
                         int64_t list_stride, const uint32_t* nnz, int64_t nnz_stride_bytes,
                         float scale, float* dense, uint32_t* status, void* stream);

/* Optional per-kernel timing of one call (used by the benchmark for its roofline figure).
 * A trace owns HIP events (host objects, no device memory).  Pass it in sparsify_opts.trace;
 * after the stream has been synchronised, read the stages of the most recent traced call. */
typedef struct sparsify_trace sparsify_trace;
sparsify_trace* sparsify_trace_create(void);
void sparsify_trace_destroy(sparsify_trace* t);
int32_t sparsify_trace_num_stages(const sparsify_trace* t);
/* name of stage i (kernel name), valid until the next traced call */
const char* sparsify_trace_stage_name(const sparsify_trace* t, int32_t i);
/* duration of stage i in milliseconds (from the event before its launch to the event after it);
 * returns SPARSIFY_E_INVALID if i is out of range or the events are not complete */
int sparsify_trace_stage_ms(sparsify_trace* t, int32_t i, float* ms);

/* Measurement aid: copies n floats (n a positive multiple of 4; both DEVICE pointers 16-byte
 * aligned, not overlapping) with one plain kernel that reads 4n bytes and writes 4n bytes.
 * Hardware byte counters of the compressor's kernels are scaled by what they read for this one. */
int sparsify_calibration_copy(float* dst, const float* src, int64_t n, void* stream);

/* Library version string (static storage). */
const char* sparsify_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPARSIFY_H_ */
