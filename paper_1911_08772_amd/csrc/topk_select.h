// Exact Top_k, flat vectors: what the flat forms share.  The per-pass global histograms (replicated
// to spread same-address atomics), the rows and columns of the count tables that the forms with
// ordered compaction use, the kernel that clears them, and the digit choice that every workgroup
// of the next kernel makes for itself from the previous pass's histogram (same arithmetic, same
// inputs: all workgroups agree).
#pragma once
#include "common.h"
#include "gaussiank_flat.h"
#include "setup.h"
#include "topk.h"

namespace sp {

constexpr int kTopkCopies = 32;  // replicas of each pass's global histogram
constexpr int kTopkHistWords = kDigits * kTopkCopies * 256;
constexpr int kLastDigitBins = 128;  // the last digit has 7 bits

__device__ inline uint32_t* pass_hist(const Args& a, int pass) {
  return a.hist + (size_t)pass * kTopkCopies * 256;
}

// rows of tile_counts used by the forms with ordered compaction
constexpr int kRowTake = 0;   // survivors of the tile, ranked ties not included
constexpr int kRowTies = 1;   // keys equal to T (only when ties are ranked)
constexpr int kRowCand = 2;   // candidate keys the filter pass wrote for the tile
constexpr int kRowAbove = 3;  // keys known to exceed the k-th key before its last digits are
// columns of group_counts used by them
constexpr int kColTake = 0;
constexpr int kColTies = 1;

__device__ inline uint32_t* tile_row(const Args& a, int row) {
  return a.tile_counts + (size_t)row * a.max_tiles;
}

// Clears `hist_words` words of histograms and the group totals, resets the selection state.
__global__ __launch_bounds__(kBlock) void k_topk_init_fused(const Args a, uint32_t hist_words) {
  for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < hist_words; i += gridDim.x * kBlock)
    a.hist[i] = 0;
  if (blockIdx.x == 0) {
    for (uint32_t i = threadIdx.x; i < (uint32_t)(kBigMaxGroups * kNumThres); i += kBlock)
      a.group_counts[i] = 0;
    if (a.list && threadIdx.x < 64) a.list_stats[threadIdx.x] = 0;  // the lists' length and overflow words
    if (threadIdx.x == 0) {
      SegCtrl& c = a.ctrl[0];
      c.prefix = 0;
      c.k_rem = (uint32_t)a.flat_k;
      c.n_eq = 0;
      c.rank_ties = 0;
      c.select_none = 0;
      c.bad = 0;
      c.list_mode = 0;
      sparsify_result& r = a.result[0];
      clear_result(r);
      r.nnz = (uint32_t)a.flat_k;
    }
  }
}

// The digit of pass `pass` that holds the k_rem-th largest of the keys matching `prefix`, from
// the replicated histogram `hist`; run by all 256 threads of a workgroup (thread order =
// descending digit).  `lds` holds kWaves + 3 words.  Three barriers.
struct Digit {
  uint32_t prefix, k_rem, count;  // extended prefix, rank left inside the digit, keys in it
  uint32_t total;                 // keys counted by the histogram
};
__device__ inline Digit digit_from_bins(uint32_t v, int pass, uint32_t prefix, uint32_t k_rem,
                                        uint32_t* lds);

__device__ inline Digit choose_digit(const uint32_t* hist, int pass, uint32_t prefix,
                                     uint32_t k_rem, uint32_t* lds) {
  const uint32_t bin = 255u - threadIdx.x;
  uint32_t x[kTopkCopies];
#pragma unroll
  for (int r = 0; r < kTopkCopies; ++r) x[r] = hist[r * 256 + bin];  // all in flight at once
  uint32_t v = 0;
#pragma unroll
  for (int r = 0; r < kTopkCopies; ++r) v += x[r];
  return digit_from_bins(v, pass, prefix, k_rem, lds);
}

// The same with a run-time number of replicas (layer-wise calls), in two steps so that a caller
// can have the histogram on order while it still waits for the prefix and the rank.
__device__ inline uint32_t load_digit_bins(const uint32_t* hist, uint32_t copies) {
  const uint32_t bin = 255u - threadIdx.x;
  uint32_t v = 0;
  for (uint32_t r0 = 0; r0 < copies; r0 += 8) {
    uint32_t x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = (r0 + u < copies) ? hist[(size_t)(r0 + u) * 256 + bin] : 0u;
#pragma unroll
    for (int u = 0; u < 8; ++u) v += x[u];
  }
  return v;
}
__device__ inline Digit choose_digit_n(const uint32_t* hist, uint32_t copies, int pass,
                                       uint32_t prefix, uint32_t k_rem, uint32_t* lds) {
  return digit_from_bins(load_digit_bins(hist, copies), pass, prefix, k_rem, lds);
}

// `v`: this thread's bin count (thread order = descending digit).
__device__ inline Digit digit_from_bins(uint32_t v, int pass, uint32_t prefix, uint32_t k_rem,
                                        uint32_t* lds) {
  const uint32_t nbins = 1u << digit_bits(pass);
  const uint32_t bin = 255u - threadIdx.x;
  if (bin >= nbins) v = 0;
  if (threadIdx.x == 0) {  // what is read back when the rank exceeds the total: nothing chosen
    lds[kWaves] = prefix << digit_bits(pass);
    lds[kWaves + 1] = 0;
    lds[kWaves + 2] = 0;
  }
  uint32_t total;
  const uint32_t above = block_exclusive_scan<kWaves>(v, lds, &total);  // keys in higher digits
  if (above < k_rem && k_rem <= above + v) {
    lds[kWaves] = (prefix << digit_bits(pass)) | bin;
    lds[kWaves + 1] = k_rem - above;
    lds[kWaves + 2] = v;
  }
  __syncthreads();
  const Digit d = {lds[kWaves], lds[kWaves + 1], lds[kWaves + 2], total};
  return d;
}


}  // namespace sp
