// Per-call initialisation of the control blocks: for the segmented call, validation of the
// device-resident layout, the tile numbering of the segments and the per-segment quantiles.
#pragma once
#include "common.h"
#include "gaussiank.h"

namespace sp {

__device__ inline void clear_result(sparsify_result& r) {
  r.nnz = 0;
  r.rounds = 0;
  r.count[0] = r.count[1] = r.count[2] = r.count[3] = 0;
  r.flags = 0;
  r.thres_f32 = 0.0f;
  r.mean = r.std = r.z = r.thres0 = r.thres = 0.0;
  r.topk_key = 0;
  r.topk_ties_taken = 0;
  r.acc_sqnorm = 0.0;
  r.residual_sqnorm = 0.0;
}

// Plain copy of n floats (n a multiple of 4, both pointers 16-byte aligned): a kernel of known
// traffic, 4n bytes read and 4n written, against which hardware byte counters are scaled.
__global__ __launch_bounds__(kBlock) void k_calibration_copy(float* dst, const float* src, size_t n4) {
  const float4* s4 = reinterpret_cast<const float4*>(src);
  float4* d4 = reinterpret_cast<float4*>(dst);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (size_t)gridDim.x * blockDim.x)
    d4[i] = s4[i];
}

// Segmented calls: one block walks the segments in chunks of kBlock, numbers their tiles and
// their groups of kSegGroupTiles tiles, and clears the group totals.
// mode 0 = Top_k, 1 = Gaussian_k.
constexpr uint32_t kSegGroupTiles = 64;

// Largest of the values held by the threads before the calling one (thread order), and the largest
// of all: a segment may start only at or after every earlier offset, or two valid segments could
// overlap.  `lds` holds kWaves words of 8 bytes.  Two barriers.
__device__ inline int64_t block_exclusive_max(int64_t v, int64_t lowest, int64_t* lds, int64_t* all) {
  int64_t inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int64_t o = __shfl_up(inc, off, 64);
    if (lane_id() >= off && o > inc) inc = o;
  }
  int64_t before = __shfl_up(inc, 1, 64);
  if (lane_id() == 0) before = lowest;
  if (lane_id() == 63) lds[wave_id()] = inc;
  __syncthreads();
  int64_t total = lowest;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const int64_t x = lds[w];
    if (w < wave_id() && x > before) before = x;
    if (x > total) total = x;
  }
  __syncthreads();
  *all = total;
  return before;
}

// One round of the walk: what thread i learns of segment base + i.  Every workgroup that runs a
// round on the same layout gets the same answers (same arithmetic on the same inputs).
struct SegRound {
  int s;                          // the segment (base + thread), >= a.L: none
  int64_t start, end, k, o0, o1;
  uint32_t nt, tile0, ng, group0; // tiles and groups of 64 tiles (0 if bad), the first of each
  bool bad;
  uint32_t total, gtotal;         // tiles and groups numbered in this round (block-uniform)
};
// `lds_scan` holds kWaves + 1 words, `lds_max` kWaves words of 8 bytes.  Barriers.
__device__ inline SegRound seg_setup_round(const Args& a, int base, uint32_t carry, uint32_t gcarry,
                                           int64_t& off_max, uint32_t* lds_scan, int64_t* lds_max) {
  SegRound r;
  r.s = base + (int)threadIdx.x;
  const int s = r.s;
  uint32_t nt = 0;
  bool bad = true;
  int64_t start = 0, end = 0, k = 0, o0 = 0, o1 = 0;
  if (s < a.L) {
    start = a.seg_off[s];
    end = a.seg_off[s + 1];
    k = a.seg_k[s];
    o0 = a.out_off[s];
    o1 = a.out_off[s + 1];
    bad = !(start >= 0 && end > start && end <= a.d_total && k >= 1 && k <= end - start &&
            o0 >= 0 && o1 >= o0 && o1 <= a.out_cap);
    if (s == 0 && start != 0) bad = true;
    if (s == a.L - 1 && end != a.d_total) bad = true;
  }
  {  // offsets must not step back behind an earlier one (seg_off non-decreasing up to here)
    const int64_t lowest = (int64_t)1 << 63;
    int64_t round_max;
    const int64_t before = block_exclusive_max(s < a.L ? start : lowest, lowest, lds_max, &round_max);
    if (s < a.L && (start < before || start < off_max)) bad = true;
    if (round_max > off_max) off_max = round_max;
  }
  if (s < a.L && !bad) nt = seg_ntiles(start, end, a.tile_chunks);
  uint32_t total, gtotal;
  const uint32_t excl = block_exclusive_scan(nt, lds_scan, &total);
  // a layout whose valid segments overlap could number more tiles than the workspace holds
  if (s < a.L && !bad && (uint64_t)carry + excl + nt > (uint64_t)a.max_tiles) bad = true;
  const uint32_t ng = bad ? 0u : (nt + kSegGroupTiles - 1) / kSegGroupTiles;
  const uint32_t gexcl = block_exclusive_scan(ng, lds_scan, &gtotal);
  const uint32_t group0 = gcarry + gexcl;
  if (s < a.L && !bad && (uint64_t)group0 + ng > (uint64_t)a.max_groups) bad = true;  // cannot happen: see carve
  r.start = start;
  r.end = end;
  r.k = k;
  r.o0 = o0;
  r.o1 = o1;
  r.nt = bad ? 0u : nt;
  r.tile0 = carry + excl;
  r.ng = ng;
  r.group0 = group0;
  r.bad = bad;
  r.total = total;
  r.gtotal = gtotal;
  return r;
}

__device__ inline void seg_setup_body(const Args& a, int mode) {
  __shared__ uint32_t lds_scan[kWaves + 1];
  __shared__ int64_t lds_max[kWaves];
  uint32_t carry = 0;    // tiles numbered so far (block-uniform, saturating)
  uint32_t gcarry = 0;   // groups numbered so far
  int64_t off_max = 0;   // largest offset among the segments of earlier rounds
  for (int base = 0; base < a.L; base += kBlock) {
    const SegRound r = seg_setup_round(a, base, carry, gcarry, off_max, lds_scan, lds_max);
    const int s = r.s;
    if (s < a.L) {
      const bool bad = r.bad;
      a.tile_start[s] = r.tile0;
      SegCtrl& c = a.ctrl[s];
      c.start = r.start;
      c.end = r.end;
      c.k = r.k;
      c.cap = r.o1 - r.o0;
      c.out_base = r.o0;
      c.tile0 = r.tile0;
      c.ntiles = r.nt;
      c.bad = bad ? 1u : 0u;
      c.group0 = r.group0;
      c.prefix = 0;
      c.k_rem = (uint32_t)r.k;
      c.n_eq = 0;
      c.rank_ties = 0;
      c.select_none = 0;
      c.t_final = 0.0f;
      c.list_mode = 0;  // layer-wise calls with lists: set when one of the segment's stretches ran out
      c.list_count = 0;
      sparsify_result& res = a.result[s];
      clear_result(res);
      if (bad) {
        res.flags = SPARSIFY_F_BADSEGMENT;
      } else if (mode == 0) {
        if (c.cap < r.k) {
          c.select_none = 1;
          res.flags = SPARSIFY_F_OVERFLOW;
        } else {
          res.nnz = (uint32_t)r.k;
        }
      }
    }
    const uint64_t next = (uint64_t)carry + r.total;
    carry = next > 0x40000000ull ? 0x40000000u : (uint32_t)next;
    gcarry += r.gtotal;  // <= carry / 1 + L: no overflow
  }
  if (threadIdx.x == 0) a.tile_start[a.L] = carry;
  const uint32_t words = (gcarry < a.max_groups ? gcarry : a.max_groups) * (uint32_t)kNumThres;
  for (uint32_t i = threadIdx.x; i < words; i += kBlock) a.seg_groups[i] = 0;
}

__global__ __launch_bounds__(kBlock) void k_seg_setup(const Args a, int mode) { seg_setup_body(a, mode); }

}  // namespace sp
