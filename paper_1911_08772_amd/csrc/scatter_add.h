// Decompression and aggregation: dense = scale * sum over the workers p of Comp_k(acc_p), the sum
// in Eq. (2), from the workers' compacted (index, value) lists.  One kernel, no workspace, no
// floating-point atomics: the result is the fp32 sum taken worker 0 first, bit for bit.
//
// Each list is strictly ascending in index (what the compressors of this library emit), so the
// pairs that fall into a stretch of `dense` are one contiguous run of every list.  A workgroup
// owns a span of consecutive chunks of `dense`.  It finds, for every list, the run that falls
// into its span (a cooperative search: 16 lanes probe 16 places per round, so a list of tens of
// thousands of pairs takes four dependent loads instead of fifteen), numbers the runs' pairs
// list after list, loads them into registers in one batch, and then builds each chunk in LDS:
// zeros, then list after list (a barrier between lists; inside a list the indices differ, so
// its pairs commute), then one scaled, coalesced store of the chunk.  HBM traffic: 4 bytes per
// element written, 8 bytes per pair read.
//
// A few extra workgroups check the lists (strictly ascending, indices below d, counts within the
// stride) and raise a flag; pairs outside a workgroup's own span are never applied, so whatever
// the lists hold nothing is written outside `dense`.
#pragma once
#include "common.h"

namespace sp {

constexpr int kScatterMaxLists = 1024;
constexpr int kScatterRegs = 4;                            // pairs per thread per round
constexpr int kScatterRound = kBlock * kScatterRegs;       // pairs per round
constexpr int kScatterLanes = 16;                          // lanes per cooperative search
constexpr int kScatterCheckers = 64;                       // workgroups that check the lists

struct ScatterArgs {
  int64_t d;
  int32_t P;
  const uint32_t* idx;   // [P][stride]
  const float* val;      // [P][stride]
  int64_t stride;
  const uint32_t* nnz;   // nnz[p * nnz_step]
  int64_t nnz_step;      // in 4-byte words
  float scale;
  float* dense;
  uint32_t* status;
  uint32_t span_chunks;  // chunks per workgroup
  uint32_t nspans;
};

// First position j in [from, n) with list[j] >= target (n if none), found by the 16 lanes of a
// group together.  `geometric`: the first round probes from+1, from+2, from+4, ... (the answer is
// expected close to `from`).  Every lane of the wave must call this; groups whose list is done
// idle along.  Terminates on any data: the range shrinks every round.
__device__ inline uint32_t group_lower_bound(const uint32_t* list, uint32_t from, uint32_t n,
                                             uint32_t target, bool active, bool geometric) {
  const uint32_t l = (uint32_t)lane_id() & (kScatterLanes - 1);
  const int shift = (lane_id() / kScatterLanes) * kScatterLanes;
  uint32_t L = active ? from : 0u, R = active ? n : 0u;  // the answer lies in [L, R]
  bool first = geometric;
  while (__any(R > L)) {
    const uint32_t m = R - L;
    // probe positions L + off(l) - 1 with off increasing in l; off(-1) = 0
    const uint32_t step = m / (kScatterLanes + 1) + 1;
    const uint32_t off = first ? (1u << l) : (l + 1u) * step;
    const uint32_t off_prev = first ? (l ? (1u << (l - 1)) : 0u) : l * step;
    const bool inside = off <= m;                      // probe position L + off - 1 < R
    const uint32_t v = (R > L && inside) ? list[L + off - 1] : 0xFFFFFFFFu;
    const bool ge = !inside || v >= target;
    const uint32_t mask = (uint32_t)(__ballot(ge) >> shift) & 0xFFFFu;
    // first lane whose probe is >= target: the answer is in (its predecessor's probe, its probe]
    const uint32_t f = mask ? (uint32_t)__builtin_ctz(mask) : (uint32_t)kScatterLanes;
    const uint32_t lo_off = __shfl(off_prev, shift + (f < kScatterLanes ? f : kScatterLanes - 1), 64);
    const uint32_t hi_off = __shfl(off, shift + (f < kScatterLanes ? f : kScatterLanes - 1), 64);
    if (R > L) {
      if (f < kScatterLanes) {
        const uint32_t newR = (hi_off <= m) ? L + hi_off - 1 : R;
        L = L + lo_off;
        R = newR;
      } else {
        L = L + hi_off;  // every probe was below the target (and inside the range)
      }
    }
    first = false;
  }
  return L;
}

// Turns per-list counts cnt[0..P) (LDS) into offsets off[0..P] (LDS) and returns the total.
// Two barriers inside; one more before the caller may read off[].
__device__ inline uint32_t scan_lists(const uint32_t* cnt, uint32_t* off, int P, uint32_t* lds_scan) {
  constexpr int kPer = kScatterMaxLists / kBlock;  // 4 consecutive lists per thread
  uint32_t x[kPer], sum = 0;
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int p = (int)threadIdx.x * kPer + u;
    x[u] = p < P ? cnt[p] : 0u;
    sum += x[u];
  }
  uint32_t total;
  uint32_t run = block_exclusive_scan(sum, lds_scan, &total);
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int p = (int)threadIdx.x * kPer + u;
    if (p < P) off[p] = run;
    run += x[u];
  }
  if (threadIdx.x == 0) off[P] = total;
  return total;
}

// The list that flat item n belongs to: largest q with off[q] <= n (n < off[P]).
__device__ inline int list_of_item(const uint32_t* off, int P, uint32_t n) {
  int lo = 0, hi = P;  // off[lo] <= n < off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= n) lo = mid; else hi = mid;
  }
  return lo;
}

// Dynamic LDS: four tables of P (+1) words.
__host__ __device__ inline uint32_t scatter_table_words(int P) { return 4u * (uint32_t)P + 4u; }

__global__ __launch_bounds__(kBlock) void k_scatter_add(const ScatterArgs a) {
  __shared__ float tile[kChunk];
  __shared__ uint32_t lds_scan[kWaves];
  extern __shared__ uint32_t lds_tables[];
  const int P = a.P;
  uint32_t* beg = lds_tables;          // [P] first pair of the list's run
  uint32_t* cnt = beg + P;             // [P] pairs in the run
  uint32_t* len = cnt + P;             // [P] pairs in the list
  uint32_t* off = len + P;             // [P + 1] runs numbered one after the other

  if (blockIdx.x < (uint32_t)kScatterCheckers) {
    // ---- checker: slice blockIdx.x of every list ------------------------------------------------
    bool bad_count = false;
    for (int p = threadIdx.x; p < P; p += kBlock) {
      uint32_t n = a.nnz[(int64_t)p * a.nnz_step];
      if ((int64_t)n > a.stride) {
        bad_count = true;
        n = (uint32_t)a.stride;
      }
      const uint32_t s = (uint32_t)((uint64_t)n * blockIdx.x / kScatterCheckers);
      const uint32_t e = (uint32_t)((uint64_t)n * (blockIdx.x + 1) / kScatterCheckers);
      beg[p] = s;
      cnt[p] = e - s;
      len[p] = n;
    }
    __syncthreads();
    const uint32_t T = scan_lists(cnt, off, P, lds_scan);
    __syncthreads();
    bool bad = false;
    for (uint32_t base = 0; base < T; base += kScatterRound) {
#pragma unroll
      for (int r = 0; r < kScatterRegs; ++r) {
        const uint32_t n = base + r * kBlock + threadIdx.x;
        if (n < T) {
          const int q = list_of_item(off, P, n);
          const uint32_t j = beg[q] + (n - off[q]);
          const uint32_t* list = a.idx + (int64_t)q * a.stride;
          const uint32_t cur = list[j];
          const uint32_t nxt = (j + 1 < len[q]) ? list[j + 1] : 0xFFFFFFFFu;
          if (!((int64_t)cur < a.d && cur < nxt)) bad = true;
        }
      }
    }
    uint32_t flags = (bad ? 1u : 0u) | (bad_count ? 2u : 0u);
    if (__any(flags != 0)) {  // one atomic per wave that found something
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) flags |= __shfl_xor(flags, o, 64);
      if (lane_id() == 0) atomicOr(a.status, flags);
    }
    return;
  }

  // ---- one span of `dense` ------------------------------------------------------------------------
  const uint32_t span = blockIdx.x - kScatterCheckers;
  const int64_t span_elems = (int64_t)a.span_chunks * kChunk;
  const int64_t lo = (int64_t)span * span_elems;
  if (lo >= a.d) return;
  const int64_t hi = lo + span_elems < a.d ? lo + span_elems : a.d;

  // runs of the lists inside [lo, hi): 16 lanes per list, 16 lists per pass
  for (int p0 = 0; p0 < P; p0 += kBlock / kScatterLanes) {
    const int p = p0 + (int)threadIdx.x / kScatterLanes;
    const bool active = p < P;
    uint32_t n = 0;
    const uint32_t* list = a.idx;
    if (active) {
      n = a.nnz[(int64_t)p * a.nnz_step];
      if ((int64_t)n > a.stride) n = (uint32_t)a.stride;
      list = a.idx + (int64_t)p * a.stride;
    }
    const uint32_t b = group_lower_bound(list, 0u, n, (uint32_t)lo, active, false);
    // hi <= 2^31 fits; a span holds at most span_elems entries of a strictly ascending list
    uint32_t limit = n;
    if ((uint64_t)b + (uint64_t)span_elems < (uint64_t)n) limit = b + (uint32_t)span_elems;
    const uint32_t e = group_lower_bound(list, b, limit, (uint32_t)hi, active, true);
    if (active && (threadIdx.x & (kScatterLanes - 1)) == 0) {
      beg[p] = b;
      cnt[p] = e - b;
    }
  }
  __syncthreads();
  const uint32_t T = scan_lists(cnt, off, P, lds_scan);
  __syncthreads();

  uint32_t pi[kScatterRegs];
  float pv[kScatterRegs];
  int pq[kScatterRegs];
  auto load_round = [&](uint32_t base) {
#pragma unroll
    for (int r = 0; r < kScatterRegs; ++r) {
      const uint32_t n = base + r * kBlock + threadIdx.x;
      pq[r] = -1;
      pi[r] = 0;
      pv[r] = 0.0f;
      if (n < T) {
        const int q = list_of_item(off, P, n);
        const int64_t at = (int64_t)q * a.stride + beg[q] + (n - off[q]);
        pq[r] = q;
        pi[r] = a.idx[at];
        pv[r] = a.val[at];
      }
    }
  };
  const bool one_round = T <= (uint32_t)kScatterRound;
  if (one_round) load_round(0);

  for (int64_t clo = lo; clo < hi; clo += kChunk) {
    const int64_t chi = clo + kChunk < hi ? clo + kChunk : hi;
    {  // zeros
      float4* t4 = reinterpret_cast<float4*>(tile);
#pragma unroll
      for (int j = 0; j < kSlots; ++j) t4[j * kBlock + threadIdx.x] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __syncthreads();
    for (uint32_t base = 0; base < T; base += kScatterRound) {
      if (!one_round) load_round(base);
      // lists present in this round: those of its first and last item, and all between
      const uint32_t last = (base + kScatterRound < T ? base + kScatterRound : T) - 1u;
      const int q0 = list_of_item(off, P, base), q1 = list_of_item(off, P, last);
      for (int q = q0; q <= q1; ++q) {
        if (off[q + 1] == off[q]) continue;  // block-uniform: the list has nothing in this span
#pragma unroll
        for (int r = 0; r < kScatterRegs; ++r) {
          if (pq[r] == q && (int64_t)pi[r] >= clo && (int64_t)pi[r] < chi) {
            float* cell = &tile[(int64_t)pi[r] - clo];
            *cell = *cell + pv[r];  // one fp32 addition per contribution, worker order
          }
        }
        __syncthreads();
      }
    }
    // scaled store of the chunk
    if (chi - clo == kChunk) {
      const float4* t4 = reinterpret_cast<const float4*>(tile);
      float4* d4 = reinterpret_cast<float4*>(a.dense + clo);
#pragma unroll
      for (int j = 0; j < kSlots; ++j) {
        float4 x = t4[j * kBlock + threadIdx.x];
        x.x = x.x * a.scale;
        x.y = x.y * a.scale;
        x.z = x.z * a.scale;
        x.w = x.w * a.scale;
        d4[j * kBlock + threadIdx.x] = x;
      }
    } else {
      for (int64_t i = clo + threadIdx.x; i < chi; i += kBlock) a.dense[i] = tile[i - clo] * a.scale;
    }
    __syncthreads();  // the tile is zeroed again by the next chunk
  }
}

}  // namespace sp
