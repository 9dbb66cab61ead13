// Decompression and aggregation: dense = scale * sum over the workers p of Comp_k(acc_p), the sum
// in Eq. (2), from the workers' compacted (index, value) lists.  One kernel, no workspace, no
// floating-point atomics: the result is the fp32 sum taken worker 0 first, bit for bit.
//
// Each list is strictly ascending in index (what the compressors of this library emit), so the
// pairs that fall into a stretch of `dense` are one contiguous run of every list.  A workgroup
// owns a span of consecutive chunks of `dense`:
//   1. it streams zeros over the span (almost all of it stays zero);
//   2. it finds, for every list, the run that falls into the span (a cooperative search: 16 lanes
//      probe 16 places per round, so a list of tens of thousands of pairs takes four dependent
//      loads instead of fifteen);
//   3. it numbers the runs' pairs list after list and loads them into registers in one batch;
//   4. it enters the pairs' indices into a small hash table in LDS, which tells the elements that
//      receive one contribution (their value is final at once) from the few that receive several;
//      those are summed in list order, one contribution per round (the pending pair with the
//      lowest number goes next), so the number of rounds is the largest number of workers that
//      meet in one element;
//   5. it stores the touched elements over the zeros.
// Spans with more pairs than the registers hold are taken chunk by chunk, and a chunk that still
// has too many (a list denser than a quarter of the vector) is built densely in LDS, list after
// list.  HBM traffic: 4 bytes per element written, 8 bytes per pair read.
//
// A few extra workgroups check the lists (strictly ascending, indices below d, counts within the
// stride) and raise a flag; pairs outside a workgroup's own span are never applied, so whatever
// the lists hold nothing is written outside `dense`.
#pragma once
#include "common.h"

namespace sp {

constexpr int kScatterMaxLists = 1024;
constexpr int kScatterRegs = 4;                            // pairs per thread per round
constexpr int kScatterRound = kBlock * kScatterRegs;       // pairs per round: 1024
constexpr int kScatterSlots = 2 * kScatterRound;           // hash table entries
constexpr int kScatterLanes = 16;                          // lanes per cooperative search
constexpr int kScatterCheckers = 128;                      // workgroups that check the lists
constexpr int kScatterCheckRegs = 8;                       // entries per thread per checking round
constexpr uint32_t kScatterEmpty = 0xFFFFFFFFu;
static_assert(2 * kScatterSlots == kChunk, "the hash tables and the dense tile share their LDS");

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
// idle along.  Terminates on any data: the range shrinks every round, and no position outside
// [from, n) is read.
__device__ inline uint32_t group_lower_bound(const uint32_t* list, uint32_t from, uint32_t n,
                                             uint32_t target, bool active, bool geometric) {
  const uint32_t l = (uint32_t)lane_id() & (kScatterLanes - 1);
  const int shift = (lane_id() / kScatterLanes) * kScatterLanes;
  uint32_t L = active ? from : 0u, R = active ? n : 0u;  // the answer lies in [L, R]
  if (R < L) R = L;
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
    const int src = shift + (int)(f < (uint32_t)kScatterLanes ? f : (uint32_t)kScatterLanes - 1u);
    const uint32_t lo_off = __shfl(off_prev, src, 64);
    const uint32_t hi_off = __shfl(off, src, 64);
    if (R > L) {
      if (f < (uint32_t)kScatterLanes) {
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

// Dynamic LDS: five tables of P (+1) words.
__host__ __device__ inline uint32_t scatter_table_words(int P) { return 5u * (uint32_t)P + 4u; }

// The pairs of one round in registers: item number, list, index, value (item < 0: none).
struct ScatterRegs {
  uint32_t pi[kScatterRegs];
  float pv[kScatterRegs];
  int32_t item[kScatterRegs];
  int32_t list[kScatterRegs];
};

__global__ __launch_bounds__(kBlock) void k_scatter_add(const ScatterArgs a) {
  // Two hash tables of kScatterSlots words, or one dense tile of kChunk floats.
  __shared__ uint32_t lds_ab[kChunk];
  __shared__ uint32_t lds_scan[kWaves];
  extern __shared__ uint32_t lds_tables[];
  const int P = a.P;
  uint32_t* beg = lds_tables;          // [P] first pair of the list's run (current range)
  uint32_t* cnt = beg + P;             // [P] pairs in that run
  uint32_t* sbeg = cnt + P;            // [P] the same for the whole span (checker: the list's length)
  uint32_t* scnt = sbeg + P;           // [P]
  uint32_t* off = scnt + P;            // [P + 1] runs numbered one after the other

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
      sbeg[p] = n;
    }
    __syncthreads();
    const uint32_t T = scan_lists(cnt, off, P, lds_scan);
    __syncthreads();
    bool bad = false;
    for (uint32_t base = 0; base < T; base += kBlock * kScatterCheckRegs) {
      uint32_t cur[kScatterCheckRegs], nxt[kScatterCheckRegs];
#pragma unroll
      for (int r = 0; r < kScatterCheckRegs; ++r) {  // all loads first, then the comparisons
        const uint32_t n = base + r * kBlock + threadIdx.x;
        cur[r] = 0u;
        nxt[r] = 0xFFFFFFFFu;
        if (n < T) {
          const int q = list_of_item(off, P, n);
          const uint32_t j = beg[q] + (n - off[q]);
          const uint32_t* list = a.idx + (int64_t)q * a.stride;
          cur[r] = list[j];
          if (j + 1 < sbeg[q]) nxt[r] = list[j + 1];
        }
      }
#pragma unroll
      for (int r = 0; r < kScatterCheckRegs; ++r)
        if (!((int64_t)cur[r] < a.d && cur[r] < nxt[r])) bad = true;
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
  uint32_t* tab_a = lds_ab;                  // keys, later the sums of the shared elements
  uint32_t* tab_b = lds_ab + kScatterSlots;  // contributions per key, later the claims
  float* tile = reinterpret_cast<float*>(lds_ab);

  {  // zeros over the span; the touched elements are stored again at the end, after barriers
    const float zero = 0.0f * a.scale;
    for (int64_t c = lo; c < hi; c += kChunk) {
      if (c + kChunk <= hi) {
        float4* d4 = reinterpret_cast<float4*>(a.dense + c);
#pragma unroll
        for (int j = 0; j < kSlots; ++j) d4[j * kBlock + threadIdx.x] = make_float4(zero, zero, zero, zero);
      } else {
        for (int64_t i = c + threadIdx.x; i < hi; i += kBlock) a.dense[i] = zero;
      }
    }
#pragma unroll
    for (int j = 0; j < kChunk / kBlock; ++j)
      lds_ab[j * kBlock + threadIdx.x] = (j * kBlock < kScatterSlots) ? kScatterEmpty : 0u;
  }

  // Runs of the lists inside [rlo, rhi): 16 lanes per list, 16 lists per pass.  whole = true:
  // searched in the whole list (its length from nnz), results to sbeg/scnt; else searched inside
  // the span's run, results to beg/cnt.
  auto find_runs = [&](int64_t rlo, int64_t rhi, bool whole) {
    for (int p0 = 0; p0 < P; p0 += kBlock / kScatterLanes) {
      const int p = p0 + (int)threadIdx.x / kScatterLanes;
      const bool active = p < P;
      uint32_t from = 0, to = 0;
      const uint32_t* list = a.idx;
      if (active) {
        list = a.idx + (int64_t)p * a.stride;
        if (whole) {
          to = a.nnz[(int64_t)p * a.nnz_step];
          if ((int64_t)to > a.stride) to = (uint32_t)a.stride;
        } else {
          from = sbeg[p];
          to = from + scnt[p];
        }
      }
      const uint32_t b = group_lower_bound(list, from, to, (uint32_t)rlo, active, !whole);
      // [rlo, rhi) holds at most rhi - rlo entries of a strictly ascending list
      uint32_t limit = to;
      if ((uint64_t)b + (uint64_t)(rhi - rlo) < (uint64_t)to) limit = b + (uint32_t)(rhi - rlo);
      const uint32_t e = group_lower_bound(list, b, limit, (uint32_t)rhi, active, true);
      if (active && (threadIdx.x & (kScatterLanes - 1)) == 0) {
        (whole ? sbeg : beg)[p] = b;
        (whole ? scnt : cnt)[p] = e - b;
      }
    }
  };

  // Loads the pairs base .. base + 1023 of the current runs (beg/off), all loads in flight at
  // once; pairs whose index is outside [rlo, rhi) (possible only in lists that are not ascending)
  // are dropped.
  auto load_round = [&](ScatterRegs& g, uint32_t base, uint32_t T, int64_t rlo, int64_t rhi) {
#pragma unroll
    for (int r = 0; r < kScatterRegs; ++r) {
      const uint32_t n = base + r * kBlock + threadIdx.x;
      g.item[r] = -1;
      g.list[r] = -1;
      g.pi[r] = 0;
      g.pv[r] = 0.0f;
      if (n < T) {
        const int q = list_of_item(off, P, n);
        const int64_t at = (int64_t)q * a.stride + beg[q] + (n - off[q]);
        g.item[r] = (int32_t)n;
        g.list[r] = q;
        g.pi[r] = a.idx[at];
        g.pv[r] = a.val[at];
      }
    }
#pragma unroll
    for (int r = 0; r < kScatterRegs; ++r)
      if (g.item[r] >= 0 && !((int64_t)g.pi[r] >= rlo && (int64_t)g.pi[r] < rhi)) g.item[r] = -1;
  };

  // At most kScatterRound pairs, in registers: hash, sum what is shared in item order, store.
  // On entry and on exit tab_a is all kScatterEmpty and tab_b all zero.
  auto sparse_accumulate = [&](const ScatterRegs& g) {
    uint32_t slot[kScatterRegs];
    bool shared[kScatterRegs];
#pragma unroll
    for (int r = 0; r < kScatterRegs; ++r) {
      slot[r] = 0;
      if (g.item[r] >= 0) {
        uint32_t s = (g.pi[r] * 2654435761u) >> 21;  // 11 bits
        for (int tries = 0; tries < kScatterSlots; ++tries) {  // at most 1024 keys in 2048 slots
          const uint32_t old = atomicCAS(&tab_a[s], kScatterEmpty, g.pi[r]);
          if (old == kScatterEmpty || old == g.pi[r]) break;
          s = (s + 1u) & (uint32_t)(kScatterSlots - 1);
        }
        slot[r] = s;
        atomicAdd(&tab_b[s], 1u);
      }
    }
    __syncthreads();
    bool any_shared = false;
#pragma unroll
    for (int r = 0; r < kScatterRegs; ++r) {
      shared[r] = g.item[r] >= 0 && tab_b[slot[r]] > 1u;
      any_shared = any_shared || shared[r];
    }
    float out[kScatterRegs];
#pragma unroll
    for (int r = 0; r < kScatterRegs; ++r) out[r] = 0.0f + g.pv[r];  // the element's only contribution
    if (__syncthreads_or(any_shared)) {  // (the barrier also ends the reads of tab_b above)
#pragma unroll
      for (int r = 0; r < kScatterRegs; ++r) {
        if (shared[r]) {
          tab_a[slot[r]] = 0u;             // +0.0f: the sum starts here
          tab_b[slot[r]] = kScatterEmpty;  // nobody has claimed the next turn
        }
      }
      bool pending[kScatterRegs];
#pragma unroll
      for (int r = 0; r < kScatterRegs; ++r) pending[r] = shared[r];
      bool more = true;
      while (__syncthreads_or(more)) {
        // the pending pair with the lowest item number (the earliest worker) of each element
#pragma unroll
        for (int r = 0; r < kScatterRegs; ++r)
          if (pending[r]) atomicMin(&tab_b[slot[r]], (uint32_t)g.item[r]);
        __syncthreads();
        bool mine[kScatterRegs];
#pragma unroll
        for (int r = 0; r < kScatterRegs; ++r) mine[r] = pending[r] && tab_b[slot[r]] == (uint32_t)g.item[r];
        __syncthreads();
        more = false;
#pragma unroll
        for (int r = 0; r < kScatterRegs; ++r) {
          if (mine[r]) {
            tab_a[slot[r]] = __float_as_uint(__uint_as_float(tab_a[slot[r]]) + g.pv[r]);  // one fp32 addition
            tab_b[slot[r]] = kScatterEmpty;
            pending[r] = false;
          }
          more = more || pending[r];
        }
      }
#pragma unroll
      for (int r = 0; r < kScatterRegs; ++r)
        if (shared[r]) out[r] = __uint_as_float(tab_a[slot[r]]);
      __syncthreads();
    }
    // several holders of one element store the same value
#pragma unroll
    for (int r = 0; r < kScatterRegs; ++r) {
      if (g.item[r] >= 0) {
        a.dense[g.pi[r]] = out[r] * a.scale;
        tab_a[slot[r]] = kScatterEmpty;
        tab_b[slot[r]] = 0u;
      }
    }
    __syncthreads();
  };

  // A chunk with more pairs than one round: built densely in the tile, round after round, list
  // after list (a barrier after every list that has pairs in the chunk), then stored whole.
  auto dense_accumulate = [&](uint32_t T, int64_t clo, int64_t chi) {
#pragma unroll
    for (int j = 0; j < kChunk / kBlock; ++j) tile[j * kBlock + threadIdx.x] = 0.0f;
    __syncthreads();
    for (uint32_t base = 0; base < T; base += kScatterRound) {
      ScatterRegs g;
      load_round(g, base, T, clo, chi);
      const uint32_t last = (base + kScatterRound < T ? base + kScatterRound : T) - 1u;
      const int q0 = list_of_item(off, P, base), q1 = list_of_item(off, P, last);
      for (int q = q0; q <= q1; ++q) {
        if (off[q + 1] == off[q]) continue;  // block-uniform
#pragma unroll
        for (int r = 0; r < kScatterRegs; ++r) {
          if (g.item[r] >= 0 && g.list[r] == q) {
            float* cell = &tile[(int64_t)g.pi[r] - clo];
            *cell = *cell + g.pv[r];
          }
        }
        __syncthreads();
      }
    }
    for (int64_t i = clo + threadIdx.x; i < chi; i += kBlock) a.dense[i] = tile[i - clo] * a.scale;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kChunk / kBlock; ++j)
      lds_ab[j * kBlock + threadIdx.x] = (j * kBlock < kScatterSlots) ? kScatterEmpty : 0u;
    __syncthreads();
  };

  find_runs(lo, hi, true);
  __syncthreads();  // also: the hash tables are set up, and the zeros come before the later stores
  uint32_t T = scan_lists(scnt, off, P, lds_scan);
  __syncthreads();
  if (T == 0) return;
  if (T <= (uint32_t)kScatterRound) {  // the usual case: the whole span at once
    for (int p = threadIdx.x; p < P; p += kBlock) beg[p] = sbeg[p];
    __syncthreads();
    ScatterRegs g;
    load_round(g, 0, T, lo, hi);
    sparse_accumulate(g);
    return;
  }
  for (int64_t clo = lo; clo < hi; clo += kChunk) {  // dense lists: chunk by chunk
    const int64_t chi = clo + kChunk < hi ? clo + kChunk : hi;
    find_runs(clo, chi, false);
    __syncthreads();
    T = scan_lists(cnt, off, P, lds_scan);
    __syncthreads();
    if (T == 0) continue;
    if (T <= (uint32_t)kScatterRound) {
      ScatterRegs g;
      load_round(g, 0, T, clo, chi);
      sparse_accumulate(g);
    } else {
      dense_accumulate(T, clo, chi);
    }
  }
}

}  // namespace sp
