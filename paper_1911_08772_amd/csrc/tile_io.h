// Per-thread tile loads and stores.  Thread `tid` owns, in each of the kSlots slots, the four
// consecutive elements starting at tbase + (slot*kBlock + tid)*4, so one wave instruction covers
// 1 KiB of contiguous memory.  The FULL variants use aligned 16-byte accesses; the others
// predicate every element against the tile's valid range [lo, hi).
#pragma once
#include "common.h"

namespace sp {

__device__ inline int64_t slot_index(const Tile& t, int slot) {
  return t.tbase + (int64_t)(slot * kBlock + (int)threadIdx.x) * 4;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// returns the validity mask (bit e set if element e of this thread is inside the tile's range).
// STREAM marks data that will not be read again soon (non-temporal: it should not displace
// what later passes re-read from the caches).
template <bool FULL, bool STREAM = false>
__device__ inline uint32_t load_tile(const float* __restrict__ p, const Tile& t,
                                     float (&v)[kPerThread]) {
  if (FULL) {
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      const f32x4* src = reinterpret_cast<const f32x4*>(p + slot_index(t, j));
      const f32x4 q = STREAM ? __builtin_nontemporal_load(src) : *src;
      v[4 * j + 0] = q.x;
      v[4 * j + 1] = q.y;
      v[4 * j + 2] = q.z;
      v[4 * j + 3] = q.w;
    }
    return 0xFFFFu;
  }
  // ragged chunk: slots wholly inside [lo, hi) still move as one aligned float4; only the
  // slots that straddle an end of the range go element by element
  uint32_t valid = 0;
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    const int64_t i0 = slot_index(t, j);
    if (i0 >= t.lo && i0 + 4 <= t.hi) {
      const f32x4* src = reinterpret_cast<const f32x4*>(p + i0);
      const f32x4 q = STREAM ? __builtin_nontemporal_load(src) : *src;
      v[4 * j + 0] = q.x;
      v[4 * j + 1] = q.y;
      v[4 * j + 2] = q.z;
      v[4 * j + 3] = q.w;
      valid |= 0xFu << (4 * j);
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int64_t i = i0 + c;
        const bool ok = (i >= t.lo) && (i < t.hi);
        v[4 * j + c] = ok ? p[i] : 0.0f;
        valid |= (ok ? 1u : 0u) << (4 * j + c);
      }
    }
  }
  return valid;
}

// STREAM: data nobody reads again soon (non-temporal stores; full chunks only).
template <bool FULL, bool STREAM = false>
__device__ inline void store_tile(float* p, const Tile& t, const float (&v)[kPerThread],
                                  uint32_t valid) {
  if (FULL) {
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      f32x4 q;
      q.x = v[4 * j + 0];
      q.y = v[4 * j + 1];
      q.z = v[4 * j + 2];
      q.w = v[4 * j + 3];
      f32x4* dst = reinterpret_cast<f32x4*>(p + slot_index(t, j));
      if (STREAM) __builtin_nontemporal_store(q, dst);
      else *dst = q;
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    const int64_t i0 = slot_index(t, j);
    if (((valid >> (4 * j)) & 0xFu) == 0xFu) {
      float4 q;
      q.x = v[4 * j + 0];
      q.y = v[4 * j + 1];
      q.z = v[4 * j + 2];
      q.w = v[4 * j + 3];
      *reinterpret_cast<float4*>(p + i0) = q;
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if ((valid >> (4 * j + c)) & 1u) p[i0 + c] = v[4 * j + c];
    }
  }
}

}  // namespace sp
