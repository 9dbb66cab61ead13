// C ABI of the gfx950 gradient compressor: argument checks, workspace carving, kernel launches.
// Nothing here touches device memory from the host or synchronises the stream.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "common.h"
#include "gaussiank.h"
#include "gaussiank_flat.h"
#include "gaussiank_seg.h"
#include "scatter_add.h"
#include "setup.h"
#include "sparsify.h"
#include "topk.h"
#include "dgck.h"
#include "topk_filter.h"
#include "topk_seg.h"
#include "topk_flat.h"

using namespace sp;

// ---- built-in workspace of the entry point that allocates nothing ------------------------------
// One copy per GPU the library runs on, held until the process ends.  In host code the array's
// name is only a handle for the runtime's symbol lookup: the device address is looked up once per
// device (static_scratch below) and that pointer is what the kernels receive.
constexpr size_t kStaticScratchBytes = size_t(6) << 20;
constexpr int64_t kStaticMaxD = int64_t(1) << 27;  // workspace of 2^27 elements: 5.06 MiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// ---- per-kernel timing (optional) -----------------------------------------------------------
constexpr int kMaxStages = 24;
struct sparsify_trace {
  hipEvent_t ev[kMaxStages + 1];
  const char* name[kMaxStages];
  int n;
  bool ok;
};

namespace {

struct Launcher {
  hipStream_t stream;
  sparsify_trace* tr;
  hipError_t err = hipSuccess;

  void begin() {
    if (tr) {
      tr->n = 0;
      note(hipEventRecord(tr->ev[0], stream));
    }
  }
  void note(hipError_t e) {
    if (err == hipSuccess && e != hipSuccess) err = e;
  }
  template <class K, class... A>
  void run(const char* name, K kernel, dim3 grid, dim3 block, A... args) {
    if (err != hipSuccess) return;
    kernel<<<grid, block, 0, stream>>>(args...);
    note(hipGetLastError());
    if (tr && tr->n < kMaxStages) {
      tr->name[tr->n] = name;
      ++tr->n;
      note(hipEventRecord(tr->ev[tr->n], stream));
    }
  }
};

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Chunks per tile.  Short vectors (up to kOneChunkLimit chunks) use one-chunk tiles, so that there
// are enough workgroups to fill the chip.  Longer ones use at least three chunks per tile (the
// per-workgroup prologues of the count and compact kernels are then paid a third as often:
// measured 8 % faster at 14.7 M elements, slower below about 6 M) and otherwise the smallest odd
// number that keeps the vector within about four thousand tiles, so that the per-tile partials
// stay few.  Odd on purpose: with a power-of-two tile size the workgroups, which advance in step,
// sit a power of two bytes apart and crowd the same memory channels (measured: 4 chunks per tile
// 5 % slower than 3 or 5).
// Vectors of more chunks than kChunkGridFrom (123 M elements) use the chunk-per-workgroup
// accumulate and, where the selector has the larger group tables (`big_tables`: Gaussian_k and
// Top_k with a separate accumulator), keep three chunks per tile as long as those tables hold the
// tiles: measured 3 % slower than the resident form at 67 M and 100 M elements, 2 % faster at
// 134 M, 5 % at 268 M and 537 M.
constexpr int64_t kTargetTiles = 4096;
constexpr int64_t kOneChunkLimit = 1536;
constexpr uint32_t kChunkGridFrom = 30000;
uint32_t tile_chunks_of(int64_t d_total, bool big_tables) {
  const int64_t chunks = (d_total + kChunk - 1) / kChunk;
  if (chunks <= kOneChunkLimit) return 1;
  const int64_t most = (big_tables && chunks > (int64_t)kChunkGridFrom) ? kBigMaxTiles : kTargetTiles;
  uint32_t c = 3;
  while ((chunks + c - 1) / c > most) c += 2;
  return c;
}

// The workspace is sized for the finest tiling (one chunk per tile), so any tiling fits.
uint32_t max_tiles_of(int64_t d_total, int32_t L, uint32_t tile_chunks) {
  // each segment adds at most two tiles over d/tile (ragged head and tail)
  return (uint32_t)(d_total / ((int64_t)kChunk * tile_chunks) + 2 * (int64_t)L + 1);
}

// Replicas of each segment's global histogram.  Every tile of a segment adds its bins to one
// replica with device-wide atomics, and those that meet on one address are performed one after
// the other (tens of nanoseconds each): the more tiles a segment has, the more replicas it
// needs.  By the number of segments, and at least one replica per eight tiles of an average
// segment at the default tile length (54 segments of 25.6 M elements: 1 -> 8 replicas took
// 6 us off the kernel that follows the accumulate kernel).
uint32_t hist_copies_of(int64_t d_total, int32_t L) {
  const uint32_t by_segments = L >= 32 ? 1u : L >= 8 ? 4u : L >= 2 ? 16u : 32u;
  const int64_t tiles_per_segment = d_total / ((int64_t)kChunk * 3 * L);
  uint32_t by_tiles = 1;
  while (by_tiles < 32u && (int64_t)by_tiles * 8 <= tiles_per_segment) by_tiles *= 2;
  return by_segments > by_tiles ? by_segments : by_tiles;
}

// Short lists (lists.h; Top_k: topk_list.h, DGC_k: dgck.h, Gaussian_k: gaussiank_list.h): flat
// vectors long enough for the passes saved to matter.  The list buffer holds kListShare of the
// vector's length in entries (Top_k's lists are expected to take max(4 k, 0.4 % of d), the
// others' about k), split evenly among the waves of the kernel that writes them.
constexpr int64_t kListFrom = 6'000'000;
constexpr double kListShare = 0.10;
// (Layer-wise calls: Gaussian_k and Top_k with a separate acc, up to kListMaxSegments segments,
// which bounds the run table.)
constexpr int32_t kListMaxSegments = 1024;
bool list_sized(int64_t d_total, int32_t L) {
  return L <= kListMaxSegments && d_total >= kListFrom;
}
size_t list_entries(int64_t d_total) { return (size_t)(kListShare * (double)d_total) + 64 * (size_t)kWaves * kMaxMomentParts; }

// Layer-wise Top_k with lists: five of its kernels do next to nothing per tile, and what they
// cost is the dispatch of a workgroup per tile; five chunks per tile instead of three measured
// 4 % faster per call on the 54-segment layout (0.128 against 0.133 ms; seven chunks 0.131;
// layer-wise Gaussian_k is fastest with three).
constexpr uint32_t kSegTopkListTileChunks = 5;

struct Carve {
  size_t ctrl, tile_start, partial, folded, tile_counts, tile_base, tie_base, group_counts, seg_groups,
      norm_partial, hist, tile_hist, total;
  size_t list, run_table, list_stats;  // with lists only
  size_t run_entries;
  uint32_t max_groups;
};
Carve carve(int64_t d_total, int32_t L, bool lists = false) {
  const size_t mt = max_tiles_of(d_total, L, 1);
  Carve c;
  size_t off = 0;
  c.ctrl = off;        off = align_up(off + sizeof(SegCtrl) * (size_t)L);
  c.tile_start = off;  off = align_up(off + sizeof(uint32_t) * ((size_t)L + 1));
  c.partial = off;     off = align_up(off + sizeof(double) * 3 * mt);
  c.folded = off;      off = align_up(off + sizeof(double) * 3 * kMaxMomentParts);
  c.tile_counts = off; off = align_up(off + sizeof(uint32_t) * kNumThres * mt);
  c.tile_base = off;   off = align_up(off + sizeof(uint32_t) * mt);
  c.tie_base = off;    off = align_up(off + sizeof(uint32_t) * mt);
  c.group_counts = off; off = align_up(off + sizeof(uint32_t) * kBigMaxGroups * kNumThres);
  // a segment's tiles are totalled in groups of 64 of its own: at most tiles/64 + one per segment
  c.max_groups = (uint32_t)(mt / kGroupTiles + (size_t)L + 1);
  c.seg_groups = off;  off = align_up(off + sizeof(uint32_t) * kNumThres * (size_t)c.max_groups);
  c.norm_partial = off; off = align_up(off + sizeof(double) * 2 * mt);
  size_t hist_words = (size_t)kDigits * 256 * (size_t)L * hist_copies_of(d_total, L);  // [pass][segment][replica]
  if (hist_words < (size_t)kDgcHistWords) hist_words = kDgcHistWords;  // per-pass buffers (flat): 4 or 8
  c.hist = off;        off = align_up(off + sizeof(uint32_t) * hist_words);
  // per-tile histograms of the last digit: flat Top_k in place, at most kFusedMaxTiles tiles
  const size_t hist_tiles = mt < (size_t)kFusedMaxTiles ? mt : (size_t)kFusedMaxTiles;
  c.tile_hist = off;   off = align_up(off + sizeof(uint32_t) * kLastDigitBins * hist_tiles);
  c.list = c.run_table = c.list_stats = 0;
  c.run_entries = 0;
  if (lists) {  // appended, so that the layout above does not depend on them
    // one record per 256-element run of every chunk of every tile: the vector's chunks plus, per
    // segment, the ragged head and tail tiles at the default tile length
    const size_t chunks = (size_t)((d_total + kChunk - 1) / kChunk);
    // (or at the tile length that layer-wise Top_k prefers with its lists)
    size_t tc_most = tile_chunks_of(d_total, false);
    if (tc_most < kSegTopkListTileChunks) tc_most = kSegTopkListTileChunks;
    c.run_entries = (chunks + tc_most * (2 * (size_t)L + 1)) * kRunsPerChunk;
    c.list_stats = off;  off = align_up(off + sizeof(uint32_t) * 2 * kListStatCopies);
    c.run_table = off;   off = align_up(off + sizeof(uint2) * c.run_entries);
    c.list = off;        off = align_up(off + sizeof(uint2) * list_entries(d_total));
  }
  c.total = off;
  return c;
}

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

struct Range {
  uintptr_t b, e;
};
Range range_of(const void* p, size_t bytes) {
  return Range{reinterpret_cast<uintptr_t>(p), reinterpret_cast<uintptr_t>(p) + bytes};
}
bool overlap(Range x, Range y) { return x.b < y.e && y.b < x.e; }

// Common checks of the buffers; fills the workspace pointers of `a`.
int prepare(Args& a, int32_t L, int64_t d_total, const float* grad, float* residual, float* acc,
            uint32_t* out_idx, float* out_val, int64_t out_cap, sparsify_result* result,
            void* workspace, size_t workspace_bytes, const sparsify_opts* opts) {
  if (L < 1 || L > (1 << 20) || d_total < 1 || d_total >= (int64_t(1) << 31)) return SPARSIFY_E_INVALID;
  if (!grad || !residual || !acc || !out_idx || !out_val || !result || out_cap < 1)
    return SPARSIFY_E_INVALID;
  if (misaligned(grad, 16) || misaligned(residual, 16) || misaligned(acc, 16) ||
      misaligned(out_idx, 16) || misaligned(out_val, 16) || misaligned(result, 8))
    return SPARSIFY_E_INVALID;
  double tail_div = 2.0;
  int32_t ddof = 1;
  if (opts) {
    tail_div = opts->tail_div;
    ddof = opts->ddof;
    if (!(tail_div >= 1.0) || !(tail_div <= 1e300) || (ddof != 0 && ddof != 1))
      return SPARSIFY_E_INVALID;
  }
  Carve cv = carve(d_total, L);
  if (!workspace || misaligned(workspace, kAlign) || workspace_bytes < cv.total)
    return SPARSIFY_E_WORKSPACE;
  bool lists = false;
  if (list_sized(d_total, L)) {  // the larger layout extends the smaller one
    const Carve big = carve(d_total, L, true);
    if (workspace_bytes >= big.total) {
      cv = big;
      lists = true;
    }
  }

  const size_t vec = sizeof(float) * (size_t)d_total;
  const Range rg = range_of(grad, vec), rr = range_of(residual, vec), ra = range_of(acc, vec);
  const Range ri = range_of(out_idx, 4 * (size_t)out_cap), rv = range_of(out_val, 4 * (size_t)out_cap);
  const Range rs = range_of(result, sizeof(sparsify_result) * (size_t)L);
  const Range rw = range_of(workspace, cv.total);
  const bool inplace = (acc == residual);
  const Range all[] = {rg, rr, ra, ri, rv, rs, rw};
  for (int i = 0; i < 7; ++i)
    for (int j = i + 1; j < 7; ++j) {
      if (inplace && i == 1 && j == 2) continue;
      if (overlap(all[i], all[j])) return SPARSIFY_E_INVALID;
    }

  char* w = static_cast<char*>(workspace);
  std::memset(&a, 0, sizeof(a));
  a.L = L;
  a.inplace = inplace ? 1 : 0;
  a.d_total = d_total;
  a.out_cap = out_cap;
  a.grad = grad;
  a.resid = residual;
  a.acc = acc;
  a.out_idx = out_idx;
  a.out_val = out_val;
  a.result = result;
  a.ctrl = reinterpret_cast<SegCtrl*>(w + cv.ctrl);
  a.tile_start = reinterpret_cast<uint32_t*>(w + cv.tile_start);
  a.partial = reinterpret_cast<double*>(w + cv.partial);
  a.folded = reinterpret_cast<double*>(w + cv.folded);
  a.tile_counts = reinterpret_cast<uint32_t*>(w + cv.tile_counts);
  a.tile_base = reinterpret_cast<uint32_t*>(w + cv.tile_base);
  a.tie_base = reinterpret_cast<uint32_t*>(w + cv.tie_base);
  a.group_counts = reinterpret_cast<uint32_t*>(w + cv.group_counts);
  a.seg_groups = reinterpret_cast<uint32_t*>(w + cv.seg_groups);
  a.max_groups = cv.max_groups;
  a.norm_partial = reinterpret_cast<double*>(w + cv.norm_partial);
  a.norms = (opts && opts->error_norms) ? 1 : 0;
  a.hist = reinterpret_cast<uint32_t*>(w + cv.hist);
  a.tile_hist = reinterpret_cast<uint32_t*>(w + cv.tile_hist);
  a.hist_copies = hist_copies_of(d_total, L);
  if (lists) {
    a.list = reinterpret_cast<uint2*>(w + cv.list);
    a.run_table = reinterpret_cast<uint2*>(w + cv.run_table);
    a.list_stats = reinterpret_cast<uint32_t*>(w + cv.list_stats);
    a.run_cap = (uint32_t)cv.run_entries;
  }
  a.tile_chunks = tile_chunks_of(d_total, false);
  if (opts && opts->tile_chunks != 0) {
    if (opts->tile_chunks < 0 || opts->tile_chunks > (1 << 20)) return SPARSIFY_E_INVALID;
    a.tile_chunks = (uint32_t)opts->tile_chunks;
  }
  a.max_tiles = max_tiles_of(d_total, L, 1);
  a.ddof = ddof;
  a.tail_div = tail_div;
  return SPARSIFY_OK;
}

// Compute units of the current device (cached; a conservative figure if the runtime cannot tell).
uint32_t compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return 256;
  return (uint32_t)cus;
}

// Whether the compaction kernels read acc with the non-temporal hint (it is acc's last use in the
// call).  It pays where one vector still fits the last-level cache (256 MB) but the call's three
// do not: acc then no longer displaces the new residual, which the next call's accumulate kernel
// reads first.  Measured over chains of calls: 8 % faster per call at 42 M elements, 7 % at 50 M,
// 1 % at 67 M; no difference at 25.6 M and 33.5 M; 2 % slower at 100 M.
// In the same range the Gaussian_k accumulate kernel (separate acc) stores acc with that hint:
// the count kernel then finds less of acc in the cache and slows down, the accumulate kernel gains
// more (per call: 2 % faster at 50 M elements, 4 % at 59 M, 5 % at 66 M; no difference at 42 M;
// 3-5 % slower at 84 M and 100 M, and slightly slower at 25.6 M, where it is not used).
// With lists a workgroup of the compact kernel takes this many tiles (a divisor of the group
// size): the tables every workgroup reads are then read a fraction as often, and a wave writes
// one or two tiles' pairs.  Measured (kernel, event to event): 25.6 M elements 12.3 us with one
// tile, 10.0 with two or four, 11.8 with eight, 15.1 with sixteen; 66 M elements 17.2 / 14.8 /
// 18.1 us with two / four / eight; 268 M elements (the larger tables) 87 us with one, 64 with
// two, 36 with eight or sixteen.
constexpr uint32_t kListCompactTiles = 4, kBigListCompactTiles = 8;
static_assert(kGroupTiles % kListCompactTiles == 0 && kBigGroupTiles % kBigListCompactTiles == 0, "a workgroup's tiles share a group");
constexpr int64_t kStreamAccFrom = 40'000'000, kStreamAccBelow = 80'000'000;
bool stream_acc(const Args& a) { return a.d_total >= kStreamAccFrom && a.d_total < kStreamAccBelow; }
// Gaussian_k with lists reads acc once (the count kernel) and the hints pay from a shorter
// vector on: per call 4.5 % faster at 33.5 M elements, no difference at 30 M and below.
constexpr int64_t kStreamAccListFrom = 32'000'000;

// Layer-wise Gaussian_k: three launches for up to 256 segments, setup + three beyond (gaussiank_seg.h).
void launch_gaussiank_seg(Launcher& ln, const Args& a, uint32_t tiles) {
  const dim3 blk(kBlock);
  if (a.L <= kBlock) {  // the accumulate kernel's workgroups find their segments themselves
    ln.run("accum_moments", k_accum_moments_seg_setup, dim3(tiles + 1), blk, a);
  } else {
    ln.run("seg_setup", k_seg_setup, dim3(1), blk, a, 1);
    ln.run("accum_moments", k_accum_moments_seg, dim3(tiles), blk, a);
  }
  ln.run("gk_count", k_gk_count_seg, dim3(tiles), blk, a);
  if (a.norms) {
    ln.run("gk_compact", k_gk_compact_seg<true>, dim3(tiles), blk, a);
    ln.run("norms", k_norms_finalize<true>, dim3(a.L), dim3(kFinBlock), a);
  } else {
    ln.run("gk_compact", k_gk_compact_seg<false>, dim3(tiles), blk, a);
  }
}

// Flat Gaussian_k: three launches (gaussiank_flat.h), four for long vectors.
void launch_gaussiank_flat(Launcher& ln, Args& a, uint32_t tiles) {
  const dim3 blk(kBlock);
  // The streaming grid of the accumulate kernel: one workgroup per compute unit (measured on 256
  // CUs: 256 workgroups beat 512 and 1024 by about 1.5 % end to end, and the count kernel's
  // prologue has fewer partials to merge; 128 or 384 are clearly worse).
  static const uint32_t cus = compute_units();
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  uint32_t want = cus < (uint32_t)kMaxMomentParts ? cus : (uint32_t)kMaxMomentParts;
  if (want > nchunks) want = nchunks;
  if (want > a.max_tiles) want = a.max_tiles;
  if (want < 1) want = 1;
  a.moment_parts = want;
  a.compact_tiles = 1;
  a.flat_tiles = tiles;
  if (a.list) {  // gaussiank_list.h: a stretch of the list buffer per wave of the count kernel
    a.list_cap = (uint32_t)(list_entries(a.d_total) / ((size_t)tiles * kWaves));
    a.list_last = (uint32_t)(list_entries(a.d_total) - 1);
    a.compact_tiles = nchunks > kChunkGridFrom ? kBigListCompactTiles : kListCompactTiles;
  }
  const dim3 cgrid((tiles + a.compact_tiles - 1) / a.compact_tiles);
  if (nchunks > kChunkGridFrom) {  // (flat_call has checked that the group tables hold `tiles`)
    // long vector: one chunk per workgroup and a fold of the partials, then short tiles in
    // groups of kBigGroupTiles
    a.moment_parts = nchunks < (uint32_t)kMaxMomentParts ? nchunks : (uint32_t)kMaxMomentParts;
    a.use_folded = 1;
    ln.run("accum_moments", k_accum_moments_chunks, dim3(nchunks + 1), blk, a);
    ln.run("fold_moments", k_fold_moments, dim3(a.moment_parts), blk, a);
    ln.run("gk_count", k_gk_count_fused<kBigGroupTiles>, dim3(tiles), blk, a);
    if (a.norms) {
      ln.run("gk_compact", k_gk_compact_fused<true, kBigGroupTiles, kBigMaxGroups, false>, cgrid, blk, a);
      ln.run("norms", k_norms_finalize<false>, dim3(1), dim3(kFinBlock), a);
    } else {
      ln.run("gk_compact", k_gk_compact_fused<false, kBigGroupTiles, kBigMaxGroups, false>, cgrid, blk, a);
    }
    return;
  }
  {
    // (with lists, acc is stored with the hint from 32 M elements up to the 123 M this branch
    // serves: per call 11 % faster at 80 M elements, 6 % at 90 M, 1 % from 100 M to 120 M)
    const bool nt_store = (stream_acc(a) || (a.list && a.d_total >= kStreamAccListFrom)) && !a.inplace;
    if (nt_store) ln.run("accum_moments", k_accum_moments_fused<true>, dim3(want + 1), blk, a);
    else ln.run("accum_moments", k_accum_moments_fused<false>, dim3(want + 1), blk, a);
    // with lists the count kernel is acc's last reader: from 32 M elements (up to the 123 M this
    // branch serves) it reads acc with the non-temporal hint (per call: 11 % faster at 66 M
    // elements, 2 % at 100 M, no difference at 85 M; slower beyond 123 M)
    if (a.list && a.d_total >= kStreamAccListFrom) ln.run("gk_count", k_gk_count_fused<kGroupTiles, true>, dim3(tiles), blk, a);
    else ln.run("gk_count", k_gk_count_fused<kGroupTiles>, dim3(tiles), blk, a);
    if (a.norms) {
      if (stream_acc(a)) ln.run("gk_compact", k_gk_compact_fused<true, kGroupTiles, kMaxGroups, true>, cgrid, blk, a);
      else ln.run("gk_compact", k_gk_compact_fused<true, kGroupTiles, kMaxGroups, false>, cgrid, blk, a);
      ln.run("norms", k_norms_finalize<false>, dim3(1), dim3(kFinBlock), a);
    } else {
      if (stream_acc(a)) ln.run("gk_compact", k_gk_compact_fused<false, kGroupTiles, kMaxGroups, true>, cgrid, blk, a);
      else ln.run("gk_compact", k_gk_compact_fused<false, kGroupTiles, kMaxGroups, false>, cgrid, blk, a);
    }
  }
}

void launch_topk_flat_rest(Launcher& ln, const Args& a, uint32_t tiles, uint32_t nchunks, uint32_t resident);

// Flat Top_k.  Separate acc: seven launches with candidate filtering (topk_filter.h); in place:
// seven launches with three more digit passes over acc (topk_flat.h).  flat_call has checked
// that the group tables hold `tiles`.
void launch_topk_flat(Launcher& ln, const Args& a, uint32_t tiles) {
  const dim3 blk(kBlock);
  const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
  static const uint32_t cus = compute_units();
  const uint32_t resident = cus < nchunks ? cus : nchunks;
  Args al = a;  // short-list form (topk_list.h): the first two launches differ, the rest is shared
  if (a.list) {
    // (the resident grid at every length: one chunk per workgroup in dispatch order, which the
    // accumulate kernels without lists use beyond 123 M elements, measured 6 % slower here)
    al.list_cap = (uint32_t)(list_entries(a.d_total) / ((size_t)resident * kWaves));
    al.list_last = (uint32_t)(list_entries(a.d_total) - 1);
    ln.run("topk_init", k_topk_init_list, dim3(32), blk, al, (uint32_t)kTopkHistWords);
    ln.run("topk_accum_hist", k_topk_accum_list<false>, dim3(resident), blk, al);
  }
  launch_topk_flat_rest(ln, al, tiles, nchunks, resident);
}
void launch_topk_flat_rest(Launcher& ln, const Args& a, uint32_t tiles, uint32_t nchunks, uint32_t resident) {
  const dim3 blk(kBlock);
  const dim3 pg(tiles);
  if (!a.inplace) {
    const bool big = nchunks > kChunkGridFrom;  // long vector: larger group tables
    // one wave per tile's candidate list, several lists per wave when there are many tiles
    uint32_t lists = (tiles + kWaves - 1) / kWaves;
    if (lists > 4096) lists = 4096;
    const dim3 cg(lists);
    if (!a.list) {
      ln.run("topk_init", k_topk_init_fused, dim3(32), blk, a, (uint32_t)kTopkHistWords);
      if (big) ln.run("topk_accum_hist", k_topk_accum_hist_chunks, dim3(nchunks), blk, a);
      else ln.run("topk_accum_hist", k_topk_accum_hist_resident, dim3(resident), blk, a);
    }
    ln.run("topk_filter", k_topk_filter, pg, blk, a);
    ln.run("topk_cand2", k_topk_cand_hist, cg, blk, a, 2);
    ln.run("topk_cand3", k_topk_cand_hist, cg, blk, a, 3);
    if (big) {
      ln.run("topk_final", k_topk_cand_final<kBigGroupTiles>, cg, blk, a);
      if (a.norms) ln.run("topk_compact", k_topk_compact_ordered<true, kBigGroupTiles, kBigMaxGroups, false>, pg, blk, a);
      else ln.run("topk_compact", k_topk_compact_ordered<false, kBigGroupTiles, kBigMaxGroups, false>, pg, blk, a);
    } else {
      ln.run("topk_final", k_topk_cand_final<kGroupTiles>, cg, blk, a);
      if (a.norms) ln.run("topk_compact", k_topk_compact_ordered<true, kGroupTiles, kMaxGroups, false>, pg, blk, a);
      else if (stream_acc(a)) ln.run("topk_compact", k_topk_compact_ordered<false, kGroupTiles, kMaxGroups, true>, pg, blk, a);
      else ln.run("topk_compact", k_topk_compact_ordered<false, kGroupTiles, kMaxGroups, false>, pg, blk, a);
    }
  } else {
    if (!a.list) {
      ln.run("topk_init", k_topk_init_fused, dim3(32), blk, a, (uint32_t)kTopkHistWords);
      ln.run("topk_accum_hist", k_topk_accum_hist_resident, dim3(resident), blk, a);
    }
    ln.run("topk_hist1", k_topk_hist_fused<false>, pg, blk, a, 1);
    ln.run("topk_hist2", k_topk_hist_fused<false>, pg, blk, a, 2);
    ln.run("topk_hist3", k_topk_hist_fused<true>, pg, blk, a, 3);
    ln.run("topk_ties", k_topk_ties_fused, dim3((tiles + kWaves - 1) / kWaves), blk, a);
    if (a.norms) ln.run("topk_compact", k_topk_compact_ordered<true, kGroupTiles, kMaxGroups, false>, pg, blk, a);
    else ln.run("topk_compact", k_topk_compact_ordered<false, kGroupTiles, kMaxGroups, false>, pg, blk, a);
  }
  if (a.norms) ln.run("norms", k_norms_finalize<false>, dim3(1), dim3(kFinBlock), a);
}

// Layer-wise Top_k (after k_seg_setup).  Separate acc: six launches with candidate filtering
// (topk_seg.h); in place: twelve launches, a single-workgroup digit choice per segment after
// every pass (topk.h).
void launch_topk_seg(Launcher& ln, const Args& a, uint32_t tiles) {
  const dim3 blk(kBlock);
  const dim3 pg(tiles);
  if (!a.inplace) {
    if (a.list) ln.run("topk_accum_hist", k_topk_accum_list_seg, pg, blk, a);
    else ln.run("topk_accum_hist", k_topk_accum_hist, pg, blk, a);
    ln.run("topk_filter", k_topk_filter_seg, pg, blk, a);
    ln.run("topk_cand2", k_topk_cand_hist_seg, pg, blk, a, 2);
    ln.run("topk_cand3", k_topk_cand_hist_seg, pg, blk, a, 3);
    ln.run("topk_final", k_topk_cand_final_seg, pg, blk, a);
    if (a.norms) ln.run("topk_compact", k_topk_compact_ordered_seg<true>, pg, blk, a);
    else ln.run("topk_compact", k_topk_compact_ordered_seg<false>, pg, blk, a);
  } else {
    const dim3 fin(kFinBlock);
    ln.run("topk_accum_hist", k_topk_accum_hist, pg, blk, a);
    ln.run("topk_select0", k_topk_select, dim3(a.L), fin, a, 0);
    ln.run("topk_hist1", k_topk_hist<false>, pg, blk, a, 1);
    ln.run("topk_select1", k_topk_select, dim3(a.L), fin, a, 1);
    ln.run("topk_hist2", k_topk_hist<false>, pg, blk, a, 2);
    ln.run("topk_select2", k_topk_select, dim3(a.L), fin, a, 2);
    ln.run("topk_hist3", k_topk_hist<true>, pg, blk, a, 3);
    ln.run("topk_select3", k_topk_select, dim3(a.L), fin, a, 3);
    ln.run("topk_tie_count", k_topk_tie_count, dim3(tiles), blk, a);
    ln.run("topk_tie_scan", k_topk_tie_scan, dim3(a.L), fin, a);
    if (a.norms) ln.run("topk_compact", k_topk_compact<true>, dim3(tiles), blk, a);
    else ln.run("topk_compact", k_topk_compact<false>, dim3(tiles), blk, a);
  }
  if (a.norms) ln.run("norms", k_norms_finalize<true>, dim3(a.L), dim3(kFinBlock), a);
}

// DGC_k: eleven launches; twelve with the lists, where the sample comes first and the accumulate
// pass already knows the sample's threshold (dgck.h).
void launch_dgck(Launcher& ln, const Args& a0, uint32_t tiles) {
  const dim3 blk(kBlock), pg(tiles), cg((tiles + kWaves - 1) / kWaves);
  Args a = a0;
  ln.run("dgck_init", k_topk_init_fused, dim3(64), blk, a, (uint32_t)kDgcHistWords);
  if (a.list) {
    const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
    static const uint32_t cus = compute_units();
    const uint32_t resident = cus < nchunks ? cus : nchunks;
    a.list_cap = (uint32_t)(list_entries(a.d_total) / ((size_t)resident * kWaves));
    a.list_last = (uint32_t)(list_entries(a.d_total) - 1);
    const int64_t per_wg = (int64_t)kBlock * kSampleBatch;
    ln.run("dgck_sample", k_dgck_sample, dim3((uint32_t)((a.sample_m + per_wg - 1) / per_wg)), blk, a);
  } else {
    ln.run("dgck_accum_sample", k_dgck_accum_sample, pg, blk, a);
  }
  ln.run("dgck_sample1", k_dgck_lists_hist, cg, blk, a, 1);
  ln.run("dgck_sample2", k_dgck_lists_hist, cg, blk, a, 2);
  ln.run("dgck_sample3", k_dgck_lists_hist, cg, blk, a, 3);
  if (a.list) {
    const uint32_t nchunks = (uint32_t)((a.d_total + kChunk - 1) / kChunk);
    static const uint32_t cus = compute_units();
    ln.run("dgck_accum_list", k_topk_accum_list<true>, dim3(cus < nchunks ? cus : nchunks), blk, a);
  }
  ln.run("dgck_filter", k_dgck_filter, pg, blk, a);
  ln.run("dgck_kept1", k_dgck_lists_hist, cg, blk, a, 5);
  ln.run("dgck_kept2", k_dgck_lists_hist, cg, blk, a, 6);
  ln.run("dgck_kept3", k_dgck_lists_hist, cg, blk, a, 7);
  ln.run("dgck_final", k_dgck_final, cg, blk, a);
  if (a.norms) {
    ln.run("dgck_compact", k_topk_compact_ordered<true, kGroupTiles, kMaxGroups, false>, pg, blk, a);
    ln.run("norms", k_norms_finalize<false>, dim3(1), dim3(kFinBlock), a);
  } else {
    if (stream_acc(a)) ln.run("dgck_compact", k_topk_compact_ordered<false, kGroupTiles, kMaxGroups, true>, pg, blk, a);
    else ln.run("dgck_compact", k_topk_compact_ordered<false, kGroupTiles, kMaxGroups, false>, pg, blk, a);
  }
}

enum { kSelGaussian = 0, kSelTopk = 1, kSelDgc = 2 };

// Device address of this device's copy of `scratch`, looked up on the first call made with that
// device current and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPARSIFY_E_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SPARSIFY_E_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SPARSIFY_OK;
}

int flat_call(int selector, int64_t d, int64_t k, const float* grad, float* residual, float* acc,
              uint32_t* out_idx, float* out_val, int64_t cap, sparsify_result* result,
              void* workspace, size_t workspace_bytes, const sparsify_opts* opts, void* stream) {
  if (k < 1 || k > d) return SPARSIFY_E_INVALID;
  if (selector != kSelGaussian && cap < k) return SPARSIFY_E_INVALID;
  Args a;
  const int rc = prepare(a, 1, d, grad, residual, acc, out_idx, out_val, cap, result, workspace,
                         workspace_bytes, opts);
  if (rc != SPARSIFY_OK) return rc;
  a.flat_k = k;
  a.flat_cap = cap;
  // the short-list forms: no norms asked for, k small enough for the lists' share of the
  // workspace, where the workspace has room at all (prepare)
  // (Top_k's and DGC_k's lists are built to hold about four times k entries, Gaussian_k's about k)
  const double list_need = selector == kSelGaussian ? 2.0 * (double)k : 2.0 * kListAim * (double)k;
  if (a.norms || (opts && opts->short_list < 0) || list_need > kListShare * (double)d) a.list = nullptr;
  if (!(opts && opts->tile_chunks != 0))
    a.tile_chunks = tile_chunks_of(d, selector == kSelGaussian || (selector == kSelTopk && !a.inplace));
  const uint32_t tiles = seg_ntiles(0, d, a.tile_chunks);
  if (selector == kSelGaussian || selector == kSelTopk) {
    // a forced tile length must leave no more tiles than the group tables hold (the larger
    // tables serve long vectors, except Top_k in place)
    const bool big = (d + kChunk - 1) / kChunk > (int64_t)kChunkGridFrom &&
                     !(selector == kSelTopk && a.inplace);
    if (tiles > (uint32_t)(big ? kBigMaxTiles : kFusedMaxTiles)) return SPARSIFY_E_INVALID;
  }
  if (selector == kSelDgc) {
    // the per-tile key lists live in the residual buffer and the list kernels use one lane per
    // group of tiles: separate acc and at most kFusedMaxTiles tiles
    if (a.inplace || tiles > (uint32_t)kFusedMaxTiles) return SPARSIFY_E_INVALID;
    int64_t S = 100;
    if (opts && opts->sample_stride != 0) S = opts->sample_stride;
    if (S < 1) return SPARSIFY_E_INVALID;
    a.sample_stride = S;
    a.sample_m = (d + S - 1) / S;
    a.sample_k = (k * a.sample_m + d - 1) / d;
    a.sample_seed = opts ? opts->sample_seed : 0;
    // (the sample's keys wait in the list buffer until the accumulate pass overwrites it)
    if ((size_t)a.sample_m > list_entries(d)) a.list = nullptr;
  }
  Launcher ln{static_cast<hipStream_t>(stream),
              opts ? static_cast<sparsify_trace*>(opts->trace) : nullptr};
  ln.begin();
  if (selector == kSelGaussian) {
    launch_gaussiank_flat(ln, a, tiles);
  } else if (selector == kSelTopk) {
    launch_topk_flat(ln, a, tiles);
  } else {
    launch_dgck(ln, a, tiles);
  }
  if (ln.tr) ln.tr->ok = (ln.err == hipSuccess);
  return ln.err == hipSuccess ? SPARSIFY_OK : SPARSIFY_E_LAUNCH;
}

}  // namespace

extern "C" {

const char* sparsify_version(void) { return "sparsify 0.1 (gfx950)"; }

size_t sparsify_workspace_bytes_min(int64_t d_total, int32_t num_segments) {
  if (d_total < 1 || d_total >= (int64_t(1) << 31) || num_segments < 1 || num_segments > (1 << 20))
    return 0;
  return carve(d_total, num_segments).total;
}

size_t sparsify_workspace_bytes(int64_t d_total, int32_t num_segments) {
  if (d_total < 1 || d_total >= (int64_t(1) << 31) || num_segments < 1 || num_segments > (1 << 20))
    return 0;
  return carve(d_total, num_segments, list_sized(d_total, num_segments)).total;
}

int sparsify_gaussiank(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                       uint32_t* out_idx, float* out_val, int64_t cap, sparsify_result* result,
                       void* workspace, size_t workspace_bytes, const sparsify_opts* opts,
                       void* stream) {
  return flat_call(kSelGaussian, d, k, grad, residual, acc, out_idx, out_val, cap, result, workspace,
                   workspace_bytes, opts, stream);
}

int sparsify_gaussiank_static(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                              uint32_t* out_idx, float* out_val, int64_t cap,
                              sparsify_result* result, const sparsify_opts* opts, void* stream) {
  if (d > kStaticMaxD) return SPARSIFY_E_WORKSPACE;  // beyond what the built-in workspace holds
  if (d < 1 || k < 1 || k > d) return SPARSIFY_E_INVALID;
  static_assert(kStaticScratchBytes % 256 == 0, "the workspace is carved in 256-byte units");
  if (carve(d, 1).total > kStaticScratchBytes) return SPARSIFY_E_WORKSPACE;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != SPARSIFY_OK) return rc;
  return flat_call(kSelGaussian, d, k, grad, residual, acc, out_idx, out_val, cap, result, ws,
                   kStaticScratchBytes, opts, stream);
}

int sparsify_topk(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                  uint32_t* out_idx, float* out_val, int64_t cap, sparsify_result* result,
                  void* workspace, size_t workspace_bytes, const sparsify_opts* opts,
                  void* stream) {
  return flat_call(kSelTopk, d, k, grad, residual, acc, out_idx, out_val, cap, result, workspace,
                   workspace_bytes, opts, stream);
}

int sparsify_dgck(int64_t d, int64_t k, const float* grad, float* residual, float* acc,
                  uint32_t* out_idx, float* out_val, int64_t cap, sparsify_result* result,
                  void* workspace, size_t workspace_bytes, const sparsify_opts* opts,
                  void* stream) {
  return flat_call(kSelDgc, d, k, grad, residual, acc, out_idx, out_val, cap, result, workspace,
                   workspace_bytes, opts, stream);
}

int sparsify_segmented(int32_t num_segments, int64_t d_total, const int64_t* seg_off,
                       const int64_t* seg_k, int32_t mode, const float* grad, float* residual,
                       float* acc, uint32_t* out_idx, float* out_val, const int64_t* out_off,
                       int64_t out_cap, sparsify_result* results, void* workspace,
                       size_t workspace_bytes, const sparsify_opts* opts, void* stream) {
  if ((mode != 0 && mode != 1) || !seg_off || !seg_k || !out_off) return SPARSIFY_E_INVALID;
  if (misaligned(seg_off, 8) || misaligned(seg_k, 8) || misaligned(out_off, 8))
    return SPARSIFY_E_INVALID;
  Args a;
  const int rc = prepare(a, num_segments, d_total, grad, residual, acc, out_idx, out_val, out_cap,
                         results, workspace, workspace_bytes, opts);
  if (rc != SPARSIFY_OK) return rc;
  a.seg_off = seg_off;
  a.seg_k = seg_k;
  a.out_off = out_off;
  if (mode == 0 && a.list && !a.inplace && !a.norms && !(opts && (opts->short_list < 0 || opts->tile_chunks != 0)) &&
      a.tile_chunks < kSegTopkListTileChunks)
    a.tile_chunks = kSegTopkListTileChunks;
  // upper bound of the tile count for this tiling; surplus workgroups exit at once
  const uint32_t tiles = max_tiles_of(d_total, num_segments, a.tile_chunks);
  // short lists (gaussiank_seg.h; topk_seg.h, with a separate acc): without the norms, where the
  // workspace has room (prepare) and the run table holds this tiling's runs
  if ((mode == 0 && a.inplace) || a.norms || (opts && opts->short_list < 0) ||
      (uint64_t)tiles * a.tile_chunks * kRunsPerChunk > (uint64_t)a.run_cap)
    a.list = nullptr;
  if (a.list) {
    a.list_cap = (uint32_t)(list_entries(d_total) / ((size_t)tiles * kWaves));
    a.list_last = (uint32_t)(list_entries(d_total) - 1);
    if (a.list_cap < 1) a.list = nullptr;
  }
  Launcher ln{static_cast<hipStream_t>(stream),
              opts ? static_cast<sparsify_trace*>(opts->trace) : nullptr};
  ln.begin();
  if (mode == 1) {
    launch_gaussiank_seg(ln, a, tiles);
  } else {
    // the setup kernel's other workgroups clear the histograms ([pass][segment][replica][256]: at
    // most 2^30 words) and, with lists, sample the segments (topk_seg.h)
    const size_t n = (size_t)kDigits * 256 * (size_t)num_segments * a.hist_copies;
    const unsigned fill_wgs = (unsigned)((n + 1023) / 1024 < 1024 ? (n + 1023) / 1024 : 1024);
    const unsigned samplers = a.list ? (unsigned)num_segments : 0u;
    ln.run("seg_setup", k_topk_seg_setup, dim3(1 + samplers + fill_wgs), dim3(kBlock), a, (uint32_t)n, samplers);
    launch_topk_seg(ln, a, tiles);
  }
  if (ln.tr) ln.tr->ok = (ln.err == hipSuccess);
  return ln.err == hipSuccess ? SPARSIFY_OK : SPARSIFY_E_LAUNCH;
}

int sparsify_scatter_add(int64_t d, int32_t num_lists, const uint32_t* idx, const float* val,
                         int64_t list_stride, const uint32_t* nnz, int64_t nnz_stride_bytes,
                         float scale, float* dense, uint32_t* status, void* stream) {
  if (d < 1 || d >= (int64_t(1) << 31) || num_lists < 1 || num_lists > kScatterMaxLists ||
      list_stride < 1 || list_stride >= (int64_t(1) << 31))
    return SPARSIFY_E_INVALID;
  if (!idx || !val || !nnz || !dense || !status || nnz_stride_bytes < 4 || (nnz_stride_bytes & 3) != 0)
    return SPARSIFY_E_INVALID;
  if (misaligned(idx, 4) || misaligned(val, 4) || misaligned(nnz, 4) || misaligned(status, 4) ||
      misaligned(dense, 16))
    return SPARSIFY_E_INVALID;
  const size_t pairs = (size_t)num_lists * (size_t)list_stride;
  const Range rd = range_of(dense, 4 * (size_t)d);
  const Range others[] = {range_of(idx, 4 * pairs), range_of(val, 4 * pairs),
                          range_of(nnz, (size_t)(num_lists - 1) * (size_t)nnz_stride_bytes + 4),
                          range_of(status, 4)};
  for (const Range& r : others)
    if (overlap(rd, r)) return SPARSIFY_E_INVALID;
  if (overlap(others[3], others[0]) || overlap(others[3], others[1]) || overlap(others[3], others[2]))
    return SPARSIFY_E_INVALID;

  ScatterArgs a;
  a.d = d;
  a.P = num_lists;
  a.idx = idx;
  a.val = val;
  a.stride = list_stride;
  a.nnz = nnz;
  a.nnz_step = nnz_stride_bytes / 4;
  a.scale = scale;
  a.dense = dense;
  a.status = status;
  // Spans of whole chunks.  Four chunks per span measured best at 25.6 M and 66 M elements (one
  // search per list per span, against 3 and 6 % more time with 3 and 8, 70 % more with 1); fewer
  // when the vector is short (at least about a thousand workgroups) or when the lists can be so
  // dense that a span's pairs would not fit one register round of 1024: their counts are on the
  // device, so the stride is what the host knows, and lists are taken to be a quarter full.
  const int64_t chunks = (d + kChunk - 1) / kChunk;
  int64_t span = 4;
  if (span > chunks / 1024) span = chunks / 1024;
  const int64_t by_density = d / ((int64_t)num_lists * list_stride);  // = 4096 pairs a span / 4096
  if (span > by_density) span = by_density;
  if (span < 1) span = 1;
  a.span_chunks = (uint32_t)span;
  a.nspans = (uint32_t)((chunks + span - 1) / span);
  hipStream_t st = static_cast<hipStream_t>(stream);
  k_scatter_add<<<dim3(kScatterCheckers + a.nspans), dim3(kBlock),
                  sizeof(uint32_t) * scatter_table_words(num_lists), st>>>(a);
  return hipGetLastError() == hipSuccess ? SPARSIFY_OK : SPARSIFY_E_LAUNCH;
}

int sparsify_calibration_copy(float* dst, const float* src, int64_t n, void* stream) {
  if (!dst || !src || n < 4 || (n & 3) != 0 || misaligned(dst, 16) || misaligned(src, 16))
    return SPARSIFY_E_INVALID;
  if (overlap(range_of(dst, 4 * (size_t)n), range_of(src, 4 * (size_t)n))) return SPARSIFY_E_INVALID;
  const size_t n4 = (size_t)n / 4;
  const size_t want = (n4 + kBlock - 1) / kBlock;
  k_calibration_copy<<<dim3((unsigned)(want < 65536 ? want : 65536)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream)>>>(dst, src, n4);
  return hipGetLastError() == hipSuccess ? SPARSIFY_OK : SPARSIFY_E_LAUNCH;
}

sparsify_trace* sparsify_trace_create(void) {
  sparsify_trace* t = new (std::nothrow) sparsify_trace();
  if (!t) return nullptr;
  t->n = 0;
  t->ok = false;
  for (int i = 0; i <= kMaxStages; ++i) {
    if (hipEventCreate(&t->ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(t->ev[j]);
      delete t;
      return nullptr;
    }
  }
  return t;
}

void sparsify_trace_destroy(sparsify_trace* t) {
  if (!t) return;
  for (int i = 0; i <= kMaxStages; ++i) (void)hipEventDestroy(t->ev[i]);
  delete t;
}

int32_t sparsify_trace_num_stages(const sparsify_trace* t) { return t ? t->n : 0; }

const char* sparsify_trace_stage_name(const sparsify_trace* t, int32_t i) {
  return (t && i >= 0 && i < t->n) ? t->name[i] : "";
}

int sparsify_trace_stage_ms(sparsify_trace* t, int32_t i, float* ms) {
  if (!t || !ms || i < 0 || i >= t->n || !t->ok) return SPARSIFY_E_INVALID;
  return hipEventElapsedTime(ms, t->ev[i], t->ev[i + 1]) == hipSuccess ? SPARSIFY_OK
                                                                       : SPARSIFY_E_INVALID;
}

}  // extern "C"
