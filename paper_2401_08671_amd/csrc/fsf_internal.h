// Internal declarations shared by the C-ABI layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <stdint.h>

#include "fsf.h"
#include "fsf_measure.h"

namespace fsf {

// Everything a kernel needs to know about one pass; passed by value to every launch.
struct Pass {
  int32_t n_q_heads, n_kv_heads, group;  // group = n_q_heads / n_kv_heads
  int32_t head_dim, block_size, window;
  float scale;
  int32_t dtype;
  int32_t n_seqs, max_blocks, n_tokens;
  const fsf_seq_desc* descs;    // device
  const int32_t* block_tables;  // device
};

// Index of the sequence that owns token row t (descriptors are sorted by q_offset).
__device__ __forceinline__ int find_seq(const fsf_seq_desc* descs, int n_seqs, int t) {
  int lo = 0, hi = n_seqs - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (descs[mid].q_offset <= t)
      lo = mid;
    else
      hi = mid - 1;
  }
  return lo;
}

// Load an int32 whose address is the same for every lane of the wave through the scalar
// cache.  Besides saving vector registers this keeps the load out of the vector-memory
// counter, whose in-order waits would otherwise serialise it with bulk K/V traffic in flight.
__device__ __forceinline__ int32_t load_uniform_i32(const int32_t* ptr) {
  const uint64_t a = reinterpret_cast<uint64_t>(ptr);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
  const auto* cp = reinterpret_cast<const __attribute__((address_space(4))) int32_t*>(
      (static_cast<uint64_t>(hi) << 32) | lo);
  return *cp;
}

// ---------------------------------------------------------------------------------------
// Matrix-core path (bf16/f16, head_dim 128, block_size 16 * 2^k, group <= 16).
//
// Work is cut on the device by a one-workgroup planning kernel; the host evaluates the
// same formulas on its copy of the descriptors to size the grids.
//   streaming sequences: generation rows (n_new == 1) and short prompt chunks, the 2..30-row
//     chunks and remainders that filling the token budget exactly produces (paper Sec. 3.2):
//     "items" = (sequence, slice of rows, run of about split_blocks cache blocks).  A slice is
//     as many consecutive rows as fit, with the query heads of one KV head, into the 16 columns
//     of a streaming unit (16 / group rows); a chunk of at most stream_max_slices slices streams
//   other prompt chunks: "tiles" = (sequence, kPrefillTileM consecutive rows)
// ---------------------------------------------------------------------------------------
constexpr int kHeadDim = 128;
constexpr int kPrefillTileM = 256;   // query rows per prefill workgroup (4 waves x 64 rows)
constexpr int kMaxDecodeItemsExtra = 8192;  // items beyond one per sequence (bounds the workspace)
constexpr int kStreamCols = 16;             // (row, query head) columns of a streaming unit
constexpr int kMaxStreamSlices = 16;        // upper limit of stream_max_slices
constexpr int kDefaultStreamSlices = 2;     // chunks of up to 2 slices stream by default
// Prompt-chunk tiles may have their key range cut into parts, one workgroup each, which store
// unnormalised partial results that a merge kernel combines.  Two cases (decided on the host
// from counts and step numbers, passed by value):
//   heavy tiles  a tile that alone would outlast the rest of the pass (a short remainder of a
//                prompt over its long cached prefix, next to the first chunk of the next
//                prompt; or any tile when there is less than one round of workgroups):
//                up to kMaxHeavyTiles of them, each with its own number of parts; started first
//   tail tiles   when the last round of workgroups is at most half full, the tiles of that
//                round (the lowest tile indices that are not heavy), the same number of parts
//                each; started last
// Workgroups are numbered (tile, part)-major: all parts of the heavy tiles, then the whole
// tiles by descending tile index (within a chunk: most keys first), then the tail tiles.
constexpr int kMaxHeavyTiles = 4;
constexpr int kMaxPrefillSplitUnits = 512;  // (tile, head, part) workgroups with partial results (bounds the workspace)
constexpr int kPrefillPartRowFloats = 136;  // a partial row: O 128 floats, m, l, padding to a multiple of 16 bytes
constexpr int kPrefillMinPartSteps = 8;     // no part is shorter than this many 64-key steps

// Visible key range of the row at position pos.
__host__ __device__ inline void visible_range(int pos, int window, int& lo, int& hi) {
  hi = pos;
  lo = (window > 0 && pos - window + 1 > 0) ? pos - window + 1 : 0;
}

// Number of items a generation row over nblk cache blocks is cut into: about split_blocks
// blocks each, but never so fine that an item holds fewer than min_item_blocks blocks
// (short items pay more for their start-up and merge than the better balance returns).
__host__ __device__ inline int decode_splits(int nblk, int split_blocks, int min_item_blocks) {
  const int want = (nblk + split_blocks - 1) / split_blocks;
  const int cap = nblk / min_item_blocks > 1 ? nblk / min_item_blocks : 1;
  return want < cap ? want : cap;
}

// Rows of a streaming sequence per unit, and the units ("slices") its rows take.
__host__ __device__ inline int stream_rows_per_slice(int group) { return kStreamCols / group; }
__host__ __device__ inline int stream_slices(int n_new, int group) {
  const int rps = stream_rows_per_slice(group);
  return (n_new + rps - 1) / rps;
}
// Does the sequence take the streaming kernel (else its rows are tiled for the matrix-core kernel)?
__host__ __device__ inline bool is_streaming(int n_new, int group, int max_slices) {
  return n_new == 1 || stream_slices(n_new, group) <= max_slices;
}

// What a sequence contributes: streaming items (slices x key cuts), prompt-chunk tiles, and
// partial-result rows (cuts x rows, for sequences whose keys are cut at all).  The key cuts are
// taken over the cache blocks that any row of the sequence sees; every slice uses the same cuts.
struct SeqWork {
  int dec_items, pre_tiles, cuts, prows;
};
__host__ __device__ inline SeqWork seq_work(int n_new, int n_cached, int window, int block_size, int group,
                                            int max_slices, int split_blocks, int min_item_blocks) {
  SeqWork w = {0, 0, 0, 0};
  if (is_streaming(n_new, group, max_slices)) {
    int lo, hi, tmp;
    visible_range(n_cached, window, lo, tmp);
    visible_range(n_cached + n_new - 1, window, tmp, hi);
    const int nblk = hi / block_size - lo / block_size + 1;
    w.cuts = decode_splits(nblk, split_blocks, min_item_blocks);
    w.dec_items = stream_slices(n_new, group) * w.cuts;
    w.prows = w.cuts > 1 ? w.cuts * n_new : 0;
  } else {
    w.pre_tiles = (n_new + kPrefillTileM - 1) / kPrefillTileM;
  }
  return w;
}

struct PrefillSplit {
  int32_t n_heavy;
  int32_t heavy_tile[kMaxHeavyTiles];   // tile indices, descending
  int32_t heavy_parts[kMaxHeavyTiles];  // >= 2 each
  int32_t tail_tiles;                   // how many of the lowest non-heavy tile indices are split
  int32_t tail_parts;                   // into this many parts each (>= 2 if tail_tiles > 0)
};

struct PrefillWork {
  int tile, part, n_parts;
  int slab;  // (tile, part) number in the partial-result buffer, -1 for an unsplit tile
};

__host__ __device__ inline int prefill_heavy_groups(const PrefillSplit& sp) {
  int n = 0;
  for (int k = 0; k < sp.n_heavy; ++k) n += sp.heavy_parts[k];
  return n;
}

// a-th lowest tile index that is not a heavy tile
__host__ __device__ inline int prefill_nth_plain_tile(int a, const PrefillSplit& sp) {
  int tile = a;
  for (int k = sp.n_heavy - 1; k >= 0; --k)  // ascending
    if (sp.heavy_tile[k] <= tile) ++tile;
  return tile;
}

// number of (tile, part) groups; workgroups = groups x query heads
__host__ __device__ inline int prefill_groups(int n_tiles, const PrefillSplit& sp) {
  return prefill_heavy_groups(sp) + (n_tiles - sp.n_heavy - sp.tail_tiles) + sp.tail_tiles * sp.tail_parts;
}

__host__ __device__ inline PrefillWork prefill_group_to_work(int g, int n_tiles, const PrefillSplit& sp) {
  PrefillWork w;
  const int heavy = prefill_heavy_groups(sp);
  if (g < heavy) {
    int k = 0, start = 0;
    while (g >= start + sp.heavy_parts[k]) start += sp.heavy_parts[k++];
    w.tile = sp.heavy_tile[k];
    w.part = g - start;
    w.n_parts = sp.heavy_parts[k];
    w.slab = g;
    return w;
  }
  g -= heavy;
  const int n_plain = n_tiles - sp.n_heavy;
  const int n_whole = n_plain - sp.tail_tiles;
  if (g < n_whole) {  // descending tile index among the plain tiles above the tail
    w.tile = prefill_nth_plain_tile(n_plain - 1 - g, sp);
    w.part = 0;
    w.n_parts = 1;
    w.slab = -1;
    return w;
  }
  g -= n_whole;
  const int a = sp.tail_tiles - 1 - g / sp.tail_parts;  // ascending ordinal of the tail tile
  w.tile = prefill_nth_plain_tile(a, sp);
  w.part = g % sp.tail_parts;
  w.n_parts = sp.tail_parts;
  w.slab = heavy + a * sp.tail_parts + w.part;
  return w;
}

// j-th split tile (heavy tiles first, then tail tiles ascending): its index, parts and first slab
__host__ __device__ inline PrefillWork prefill_split_tile(int j, const PrefillSplit& sp) {
  PrefillWork w;
  w.part = 0;
  if (j < sp.n_heavy) {
    w.tile = sp.heavy_tile[j];
    w.n_parts = sp.heavy_parts[j];
    w.slab = 0;
    for (int k = 0; k < j; ++k) w.slab += sp.heavy_parts[k];
  } else {
    const int a = j - sp.n_heavy;
    w.tile = prefill_nth_plain_tile(a, sp);
    w.n_parts = sp.tail_parts;
    w.slab = prefill_heavy_groups(sp) + a * sp.tail_parts;
  }
  return w;
}

// 64-key steps a prompt-chunk tile walks: rows [i0, i1) of a chunk with n_cached tokens before it
__host__ __device__ inline int prefill_tile_steps(int n_cached, int i0, int i1, int window) {
  int lo, hi, tmp;
  visible_range(n_cached + i0, window, lo, tmp);
  visible_range(n_cached + i1 - 1, window, tmp, hi);
  return (hi - (lo & ~63)) / 64 + 1;
}

// A streaming item as its units find it: one 32-byte record per launch slot, written by the
// planning kernel, so that a unit starts from one load instead of a chain of four dependent ones
// (launch slot -> item -> sequence -> descriptor and item offset), and a wave that walks several
// units can have the next record on its way while it works.
struct __attribute__((aligned(32))) UnitRec {
  int32_t seq;         // sequence index (block-table row)
  int32_t idx;         // the item's index among its sequence's items (slice-major)
  int32_t n_new, n_cached, q_offset;  // the sequence's descriptor
  int32_t prow_start;  // first partial-result row of the sequence (used when its keys are cut)
  int32_t pad[2];
};

struct FastPlan {
  int32_t* dec_item_start;  // [n_seqs + 1] exclusive prefix of streaming items per sequence
  int32_t* pre_tile_start;  // [n_seqs + 1] exclusive prefix of prefill tiles per sequence
  int32_t* dec_prow_start;  // [n_seqs + 1] exclusive prefix of partial-result rows per sequence
  UnitRec* dec_rec;         // [items]  what a streaming unit needs of its item, in launch order (items with
                            //          the most cache blocks first)
  int32_t* pre_tile_seq;    // [tiles]  sequence index of every prefill tile
  int32_t* split_rows;      // [n_split_rows, 2] (sequence, row) of every row whose keys were cut
  float* part_ml;           // [partial rows, n_q_heads, 2]   running max (log2 domain) and sum per cut
  float* part_acc;          // [partial rows, n_q_heads, 128] unnormalised outputs per cut
  float* pre_part;          // [slab, 256 rows, n_q_heads, 136] partial results of split tiles
  int32_t split_blocks;     // target cache blocks per streaming item
  int32_t min_item_blocks;  // no cut leaves an item with fewer blocks than this
  int32_t stream_max_slices;  // chunks of at most this many slices take the streaming kernel
  int32_t n_dec_items, n_pre_tiles, n_split_rows;  // host-side totals (grid sizes)
  PrefillSplit split;       // which prompt-chunk tiles are cut along their keys
  int32_t decode_hold;      // host side: streaming waves may hold finished rows back (see attn_decode_kernel in attn_fast.hip)
};

hipError_t launch_plan(const Pass& p, const FastPlan& f, hipStream_t stream);
// reserve_units > 0: the streaming kernel leaves that many compute units entirely empty (for
// prompt-chunk tiles running beside it on another stream); 0: it may use every wave slot
hipError_t launch_attn_decode(const Pass& p, const FastPlan& f, const void* q, const void* k_cache,
                              const void* v_cache, void* out, hipStream_t stream, int reserve_units = 0);
hipError_t launch_attn_merge(const Pass& p, const FastPlan& f, void* out, hipStream_t stream);
hipError_t launch_prefill_merge(const Pass& p, const FastPlan& f, void* out, hipStream_t stream);
// persistent_groups > 0: that many workgroups walk all tiles (the kernel occupies that many compute units)
hipError_t launch_attn_prefill(const Pass& p, const FastPlan& f, const void* q, const void* k_cache,
                               const void* v_cache, void* out, hipStream_t stream, int persistent_groups = 0);
// prompt-chunk tiles and generation-row items in ONE launch, so the two kinds of work overlap
hipError_t launch_attn_fused(const Pass& p, const FastPlan& f, const void* q, const void* k_cache,
                             const void* v_cache, void* out, hipStream_t stream);

// A kernel that uses more than 64 KB of dynamic LDS has to ask for it, once per device: called
// before every such launch, does the asking on the first call on each device.
template <auto Kernel>
inline hipError_t allow_lds_bytes(int bytes) {
  constexpr int kMaxDevices = 64;
  static std::atomic<bool> done[kMaxDevices];
  int dev = 0;
  if (const hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!done[dev].load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done[dev].store(true, std::memory_order_release);
  }
  return hipSuccess;
}

// Compute units of the current device (asked once; 256 if the runtime does not say).
inline int device_compute_units() {
  static const int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 1)
      cu = 256;
    return cu;
  }();
  return n;
}

// Optional per-kernel timing (see fsf_profile_enable): brackets a launch with HIP events.
struct PhaseTimer {
  PhaseTimer(int phase, hipStream_t stream);
  ~PhaseTimer();
  int phase_;
  hipStream_t stream_;
  hipEvent_t start_;
  bool on_;
};

hipError_t launch_kv_append(const Pass& p, const void* k_new, const void* v_new, void* k_cache,
                            void* v_cache, hipStream_t stream);
hipError_t launch_kv_append_rotary(const Pass& p, const void* k_new, const void* v_new, void* k_cache,
                                   void* v_cache, const float* cos_sin, hipStream_t stream);
hipError_t launch_rotary_q(const Pass& p, void* q, const float* cos_sin, hipStream_t stream);

// y[M, N] = x[M, K] . w[N, K]^T on the matrix cores (N % 256 == 0, K % 64 == 0, bf16 / f16).
// workspace (may be null): room for fp32 partial results where cutting k into parts pays.
hipError_t launch_linear(int dtype, const void* x, const void* w, void* y, int M, int N, int K, void* workspace,
                         size_t workspace_bytes, hipStream_t stream);
// parts k would be cut into with a workspace of that size (1: no cut, no workspace used)
int linear_splits(int M, int N, int K, int cus, size_t workspace_bytes);

hipError_t launch_attn_generic(const Pass& p, const void* q, const void* k_cache,
                               const void* v_cache, void* out, hipStream_t stream);

}  // namespace fsf
