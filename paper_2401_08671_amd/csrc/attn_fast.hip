// Kernels of the matrix-core attention path and their launchers.
//
// A Dynamic SplitFuse pass mixes prompt chunks (dense, matrix-core bound) with one-token
// generations (streaming, HBM bound) at a fixed token budget (paper Sec. 3.2).  Each kind of
// work gets its own launch with the workgroup shape that suits it: 256-thread tiles with
// 64 KB of LDS, two to a compute unit, for the chunks; for the streaming work one eight-wave
// workgroup per compute unit, a persistent grid that walks the (sequence, KV head, key range)
// units (a 64-thread kernel, one unit per workgroup, serves passes too small to fill the
// chip).  Both kernels fill the register file at two waves per SIMD, so they cannot share a
// compute unit; a single fused grid (kept behind a flag: it saves one launch for tiny
// passes) measured no faster than the sum.  A persistent form of the tile kernel can run
// beside the streaming grid on compute units that grid leaves free (an option, off by
// default).
#include "attn_decode_body.h"
#include "attn_prefill_body.h"

namespace fsf {
namespace {

constexpr int kThreads = 64 * kPrefillWaves;
constexpr int kUnitsPerGroup = kThreads / 64;  // generation-row units (waves) per workgroup

// Prefill workgroups: (tile, part) groups in their start order, query heads innermost.
__device__ __forceinline__ PrefillWork prefill_block_to_work(const Pass& p, const FastPlan& f, int block,
                                                             int& hq) {
  const int g = block / p.n_q_heads;
  hq = block - g * p.n_q_heads;
  return prefill_group_to_work(g, f.n_pre_tiles, f.split);
}


template <int DT, typename T>
__global__ __launch_bounds__(kThreads, 1) void attn_prefill_kernel(Pass p, FastPlan f,
                                                                 const T* __restrict__ q,
                                                                 const T* __restrict__ kc,
                                                                 const T* __restrict__ vc,
                                                                 T* __restrict__ out) {
  __shared__ __attribute__((aligned(1024))) char lds[kPrefillLdsBytes];
  int hq;
  const PrefillWork w = prefill_block_to_work(p, f, blockIdx.x, hq);
  prefill_tile<DT, T>(p, f, q, kc, vc, out, w, hq, (lds_char*)lds);
}

// The same tiles walked by a fixed number of workgroups (workgroup j takes tiles j, j + grid, ...
// in start order): the kernel then occupies exactly gridDim.x compute units however long it runs
// and whatever else is on the chip, which is what running it beside the streaming kernel needs.
template <int DT, typename T>
__global__ __launch_bounds__(kThreads, 1) void attn_prefill_persistent_kernel(Pass p, FastPlan f,
                                                                            const T* __restrict__ q,
                                                                            const T* __restrict__ kc,
                                                                            const T* __restrict__ vc,
                                                                            T* __restrict__ out, int n_blocks) {
  __shared__ __attribute__((aligned(1024))) char lds[kPrefillLdsBytes];
  for (int b = blockIdx.x; b < n_blocks; b += gridDim.x) {
    int hq;
    const PrefillWork w = prefill_block_to_work(p, f, b, hq);
    prefill_tile<DT, T>(p, f, q, kc, vc, out, w, hq, (lds_char*)lds);
    __syncthreads();  // the next tile's copies overwrite LDS slots that slower waves may still read
  }
}

// One generation-row unit per 64-thread workgroup: a finished unit frees its slot at once,
// which measured best on the short-sequence batches.
// hold_slots == 0: one unit per workgroup, results stored at once.  hold_slots > 0: the grid
// is one round of resident waves, every wave walks its share of the units (in launch order,
// back and forth over the rounds so that every wave gets long and short ones) and keeps the
// finished rows of up to hold_slots units in LDS; they are stored when the wave is done (or the
// slots are full).  The rows' writes then come at the end of the kernel, when the reads thin
// out, instead of being sprinkled into the read stream, where they cost several times their bytes.
template <int DT, typename T, bool kBlock16>
__global__ __launch_bounds__(64, 2) void attn_decode_single_kernel(Pass p, FastPlan f,
                                                                const T* __restrict__ q,
                                                                const T* __restrict__ kc,
                                                                const T* __restrict__ vc,
                                                                T* __restrict__ out, int hold_slots) {
  extern __shared__ __attribute__((aligned(16))) char decode_lds[];
  lds_char* stage = (lds_char*)decode_lds;
  if (hold_slots == 0) {
    const int slot = (int)blockIdx.x / p.n_kv_heads;
    decode_unit<DT, T, kBlock16>(p, f, q, kc, vc, out, load_unit_rec(f, slot), (int)blockIdx.x - slot * p.n_kv_heads,
                                 threadIdx.x, stage, nullptr);
    return;
  }
  const int row_bytes = p.group * kHeadDim * (int)sizeof(T);
  lds_char* hold = stage + kDecodeStageBytes;
  auto* dst = reinterpret_cast<__attribute__((address_space(3))) int64_t*>(hold + hold_slots * row_bytes);
  const int n_units = f.n_dec_items * p.n_kv_heads;
  const int G = gridDim.x, lane = threadIdx.x;
  int held = 0;
  auto flush = [&] {
    for (int s = 0; s < held; ++s) store_rows(reinterpret_cast<char*>(out) + dst[s], hold + s * row_bytes, row_bytes, lane);
    held = 0;
  };
  for (int round = 0; round * G < n_units; ++round) {
    const int unit = round * G + ((round & 1) ? G - 1 - (int)blockIdx.x : (int)blockIdx.x);
    if (unit >= n_units) continue;
    const int slot = unit / p.n_kv_heads;
    const int64_t d = decode_unit<DT, T, kBlock16>(p, f, q, kc, vc, out, load_unit_rec(f, slot), unit - slot * p.n_kv_heads,
                                                   lane, stage, hold + held * row_bytes);
    if (d >= 0) {  // the same in every lane
      if (lane == 0) dst[held] = d;
      ++held;
    }
    __builtin_amdgcn_wave_barrier();
    if (held == hold_slots) flush();
  }
  flush();
}

// The same walk with eight waves to a workgroup and so much LDS that a workgroup has a compute
// unit to itself: a grid of fewer workgroups than compute units then leaves whole units empty,
// wherever the dispatcher puts it and whatever starts first.  That is what lets prompt-chunk
// tiles (which need a whole empty unit each: a tile wave takes a SIMD's entire register file) run
// on a second stream beside the streaming kernel.  (The streaming kernel's grid is one round of
// waves that are all meant to be resident at once; a single wave slot taken by other work makes
// one of them start only when another has finished, and the launch lasts up to twice as long:
// measured +11 % beside one foreign wave, +23 % beside one prompt-chunk workgroup.)
constexpr int kWideWaves = 8;
template <int DT, typename T, bool kBlock16>
__global__ __launch_bounds__(64 * kWideWaves) void attn_decode_kernel(Pass p, FastPlan f,
                                                                           const T* __restrict__ q,
                                                                           const T* __restrict__ kc,
                                                                           const T* __restrict__ vc,
                                                                           T* __restrict__ out, int hold_slots,
                                                                           int lds_per_wave) {
  extern __shared__ __attribute__((aligned(16))) char decode_lds[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  lds_char* stage = (lds_char*)decode_lds + wave * lds_per_wave;
  const int row_bytes = p.group * kHeadDim * (int)sizeof(T);
  lds_char* hold = stage + kDecodeStageBytes;
  auto* dst = reinterpret_cast<__attribute__((address_space(3))) int64_t*>(hold + hold_slots * row_bytes);
  const int n_units = f.n_dec_items * p.n_kv_heads;
  // Which slot of the launch order a wave takes.  Where a workgroup's eight waves cover whole
  // sequences' KV heads (1, 2, 4 or 8 of them), consecutive slots: the workgroup then streams
  // whole cache blocks, contiguous in memory (measured on 8 KV heads: 2..4 % faster).  Otherwise
  // wave w of workgroup b takes slot w * groups + b: the eight waves of a compute unit then hold
  // units far apart in the launch order (other sequences, other lengths), as single-wave workgroups
  // dealt out in turn would; eight of a sequence's 40 heads side by side run in lockstep through
  // the same blocks and were 6 % slower on the long-prompt stream.
  const int G = gridDim.x * kWideWaves;
  const int me = (kWideWaves % p.n_kv_heads == 0) ? blockIdx.x * kWideWaves + wave : wave * (int)gridDim.x + (int)blockIdx.x;
  int held = 0;
  auto flush = [&] {
    for (int s = 0; s < held; ++s) store_rows(reinterpret_cast<char*>(out) + dst[s], hold + s * row_bytes, row_bytes, lane);
    held = 0;
  };
  for (int round = 0; round * G < n_units; ++round) {
    const int unit = round * G + ((round & 1) ? G - 1 - me : me);
    if (unit >= n_units) continue;
    const int slot = unit / p.n_kv_heads;
    const int64_t d = decode_unit<DT, T, kBlock16>(p, f, q, kc, vc, out, load_unit_rec(f, slot), unit - slot * p.n_kv_heads,
                                                   lane, stage, hold + held * row_bytes);
    if (d >= 0) {  // the same in every lane
      if (lane == 0) dst[held] = d;
      ++held;
    }
    __builtin_amdgcn_wave_barrier();
    if (held == hold_slots) flush();
  }
  flush();
}

template <int DT, typename T>
__global__ __launch_bounds__(kThreads, 1) void attn_fused_kernel(Pass p, FastPlan f,
                                                               const T* __restrict__ q,
                                                               const T* __restrict__ kc,
                                                               const T* __restrict__ vc,
                                                               T* __restrict__ out) {
  __shared__ __attribute__((aligned(1024))) char lds[kPrefillLdsBytes];
  // Workgroup numbering spreads the prompt-chunk tiles evenly through the generation-row
  // groups (and vice versa).  A tile workgroup fills a compute unit, so at any moment a small,
  // steady share of the chip does matrix-core work while the rest keeps HBM saturated.
  const int n_pre = f.n_pre_tiles * p.n_q_heads;
  const int n_dec = (f.n_dec_items * p.n_kv_heads + kUnitsPerGroup - 1) / kUnitsPerGroup;
  const int64_t total = (int64_t)n_pre + n_dec;
  const int b = blockIdx.x;
  const int pre_before = (int)((int64_t)b * n_pre / total);        // tiles among workgroups [0, b)
  const int pre_upto = (int)(((int64_t)b + 1) * n_pre / total);    // ... among [0, b]
  const bool is_prefill = pre_upto > pre_before;
  const int idx = is_prefill ? pre_before : b - pre_before;
  if (is_prefill) {  // uniform per workgroup
    int hq;
    const PrefillWork w = prefill_block_to_work(p, f, idx, hq);  // the fused grid is launched without split tiles
    prefill_tile<DT, T>(p, f, q, kc, vc, out, w, hq, (lds_char*)lds);
  } else {
    const int unit = idx * kUnitsPerGroup + (threadIdx.x >> 6);
    if (unit >= f.n_dec_items * p.n_kv_heads) return;
    // (the host launches this kernel for blocks of 32 tokens or more only)
    const int slot = unit / p.n_kv_heads;
    decode_unit<DT, T, false>(p, f, q, kc, vc, out, load_unit_rec(f, slot), unit - slot * p.n_kv_heads, threadIdx.x & 63,
                              (lds_char*)lds + (threadIdx.x >> 6) * kDecodeStageBytes, nullptr);
  }
}

unsigned decode_groups(const Pass& p, const FastPlan& f) {
  const int64_t units = (int64_t)f.n_dec_items * p.n_kv_heads;
  return (unsigned)((units + kUnitsPerGroup - 1) / kUnitsPerGroup);
}

}  // namespace

#define FSF_LAUNCH(KERNEL, GRID)                                                                   \
  if (p.dtype == FSF_BF16)                                                                         \
    KERNEL<FSF_BF16, bf16_t><<<GRID, kThreads, 0, stream>>>(                                       \
        p, f, (const bf16_t*)q, (const bf16_t*)k_cache, (const bf16_t*)v_cache, (bf16_t*)out);     \
  else                                                                                             \
    KERNEL<FSF_F16, f16_t><<<GRID, kThreads, 0, stream>>>(                                         \
        p, f, (const f16_t*)q, (const f16_t*)k_cache, (const f16_t*)v_cache, (f16_t*)out);

hipError_t launch_attn_prefill(const Pass& p, const FastPlan& f, const void* q, const void* k_cache,
                               const void* v_cache, void* out, hipStream_t stream, int persistent_groups) {
  if (f.n_pre_tiles == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_PREFILL, stream);
  const unsigned grid = (unsigned)prefill_groups(f.n_pre_tiles, f.split) * p.n_q_heads;
  if (persistent_groups > 0) {
    const unsigned g = std::min<unsigned>(grid, (unsigned)persistent_groups);
    if (p.dtype == FSF_BF16)
      attn_prefill_persistent_kernel<FSF_BF16, bf16_t><<<g, kThreads, 0, stream>>>(
          p, f, (const bf16_t*)q, (const bf16_t*)k_cache, (const bf16_t*)v_cache, (bf16_t*)out, (int)grid);
    else
      attn_prefill_persistent_kernel<FSF_F16, f16_t><<<g, kThreads, 0, stream>>>(
          p, f, (const f16_t*)q, (const f16_t*)k_cache, (const f16_t*)v_cache, (f16_t*)out, (int)grid);
    return hipGetLastError();
  }
  FSF_LAUNCH(attn_prefill_kernel, grid)
  return hipGetLastError();
}

hipError_t launch_attn_decode(const Pass& p, const FastPlan& f, const void* q, const void* k_cache,
                              const void* v_cache, void* out, hipStream_t stream, int reserve_units) {
  if (f.n_dec_items == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_DECODE, stream);
  const unsigned n_units = (unsigned)f.n_dec_items * p.n_kv_heads;
  const int row_bytes = p.group * kHeadDim * 2;
  const bool b16 = p.block_size == 16;
  const unsigned slots = 8u * (unsigned)device_compute_units();
  if (n_units > slots && f.decode_hold == 1) {
    // More units than wave slots: one round of waves that hold their results back, as one
    // workgroup of eight waves per compute unit (on all units but the reserved ones).  LDS per
    // wave: the staging area, up to 10 KB of finished rows, their addresses; at least 12 KB, so
    // that a workgroup takes 96 KB and no second one fits beside it: every unit then holds exactly
    // eight waves (single-wave workgroups spread unevenly over the units: 2..4 % slower).
    const unsigned groups = (unsigned)std::max(1, device_compute_units() - reserve_units);
    const int per_wave = (int)((n_units + groups * kWideWaves - 1) / (groups * kWideWaves));
    const int hold_slots = std::max(1, std::min(per_wave, (10 * 1024) / row_bytes));
    const int lds_per_wave = std::max(12 * 1024, (kDecodeStageBytes + hold_slots * (row_bytes + 8) + 15) & ~15);
    const size_t lds_bytes = (size_t)lds_per_wave * kWideWaves;
#define FSF_DECODE_WIDE(DT, T, B16)                                                                              \
  {                                                                                                              \
    if (const hipError_t e = allow_lds_bytes<&attn_decode_kernel<DT, T, B16>>(160 * 1024); e != hipSuccess)      \
      return e;                                                                                                  \
    attn_decode_kernel<DT, T, B16><<<groups, 64 * kWideWaves, lds_bytes, stream>>>(                         \
        p, f, (const T*)q, (const T*)k_cache, (const T*)v_cache, (T*)out, hold_slots, lds_per_wave);             \
  }
    if (p.dtype == FSF_BF16) {
      if (b16) FSF_DECODE_WIDE(FSF_BF16, bf16_t, true) else FSF_DECODE_WIDE(FSF_BF16, bf16_t, false)
    } else {
      if (b16) FSF_DECODE_WIDE(FSF_F16, f16_t, true) else FSF_DECODE_WIDE(FSF_F16, f16_t, false)
    }
#undef FSF_DECODE_WIDE
    return hipGetLastError();
  }
  // one unit per single-wave workgroup, results stored at once; or (decode_hold == 2, kept for
  // comparison) one round of single-wave workgroups that hold their results back
  unsigned grid = n_units;
  int hold_slots = 0;
  if (n_units > slots && f.decode_hold == 2) {
    grid = slots;
    hold_slots = std::min((int)((n_units + slots - 1) / slots), (10 * 1024) / row_bytes);
  }
  const size_t lds_bytes = kDecodeStageBytes + (size_t)hold_slots * (row_bytes + 8);
#define FSF_DECODE(DT, T, B16)                 \
  attn_decode_single_kernel<DT, T, B16><<<grid, 64, lds_bytes, stream>>>(p, f, (const T*)q, (const T*)k_cache, \
                                                                  (const T*)v_cache, (T*)out, hold_slots)
  if (p.dtype == FSF_BF16) {
    if (b16) FSF_DECODE(FSF_BF16, bf16_t, true); else FSF_DECODE(FSF_BF16, bf16_t, false);
  } else {
    if (b16) FSF_DECODE(FSF_F16, f16_t, true); else FSF_DECODE(FSF_F16, f16_t, false);
  }
#undef FSF_DECODE
  return hipGetLastError();
}

hipError_t launch_attn_fused(const Pass& p, const FastPlan& f, const void* q, const void* k_cache,
                             const void* v_cache, void* out, hipStream_t stream) {
  const unsigned grid = (unsigned)f.n_pre_tiles * p.n_q_heads + decode_groups(p, f);
  if (grid == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_FUSED, stream);
  FSF_LAUNCH(attn_fused_kernel, grid)
  return hipGetLastError();
}

#undef FSF_LAUNCH

}  // namespace fsf

