// Kernels of the matrix-core attention path and their launchers.
//
// A Dynamic SplitFuse pass mixes prompt chunks (dense, matrix-core bound) with one-token
// generations (streaming, HBM bound) at a fixed token budget (paper Sec. 3.2).  By default
// each kind of work gets its own launch with the workgroup shape that suits it (256-thread
// tiles with 64 KB of LDS, two to a compute unit; 64-thread streaming units).  Both kernels
// fill the register file at two waves per SIMD, so they cannot share a compute unit and a
// single fused grid (kept behind a flag: it saves one launch for tiny passes) measured no
// faster than the sum.
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

// One generation-row unit per 64-thread workgroup: a finished unit frees its slot at once,
// which measured best on the short-sequence batches.
// hold_slots == 0: one unit per workgroup, results stored at once.  hold_slots > 0: the grid
// is one round of resident waves, every wave walks its share of the units (in launch order,
// back and forth over the rounds so that every wave gets long and short ones) and keeps the
// finished rows of up to hold_slots units in LDS; they are stored when the wave is done (or the
// slots are full).  The rows' writes then come at the end of the kernel, when the reads thin
// out, instead of being sprinkled into the read stream, where they cost several times their bytes.
template <int DT, typename T, bool kBlock16>
__global__ __launch_bounds__(64, 2) void attn_decode_kernel(Pass p, FastPlan f,
                                                                const T* __restrict__ q,
                                                                const T* __restrict__ kc,
                                                                const T* __restrict__ vc,
                                                                T* __restrict__ out, int hold_slots) {
  extern __shared__ __attribute__((aligned(16))) char decode_lds[];
  lds_char* stage = (lds_char*)decode_lds;
  if (hold_slots == 0) {
    decode_unit<DT, T, kBlock16>(p, f, q, kc, vc, out, blockIdx.x, threadIdx.x, stage, nullptr);
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
    const int64_t d = decode_unit<DT, T, kBlock16>(p, f, q, kc, vc, out, unit, lane, stage, hold + held * row_bytes);
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
    decode_unit<DT, T, false>(p, f, q, kc, vc, out, unit, threadIdx.x & 63,
                              (lds_char*)lds + (threadIdx.x >> 6) * kDecodeStageBytes, nullptr);
  }
}

int decode_compute_units() {
  static int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 1)
      cu = 256;
    return cu;
  }();
  return n;
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
                               const void* v_cache, void* out, hipStream_t stream) {
  if (f.n_pre_tiles == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_PREFILL, stream);
  const unsigned grid = (unsigned)prefill_groups(f.n_pre_tiles, f.split) * p.n_q_heads;
  FSF_LAUNCH(attn_prefill_kernel, grid)
  return hipGetLastError();
}

hipError_t launch_attn_decode(const Pass& p, const FastPlan& f, const void* q, const void* k_cache,
                              const void* v_cache, void* out, hipStream_t stream) {
  if (f.n_dec_items == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_DECODE, stream);
  const unsigned n_units = (unsigned)f.n_dec_items * p.n_kv_heads;
  // With more units than wave slots (two waves per SIMD): one round of waves that hold their
  // results back.  LDS per wave: the staging area, up to 10 KB of finished rows, their addresses.
  unsigned grid = n_units;
  int hold_slots = 0;
  const unsigned slots = 8u * (unsigned)decode_compute_units();
  const int row_bytes = p.group * kHeadDim * 2;
  if (n_units > slots && f.decode_hold) {
    grid = slots;
    const int per_wave = (int)((n_units + slots - 1) / slots);
    hold_slots = std::min(per_wave, (10 * 1024) / row_bytes);
  }
  const size_t lds_bytes = kDecodeStageBytes + (size_t)hold_slots * (row_bytes + 8);
#define FSF_DECODE(DT, T, B16)                 \
  attn_decode_kernel<DT, T, B16><<<grid, 64, lds_bytes, stream>>>(p, f, (const T*)q, (const T*)k_cache, \
                                                                  (const T*)v_cache, (T*)out, hold_slots)
  const bool b16 = p.block_size == 16;
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

