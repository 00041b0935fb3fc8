// Generic ragged blocked-KV attention: any dtype, any head_dim <= 256, any block size.
//
// Computes, for every new row of every sequence, causal (optionally windowed) softmax
// attention over the sequence's cached + new tokens read through the block table
// (paper Sec. 2: prompt passes and generation passes; Sec. 2.1: blocked cache; Sec. 3.2:
// a prompt chunk attends to the chunks cached by earlier passes).
//
// Correctness-first path: one wavefront per (token row, query head), fp32 throughout.
// Keys are taken 64 at a time: lane j scores key k0+j, the wave reduces max and sum with
// shuffles (running softmax), then the 64 weights are broadcast one by one while the
// lanes own the output's d columns.  Only visible keys are ever read, so stale cache
// slots cannot leak into the result.  The bf16/f16 head_dim-128 shapes use the matrix
// core kernels instead; this kernel serves fp32 and every other shape.
#include <math.h>

#include "fsf_internal.h"
#include "numeric.h"

namespace fsf {
namespace {

constexpr int kWaves = 4;
constexpr int kMaxD = 256;

__device__ __forceinline__ float wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

template <typename T>
__global__ __launch_bounds__(kWaves * 64) void attn_generic_kernel(Pass p, const T* __restrict__ q,
                                                                   const T* __restrict__ kc,
                                                                   const T* __restrict__ vc,
                                                                   T* __restrict__ out) {
  __shared__ float q_lds[kWaves][kMaxD];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t n_items = (int64_t)p.n_tokens * p.n_q_heads;
  int64_t item = (int64_t)blockIdx.x * kWaves + wave;
  const bool live = item < n_items;
  if (!live) item = n_items - 1;  // keep the wave in the barrier; its result is dropped

  const int t = (int)(item / p.n_q_heads);
  const int hq = (int)(item - (int64_t)t * p.n_q_heads);
  const int hk = hq / p.group;
  const int d = p.head_dim, B = p.block_size;
  const int s = find_seq(p.descs, p.n_seqs, t);
  const fsf_seq_desc sd = p.descs[s];
  const int pos = sd.n_cached + (t - sd.q_offset);
  const int hi = pos;
  const int lo = (p.window > 0 && pos - p.window + 1 > 0) ? pos - p.window + 1 : 0;
  const int32_t* bt = p.block_tables + (int64_t)s * p.max_blocks;

  const T* qrow = q + ((int64_t)t * p.n_q_heads + hq) * d;
  for (int e = lane; e < d; e += 64) q_lds[wave][e] = to_float(qrow[e]);
  __syncthreads();

  float m = -INFINITY, l = 0.f;
  float acc[kMaxD / 64] = {0.f, 0.f, 0.f, 0.f};

  for (int k0 = lo; k0 <= hi; k0 += 64) {
    const int key = k0 + lane;
    const bool vis = key <= hi;
    float sc = -INFINITY;
    if (vis) {
      const int64_t blk = bt[key / B];
      const T* krow = kc + ((blk * p.n_kv_heads + hk) * B + key % B) * d;
      float dot = 0.f;
      for (int e = 0; e < d; ++e) dot += q_lds[wave][e] * to_float(krow[e]);
      sc = dot * p.scale;
    }
    const float m_new = fmaxf(m, wave_max(sc));  // finite: key k0 is always visible
    const float corr = expf(m - m_new);          // first chunk: exp(-inf) = 0
    const float pr = vis ? expf(sc - m_new) : 0.f;
    l = l * corr + wave_sum(pr);
#pragma unroll
    for (int e = 0; e < kMaxD / 64; ++e) acc[e] *= corr;
    const int cnt = (hi - k0 + 1) < 64 ? (hi - k0 + 1) : 64;
    for (int jj = 0; jj < cnt; ++jj) {
      const float pj = __shfl(pr, jj);
      const int kj = k0 + jj;
      const int64_t blk = bt[kj / B];
      const T* vrow = vc + ((blk * p.n_kv_heads + hk) * B + kj % B) * d;
#pragma unroll
      for (int e = 0; e < kMaxD / 64; ++e) {
        const int col = lane + 64 * e;
        if (col < d) acc[e] += pj * to_float(vrow[col]);
      }
    }
    m = m_new;
  }

  if (live) {
    T* orow = out + ((int64_t)t * p.n_q_heads + hq) * d;
    const float inv = 1.f / l;
#pragma unroll
    for (int e = 0; e < kMaxD / 64; ++e) {
      const int col = lane + 64 * e;
      if (col < d) orow[col] = from_float<T>(acc[e] * inv);
    }
  }
}

}  // namespace

hipError_t launch_attn_generic(const Pass& p, const void* q, const void* k_cache,
                               const void* v_cache, void* out, hipStream_t stream) {
  const int64_t n_items = (int64_t)p.n_tokens * p.n_q_heads;
  if (n_items == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_GENERIC, stream);
  const unsigned grid = (unsigned)((n_items + kWaves - 1) / kWaves);
  switch (p.dtype) {
    case FSF_F32:
      attn_generic_kernel<float><<<grid, kWaves * 64, 0, stream>>>(
          p, (const float*)q, (const float*)k_cache, (const float*)v_cache, (float*)out);
      break;
    case FSF_BF16:
      attn_generic_kernel<bf16_t><<<grid, kWaves * 64, 0, stream>>>(
          p, (const bf16_t*)q, (const bf16_t*)k_cache, (const bf16_t*)v_cache, (bf16_t*)out);
      break;
    case FSF_F16:
      attn_generic_kernel<f16_t><<<grid, kWaves * 64, 0, stream>>>(
          p, (const f16_t*)q, (const f16_t*)k_cache, (const f16_t*)v_cache, (f16_t*)out);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace fsf
