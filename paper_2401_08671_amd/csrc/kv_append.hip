// KV-cache append: scatter this pass's K/V rows into their cache blocks, bit for bit.
//
// Paper Sec. 2 (a pass adds its tokens to the sequence's cache) and Sec. 2.1 (the cache is
// a pool of fixed-size blocks).  Token i of sequence s sits at position p = n_cached + i,
// i.e. block block_tables[s][p / B], slot p % B.  Pure copy: HBM bound, a fraction of a
// percent of the attention traffic.
//
// One workgroup per token.  A token's K row is n_kv_heads * d contiguous elements in
// k_new; in the cache head h of that row is a contiguous d-element run at
// [blk][h][slot][:].  Threads move 16-byte (or 4-byte) units, so each head run is written
// with whole-wave coalesced stores.
//
// Rotary variant: the K row is rotated by the angles of its position on the way (the rotary
// position embedding of the Llama family the paper's evaluation serves, Sec. 4.1; half-split
// pairing: element i with i + d/2).  The arithmetic is fixed so that the cache stays
// bit-exact against a reference: float32 products and their sum or difference, each rounded
// to nearest even and never fused, then one rounding to the storage type.  cos and sin come
// from a table the caller supplies, so no transcendental is evaluated here.
#include "fsf_internal.h"
#include "numeric.h"

namespace fsf {
namespace {

template <typename Unit>
__global__ __launch_bounds__(256) void kv_append_kernel(Pass p, const Unit* __restrict__ k_new,
                                                        const Unit* __restrict__ v_new,
                                                        Unit* __restrict__ k_cache,
                                                        Unit* __restrict__ v_cache,
                                                        int units_per_head) {
  const int t = blockIdx.x;
  const int s = find_seq(p.descs, p.n_seqs, t);
  const fsf_seq_desc d = p.descs[s];
  const int pos = d.n_cached + (t - d.q_offset);
  const int64_t blk = p.block_tables[(int64_t)s * p.max_blocks + pos / p.block_size];
  const int slot = pos % p.block_size;

  const int row_units = p.n_kv_heads * units_per_head;
  const int64_t src = (int64_t)t * row_units;
  // cache element [blk][h][slot][0] in units
  const int64_t blk_base = blk * p.n_kv_heads * (int64_t)p.block_size * units_per_head;
  for (int u = threadIdx.x; u < row_units; u += blockDim.x) {
    const int h = u / units_per_head;
    const int w = u - h * units_per_head;
    const int64_t dst = blk_base + ((int64_t)h * p.block_size + slot) * units_per_head + w;
    k_cache[dst] = k_new[src + u];
    v_cache[dst] = v_new[src + u];
  }
}

// One workgroup per token; a thread rotates one (i, i + d/2) pair of one head at a time and
// copies the matching V elements.  T is the storage type.
template <typename T>
__global__ __launch_bounds__(256) void kv_append_rotary_kernel(Pass p, const T* __restrict__ k_new,
                                                               const T* __restrict__ v_new,
                                                               T* __restrict__ k_cache,
                                                               T* __restrict__ v_cache,
                                                               const float2* __restrict__ cos_sin) {
// Products and sums below must stay separate roundings: the compiler's default would fuse
// them into multiply-adds (the *_rn intrinsics are plain operators and fuse as well).
#pragma clang fp contract(off)
  const int t = blockIdx.x;
  const int s = find_seq(p.descs, p.n_seqs, t);
  const fsf_seq_desc d = p.descs[s];
  const int pos = d.n_cached + (t - d.q_offset);
  const int64_t blk = p.block_tables[(int64_t)s * p.max_blocks + pos / p.block_size];
  const int slot = pos % p.block_size;
  const int half = p.head_dim / 2;
  const float2* cs = cos_sin + (int64_t)pos * half;
  const int64_t src = (int64_t)t * p.n_kv_heads * p.head_dim;
  const int64_t blk_base = blk * p.n_kv_heads * (int64_t)p.block_size * p.head_dim;
  for (int u = threadIdx.x; u < p.n_kv_heads * half; u += blockDim.x) {
    const int h = u / half;
    const int i = u - h * half;
    const int64_t in = src + (int64_t)h * p.head_dim + i;
    const int64_t dst = blk_base + ((int64_t)h * p.block_size + slot) * p.head_dim + i;
    const float a = to_float(k_new[in]), b = to_float(k_new[in + half]);
    const float2 c = cs[i];
    const float ac = a * c.x, bs = b * c.y, bc = b * c.x, as = a * c.y;
    k_cache[dst] = from_float<T>(ac - bs);
    k_cache[dst + half] = from_float<T>(bc + as);
    v_cache[dst] = v_new[in];
    v_cache[dst + half] = v_new[in + half];
  }
}

// The same rotation applied in place to the query rows [T, n_q_heads, d]: one workgroup per
// token, a thread per (head, pair).
template <typename T>
__global__ __launch_bounds__(256) void rotary_q_kernel(Pass p, T* __restrict__ q, const float2* __restrict__ cos_sin) {
#pragma clang fp contract(off)
  const int t = blockIdx.x;
  const int s = find_seq(p.descs, p.n_seqs, t);
  const fsf_seq_desc d = p.descs[s];
  const int pos = d.n_cached + (t - d.q_offset);
  const int half = p.head_dim / 2;
  const float2* cs = cos_sin + (int64_t)pos * half;
  T* row = q + (int64_t)t * p.n_q_heads * p.head_dim;
  for (int u = threadIdx.x; u < p.n_q_heads * half; u += blockDim.x) {
    const int h = u / half;
    const int i = u - h * half;
    T* x = row + h * p.head_dim + i;
    const float a = to_float(x[0]), b = to_float(x[half]);
    const float2 c = cs[i];
    const float ac = a * c.x, bs = b * c.y, bc = b * c.x, as = a * c.y;
    x[0] = from_float<T>(ac - bs);
    x[half] = from_float<T>(bc + as);
  }
}

}  // namespace

hipError_t launch_rotary_q(const Pass& p, void* q, const float* cos_sin, hipStream_t stream) {
  if (p.n_tokens == 0 || p.n_seqs == 0) return hipSuccess;
  const float2* cs = reinterpret_cast<const float2*>(cos_sin);
  if (p.dtype == FSF_F32)
    rotary_q_kernel<float><<<p.n_tokens, 256, 0, stream>>>(p, (float*)q, cs);
  else if (p.dtype == FSF_BF16)
    rotary_q_kernel<bf16_t><<<p.n_tokens, 256, 0, stream>>>(p, (bf16_t*)q, cs);
  else
    rotary_q_kernel<f16_t><<<p.n_tokens, 256, 0, stream>>>(p, (f16_t*)q, cs);
  return hipGetLastError();
}

hipError_t launch_kv_append_rotary(const Pass& p, const void* k_new, const void* v_new, void* k_cache,
                                   void* v_cache, const float* cos_sin, hipStream_t stream) {
  if (p.n_tokens == 0 || p.n_seqs == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_APPEND, stream);
  const float2* cs = reinterpret_cast<const float2*>(cos_sin);
  if (p.dtype == FSF_F32)
    kv_append_rotary_kernel<float><<<p.n_tokens, 256, 0, stream>>>(p, (const float*)k_new, (const float*)v_new,
                                                                  (float*)k_cache, (float*)v_cache, cs);
  else if (p.dtype == FSF_BF16)
    kv_append_rotary_kernel<bf16_t><<<p.n_tokens, 256, 0, stream>>>(p, (const bf16_t*)k_new, (const bf16_t*)v_new,
                                                                   (bf16_t*)k_cache, (bf16_t*)v_cache, cs);
  else
    kv_append_rotary_kernel<f16_t><<<p.n_tokens, 256, 0, stream>>>(p, (const f16_t*)k_new, (const f16_t*)v_new,
                                                                  (f16_t*)k_cache, (f16_t*)v_cache, cs);
  return hipGetLastError();
}

hipError_t launch_kv_append(const Pass& p, const void* k_new, const void* v_new, void* k_cache,
                            void* v_cache, hipStream_t stream) {
  if (p.n_tokens == 0 || p.n_seqs == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_APPEND, stream);
  const int esize = p.dtype == FSF_F32 ? 4 : 2;
  const int head_bytes = p.head_dim * esize;
  const uintptr_t all = (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_cache | (uintptr_t)v_cache;
  if (head_bytes % 16 == 0 && (all & 15) == 0) {  // 16-byte units need 16-byte aligned tensors
    kv_append_kernel<uint4><<<p.n_tokens, 256, 0, stream>>>(
        p, (const uint4*)k_new, (const uint4*)v_new, (uint4*)k_cache, (uint4*)v_cache,
        head_bytes / 16);
  } else {
    kv_append_kernel<uint32_t><<<p.n_tokens, 256, 0, stream>>>(
        p, (const uint32_t*)k_new, (const uint32_t*)v_new, (uint32_t*)k_cache,
        (uint32_t*)v_cache, head_bytes / 4);
  }
  return hipGetLastError();
}

}  // namespace fsf
