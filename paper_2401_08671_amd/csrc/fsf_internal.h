// Internal declarations shared by the C-ABI layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fsf.h"

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

hipError_t launch_kv_append(const Pass& p, const void* k_new, const void* v_new, void* k_cache,
                            void* v_cache, hipStream_t stream);

hipError_t launch_attn_generic(const Pass& p, const void* q, const void* k_cache,
                               const void* v_cache, void* out, hipStream_t stream);

}  // namespace fsf
