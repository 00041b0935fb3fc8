// Work planning and split merging for the matrix-core attention path.
//
// A pass mixes one-row generations with prompt chunks of any length (paper Sec. 3.2), so
// work per sequence is ragged.  plan_kernel turns the descriptors into exclusive prefix
// arrays (streaming items, prefill tiles, partial-result rows) plus item->sequence and
// tile->sequence tables, so every wave of the compute kernels finds its work with one load; no
// host-to-device copy is needed.  The streaming items are also put in launch order, those with
// the most cache blocks first (a counting sort by block count): units of similar length then
// run side by side and the longest do not end up in the tail (+2..3 % on the generation-row
// kernel against descriptor order).
//
// merge_kernel combines the partial results of a generation row whose visible keys were
// split across several workgroups: with per-split running maximum m_k (log2 domain),
// sum l_k and unnormalised output a_k,
//     m = max_k m_k,  l = sum_k l_k 2^(m_k - m),  out = sum_k a_k 2^(m_k - m) / l.
#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {
namespace {

constexpr int kPlanThreads = 1024;

// Inclusive prefix sum over the workgroup's kPlanThreads values (one per thread): shuffles inside
// each wave, then the 16 wave totals through LDS.  `totals` holds one int per wave.
__device__ __forceinline__ int block_inclusive_scan(int v, int* totals) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int a = __shfl_up(v, off);
    if (lane >= off) v += a;
  }
  __syncthreads();  // totals may still be read from the previous scan
  if (lane == 63) totals[wave] = v;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += totals[w];
  return v + before;
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(Pass p, FastPlan f) {
  __shared__ int s_bucket[kPlanThreads];  // streaming items per block count, largest count first
  __shared__ int s_totals[4][kPlanThreads / 64];
  const int tid = threadIdx.x;
  s_bucket[tid] = 0;
  const int per = (p.n_seqs + kPlanThreads - 1) / kPlanThreads;
  const int s0 = tid * per;
  const int s1 = min(s0 + per, p.n_seqs);
  auto work_of = [&](int s) {
    return seq_work(p.descs[s].n_new, p.descs[s].n_cached, p.window, p.block_size, p.group, f.stream_max_slices,
                    f.split_blocks, f.min_item_blocks);
  };
  int dec = 0, pre = 0, spl = 0, prw = 0;
  for (int s = s0; s < s1; ++s) {
    const SeqWork w = work_of(s);
    dec += w.dec_items;
    pre += w.pre_tiles;
    spl += w.cuts > 1 ? p.descs[s].n_new : 0;  // rows whose keys were cut
    prw += w.prows;
  }
  // inclusive scans over the per-thread sums
  const int dec_incl = block_inclusive_scan(dec, s_totals[0]);
  const int pre_incl = block_inclusive_scan(pre, s_totals[1]);
  const int spl_incl = block_inclusive_scan(spl, s_totals[2]);
  const int prw_incl = block_inclusive_scan(prw, s_totals[3]);
  int dec_run = dec_incl - dec, pre_run = pre_incl - pre, spl_run = spl_incl - spl, prw_run = prw_incl - prw;  // exclusive
  for (int s = s0; s < s1; ++s) {
    f.dec_item_start[s] = dec_run;
    f.pre_tile_start[s] = pre_run;
    f.dec_prow_start[s] = prw_run;
    const SeqWork w = work_of(s);
    for (int k = 0; k < w.pre_tiles; ++k) f.pre_tile_seq[pre_run + k] = s;
    if (w.cuts > 1)
      for (int r = 0; r < p.descs[s].n_new; ++r, ++spl_run) {
        f.split_rows[2 * spl_run] = s;
        f.split_rows[2 * spl_run + 1] = r;
      }
    dec_run += w.dec_items;
    pre_run += w.pre_tiles;
    prw_run += w.prows;
  }
  if (tid == kPlanThreads - 1) {
    f.dec_item_start[p.n_seqs] = dec_incl;
    f.pre_tile_start[p.n_seqs] = pre_incl;
    f.dec_prow_start[p.n_seqs] = prw_incl;
  }
  // ---- launch order of the streaming items: counting sort, most blocks first
  auto bucket_of = [&](int s, int cuts) {  // all items of a sequence hold about nblk / cuts blocks
    int lo, hi, tmp;
    visible_range(p.descs[s].n_cached, p.window, lo, tmp);
    visible_range(p.descs[s].n_cached + p.descs[s].n_new - 1, p.window, tmp, hi);
    const int per_item = (hi / p.block_size - lo / p.block_size + cuts) / cuts;
    return kPlanThreads - 1 - min(per_item, kPlanThreads - 1);
  };
  __syncthreads();  // s_bucket zeroed by every thread above
  for (int s = s0; s < s1; ++s) {
    const SeqWork w = work_of(s);
    if (w.dec_items > 0) atomicAdd(&s_bucket[bucket_of(s, w.cuts)], w.dec_items);
  }
  __syncthreads();
  const int mine = s_bucket[tid];
  const int start = block_inclusive_scan(mine, s_totals[0]) - mine;  // scan over the buckets
  s_bucket[tid] = start;  // next free launch slot of the bucket (every thread touches its own entry only)
  __syncthreads();
  prw_run = prw_incl - prw;
  for (int s = s0; s < s1; ++s) {
    const SeqWork w = work_of(s);
    if (w.dec_items > 0) {
      const int pos = atomicAdd(&s_bucket[bucket_of(s, w.cuts)], w.dec_items);
      const fsf_seq_desc sd = p.descs[s];
      for (int k = 0; k < w.dec_items; ++k)
        f.dec_rec[pos + k] = UnitRec{s, k, sd.n_new, sd.n_cached, sd.q_offset, prw_run, {0, 0}};
    }
    prw_run += w.prows;
  }
}

// One wave per (row whose keys were cut, query head).  Maximum and sum: lane k takes cuts k,
// k + 64, ... and the wave reduces; outputs: lanes own two columns each and walk the cuts four at
// a time, so that the loads of several cuts are in flight together (the walk is latency-bound: a
// long sequence alone in a pass has a hundred cuts and nothing else to hide behind).
// Partial row of (cut k, row r) of a sequence: dec_prow_start[s] + k * n_new + r.
template <typename T>
__global__ __launch_bounds__(64) void merge_kernel(Pass p, FastPlan f, T* __restrict__ out) {
  const int s = f.split_rows[2 * (blockIdx.x / p.n_q_heads)];
  const int r = f.split_rows[2 * (blockIdx.x / p.n_q_heads) + 1];
  const int hq = blockIdx.x % p.n_q_heads;
  const int n_new = p.descs[s].n_new;
  const int n_splits = (f.dec_prow_start[s + 1] - f.dec_prow_start[s]) / n_new;
  const int64_t prow0 = (int64_t)f.dec_prow_start[s] + r;
  const int lane = threadIdx.x;
  const float* ml = f.part_ml + (prow0 * p.n_q_heads + hq) * 2;
  const int64_t ml_stride = (int64_t)n_new * p.n_q_heads * 2;  // cut to cut
  float m = -INFINITY;
  for (int k = lane; k < n_splits; k += 64) m = fmaxf(m, ml[k * ml_stride]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  float l = 0.f;
  for (int k = lane; k < n_splits; k += 64) l += ml[k * ml_stride + 1] * fast_exp2(ml[k * ml_stride] - m);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
  const float* acc = f.part_acc + (prow0 * p.n_q_heads + hq) * kHeadDim + lane * 2;
  const int64_t acc_stride = (int64_t)n_new * p.n_q_heads * kHeadDim;
  float a0 = 0.f, a1 = 0.f;
  int k = 0;
  for (; k + 4 <= n_splits; k += 4) {
    float2 a[4];
    float w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      a[u] = *reinterpret_cast<const float2*>(acc + (k + u) * acc_stride);
      w[u] = fast_exp2(ml[(k + u) * ml_stride] - m);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      a0 += a[u].x * w[u];
      a1 += a[u].y * w[u];
    }
  }
  for (; k < n_splits; ++k) {
    const float2 a = *reinterpret_cast<const float2*>(acc + k * acc_stride);
    const float w = fast_exp2(ml[k * ml_stride] - m);
    a0 += a.x * w;
    a1 += a.y * w;
  }
  const float inv = 1.f / l;
  T* orow = out + ((int64_t)(p.descs[s].q_offset + r) * p.n_q_heads + hq) * kHeadDim;
  orow[lane * 2] = from_float<T>(a0 * inv);
  orow[lane * 2 + 1] = from_float<T>(a1 * inv);
}

// Split prompt-chunk tiles: one wave per (row of a split tile, query head) combines the
// partial results of that row's parts in the same way; lanes own two output columns each.
template <typename T>
__global__ __launch_bounds__(64) void prefill_merge_kernel(Pass p, FastPlan f, T* __restrict__ out) {
  const int hq = blockIdx.x % p.n_q_heads;
  const int jrow = blockIdx.x / p.n_q_heads;  // split tile number * kPrefillTileM + row inside the tile
  const PrefillWork w = prefill_split_tile(jrow / kPrefillTileM, f.split);
  const int row = jrow % kPrefillTileM;
  const int s = f.pre_tile_seq[w.tile];
  const int i = (w.tile - f.pre_tile_start[s]) * kPrefillTileM + row;  // row of the chunk
  if (i >= p.descs[s].n_new) return;
  const int lane = threadIdx.x;
  const int64_t part_stride = (int64_t)kPrefillTileM * p.n_q_heads * kPrefillPartRowFloats;  // slab to slab
  const float* part = f.pre_part + (((int64_t)w.slab * kPrefillTileM + row) * p.n_q_heads + hq) * kPrefillPartRowFloats;
  float m = -INFINITY;
  for (int k = 0; k < w.n_parts; ++k) m = fmaxf(m, part[k * part_stride + kHeadDim]);
  float l = 0.f, a0 = 0.f, a1 = 0.f;
  for (int k = 0; k < w.n_parts; ++k) {
    const float* pk = part + k * part_stride;
    const float w = fast_exp2(pk[kHeadDim] - m);
    l += pk[kHeadDim + 1] * w;
    const float2 a = *reinterpret_cast<const float2*>(pk + lane * 2);
    a0 += a.x * w;
    a1 += a.y * w;
  }
  const float inv = 1.f / l;
  T* orow = out + ((int64_t)(p.descs[s].q_offset + i) * p.n_q_heads + hq) * kHeadDim;
  orow[lane * 2] = from_float<T>(a0 * inv);
  orow[lane * 2 + 1] = from_float<T>(a1 * inv);
}

}  // namespace

hipError_t launch_plan(const Pass& p, const FastPlan& f, hipStream_t stream) {
  PhaseTimer timer(FSF_PHASE_PLAN, stream);
  plan_kernel<<<1, kPlanThreads, 0, stream>>>(p, f);
  return hipGetLastError();
}

hipError_t launch_attn_merge(const Pass& p, const FastPlan& f, void* out, hipStream_t stream) {
  if (f.n_split_rows == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_MERGE, stream);
  const unsigned grid = (unsigned)f.n_split_rows * p.n_q_heads;
  if (p.dtype == FSF_BF16)
    merge_kernel<bf16_t><<<grid, 64, 0, stream>>>(p, f, (bf16_t*)out);
  else
    merge_kernel<f16_t><<<grid, 64, 0, stream>>>(p, f, (f16_t*)out);
  return hipGetLastError();
}

hipError_t launch_prefill_merge(const Pass& p, const FastPlan& f, void* out, hipStream_t stream) {
  const int n_split = f.split.n_heavy + f.split.tail_tiles;
  if (n_split == 0) return hipSuccess;
  PhaseTimer timer(FSF_PHASE_MERGE, stream);
  const unsigned grid = (unsigned)n_split * kPrefillTileM * p.n_q_heads;
  if (p.dtype == FSF_BF16)
    prefill_merge_kernel<bf16_t><<<grid, 64, 0, stream>>>(p, f, (bf16_t*)out);
  else
    prefill_merge_kernel<f16_t><<<grid, 64, 0, stream>>>(p, f, (f16_t*)out);
  return hipGetLastError();
}

}  // namespace fsf
