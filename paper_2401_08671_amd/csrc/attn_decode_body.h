// Device code for streaming sequences: generation rows (n_new == 1) and short prompt chunks;
// split-KV attention streaming the blocked cache once.
//
// A generation pass adds one token and attends to the whole cached history (paper Sec. 2),
// so every visible K/V byte is used exactly once per KV head: the kernel is bound by HBM
// bandwidth.  One wavefront handles one (sequence, slice of rows, KV head, run of cache
// blocks); the query heads that share the KV head (GQA group, up to 16) sit side by side in the
// N dimension of the matrix-core tiles, so K/V are read once for the whole group.
//
// Dynamic SplitFuse fills the token budget exactly, so a pass usually ends in a chunk of a few
// rows of the next prompt, and the last chunk of a prompt is a short remainder over a long cached
// prefix (Sec. 3.2).  Such a chunk costs its K/V bytes, not its flops, exactly like a generation
// row, so its rows share the 16 columns with the heads: column n is (row n / group, head
// n % group) of a slice of 16 / group consecutive rows, each column with its own causal
// bound, and the slice's K/V are read once at streaming rate.
//
// Per step of 32 keys (two 16-key tiles a, b), with lane = (n = lane%16, kg = lane/16):
//   S^T[key, head] = K[key, :] . Q[head, :]    8x mfma 16x16x32; A = K rows straight from
//                                              global memory (16 B per lane), B = Q
//   lane then owns 8 scores of ONE head n: keys 4kg+r (tile a) and 16+4kg+r (tile b);
//   running softmax in registers; the max/sum across kg = lanes n, n+16, n+32, n+48 is a
//   two-step xor shuffle
//   O^T[d, head] += V^T[d, keys] . P^T[keys, head]   8x mfma 16x16x32; the 8 probabilities a
//                                              lane owns are exactly its B-operand slots;
//                                              A = V^T is built in-lane: the lane loads the
//                                              same 8 d-columns (16 B) of its 8 keys and
//                                              transposes 8x8 with byte permutes.
// Results leave through LDS, so that every store instruction writes whole contiguous rows (in
// the accumulator layout a lane's 16 bytes sit 64 bytes apart), with non-temporal stores, and
// a wave that walks several units keeps their rows there until it is done: writes sprinkled into
// the saturated read stream cost this kernel many times their bytes (with 8 query heads per KV
// head about 7 % of its time).
// Loads for the next step are issued before the current step is computed (two register
// buffers).  Rows outside [lo, hi] are masked with selects, never multiplied: stale or
// poisoned cache slots cannot leak; V rows of masked keys are zeroed.
#pragma once

#include <math.h>

#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {

struct StepBuf {
  frag8 k[2][4];  // [tile][k-step]: K[key = tile*16 + n][d = (4t + kg)*8 ..+8]
  frag8 v[8];     // [e]: V[key = (e/4)*16 + 4kg + e%4][d = n*8 ..+8]
};

// kBlock16: cache blocks of 16 tokens, so the two 16-key tiles of a step lie in two blocks (the
// second is clamped to blk_last, the unit's last block; its keys are then masked).  Otherwise a
// step lies inside one block (block size a multiple of 32, steps start at multiples of 32).
template <typename T, bool kBlock16>
__device__ __forceinline__ void load_step(StepBuf& b, const T* __restrict__ kc,
                                          const T* __restrict__ vc, const int32_t* bt, int key0,
                                          int B, int n_kv_heads, int hk, int n, int kg, int blk_last) {
  if constexpr (kBlock16) {
    const int blk_a = key0 >> 4;  // uniform; key0 is a multiple of 16
    const int blk_b = min(blk_a + 1, blk_last);
    const int64_t phys_a = load_uniform_i32(bt + blk_a), phys_b = load_uniform_i32(bt + blk_b);
    const int64_t base_a = (phys_a * n_kv_heads + hk) * (16 * kHeadDim);
    const int64_t base_b = (phys_b * n_kv_heads + hk) * (16 * kHeadDim);
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const T* kb = kc + (tile ? base_b : base_a);
#pragma unroll
      for (int t = 0; t < 4; ++t) b.k[tile][t] = load_frag8_stream(kb + n * kHeadDim + (4 * t + kg) * 8);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e)
      b.v[e] = load_frag8_stream(vc + ((e >> 2) ? base_b : base_a) + (4 * kg + (e & 3)) * kHeadDim + n * 8);
    return;
  }
  const int blk = key0 / B;                      // uniform
  const int64_t phys = load_uniform_i32(bt + blk);
  const int slot0 = key0 - blk * B;
  const int64_t base = ((phys * n_kv_heads + hk) * B + slot0) * kHeadDim;
  const T* kb = kc + base;
  const T* vb = vc + base;
#pragma unroll
  for (int tile = 0; tile < 2; ++tile)
#pragma unroll
    for (int t = 0; t < 4; ++t)
      b.k[tile][t] = load_frag8_stream(kb + (tile * 16 + n) * kHeadDim + (4 * t + kg) * 8);
#pragma unroll
  for (int e = 0; e < 8; ++e)
    b.v[e] = load_frag8_stream(vb + ((e >> 2) * 16 + 4 * kg + (e & 3)) * kHeadDim + n * 8);
}

// [lo, hi]: keys the lane's column counts (its row's visible keys inside the unit); [nm_lo, nm_hi]:
// keys that every column of the unit counts (a step inside needs no mask); [v_lo, v_hi]: keys that
// any column counts (the V rows of all others are zeroed: they may be stale or not the unit's).
template <int DT>
__device__ __forceinline__ void compute_step(StepBuf& b, const frag8 (&qf)[4], f32x4_t (&acc)[8],
                                             float& m, float& l, float sl2, int key0, int lo,
                                             int hi, int nm_lo, int nm_hi, int v_lo, int v_hi, int kg) {
  using M = Mma<DT>;
  f32x4_t sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    sa = M::mfma16(b.k[0][t], qf[t], sa);
    sb = M::mfma16(b.k[1][t], qf[t], sb);
  }
  float s[8];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    s[r] = sa[r] * sl2;
    s[4 + r] = sb[r] * sl2;
  }
  const bool boundary = key0 < nm_lo || key0 + 31 > nm_hi;  // uniform
  if (boundary) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int key = key0 + (e >> 2) * 16 + 4 * kg + (e & 3);
      if (key < lo || key > hi) s[e] = -INFINITY;
      if (key < v_lo || key > v_hi) b.v[e] = zero_frag8();
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx);  // m starts finite, so m_new is finite
  const float corr = fast_exp2(m - m_new);
  m = m_new;
  float pr[8], sum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    pr[e] = fast_exp2(s[e] - m_new);
    sum += pr[e];
  }
  l = l * corr + sum;  // per-lane partial; the four kg lanes are added at the end
#pragma unroll
  for (int c = 0; c < 8; ++c)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[c][r] *= corr;
  frag8 pf;
#pragma unroll
  for (int j = 0; j < 4; ++j) pf.w[j] = M::pack2(pr[2 * j], pr[2 * j + 1]);
  // V^T fragments: column c of the lane's 8 d-columns, over its 8 keys
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    frag8 a;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t w0 = b.v[2 * j].w[c >> 1], w1 = b.v[2 * j + 1].w[c >> 1];
      a.w[j] = (c & 1) ? pack_hi16(w0, w1) : pack_lo16(w0, w1);
    }
    acc[c] = M::mfma16(a, pf, acc[c]);
  }
}

constexpr int kDecodeStageBytes = 16 * kHeadDim * 4;  // per wave: 16 heads x 128 floats

typedef __attribute__((address_space(3))) char decode_lds_char;

// n_bytes of finished rows from LDS to global memory, 16 bytes per lane, consecutive lanes to
// consecutive addresses, non-temporal
__device__ __forceinline__ void store_rows(char* dst, decode_lds_char* src, int n_bytes, int lane) {
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) u4 lds_u4;
  for (int off = lane * 16; off < n_bytes; off += 1024)
    __builtin_nontemporal_store(*reinterpret_cast<lds_u4*>(src + off), reinterpret_cast<u4*>(dst + off));
}

// The record of launch slot `slot`, as two 16-byte loads from an address that is the same in every lane.
__device__ __forceinline__ UnitRec load_unit_rec(const FastPlan& f, int slot) {
  typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
  const i32x4* r = reinterpret_cast<const i32x4*>(f.dec_rec + slot);
  const i32x4 a = r[0], b = r[1];
  return UnitRec{a[0], a[1], a[2], a[3], b[0], b[1], {0, 0}};
}

// One wavefront: unit = (launch slot, kv head); rec = the slot's record (item = a slice of a
// sequence's rows and a run of its cache blocks).  stage: kDecodeStageBytes of LDS that belong to this wave alone.
// hold: if not null, the finished rows of an uncut one-row unit (g heads x 256 bytes) are left
// there instead of being stored, and the byte offset in `out` where they belong is returned for
// the caller to store them later; otherwise, for units of several rows and for units that
// write partial results, -1.
template <int DT, typename T, bool kBlock16, bool kDouble = true>
__device__ __forceinline__ int64_t decode_unit(const Pass& p, const FastPlan& f, const T* __restrict__ q,
                                               const T* __restrict__ kc, const T* __restrict__ vc,
                                               T* __restrict__ out, const UnitRec& rec, int hk, int lane,
                                               decode_lds_char* stage, decode_lds_char* hold) {
  const int n = lane & 15, kg = lane >> 4;
  const int s = rec.seq;
  const fsf_seq_desc sd = {rec.n_new, rec.n_cached, rec.q_offset, 0};
  const int B = p.block_size;
  const int g = p.group;
  // the sequence's key cuts: over the blocks any of its rows sees, the same for every slice
  int lo_seq, hi_seq, tmp;
  visible_range(sd.n_cached, p.window, lo_seq, tmp);
  visible_range(sd.n_cached + sd.n_new - 1, p.window, tmp, hi_seq);
  const int b_lo = lo_seq / B, b_hi = hi_seq / B;
  const int nblk = b_hi - b_lo + 1;
  const int n_splits = decode_splits(nblk, f.split_blocks, f.min_item_blocks);
  const int idx = rec.idx;  // slice-major
  const int slice = idx / n_splits;
  const int split = idx - slice * n_splits;
  // the slice's rows, and the keys they see
  const int rps = stream_rows_per_slice(g);
  const int r0 = slice * rps;
  const int rows = min(rps, sd.n_new - r0);  // >= 1
  int lo_u, hi_u, lo_last;                   // keys any row sees; first key the last row sees
  visible_range(sd.n_cached + r0, p.window, lo_u, tmp);
  visible_range(sd.n_cached + r0 + rows - 1, p.window, lo_last, hi_u);
  const int hi_first = sd.n_cached + r0;     // last key the first row sees
  // even cut: split k owns blocks [k*nblk/n_splits, (k+1)*nblk/n_splits), never empty
  const int blk0 = b_lo + (int)((int64_t)split * nblk / n_splits);
  const int blk1 = b_lo + (int)((int64_t)(split + 1) * nblk / n_splits) - 1;
  const int key_begin = max(blk0 * B, lo_u & ~31);
  const int key_end = min((blk1 + 1) * B - 1, hi_u);  // inclusive; below key_begin if no row of the slice sees the cut
  // keys this unit counts: a step may reach past them (into the next unit's blocks when the
  // block size is 16, past the window or the last token otherwise); those scores are masked
  const int vis_lo = max(lo_u, key_begin), vis_hi = key_end;
  const int32_t* bt = p.block_tables + (int64_t)s * p.max_blocks;

  // column n = (row r0 + n / g, head hk * g + n % g)
  const int r = n / g;
  const int h = n - r * g;
  const bool col_live = r < rows;
  const int row = r0 + (col_live ? r : rows - 1);
  const int hq = hk * g + (col_live ? h : 0);
  int lo_n, hi_n;
  visible_range(sd.n_cached + row, p.window, lo_n, hi_n);
  lo_n = max(lo_n, vis_lo);
  hi_n = min(hi_n, vis_hi);
  const int nm_lo = max(lo_last, vis_lo), nm_hi = min(hi_first, vis_hi);
  frag8 qf[4];
  {
    const T* qrow = q + ((int64_t)(sd.q_offset + row) * p.n_q_heads + hq) * kHeadDim;
#pragma unroll
    for (int t = 0; t < 4; ++t) qf[t] = col_live ? load_frag8(qrow + (4 * t + kg) * 8) : zero_frag8();
  }
  f32x4_t acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m = -1e30f, l = 0.f;
  const float sl2 = p.scale * 1.4426950408889634f;

  if (key_end >= key_begin) {
  if constexpr (kDouble) {
  // Two register buffers.  The steady-state loop issues every load unconditionally, so the
  // compiler's in-order wait counts let step i compute while all of step i+1 is in flight.
  StepBuf b0, b1;
  const int n_steps = (key_end - key_begin) / 32 + 1;
  int i = 0;
  load_step<T, kBlock16>(b0, kc, vc, bt, key_begin, B, p.n_kv_heads, hk, n, kg, blk1);
  for (; i + 2 < n_steps; i += 2) {
    const int key0 = key_begin + 32 * i;
    load_step<T, kBlock16>(b1, kc, vc, bt, key0 + 32, B, p.n_kv_heads, hk, n, kg, blk1);
    compute_step<DT>(b0, qf, acc, m, l, sl2, key0, lo_n, hi_n, nm_lo, nm_hi, vis_lo, vis_hi, kg);
    load_step<T, kBlock16>(b0, kc, vc, bt, key0 + 64, B, p.n_kv_heads, hk, n, kg, blk1);
    compute_step<DT>(b1, qf, acc, m, l, sl2, key0 + 32, lo_n, hi_n, nm_lo, nm_hi, vis_lo, vis_hi, kg);
  }
  {
    const int key0 = key_begin + 32 * i;
    if (n_steps - i == 2) {
      load_step<T, kBlock16>(b1, kc, vc, bt, key0 + 32, B, p.n_kv_heads, hk, n, kg, blk1);
      compute_step<DT>(b0, qf, acc, m, l, sl2, key0, lo_n, hi_n, nm_lo, nm_hi, vis_lo, vis_hi, kg);
      compute_step<DT>(b1, qf, acc, m, l, sl2, key0 + 32, lo_n, hi_n, nm_lo, nm_hi, vis_lo, vis_hi, kg);
    } else {
      compute_step<DT>(b0, qf, acc, m, l, sl2, key0, lo_n, hi_n, nm_lo, nm_hi, vis_lo, vis_hi, kg);
    }
  }

  } else {
    // one register buffer: latency is hidden by the other waves of the compute unit
    StepBuf b0;
    for (int key0 = key_begin; key0 <= key_end; key0 += 32) {
      load_step<T, kBlock16>(b0, kc, vc, bt, key0, B, p.n_kv_heads, hk, n, kg, blk1);
      compute_step<DT>(b0, qf, acc, m, l, sl2, key0, lo_n, hi_n, nm_lo, nm_hi, vis_lo, vis_hi, kg);
    }
  }
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  // acc[c][r4] is output column d = (4kg + r4)*8 + c of column n.  The g heads of a row are
  // adjacent in memory (out and the partial buffer alike): staged column-major in LDS (a row's
  // heads side by side), then written 16 bytes per lane, consecutive lanes to consecutive addresses.
  typedef uint32_t stage_u4 __attribute__((ext_vector_type(4)));
  typedef float stage_f4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) stage_u4 lds_u4;
  typedef __attribute__((address_space(3))) stage_f4 lds_f4;
  if (n_splits == 1) {
    // (a flag, not a comparison of the pointers: the staging area may sit at LDS address 0, which is
    // also what a null LDS pointer compares equal to)
    const bool held = hold && sd.n_new == 1;
    decode_lds_char* staged = held ? hold : stage;
    if (col_live) {
      const float inv = 1.f / l;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        stage_u4 w;
        w.x = Mma<DT>::pack2(acc[0][r4] * inv, acc[1][r4] * inv);
        w.y = Mma<DT>::pack2(acc[2][r4] * inv, acc[3][r4] * inv);
        w.z = Mma<DT>::pack2(acc[4][r4] * inv, acc[5][r4] * inv);
        w.w = Mma<DT>::pack2(acc[6][r4] * inv, acc[7][r4] * inv);
        *reinterpret_cast<lds_u4*>(staged + n * (kHeadDim * 2) + (4 * kg + r4) * 16) = w;
      }
    }
    __builtin_amdgcn_wave_barrier();  // one wave: its LDS accesses complete in program order
    const int64_t row_stride = (int64_t)p.n_q_heads * kHeadDim * (int64_t)sizeof(T);
    const int64_t dst = ((int64_t)(sd.q_offset + r0) * p.n_q_heads + hk * g) * kHeadDim * (int64_t)sizeof(T);
    if (held) return dst;
    for (int rr = 0; rr < rows; ++rr)
      store_rows(reinterpret_cast<char*>(out) + dst + rr * row_stride, staged + rr * g * (kHeadDim * 2), g * kHeadDim * 2, lane);
    __builtin_amdgcn_wave_barrier();  // the staging area is reused by the wave's next unit
  } else {
    // partial row of (cut, row): dec_prow_start[s] + cut * n_new + row
    const int64_t prow0 = (int64_t)rec.prow_start + (int64_t)split * sd.n_new + r0;
    if (col_live) {
      if (kg == 0) {
        const int64_t pi = (prow0 + r) * p.n_q_heads + hq;
        f.part_ml[pi * 2] = m;
        f.part_ml[pi * 2 + 1] = l;
      }
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const stage_f4 lo4 = {acc[0][r4], acc[1][r4], acc[2][r4], acc[3][r4]};
        const stage_f4 hi4 = {acc[4][r4], acc[5][r4], acc[6][r4], acc[7][r4]};
        *reinterpret_cast<lds_f4*>(stage + n * (kHeadDim * 4) + (4 * kg + r4) * 32) = lo4;
        *reinterpret_cast<lds_f4*>(stage + n * (kHeadDim * 4) + (4 * kg + r4) * 32 + 16) = hi4;
      }
    }
    __builtin_amdgcn_wave_barrier();
    const int n_bytes = g * kHeadDim * 4;
    for (int rr = 0; rr < rows; ++rr) {
      char* pbase = reinterpret_cast<char*>(f.part_acc + ((prow0 + rr) * p.n_q_heads + hk * g) * kHeadDim);
      decode_lds_char* src = stage + rr * n_bytes;
#pragma unroll
      for (int j = 0; j < 8; ++j) {  // 1 KB = 2 heads per instruction
        const int off = j * 1024 + lane * 16;
        if (off < n_bytes) __builtin_nontemporal_store(*reinterpret_cast<lds_f4*>(src + off), reinterpret_cast<stage_f4*>(pbase + off));
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
  return -1;
}


}  // namespace fsf
