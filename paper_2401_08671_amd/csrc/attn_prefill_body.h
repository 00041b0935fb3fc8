// Device code for prompt chunks (n_new > 1): tiled matrix-core attention over the blocked cache.
//
// A chunk of a split prompt attends causally to its own rows and to every chunk cached by
// earlier passes (paper Sec. 3.2 rule 1; Sec. 2 prompt processing).  Work is dense
// contraction: 4*d flops per (row, visible key), so it belongs on the matrix cores.
//
// One workgroup (8 waves) owns a tile of 8*32*NQ consecutive rows of one sequence and one
// query head; wave w owns 32*NQ of them.  Keys are taken 64 at a time (never straddling a
// cache block since block_size % 64 == 0), gathered through the block table:
//   HBM/L2 -> LDS directly (global_load_lds, 16 bytes per lane, no registers, no VALU).
//     Both tiles stay row-major [64 keys][128 d]; the lane -> global chunk mapping applies an
//     XOR swizzle so the later reads are bank-conflict free:
//       K: 16-byte chunk c of key row r sits at chunk c ^ (r & 7)
//       V: 32-byte segment s of key row r sits at segment s ^ (r & 7)
//     Rows past the sequence's last token are fetched from its last token instead: their
//     scores are masked, and a finite stand-in keeps 0 * garbage out of the second product.
//   S^T[key, row] = K . Q^T     A = K rows (ds_read_b128), B = Q^T held in registers
//   running softmax per row in registers: a lane owns 32 scores of one row per q-tile, the
//   max across the two half-waves is one xor-32 shuffle; the running reference is only
//   raised when a maximum outgrows it by 2^8 (lazy rescale), so the accumulators are not
//   touched by VALU code in the steady state
//   O^T[d, row] += V^T . P^T    A = V^T read from the row-major V tile with the transposing
//                               LDS read (ds_read_b64_tr_b16: a 16-lane group reads 4 keys x
//                               16 d and each lane receives 4 keys of one d); B = P^T = the
//                               lane's own probabilities, no cross-lane movement
// Four LDS stages (separate arrays, so the compiler can tell the stages being filled from
// the stage being read): the copies for steps j+1..j+3 are in flight while step j is
// computed, which hides the HBM/L2 latency of a gathered block; one barrier per step.
#pragma once

#include <math.h>

#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {

constexpr int kPrefillWaves = 8;
constexpr int NQ = kPrefillTileM / (32 * kPrefillWaves);  // 32-row q-tiles per wave
constexpr int kStages = 4;                                // LDS stages (prefetch distance kStages - 1)
constexpr int kKeysPerStep = 64;
constexpr int kTileBytes = 64 * 256;         // one K or V tile: [64 keys][128 d] of 2-byte elements
constexpr int kStageBytes = 2 * kTileBytes;  // K tile + V tile
constexpr int kFragAhead = 4;                // K fragments in flight from LDS (k-steps)
constexpr int kVAhead = 4;                   // V^T fragments in flight from LDS
constexpr float kLazyLog2 = 8.f;             // running-max slack before accumulators are rescaled

typedef __attribute__((address_space(3))) char lds_char;
typedef short v4s16 __attribute__((ext_vector_type(4)));

// Start the asynchronous copy of one 64-key step (K and V tiles) into an LDS stage.
// Each of the 8 waves copies 8 key rows: 2 instructions x (4 rows x 256 B) per tile.
constexpr int kCopyInstrPerStep = 2 * (64 / kPrefillWaves / 4);  // per wave: K + V
template <typename T>
__device__ __forceinline__ void stage_step(lds_char* stage, const T* __restrict__ kc,
                                           const T* __restrict__ vc, const int32_t* bt, int key0,
                                           int B, int n_kv_heads, int hk, int wave, int lane,
                                           int kv_last) {
  const int blk = key0 / B;
  const int64_t phys = load_uniform_i32(bt + blk);
  const int64_t base = ((phys * n_kv_heads + hk) * B + (key0 - blk * B)) * kHeadDim;
  const char* kb = reinterpret_cast<const char*>(kc + base);
  const char* vb = reinterpret_cast<const char*>(vc + base);
  const int max_row = kv_last - key0;  // >= 0: last row of this step that holds a written token
  const int pc = lane & 15;            // physical 16-byte chunk this lane fills
#pragma unroll
  for (int i = 0; i < 64 / kPrefillWaves / 4; ++i) {
    const int row0 = wave * (64 / kPrefillWaves) + i * 4;  // first of the 4 rows this instruction fills (uniform)
    const int row = row0 + (lane >> 4);
    const int src_row = row < max_row ? row : max_row;
    const char* ksrc = kb + src_row * 256 + ((pc ^ (row & 7)) << 4);
    const char* vsrc = vb + src_row * 256 + ((pc ^ ((row & 7) << 1)) << 4);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ksrc,
                                     (__attribute__((address_space(3))) void*)(stage + row0 * 256),
                                     16, 0, 0);
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)vsrc,
        (__attribute__((address_space(3))) void*)(stage + kTileBytes + row0 * 256), 16, 0, 0);
  }
}

// byte offset of 16-byte chunk `chunk` of key row `key` in the K tile
__device__ __forceinline__ int k_lds_off(int key, int chunk) {
  return key * 256 + ((chunk ^ (key & 7)) << 4);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ frag8 lds_load_frag8(const lds_char* ptr) {
  const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(ptr);
  return frag8{{v[0], v[1], v[2], v[3]}};
}

// 8 storage elements V[keys][d] for the A operand of O^T += V^T P^T: lane (d = mt*32 + l32,
// k-group hg), k-step u.  Slots 0..3 are keys 16u + 4hg + 0..3, slots 4..7 keys 16u + 8 + 4hg
// + 0..3 (the order in which the first product leaves the probabilities in registers).
// ds_read_b64_tr_b16 works on 16-lane groups: the group's lanes point at 4 key rows x 4
// 8-byte units (lane s: row s/4, unit s%4) and lane i receives, for d = unit_base + i, the
// 4 keys.  Group g of the wave covers d half (g & 1) and k-group g >> 1.
__device__ __forceinline__ frag8 load_vt_frag(const lds_char* vtile, int u, int mt, int lane) {
  const int s = lane & 15, g = lane >> 4;
  const int hg = g >> 1, dhalf = g & 1;
  const int seg = 2 * mt + dhalf;  // logical 32-byte segment of the row
  frag8 f;
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int row = 16 * u + 8 * r + 4 * hg + (s >> 2);
    const int off = row * 256 + ((seg ^ (row & 7)) << 5) + ((s & 3) << 3);
    const v4s16 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (v4s16 __attribute__((address_space(3)))*)(vtile + off));
    const uint2 w = __builtin_bit_cast(uint2, v);
    f.w[2 * r] = w.x;
    f.w[2 * r + 1] = w.y;
  }
  return f;
}

struct PrefillState {
  f32x16_t acc[4][NQ];
  float m_run[NQ], l_run[NQ];
};

// One 64-key step for one wave, reading the tiles of `stage`.
template <int DT>
__device__ __forceinline__ void prefill_compute_step(PrefillState& st, const lds_char* stage,
                                                     const frag8 (&qf)[NQ][8],
                                                     const int (&row_pos)[NQ], int key0, int window,
                                                     float sl2, bool need_mask, int l32, int hg,
                                                     int lane) {
  using M = Mma<DT>;
  const lds_char* kl = stage;
  const lds_char* vl = stage + kTileBytes;

  // ---- S^T = K . Q^T ; K fragments are fetched from LDS kFragAhead k-steps ahead of their use
  f32x16_t sc[2][NQ];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[kt][qt][r] = 0.f;
  {
    frag8 kf[kFragAhead][2];
#pragma unroll
    for (int t = 0; t < kFragAhead; ++t)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        kf[t][kt] = lds_load_frag8(kl + k_lds_off(kt * 32 + l32, 2 * t + hg));
#pragma unroll
    for (int t = 0; t < 8; ++t) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt)
          sc[kt][qt] = M::mfma32(kf[t % kFragAhead][kt], qf[qt][t], sc[kt][qt]);
        if (t + kFragAhead < 8)
          kf[t % kFragAhead][kt] =
              lds_load_frag8(kl + k_lds_off(kt * 32 + l32, 2 * (t + kFragAhead) + hg));
      }
    }
    // pin the issue order: kFragAhead k-steps of LDS reads up front, then reads and MFMAs in turn
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * kFragAhead, 0);
#pragma unroll
    for (int t = 0; t < 8 - kFragAhead; ++t) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * NQ, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * NQ * kFragAhead, 0);
  }

  // ---- mask, row maxima, and the (rare) raise of the running reference
  if (need_mask) {
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
      int rlo, rhi;
      visible_range(row_pos[qt], window, rlo, rhi);  // rows past the tile: rhi = -1, nothing visible
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + kt * 32 + 8 * (r >> 2) + 4 * hg + (r & 3);
          if (key < rlo || key > rhi) sc[kt][qt][r] = -INFINITY;
        }
    }
  }
  // Lazy rescale: the running reference m_run only has to bound the scores from above
  // loosely.  It is raised (and acc, l rescaled) only when a row's maximum outgrows it by
  // more than 2^kLazyLog2, so probabilities stay <= 2^kLazyLog2.
  float m_cand[NQ];
  bool raise = false;
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[kt][qt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    m_cand[qt] = fmaxf(st.m_run[qt], mx * sl2);
    raise |= m_cand[qt] - st.m_run[qt] > kLazyLog2;
  }
  if (__builtin_amdgcn_ballot_w64(raise) != 0) {
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
      const float m_new = (m_cand[qt] - st.m_run[qt] > kLazyLog2) ? m_cand[qt] : st.m_run[qt];
      const float corr = fast_exp2(st.m_run[qt] - m_new);
      st.m_run[qt] = m_new;
      st.l_run[qt] *= corr;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.acc[mt][qt][r] *= corr;
    }
  }

  // ---- probabilities and P^T fragments
  frag8 pfr[NQ][4];
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    const float m_ref = st.m_run[qt];
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = fast_exp2(fmaf(sc[kt][qt][r], sl2, -m_ref));
        sc[kt][qt][r] = pr;
        sum += pr;
      }
    st.l_run[qt] += sum;
    // k-step u of the second product covers keys 16u..16u+15: registers 8(u%2)..+7 of tile u/2
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
        pfr[qt][u].w[jj] = M::pack2(sc[u >> 1][qt][8 * (u & 1) + 2 * jj],
                                    sc[u >> 1][qt][8 * (u & 1) + 2 * jj + 1]);
  }

  // ---- O^T += V^T . P^T ; V^T fragments come from LDS kVAhead MFMAs ahead of their use
  frag8 vf[kVAhead];  // rolling window over i = u*4 + mt
#pragma unroll
  for (int i = 0; i < kVAhead; ++i) vf[i] = load_vt_frag(vl, i >> 2, i & 3, lane);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int u = i >> 2, mt = i & 3;
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
      st.acc[mt][qt] = M::mfma32(vf[i % kVAhead], pfr[qt][u], st.acc[mt][qt]);
    if (i + kVAhead < 16)
      vf[i % kVAhead] = load_vt_frag(vl, (i + kVAhead) >> 2, (i + kVAhead) & 3, lane);
  }
  __builtin_amdgcn_sched_group_barrier(0x100, 2 * kVAhead, 1);
#pragma unroll
  for (int i = 0; i < 16 - kVAhead; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, NQ, 1);
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, NQ * kVAhead, 1);
}

// One workgroup of 32*kPrefillWaves threads: tile = index into the pass's prefill tiles,
// hq = query head.  lds0..lds3: LDS stages of kStageBytes each (distinct arrays).
template <int DT, typename T>
__device__ __forceinline__ void prefill_tile(const Pass& p, const FastPlan& f,
                                             const T* __restrict__ q, const T* __restrict__ kc,
                                             const T* __restrict__ vc, T* __restrict__ out, int tile,
                                             int hq, lds_char* lds0, lds_char* lds1, lds_char* lds2,
                                             lds_char* lds3) {
  using M = Mma<DT>;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, hg = lane >> 5;
  const int hk = hq / p.group;
  const int s = f.pre_tile_seq[tile];  // written by the planning kernel
  const fsf_seq_desc sd = p.descs[s];
  const int B = p.block_size;
  const int n_new = sd.n_new, c = sd.n_cached;
  const int i0 = (tile - f.pre_tile_start[s]) * kPrefillTileM;  // first row of the tile
  const int i1 = min(i0 + kPrefillTileM, n_new);                // one past its last row
  const int32_t* bt = p.block_tables + (int64_t)s * p.max_blocks;

  // key range of the whole tile (all waves walk the same steps: they share the LDS tiles)
  int lo_t, hi_t, tmp;
  visible_range(c + i0, p.window, lo_t, tmp);
  visible_range(c + i1 - 1, p.window, tmp, hi_t);
  const int key_begin = lo_t & ~(kKeysPerStep - 1);
  const int kv_last = c + n_new - 1;  // last cache position this sequence has written

  // this wave's rows
  const int w_i0 = i0 + wave * 32 * NQ;
  const int w_i1 = min(w_i0 + 32 * NQ, i1);  // may be <= w_i0: wave has no live row
  const bool wave_live = w_i0 < i1;
  int w_lo_min = 0, w_lo_max = 0, w_hi_min = 0, w_hi_max = -1;
  if (wave_live) {
    visible_range(c + w_i0, p.window, w_lo_min, w_hi_min);
    visible_range(c + w_i1 - 1, p.window, w_lo_max, w_hi_max);
  }

  // Q^T fragments (B operand): lane = (row l32 of q-tile, k-group hg), k-step t -> d chunk 2t+hg
  frag8 qf[NQ][8];
  int row_pos[NQ];  // absolute position of the lane's row per q-tile (rows past the tile: -1)
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    const int i = w_i0 + qt * 32 + l32;
    const bool live = i < i1;
    row_pos[qt] = live ? c + i : -1;
    const int ic = live ? i : (i1 - 1);
    const T* qrow = q + ((int64_t)(sd.q_offset + ic) * p.n_q_heads + hq) * kHeadDim;
#pragma unroll
    for (int t = 0; t < 8; ++t) qf[qt][t] = load_frag8(qrow + (2 * t + hg) * 8);
  }

  PrefillState st;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.acc[mt][qt][r] = 0.f;
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    st.m_run[qt] = -1e30f;
    st.l_run[qt] = 0.f;
  }
  const float sl2 = p.scale * 1.4426950408889634f;

  // Copies run kStages-1 steps ahead.  The loop is unrolled by kStages so that every
  // sub-iteration names its stages statically.  A wave waits for its own part of step j with
  // vmcnt(newer copy instructions), the barrier extends that to the whole workgroup and also
  // says that everyone is done reading the stage that step j+3 will overwrite.
  lds_char* const stages[kStages] = {lds0, lds1, lds2, lds3};
#pragma unroll
  for (int a = 0; a < kStages - 1; ++a)
    if (key_begin + a * kKeysPerStep <= hi_t)
      stage_step(stages[a], kc, vc, bt, key_begin + a * kKeysPerStep, B, p.n_kv_heads, hk, wave, lane, kv_last);

  for (int key0 = key_begin; key0 <= hi_t; key0 += kStages * kKeysPerStep) {
#pragma unroll
    for (int sub = 0; sub < kStages; ++sub) {
      const int k0 = key0 + sub * kKeysPerStep;
      if (k0 > hi_t) break;
      // copy instructions of this wave issued after those of step k0
      const int newer = min(kStages - 2, (hi_t - k0) / kKeysPerStep);
      // (0x0070 = expcnt unused, lgkmcnt(0): this wave's LDS reads of the previous step are back)
      if (newer >= 2)
        __builtin_amdgcn_s_waitcnt(0x0070 | (2 * kCopyInstrPerStep));
      else if (newer == 1)
        __builtin_amdgcn_s_waitcnt(0x0070 | kCopyInstrPerStep);
      else
        __builtin_amdgcn_s_waitcnt(0x0070);
      // bare barrier: a full __syncthreads() would also wait for the copies still in flight
      __builtin_amdgcn_s_barrier();
      if (k0 + (kStages - 1) * kKeysPerStep <= hi_t)
        stage_step(stages[(sub + kStages - 1) % kStages], kc, vc, bt, k0 + (kStages - 1) * kKeysPerStep, B,
                   p.n_kv_heads, hk, wave, lane, kv_last);
      // hidden from every row of this wave?
      if (!wave_live || k0 > w_hi_max || k0 + kKeysPerStep - 1 < w_lo_min) continue;
      const bool need_mask =
          k0 + kKeysPerStep - 1 > w_hi_min || k0 < w_lo_max || w_i1 - w_i0 < 32 * NQ;
      prefill_compute_step<DT>(st, stages[sub], qf, row_pos, k0, p.window, sl2, need_mask, l32, hg, lane);
    }
  }

  // ---- normalise and store: acc[mt][qt][r] is column d = 32mt + 8(r/4) + 4hg + r%4 of the lane's row
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    float l = st.l_run[qt];
    l += __shfl_xor(l, 32);
    if (row_pos[qt] < 0) continue;
    const float inv = 1.f / l;
    const int i = row_pos[qt] - c;
    T* orow = out + ((int64_t)(sd.q_offset + i) * p.n_q_heads + hq) * kHeadDim;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        uint2 w;
        w.x = M::pack2(st.acc[mt][qt][4 * rq] * inv, st.acc[mt][qt][4 * rq + 1] * inv);
        w.y = M::pack2(st.acc[mt][qt][4 * rq + 2] * inv, st.acc[mt][qt][4 * rq + 3] * inv);
        *reinterpret_cast<uint2*>(orow + 32 * mt + 8 * rq + 4 * hg) = w;
      }
  }
}

}  // namespace fsf
