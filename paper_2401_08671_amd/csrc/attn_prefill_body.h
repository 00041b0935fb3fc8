// Device code for prompt chunks (n_new > 1): tiled matrix-core attention over the blocked cache.
//
// A chunk of a split prompt attends causally to its own rows and to every chunk cached by
// earlier passes (paper Sec. 3.2 rule 1; Sec. 2 prompt processing).  Work is dense
// contraction: 4*d flops per (row, visible key), so it belongs on the matrix cores.
//
// One workgroup (4 waves) owns a tile of 4*32*NQ consecutive rows of one sequence and one
// query head; wave w owns 32*NQ of them.  Keys are taken 64 at a time (never straddling a
// cache block since block_size % 64 == 0), gathered through the block table:
//   global -> registers (prefetched one step ahead) -> LDS
//     K   [64 keys][128 d], 16-byte chunks XOR-swizzled by key so that the 32x32x16
//         A-operand reads (32 consecutive keys, one chunk) spread over all banks
//     V^T [128 d][64 key slots]: transposed in registers (byte permutes) on the way in, with
//         the key order inside each 16 permuted so that the 8 keys a lane owns after the
//         first product are 16 contiguous bytes
//   S^T[key, row] = K . Q^T          (A = K from LDS, B = Q^T held in registers)
//   running softmax per row: a lane owns 32 scores of one row per q-tile, max/sum across
//   the two half-waves by one xor-32 shuffle
//   O^T[d, row] += V^T . P^T         (A = V^T from LDS, B = P^T = the lane's own scores,
//                                    no cross-lane movement)
// Masking (causal diagonal, window edge, rows past the chunk end) uses selects on the
// scores; wave-level tests skip steps that are entirely hidden from the wave's rows.
#pragma once

#include <math.h>

#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {

constexpr int NQ = kPrefillTileM / 128;  // 32-row q-tiles per wave
constexpr int kKeysPerStep = 64;
constexpr int kKTileBytes = 64 * 256;            // K tile [64 keys][128 d]
constexpr int kStageBytes = kKTileBytes + 128 * 128;  // + V^T tile [128 d][64 keys]
constexpr int kFragAhead = 4;                     // K fragments in flight from LDS (k-steps)
constexpr int kVAhead = 4;                        // V^T fragments in flight from LDS
constexpr int kPrefillLdsBytes = 2 * kStageBytes;
constexpr float kLazyLog2 = 8.f;  // running-max slack before accumulators are rescaled

struct Prefetch {
  frag8 k[4];
  frag8 v[4];
};

template <typename T>
__device__ __forceinline__ void prefetch_step(Prefetch& pf, const T* __restrict__ kc,
                                              const T* __restrict__ vc, const int32_t* bt,
                                              int key0, int B, int n_kv_heads, int hk, int tid,
                                              int kv_last) {
  const int blk = key0 / B;
  const int64_t phys = bt[blk];
  const int64_t base = ((phys * n_kv_heads + hk) * B + (key0 - blk * B)) * kHeadDim;
  const T* kb = kc + base;
  const T* vb = vc + base;
  const int dchunk = tid & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (tid >> 4) + 16 * i;
    pf.k[i] = load_frag8(kb + row * kHeadDim + dchunk * 8);
  }
  const int j = tid >> 4;  // keys 4j .. 4j+3
#pragma unroll
  for (int i = 0; i < 4; ++i) pf.v[i] = load_frag8(vb + (4 * j + i) * kHeadDim + dchunk * 8);
  // slots past the sequence's last token were never written: their V must not meet a
  // zero probability as NaN or Inf, so they are cleared (their scores are masked anyway)
  if (key0 + kKeysPerStep - 1 > kv_last) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (key0 + 4 * j + i > kv_last) pf.v[i] = zero_frag8();
  }
}

// byte offset of 16-byte chunk `chunk` of key row `key` in the K tile
__device__ __forceinline__ int k_lds_off(int key, int chunk) {
  return key * 256 + ((chunk ^ (key & 7)) << 4);
}
// byte offset of 16-byte chunk `chunk` (8 key slots) of row d in the V^T tile
__device__ __forceinline__ int vt_lds_off(int d, int chunk) {
  return d * 128 + ((chunk ^ ((d ^ (d >> 3)) & 7)) << 4);
}

__device__ __forceinline__ void store_step(const Prefetch& pf, char* k_lds, char* vt_lds, int tid) {
  const int dchunk = tid & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (tid >> 4) + 16 * i;
    *reinterpret_cast<uint4*>(k_lds + k_lds_off(row, dchunk)) =
        uint4{pf.k[i].w[0], pf.k[i].w[1], pf.k[i].w[2], pf.k[i].w[3]};
  }
  // V: this thread holds keys 4j..4j+3 x 8 d-columns; write 8 rows of 4 keys (8 bytes each)
  const int j = tid >> 4;
  const int key16 = (4 * j) & 15;
  const int b3 = (key16 >> 3) & 1, b2 = (key16 >> 2) & 1;
  const int chunk = 2 * (j >> 2) + b2;  // (16-key group)*2 + half
  const int sub = b3 * 8;               // byte offset inside the 16-byte chunk
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const uint32_t a0 = pf.v[0].w[c >> 1], a1 = pf.v[1].w[c >> 1];
    const uint32_t a2 = pf.v[2].w[c >> 1], a3 = pf.v[3].w[c >> 1];
    uint2 w;
    w.x = (c & 1) ? pack_hi16(a0, a1) : pack_lo16(a0, a1);
    w.y = (c & 1) ? pack_hi16(a2, a3) : pack_lo16(a2, a3);
    const int d = dchunk * 8 + c;
    *reinterpret_cast<uint2*>(vt_lds + vt_lds_off(d, chunk) + sub) = w;
  }
}

// One workgroup of 256 threads: tile = index into the pass's prefill tiles, hq = query head.
// lds: kPrefillLdsBytes of workgroup-shared memory.
template <int DT, typename T>
__device__ __forceinline__ void prefill_tile(const Pass& p, const FastPlan& f, const T* __restrict__ q,
                                             const T* __restrict__ kc, const T* __restrict__ vc,
                                             T* __restrict__ out, int tile, int hq, char* lds) {
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
  int row_pos[NQ];  // absolute position of the lane's row per q-tile (clamped rows: -1)
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

  f32x16_t acc[4][NQ];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][qt][r] = 0.f;
  float m_run[NQ], l_run[NQ];
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    m_run[qt] = -1e30f;
    l_run[qt] = 0.f;
  }
  const float sl2 = p.scale * 1.4426950408889634f;

  // Two LDS stages: while step j is computed from stage j&1, step j+1 sits in registers on its
  // way to stage (j+1)&1 and step j+2 is in flight from HBM/L2.  One barrier per step.
  Prefetch pre;
  prefetch_step(pre, kc, vc, bt, key_begin, B, p.n_kv_heads, hk, tid, kv_last);
  store_step(pre, lds, lds + kKTileBytes, tid);
  if (key_begin + kKeysPerStep <= hi_t)
    prefetch_step(pre, kc, vc, bt, key_begin + kKeysPerStep, B, p.n_kv_heads, hk, tid, kv_last);

  int stage = 0;
  for (int key0 = key_begin; key0 <= hi_t; key0 += kKeysPerStep, stage ^= 1) {
    __syncthreads();  // stage `stage` is complete; everyone is done reading stage^1
    if (key0 + kKeysPerStep <= hi_t) {
      store_step(pre, lds + (stage ^ 1) * kStageBytes, lds + (stage ^ 1) * kStageBytes + kKTileBytes, tid);
      if (key0 + 2 * kKeysPerStep <= hi_t)
        prefetch_step(pre, kc, vc, bt, key0 + 2 * kKeysPerStep, B, p.n_kv_heads, hk, tid, kv_last);
    }
    // hidden from every row of this wave?
    if (!wave_live || key0 > w_hi_max || key0 + kKeysPerStep - 1 < w_lo_min) continue;
    const char* kl = lds + stage * kStageBytes;
    const char* vl = kl + kKTileBytes;

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
        for (int kt = 0; kt < 2; ++kt) kf[t][kt] = load_frag8(kl + k_lds_off(kt * 32 + l32, 2 * t + hg));
#pragma unroll
      for (int t = 0; t < 8; ++t) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
          for (int qt = 0; qt < NQ; ++qt)
            sc[kt][qt] = M::mfma32(kf[t % kFragAhead][kt], qf[qt][t], sc[kt][qt]);
          if (t + kFragAhead < 8)
            kf[t % kFragAhead][kt] = load_frag8(kl + k_lds_off(kt * 32 + l32, 2 * (t + kFragAhead) + hg));
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
    const bool need_mask = key0 + kKeysPerStep - 1 > w_hi_min || key0 < w_lo_max || w_i1 - w_i0 < 32 * NQ;
    if (need_mask) {
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt) {
        int rlo, rhi;
        visible_range(row_pos[qt], p.window, rlo, rhi);  // dead rows: rhi = -1, nothing visible
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
    // more than 2^kLazyLog2, so probabilities stay <= 2^kLazyLog2 and the rescale of the
    // accumulator registers leaves the steady-state loop.
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
      m_cand[qt] = fmaxf(m_run[qt], mx * sl2);
      raise |= m_cand[qt] - m_run[qt] > kLazyLog2;
    }
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt) {
        const float m_new = (m_cand[qt] - m_run[qt] > kLazyLog2) ? m_cand[qt] : m_run[qt];
        const float corr = fast_exp2(m_run[qt] - m_new);
        m_run[qt] = m_new;
        l_run[qt] *= corr;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[mt][qt][r] *= corr;
      }
    }

    // ---- probabilities and P^T fragments
    frag8 pfr[NQ][4];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
      const float m_ref = m_run[qt];
      float sum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float pr = fast_exp2(fmaf(sc[kt][qt][r], sl2, -m_ref));
          sc[kt][qt][r] = pr;
          sum += pr;
        }
      l_run[qt] += sum;
      // k-step u of the second product covers keys 16u..16u+15: registers 8(u%2)..+7 of tile u/2
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
          pfr[qt][u].w[jj] = M::pack2(sc[u >> 1][qt][8 * (u & 1) + 2 * jj], sc[u >> 1][qt][8 * (u & 1) + 2 * jj + 1]);
    }

    // ---- O^T += V^T . P^T ; V^T fragments come from LDS kVAhead MFMAs ahead of their use
    frag8 vf[kVAhead];  // rolling window over i = u*4 + mt
#pragma unroll
    for (int i = 0; i < kVAhead; ++i) vf[i] = load_frag8(vl + vt_lds_off((i & 3) * 32 + l32, 2 * (i >> 2) + hg));
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int u = i >> 2, mt = i & 3;
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt) acc[mt][qt] = M::mfma32(vf[i % kVAhead], pfr[qt][u], acc[mt][qt]);
      if (i + kVAhead < 16)
        vf[i % kVAhead] = load_frag8(vl + vt_lds_off(((i + kVAhead) & 3) * 32 + l32, 2 * ((i + kVAhead) >> 2) + hg));
    }
    __builtin_amdgcn_sched_group_barrier(0x100, kVAhead, 1);
#pragma unroll
    for (int i = 0; i < 16 - kVAhead; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, NQ, 1);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, NQ * kVAhead, 1);
  }

  // ---- normalise and store: acc[mt][qt][r] is column d = 32mt + 8(r/4) + 4hg + r%4 of the lane's row
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    float l = l_run[qt];
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
        w.x = M::pack2(acc[mt][qt][4 * rq] * inv, acc[mt][qt][4 * rq + 1] * inv);
        w.y = M::pack2(acc[mt][qt][4 * rq + 2] * inv, acc[mt][qt][4 * rq + 3] * inv);
        *reinterpret_cast<uint2*>(orow + 32 * mt + 8 * rq + 4 * hg) = w;
      }
  }
}


}  // namespace fsf
