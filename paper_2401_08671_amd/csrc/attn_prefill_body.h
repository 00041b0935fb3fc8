// Device code for prompt chunks (n_new > 1): tiled matrix-core attention over the blocked cache.
//
// A chunk of a split prompt attends causally to its own rows and to every chunk cached by
// earlier passes (paper Sec. 3.2 rule 1; Sec. 2 prompt processing).  Work is dense
// contraction: 4*d flops per (row, visible key), so it belongs on the matrix cores.
//
// One workgroup (4 waves, one per SIMD) owns a tile of 128 consecutive rows of one sequence
// and one query head; wave w owns 32 of them.  Two workgroups share a compute unit, so every
// SIMD holds two waves that belong to different workgroups and never wait for each other:
// while one does its softmax the other keeps the matrix core busy.  (Two waves of ONE
// workgroup on a SIMD meet at the same barrier every step, start every step together and
// then queue for the same unit; measured, that costs a third of the throughput.)
//
// Keys are taken 64 at a time ("step"; never straddling a cache block since block_size % 64
// == 0), gathered through the block table:
//   HBM/L2 -> LDS directly (global_load_lds, 16 bytes per lane, no registers, no VALU).
//     Both tiles stay row-major [64 keys][128 d]; the lane -> global chunk mapping applies an
//     XOR swizzle so the later reads are bank-conflict free (64 banks):
//       K: 16-byte chunk c of key row r sits at chunk c ^ (r & 15)
//       V: 32-byte segment s of key row r sits at segment s ^ 2(r & 3)
//     Rows past the sequence's last token are fetched from its last token instead: their
//     scores are masked, and a finite stand-in keeps 0 * garbage out of the second product.
//   QK:  S^T[key, row] = K . Q^T   A = K rows (ds_read_b128), B = Q^T held in registers
//   softmax per row in registers: a lane owns 32 scores of one row, the max across the two
//     half-waves is one lane swap; the running reference is only raised when a maximum
//     outgrows it by 2^8 (lazy rescale), so the accumulators are rarely touched by VALU code
//   PV:  O^T[d, row] += V^T . P^T  A = V^T read from the row-major V tile with the transposing
//                                 LDS read (ds_read_b64_tr_b16), B = P^T = the lane's own
//                                 probabilities, no cross-lane movement
// Iteration b of a wave:  hand-over, QK(b), then PV(b-1) with the softmax of step b between
// its MFMAs ("PS"), so the vector ALU works in the shadow of the wave's own matrix work too.
//
// LDS (64 KB): two K slots and two V slots.  Hand-over b = wait for the wave's own copies of
// K(b) and V(b-1), workgroup barrier, start K(b+1) and V(b) in the slots that iteration b-1
// has finished reading.  One iteration (about 1 us) covers the latency of a gathered block.
#pragma once

#include <math.h>

#include <type_traits>

#include "attn_prefill_sequence.h"
#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {

constexpr int kPrefillWaves = 4;
static_assert(kPrefillTileM == 32 * kPrefillWaves, "one 32-row q-tile per wave");
constexpr int kRing = 2;                     // LDS slots per tile ring (K and V each)
constexpr int kKeysPerStep = 64;
constexpr int kTileBytes = 64 * 256;         // one K or V tile: [64 keys][128 d] of 2-byte elements
constexpr int kPrefillLdsBytes = 2 * kRing * kTileBytes;  // K slots 0, 1, then V slots 0, 1
constexpr int kVRingBase = kRing * kTileBytes;            // byte offset of V slot 0
constexpr float kLazyLog2 = 8.f;             // running-max slack before accumulators are rescaled
static_assert(kPrefillLdsBytes <= 65536, "LDS reads reach every slot with a 16-bit offset");
static_assert(kLazyLog2 == 8.f, "the PS sequence compares against the literal 0x41000000");

typedef __attribute__((address_space(3))) char lds_char;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Asynchronous copy of the K (or V) tile of one 64-key step into an LDS slot
// (global_load_lds: 16 bytes per lane, HBM/L2 -> LDS without passing registers).
// Each of the 4 waves copies 16 key rows with 4 instructions (4 rows x 256 B each).  The
// lane -> source-chunk mapping (which applies the swizzle) does not change from step to
// step, so a lane keeps its byte offset inside a (block, head) tile in a register and a
// copy costs a handful of scalar instructions for the tile's base address.
constexpr int kCopyInstrPerTile = 64 / kPrefillWaves / 4;
struct TileCopy {
  uint32_t lane_off[kCopyInstrPerTile];  // row*256 + swizzled chunk*16 of the lane's 16 bytes
  uint32_t lds_off[kCopyInstrPerTile];   // first byte the instruction fills inside a slot (uniform)
  template <bool kIsV>
  __device__ __forceinline__ void init(int wave, int lane) {
    const int pc = lane & 15;  // physical 16-byte chunk this lane fills
#pragma unroll
    for (int i = 0; i < kCopyInstrPerTile; ++i) {
      const int row0 = wave * (64 / kPrefillWaves) + i * 4;
      const int row = row0 + (lane >> 4);
      const int swz = kIsV ? ((row & 3) << 2) : (row & 15);
      lane_off[i] = row * 256 + ((pc ^ swz) << 4);
      lds_off[i] = row0 * 256;
    }
  }
  // tile_base: address of key row 0 of the step in the cache; slot: LDS byte address of the slot;
  // max_row: last row of the step that holds a written token (>= 0).  Rows past it are fetched
  // from row max_row instead.
  template <bool kClamp>
  __device__ __forceinline__ void issue(const char* tile_base, uint32_t slot, int max_row) const {
    // both are the same in all lanes; say so (the compiler cannot always tell)
    const uint64_t tb = reinterpret_cast<uint64_t>(tile_base);
    const uint64_t base = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(tb >> 32)) << 32) |
                          (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)tb);
#pragma unroll
    for (int i = 0; i < kCopyInstrPerTile; ++i) {
      uint32_t off = lane_off[i];
      if (kClamp) {  // only the last step of a sequence needs it
        const uint32_t row = off >> 8;
        off = ((row < (uint32_t)max_row ? row : (uint32_t)max_row) << 8) | (off & 255u);
      }
      // M0 = LDS address of lane 0's 16 bytes; lane l lands 16*l bytes further
      asm volatile("s_mov_b32 m0, %[m]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[v], %[s]\n\t"
                   :
                   : [m] "s"(__builtin_amdgcn_readfirstlane(slot + lds_off[i])), [v] "v"(off), [s] "s"(base)
                   : "memory");
    }
  }
};

// ---------------------------------------------------------------------------------------
// The whole walk of a tile over its steps is ONE fixed instruction sequence: LDS reads run a
// few fragments ahead of the MFMAs that consume them, every wait names exactly the reads it
// needs, the softmax of a step sits between the MFMAs of the PV before it, and a hand-over
// costs some twenty scalar instructions.  (Left to the compiler, the same loop issues two to
// three times as many instructions, and pinning parts of it makes its register allocation
// spill.)  Plain code around it sets the registers up and stores the result.
//
// Iteration b (b = 0 .. n_steps; both P buffers and both slot pairs alternate with b & 1):
//   hand-over b, QK(b) if step b is active for the wave, PV(b-1) if step b-1 is,
//   softmax(b) -> P buffer (b+1) & 1, with the scores of hidden keys set to -inf first where
//   the step needs it.
// Steady pairs: from an even b with  fast_lo <= b, b+1 <= fast_hi  the wave runs pairs of
// iterations without any test: both steps active, nothing masked, every copy whole.  There
// PV(b-1) and softmax(b) are one interleaved sequence (PS): row maximum (v_max3 chains,
// v_permlane32_swap for the other half-wave), lazy raise of the reference,
// p = 2^(s*scale*log2e - m), row sum, P^T register r = pack(p[2r], p[2r+1]); where the
// reference was raised the accumulators are scaled once the PV has landed.
//
// LDS addressing.  A read is  per-lane register + 16-bit immediate; the swizzles only touch
// address bits a lane fixes once:
//   K tile: lane (l32, hg) reads row kt*32 + l32, chunk 2t + hg for k-step t:
//     ka[t] = l32*256 + ((2t + hg) ^ (l32 & 15))*16, immediate = slot + kt*8192.  A
//     ds_read_b128 serves 16 lanes per clock from 64 banks, and 16 consecutive rows at one
//     logical chunk land on 16 different physical chunks.
//   V tile: ds_read_b64_tr_b16 works on 16-lane groups: the group's lanes point at 4 key rows
//     x 4 8-byte units (lane s: row s/4, unit s%4) and lane i receives, for d = unit_base + i,
//     the 4 keys.  Group g covers d half (g & 1) and key group hg = g >> 1.  For the A
//     operand of O^T += V^T P^T (lane d = mt*32 + l32, k-step u) slots 0..3 are keys 16u + 4hg
//     + 0..3 and slots 4..7 keys 16u + 8 + 4hg + 0..3 -- the order in which the first product
//     leaves the probabilities in registers:  va[mt] = V ring + x*256 + (2(mt ^ (x&3)) +
//     (g&1))*32 + (s&3)*8 with x = 4hg + s/4, immediate = slot + (16u + 8r)*256.  The read
//     serves 32 lanes per clock: 4 rows x 2 segments, spread over all 64 banks.
//
// Registers of the sequence:
//   v28 v29 temporaries of a clamped copy      v32 rhi - 4hg, v33 rlo - 4hg of the lane's row
//   (visible keys [rlo, rhi]; score register j of a lane is key 32(j/16) + 8((j%16)/4) + j%4 +
//   4hg of the step), v34 v35 the same minus the step's first key      v36..v39 V copy lane
//   offsets   v40 m  v41 l  v42 rescale factor  v43 scale*log2e   v44..v47 K copy lane offsets
//   v48 -inf   v50..v53 va   v54..v61 ka   v62..v93 Q^T fragments (k-step t: 4t..4t+3)
//   v94..v157 O^T (four 32x32 accumulators)   v158..v189 S^T (two 32x32 accumulators)
//   v190..v205, v206..v221 P^T buffers 0, 1     v222..v231 softmax temporaries
//   v232..v255 K / V^T fragments in flight
//   s60 n_steps   s61 s62 first, last active step of the wave   s63 s64 first, last step that
//   needs no mask   s65 s66 fast_lo, fast_hi   s67 last step with all 64 rows written   s68 last
//   written key - first key of the tile   s69 first key of the tile   s70 window   s71 first
//   step's index in the sequence (key/64)   s72 steps per cache block - 1   s73 log2 of steps
//   per block   s[74:75] block table of the sequence   s[76:77] K base of this head   s[78:79]
//   V base   s80 bytes per cache block   s81 LDS address of the wave's first copy row
//   s82..s89, s92, s93, s95, s96, s98, s99 temporaries   s[90:91] offset of step b's tiles   s94 physical
//   block of step b+1   s97 b
// Every block of MFMAs ends with the idle cycles the matrix core needs before vector code may
// read what the last MFMA wrote.
// The sequence itself (macro FSF_TILE_SEQUENCE, some 2000 instructions) is written by
// gen_prefill_sequence.py into attn_prefill_sequence.h; the build runs the generator first.
// ---------------------------------------------------------------------------------------
#define FSF_FRAG_REGS                                                                          \
  "v232", "v233", "v234", "v235", "v236", "v237", "v238", "v239", "v240", "v241", "v242",      \
      "v243", "v244", "v245", "v246", "v247", "v248", "v249", "v250", "v251", "v252", "v253",  \
      "v254", "v255"
#define FSF_SOFTMAX_TMP_REGS "v222", "v223", "v224", "v225", "v226", "v227", "v228", "v229", "v230", "v231"

typedef float f32x32_t __attribute__((ext_vector_type(32)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x32 __attribute__((ext_vector_type(32)));

// One workgroup of 64*kPrefillWaves threads: tile = index into the pass's prefill tiles,
// hq = query head, lds = kPrefillLdsBytes of LDS.
template <int DT, typename T>
__device__ __forceinline__ void prefill_tile(const Pass& p, const FastPlan& f,
                                             const T* __restrict__ q, const T* __restrict__ kc,
                                             const T* __restrict__ vc, T* __restrict__ out, int tile,
                                             int hq, lds_char* lds) {
  using M = Mma<DT>;
  // values that are the same in every lane are told so (the compiler cannot always tell)
  auto uni = [](uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane(x); };
  auto uni64 = [&](uint64_t x) { return ((uint64_t)uni((uint32_t)(x >> 32)) << 32) | uni((uint32_t)x); };
  const int tid = threadIdx.x;
  const int wave = uni(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31, hg = lane >> 5;
  const int hk = hq / p.group;
  const int s = f.pre_tile_seq[tile];  // written by the planning kernel
  const fsf_seq_desc sd = p.descs[s];
  const int B = p.block_size;
  const int n_new = sd.n_new, c = sd.n_cached;
  const int i0 = (tile - f.pre_tile_start[s]) * kPrefillTileM;  // first row of the tile
  const int i1 = min(i0 + kPrefillTileM, n_new);                // one past its last row

  // key range of the whole tile (all waves walk the same steps: they share the LDS tiles)
  int lo_t, hi_t, tmp;
  visible_range(c + i0, p.window, lo_t, tmp);
  visible_range(c + i1 - 1, p.window, tmp, hi_t);
  const int key_begin = lo_t & ~(kKeysPerStep - 1);
  const int n_steps = (hi_t - key_begin) / kKeysPerStep + 1;  // >= 1
  const int kv_last = c + n_new - 1;  // last cache position this sequence has written
  const int whole_hi = (kv_last - key_begin - (kKeysPerStep - 1)) >= 0
                           ? (kv_last - key_begin - (kKeysPerStep - 1)) / kKeysPerStep
                           : -1;  // last step with all 64 rows written

  // this wave's rows, and the steps that hold a key visible to one of them
  const int w_i0 = i0 + wave * 32;
  const int w_i1 = min(w_i0 + 32, i1);  // may be <= w_i0: wave has no live row
  int j_first = 0, j_last = -1;          // active steps
  int nomask_lo = 0, nomask_hi = -1;     // steps none of whose scores is hidden from any row
  if (w_i0 < i1) {
    int w_lo_min, w_lo_max, w_hi_min, w_hi_max;
    visible_range(c + w_i0, p.window, w_lo_min, w_hi_min);
    visible_range(c + w_i1 - 1, p.window, w_lo_max, w_hi_max);
    j_first = (w_lo_min - key_begin) / kKeysPerStep;
    j_last = (w_hi_max - key_begin) / kKeysPerStep;
    if (w_i1 - w_i0 == 32) {
      nomask_lo = (w_lo_max - key_begin + kKeysPerStep - 1) / kKeysPerStep;
      nomask_hi = (w_hi_min - key_begin - (kKeysPerStep - 1)) >= 0
                      ? (w_hi_min - key_begin - (kKeysPerStep - 1)) / kKeysPerStep
                      : -1;
    }
  }
  // Steady iterations b: steps b-1 and b active, step b unmasked, K(b+1) and V(b) whole, step
  // b+2 exists; an even number of them starting at an even b.
  int fast_lo = 0, fast_hi = -1;
  {
    const int lo = (max(max(j_first + 1, nomask_lo), 0) + 1) & ~1;
    const int hi = min(min(nomask_hi, j_last), min(n_steps - 3, whole_hi - 1));
    if (hi - lo + 1 >= 2) {
      fast_lo = lo;
      fast_hi = lo + ((hi - lo + 1) & ~1) - 1;
    }
  }

  // Q^T fragments (B operand): lane = (row l32, k-group hg), k-step t -> d chunk 2t+hg
  u32x32 qf;
  int row_pos;  // absolute position of the lane's row (rows past the tile: -1)
  {
    const int i = w_i0 + l32;
    const bool live = i < i1;
    row_pos = live ? c + i : -1;
    const int ic = live ? i : (i1 - 1);
    const T* qrow = q + ((int64_t)(sd.q_offset + ic) * p.n_q_heads + hq) * kHeadDim;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(qrow + (2 * t + hg) * 8);
#pragma unroll
      for (int e = 0; e < 4; ++e) qf[4 * t + e] = v[e];
    }
  }
  int rlo, rhi;
  visible_range(row_pos, p.window, rlo, rhi);  // rows past the tile: rhi = -1, nothing visible
  i32x4 thr = {rhi - 4 * hg, rlo - 4 * hg, 0, 0};

  u32x4 va;
  u32x8 ka;
  {
    const int lds0 = (int)(uintptr_t)lds;  // LDS byte address of K slot 0
    const int g = lane >> 4, sl = lane & 15;
    const int x = 4 * (g >> 1) + (sl >> 2);
#pragma unroll
    for (int t = 0; t < 8; ++t) ka[t] = lds0 + l32 * 256 + (((2 * t + hg) ^ (l32 & 15)) << 4);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
      va[mt] = lds0 + kVRingBase + x * 256 + ((2 * (mt ^ (x & 3)) + (g & 1)) << 5) + ((sl & 3) << 3);
  }

  // ---- copies.  Step j of the tile covers keys key_begin + 64 j .. + 63, which lie in cache block
  // (step0 + j) / spb of the sequence (spb = 64-key steps per block, a power of two).
  TileCopy kcopy, vcopy;
  kcopy.init<false>(wave, lane);
  vcopy.init<true>(wave, lane);
  const uint32_t lds_k0 = (uint32_t)(uintptr_t)lds;
  constexpr uint32_t kRowBytes = kHeadDim * sizeof(T);
  const int32_t* bt = p.block_tables + (int64_t)s * p.max_blocks;
  const uint32_t step0 = (uint32_t)key_begin / kKeysPerStep;
  const uint32_t spb = (uint32_t)B / kKeysPerStep;
  const uint32_t spb_shift = __builtin_ctz(spb);
  const uint64_t blk_bytes = (uint64_t)p.n_kv_heads * B * kRowBytes;  // one cache block, all heads (< 4 GiB)
  const char* const k_head = reinterpret_cast<const char*>(kc) + (uint64_t)hk * B * kRowBytes;
  const char* const v_head = reinterpret_cast<const char*>(vc) + (uint64_t)hk * B * kRowBytes;
  // K(0) goes out before the first hand-over; the sequence continues from there with
  //   off_prev   byte offset (block and position inside it, head excluded) of step b's tiles
  //   phys_next  physical block of step b+1, fetched one hand-over earlier
  uint64_t off_prev = (uint64_t)(uint32_t)load_uniform_i32(bt + (step0 >> spb_shift)) * blk_bytes +
                      (step0 & (spb - 1)) * (kKeysPerStep * kRowBytes);
  uint32_t phys_next = n_steps > 1 ? (uint32_t)load_uniform_i32(bt + ((step0 + 1) >> spb_shift)) : 0u;
  if (whole_hi < 0) kcopy.issue<true>(k_head + off_prev, lds_k0, kv_last - key_begin);
  else kcopy.issue<false>(k_head + off_prev, lds_k0, 0);

  // ---- the walk
  f32x32_t acc01, acc23, sc;
  u32x16 p0, p1;
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    acc01[r] = 0.f;
    acc23[r] = 0.f;
    sc[r] = 0.f;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    p0[r] = 0u;
    p1[r] = 0u;
  }
  f32x4_t mlcs = {-1e30f, 0.f, 0.f, p.scale * 1.4426950408889634f};  // m, l, rescale factor, scale*log2e
  u32x4 koff, voff;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    koff[i] = kcopy.lane_off[i];
    voff[i] = vcopy.lane_off[i];
  }
  const u32x4 s60 = {uni(n_steps), uni(j_first), uni(j_last), uni(nomask_lo)};
  const u32x4 s64 = {uni(nomask_hi), uni(fast_lo), uni(fast_hi), uni(whole_hi)};
  const u32x4 s68 = {uni(kv_last - key_begin), uni(key_begin), uni(p.window), uni(step0)};
  const u32x2 s72 = {uni(spb - 1), uni(spb_shift)};
  const u32x2 s80 = {uni((uint32_t)blk_bytes), uni(lds_k0 + kcopy.lds_off[0])};
  const uint64_t bt_s = uni64(reinterpret_cast<uint64_t>(bt));
  const uint64_t k_head_s = uni64(reinterpret_cast<uint64_t>(k_head));
  const uint64_t v_head_s = uni64(reinterpret_cast<uint64_t>(v_head));
  uint64_t off_prev_s = uni64(off_prev);
  uint32_t phys_next_s = uni(phys_next), b_s = uni(0u);
  const float ninf = -INFINITY;
#define FSF_TILE_OPERANDS                                                                      \
  : "+{v[94:125]}"(acc01), "+{v[126:157]}"(acc23), "+{v[158:189]}"(sc), "+{v[190:205]}"(p0),   \
    "+{v[206:221]}"(p1), "+{v[40:43]}"(mlcs), "+{v[32:35]}"(thr), "+{s[90:91]}"(off_prev_s),   \
    "+{s94}"(phys_next_s), "+{s97}"(b_s)                                                       \
  : "{v[50:53]}"(va), "{v[54:61]}"(ka), "{v[62:93]}"(qf), "{v[44:47]}"(koff),                  \
    "{v[36:39]}"(voff), "{v48}"(ninf), "{s[60:63]}"(s60), "{s[64:67]}"(s64),                   \
    "{s[68:71]}"(s68), "{s[72:73]}"(s72), "{s[74:75]}"(bt_s), "{s[76:77]}"(k_head_s),          \
    "{s[78:79]}"(v_head_s), "{s[80:81]}"(s80)                                                  \
  : "memory", "vcc", "scc", "s82", "s83", "s84", "s85", "s86", "s87", "s88", "s89", "s92",     \
    "s93", "s95", "s96", "s98", "s99", "v28", "v29", FSF_FRAG_REGS, FSF_SOFTMAX_TMP_REGS
  if constexpr (DT == FSF_BF16)
    asm volatile(FSF_TILE_SEQUENCE("v_mfma_f32_32x32x16_bf16", "v_cvt_pk_bf16_f32") FSF_TILE_OPERANDS);
  else
    asm volatile(FSF_TILE_SEQUENCE("v_mfma_f32_32x32x16_f16", "v_cvt_pk_f16_f32") FSF_TILE_OPERANDS);
#undef FSF_TILE_OPERANDS

  // ---- normalise and store: accumulator mt, register r is column d = 32mt + 8(r/4) + 4hg + r%4
  // of the lane's row
  float l = mlcs[1];
  l += __shfl_xor(l, 32);
  if (row_pos < 0) return;
  const float inv = 1.f / l;
  T* orow = out + ((int64_t)(sd.q_offset + row_pos - c) * p.n_q_heads + hq) * kHeadDim;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int e = 16 * (mt & 1) + 4 * rq;
      const f32x32_t& a = mt < 2 ? acc01 : acc23;
      uint2 w;
      w.x = M::pack2(a[e] * inv, a[e + 1] * inv);
      w.y = M::pack2(a[e + 2] * inv, a[e + 3] * inv);
      *reinterpret_cast<uint2*>(orow + 32 * mt + 8 * rq + 4 * hg) = w;
    }
}

}  // namespace fsf
