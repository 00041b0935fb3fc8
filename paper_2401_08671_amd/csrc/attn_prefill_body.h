// Device code for prompt chunks (n_new > 1): tiled matrix-core attention over the blocked cache.
//
// A chunk of a split prompt attends causally to its own rows and to every chunk cached by
// earlier passes (paper Sec. 3.2 rule 1; Sec. 2 prompt processing).  Work is dense
// contraction: 4*d flops per (row, visible key), so it belongs on the matrix cores.
//
// One workgroup (4 waves, one per SIMD) owns a tile of 256 consecutive rows of one sequence
// and one query head; wave w owns 64 of them as two 32-row blocks (rb = 0, 1).  A wave runs
// alone on its SIMD with all 512 registers: 256 vector registers for what the vector ALU
// touches (scores, probabilities, addresses) and 256 accumulation registers for what only
// the matrix core touches (O^T, Q^T, K / V^T fragments).  Every K or V^T fragment read from LDS
// feeds two MFMAs (one per row block), which halves the LDS traffic per flop of a 32-row wave,
// and the overlap of matrix and vector work is arranged inside the wave's own instruction
// stream instead of being left to the chance interleaving of two waves.
//
// Keys are taken 64 at a time ("step"), gathered through the block table.  Every wave copies 16
// of a step's key rows, and those never straddle a cache block (block_size is 16 * 2^k): with
// blocks of 16 or 32 tokens the four waves simply read their rows from different blocks.
//   HBM/L2 -> LDS directly (global_load_lds, 16 bytes per lane, no registers, no VALU).
//     Both tiles stay row-major [64 keys][128 d]; the lane -> global chunk mapping applies an
//     XOR swizzle so the later reads are bank-conflict free (64 banks):
//       K: 16-byte chunk c of key row r sits at chunk c ^ (r & 15)
//       V: 32-byte segment s of key row r sits at segment s ^ 2(r & 3)
//     Rows past the sequence's last token are fetched from its last token instead: their
//     scores are masked, and a finite stand-in keeps 0 * garbage out of the second product.
//   QK:  S^T[key, row] = K . Q^T   A = K rows (ds_read_b128), B = Q^T held in registers
//   softmax per row in registers: a lane owns 32 scores of one row per row block, the max
//     across the two half-waves is one lane swap; the running reference is only raised when a
//     maximum outgrows it by 2^8 (lazy rescale), so O^T is rarely touched by vector code
//   PV:  O^T[d, row] += V^T . P^T  A = V^T read from the row-major V tile with the transposing
//                                 LDS read (ds_read_b64_tr_b16), B = P^T = the lane's own
//                                 probabilities, no cross-lane movement
//
// Software pipeline.  Iteration b of a wave:  hand-over, PV(b-1), softmax(b), QK(b+1).  The
// three parts do not depend on each other (softmax(b) needs QK(b), done one iteration
// earlier, and produces the P^T that PV(b) consumes one iteration later), so in the steady
// state the 64 MFMAs of PV(b-1) and QK(b+1) form one stream with the ~300 vector
// instructions of softmax(b) placed between them.  S^T is double-buffered (softmax reads one
// buffer while QK fills the other); P^T is single: the conversions that write it come after
// the last MFMA of PV(b-1) has been issued.
//
// LDS (64 KB): two K slots and two V slots.  Hand-over b = wait for the wave's own copies of
// K(b+1) and V(b-1), workgroup barrier, start K(b+2) and V(b) in the slots that iteration b-1
// has finished reading.  One iteration (about 1.5 us) covers the latency of a gathered block.
#pragma once

#include <math.h>

#include <type_traits>

#include "attn_prefill_sequence.h"
#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {

constexpr int kPrefillWaves = 4;
constexpr int kRowsPerWave = 64;
static_assert(kPrefillTileM == kRowsPerWave * kPrefillWaves, "two 32-row blocks per wave");
constexpr int kRing = 2;                     // LDS slots per tile ring (K and V each)
constexpr int kKeysPerStep = 64;
constexpr int kTileBytes = 64 * 256;         // one K or V tile: [64 keys][128 d] of 2-byte elements
constexpr int kPrefillLdsBytes = 2 * kRing * kTileBytes;  // K slots 0, 1, then V slots 0, 1
constexpr int kVRingBase = kRing * kTileBytes;            // byte offset of V slot 0
static_assert(kPrefillLdsBytes <= 65536, "LDS reads reach every slot with a 16-bit offset");

typedef __attribute__((address_space(3))) char lds_char;

// A K (or V) tile of one 64-key step is copied into an LDS slot with global_load_lds (16
// bytes per lane, HBM/L2 -> LDS without passing registers).  Each of the 4 waves copies 16 key
// rows with 4 instructions (4 rows x 256 B each).  The lane -> source-chunk mapping (which
// applies the swizzle) does not change from step to step, so a lane keeps its byte offset
// relative to the wave's first row in a register and a copy costs a handful of scalar
// instructions for the address of that row (block, head, position inside the block).  Returns
// row*256 + swizzled chunk*16 of the lane's 16 bytes in copy instruction i of its wave, row
// counted from the wave's first; both swizzles depend on the row modulo 16 only.
template <bool kIsV>
__device__ __forceinline__ uint32_t copy_lane_offset(int lane, int i) {
  const int pc = lane & 15;  // physical 16-byte chunk this lane fills
  const int row = i * 4 + (lane >> 4);
  const int swz = kIsV ? ((row & 3) << 2) : (row & 15);
  return row * 256 + ((pc ^ swz) << 4);
}

// ---------------------------------------------------------------------------------------
// The whole walk of a tile over its steps is ONE fixed instruction sequence: it loads Q^T,
// walks the steps and stores the normalised result; plain code around it only computes the
// step ranges and addresses it starts from.  LDS reads run seven fragments ahead of the MFMAs
// that consume them, every wait names exactly the reads it needs, and a hand-over costs some
// thirty scalar instructions.  (Left to the compiler, the same loop issues two to three times
// as many instructions, and pinning parts of it makes its register allocation spill.)
//
// Iteration b (b = 0 .. n_steps; S^T buffers and slot pairs alternate with b & 1):
//   hand-over b, PV(b-1) if step b-1 is active for the wave, softmax(b) -> P^T if step b is
//   (with the scores of hidden keys set to -inf first where the step needs it), QK(b+1) if
//   step b+1 is.  Before iteration 0: K(0) and K(1) copied, QK(0).
// Steady pairs: from an even b with  fast_lo <= b, b+1 <= fast_hi  the wave runs pairs of
// iterations without any test: all three parts active, nothing masked, every copy whole.
// Softmax: row maximum (v_max3 chains, v_permlane32_swap for the other half-wave), lazy raise
// of the reference, p = 2^(s*scale*log2e - m) in place of the score, row sum, P^T register r =
// pack(p[2r], p[2r+1]); where the reference was raised O^T is scaled once the PV has landed.
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
// Registers of the sequence (rb = row block 0, 1):
//   v28 v29 temporaries of a clamped copy    v30 v32 rhi - 4hg, v31 v33 rlo - 4hg of the lane's
//   row in rb 0, 1 (visible keys [rlo, rhi]; score register j of a row block is key 32(j/16) +
//   8((j%16)/4) + j%4 + 4hg of the step), v34 v35 the same minus the step's first key
//   v36..v39 V copy lane offsets   v40..v43 K copy lane offsets   v44 v47 m   v45 v48 l
//   v46 v49 rescale factor   v50 scale*log2e   v51 -inf   v52..v55 va   v56..v63 ka
//   v64..v127, v128..v191 S^T buffers 0, 1 (32 rb + 16 kt + r)   v192..v223 P^T (16 rb + r)
//   v224..v227 address of the lane's output rows   v228..v231 of its query rows
//   v232..v255 temporaries
//   a0..a127 O^T (64 rb + 16 mt + r)   a128..a191 Q^T fragments (32 rb + 4 t + r)
//   a192..a255 sixteen K / V^T fragments in flight
//   s51 1 if the result is stored as a partial one   s[52:53] address of a V tile   s[88:89] s[54:55] lanes whose reference was raised, rb 0, 1
//   s[56:57] s[58:59] lanes whose row exists   s60 n_steps   s61 s62 first, last active step
//   of the wave   s63 s64 first, last step that needs no mask   s65 s66 fast_lo, fast_hi   s67
//   last step with all 64 rows written   s68 last written key of the sequence   s69
//   first key of the tile   s70 window   s71 the wave's 16-key quarter of step 0, counted from
//   the start of the sequence (first key/16 + wave)   s72 quarters per cache block - 1   s73
//   log2 of quarters per block   s[74:75] block table of the
//   sequence   s[76:77] K base of this head   s[78:79] V base   s80 bytes per cache block   s81
//   LDS address of the wave's first copy row   s82..s87, s92, s93, s95, s96 temporaries
//   s[90:91] s[98:99] byte offset of the tiles of steps b, b+1   s94 physical block of step
//   b+2   s97 b
// Every block of MFMAs ends with the idle cycles the matrix core needs before other code may
// read what the last MFMA wrote.
// The sequence itself (macro FSF_TILE_SEQUENCE, some 5000 instructions) is written by
// gen_prefill_sequence.py into attn_prefill_sequence.h; the build runs the generator first.
// ---------------------------------------------------------------------------------------
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));

// One workgroup of 64*kPrefillWaves threads: work = tile (index into the pass's prefill tiles),
// which part of how many of the tile's key range, and where a partial result goes; hq = query
// head, lds = kPrefillLdsBytes of LDS.
template <int DT, typename T>
__device__ __forceinline__ void prefill_tile(const Pass& p, const FastPlan& f,
                                             const T* __restrict__ q, const T* __restrict__ kc,
                                             const T* __restrict__ vc, T* __restrict__ out,
                                             const PrefillWork& work, int hq, lds_char* lds) {
  // values that are the same in every lane are told so (the compiler cannot always tell)
  auto uni = [](uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane(x); };
  auto uni64 = [&](uint64_t x) { return ((uint64_t)uni((uint32_t)(x >> 32)) << 32) | uni((uint32_t)x); };
  const int tid = threadIdx.x;
  const int wave = uni(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31, hg = lane >> 5;
  const int hk = hq / p.group;
  const int tile = work.tile;
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
  int key_begin = lo_t & ~(kKeysPerStep - 1);
  int n_steps = (hi_t - key_begin) / kKeysPerStep + 1;  // >= 1
  // a split tile: this workgroup walks part `part` of the steps and stores a partial result
  const bool is_split = work.slab >= 0;
  if (is_split) {
    const int s_lo = (int)((int64_t)work.part * n_steps / work.n_parts);
    const int s_hi = (int)((int64_t)(work.part + 1) * n_steps / work.n_parts);
    key_begin += s_lo * kKeysPerStep;
    n_steps = s_hi - s_lo;  // >= 1: the host keeps parts at kPrefillMinPartSteps steps or more
  }
  const int kv_last = c + n_new - 1;  // last cache position this sequence has written
  const int whole_hi = (kv_last - key_begin - (kKeysPerStep - 1)) >= 0
                           ? (kv_last - key_begin - (kKeysPerStep - 1)) / kKeysPerStep
                           : -1;  // last step with all 64 rows written

  // this wave's rows, and the steps that hold a key visible to one of them
  const int w_i0 = i0 + wave * kRowsPerWave;
  const int w_i1 = min(w_i0 + kRowsPerWave, i1);  // may be <= w_i0: wave has no live row
  int j_first = 0, j_last = -1;                   // active steps
  int nomask_lo = 0, nomask_hi = -1;              // steps none of whose scores is hidden from any row
  if (w_i0 < i1) {
    int w_lo_min, w_lo_max, w_hi_min, w_hi_max;
    visible_range(c + w_i0, p.window, w_lo_min, w_hi_min);
    visible_range(c + w_i1 - 1, p.window, w_lo_max, w_hi_max);
    // clipped to the steps this workgroup walks (all of the tile's unless it is split)
    j_first = w_lo_min > key_begin ? (w_lo_min - key_begin) / kKeysPerStep : 0;
    j_last = w_hi_max >= key_begin ? min((w_hi_max - key_begin) / kKeysPerStep, n_steps - 1) : -1;
    if (j_last < j_first) {
      j_first = 0;
      j_last = -1;
    }
    if (w_i1 - w_i0 == kRowsPerWave) {
      nomask_lo = w_lo_max > key_begin ? (w_lo_max - key_begin + kKeysPerStep - 1) / kKeysPerStep : 0;
      nomask_hi = (w_hi_min - key_begin - (kKeysPerStep - 1)) >= 0
                      ? (w_hi_min - key_begin - (kKeysPerStep - 1)) / kKeysPerStep
                      : -1;
    }
  }
  // Steady iterations b: steps b-1, b, b+1 active, step b unmasked, K(b+2) exists and it and
  // V(b) are whole; an even number of them starting at an even b.
  int fast_lo = 0, fast_hi = -1;
  {
    const int lo = (max(max(j_first + 1, nomask_lo), 0) + 1) & ~1;
    const int hi = min(min(nomask_hi, j_last - 1), min(n_steps - 3, whole_hi - 2));
    if (hi - lo + 1 >= 2) {
      fast_lo = lo;
      fast_hi = lo + ((hi - lo + 1) & ~1) - 1;
    }
  }

  // the lane's two rows: row block rb holds row w_i0 + 32 rb + l32
  i32x4 thr;           // {rhi, rlo} - 4 hg per row block; rows past the tile see nothing
  u32x4 q_ptr, o_ptr;  // addresses of the lane's part of the query rows and of the output rows
  uint64_t live[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int i = w_i0 + 32 * rb + l32;
    const bool is_live = i < i1;
    const int ic = is_live ? i : (i1 - 1);  // a stand-in row keeps the loads in bounds
    int rlo, rhi;
    visible_range(is_live ? c + i : -1, p.window, rlo, rhi);
    thr[2 * rb] = rhi - 4 * hg;
    thr[2 * rb + 1] = rlo - 4 * hg;
    const int64_t row = ((int64_t)(sd.q_offset + ic) * p.n_q_heads + hq) * kHeadDim;
    // Q^T fragment t of the lane is d chunk 2t + hg (8 elements); its output columns are
    // 32 mt + 8 rq + 4 hg + 0..3
    const uint64_t qa = reinterpret_cast<uint64_t>(q + row + 8 * hg);
    // a split tile's rows go to the partial-result buffer: [slab, row of the tile, head][136 floats]
    const int64_t prow = ((int64_t)work.slab * kPrefillTileM + (ic - i0)) * p.n_q_heads + hq;
    const uint64_t oa = is_split ? reinterpret_cast<uint64_t>(f.pre_part + prow * kPrefillPartRowFloats + 4 * hg)
                                 : reinterpret_cast<uint64_t>(out + row + 4 * hg);
    q_ptr[2 * rb] = (uint32_t)qa;
    q_ptr[2 * rb + 1] = (uint32_t)(qa >> 32);
    o_ptr[2 * rb] = (uint32_t)oa;
    o_ptr[2 * rb + 1] = (uint32_t)(oa >> 32);
    live[rb] = uni64(__ballot(is_live));
  }

  u32x4 va, koff, voff;
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
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      koff[i] = copy_lane_offset<false>(lane, i);
      voff[i] = copy_lane_offset<true>(lane, i);
    }
  }

  // ---- copies.  Step j of the tile covers keys key_begin + 64 j .. + 63; this wave copies the
  // 16 rows of "quarter" q0 + 4 j (quarters = runs of 16 keys, counted from the start of the
  // sequence), which lie in cache block quarter / qpb (qpb = quarters per block, a power of two).
  // A quarter past the last written token is replaced by the one that holds that token: the
  // sequence owns that block, and the rows copied from there are stand-ins for masked keys.
  const uint32_t lds_k0 = (uint32_t)(uintptr_t)lds;
  constexpr uint32_t kRowBytes = kHeadDim * sizeof(T);
  const int32_t* bt = p.block_tables + (int64_t)s * p.max_blocks;
  constexpr uint32_t kQuarterKeys = kKeysPerStep / kPrefillWaves;  // 16
  const uint32_t q0 = (uint32_t)key_begin / kQuarterKeys + wave;
  const uint32_t q_last = (uint32_t)kv_last / kQuarterKeys;
  const uint32_t qpb = (uint32_t)B / kQuarterKeys;
  const uint32_t qpb_shift = __builtin_ctz(qpb);
  const uint64_t blk_bytes = (uint64_t)p.n_kv_heads * B * kRowBytes;  // one cache block, all heads (< 4 GiB)
  const char* const k_head = reinterpret_cast<const char*>(kc) + (uint64_t)hk * B * kRowBytes;
  const char* const v_head = reinterpret_cast<const char*>(vc) + (uint64_t)hk * B * kRowBytes;
  // the sequence starts from the byte offsets (block and position inside it, head excluded) of
  // the tiles of steps 0 and 1 and the physical block of step 2
  auto quarter_of = [&](uint32_t j) { return min(q0 + kPrefillWaves * j, q_last); };
  auto block_of = [&](uint32_t j) { return (uint32_t)load_uniform_i32(bt + (quarter_of(j) >> qpb_shift)); };
  auto offset_of = [&](uint32_t j) {
    return (uint64_t)block_of(j) * blk_bytes + (quarter_of(j) & (qpb - 1)) * (kQuarterKeys * kRowBytes);
  };
  uint64_t off0_s = uni64(offset_of(0));
  uint64_t off1_s = uni64(n_steps > 1 ? offset_of(1) : 0);
  uint32_t phys2_s = uni(n_steps > 2 ? block_of(2) : 0u);
  uint32_t b_s = uni(0u);

  const u32x4 s60 = {uni(n_steps), uni(j_first), uni(j_last), uni(nomask_lo)};
  const u32x4 s64 = {uni(nomask_hi), uni(fast_lo), uni(fast_hi), uni(whole_hi)};
  const u32x4 s68 = {uni(kv_last), uni(key_begin), uni(p.window), uni(q0)};
  const u32x2 s72 = {uni(qpb - 1), uni(qpb_shift)};
  const u32x2 s80 = {uni((uint32_t)blk_bytes), uni(lds_k0 + wave * (64 / kPrefillWaves) * 256)};
  const uint64_t bt_s = uni64(reinterpret_cast<uint64_t>(bt));
  const uint64_t k_head_s = uni64(reinterpret_cast<uint64_t>(k_head));
  const uint64_t v_head_s = uni64(reinterpret_cast<uint64_t>(v_head));
  const float sl2 = p.scale * 1.4426950408889634f;  // scale * log2(e)
  const uint32_t partial = uni(is_split ? 1u : 0u);
#define FSF_TILE_OPERANDS                                                                          \
  : "+{s[90:91]}"(off0_s), "+{s[98:99]}"(off1_s), "+{s94}"(phys2_s), "+{s97}"(b_s)                 \
  : "{v[30:33]}"(thr), "{v[36:39]}"(voff), "{v[40:43]}"(koff), "{v50}"(sl2), "{v[52:55]}"(va),     \
    "{v[56:63]}"(ka), "{v[224:227]}"(o_ptr), "{v[228:231]}"(q_ptr), "{s51}"(partial),              \
    "{s[56:57]}"(live[0]),                                                                         \
    "{s[58:59]}"(live[1]), "{s[60:63]}"(s60), "{s[64:67]}"(s64), "{s[68:71]}"(s68),                \
    "{s[72:73]}"(s72), "{s[74:75]}"(bt_s), "{s[76:77]}"(k_head_s), "{s[78:79]}"(v_head_s),         \
    "{s[80:81]}"(s80)                                                                              \
  : "memory", "vcc", "scc", FSF_TILE_CLOBBERS
  if constexpr (DT == FSF_BF16)
    asm volatile(FSF_TILE_SEQUENCE("v_mfma_f32_32x32x16_bf16", "v_cvt_pk_bf16_f32") FSF_TILE_OPERANDS);
  else
    asm volatile(FSF_TILE_SEQUENCE("v_mfma_f32_32x32x16_f16", "v_cvt_pk_f16_f32") FSF_TILE_OPERANDS);
#undef FSF_TILE_OPERANDS
}

}  // namespace fsf
