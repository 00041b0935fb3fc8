// Linear layer over the tokens of a pass: y[t, o] = sum_k x[t, k] * w[o, k]   (bf16 / f16, fp32 accumulation).
//
// Besides attention, a forward pass applies dense projections to every token of the ragged
// batch (query/key/value and output projections, gated MLP); they are what makes a pass
// weight-bound while it holds few tokens and compute-bound once it holds many (paper Sec. 3.1),
// and so what fixes a sensible token budget.  Dense contraction: matrix cores.
//
// One workgroup (8 waves, two per SIMD, for all but small token counts) computes a BM x BN tile of
// y; a wave owns WM x WN of it as MFMA blocks (16x16x32 in the large tile shapes, 32x32x16 in the small
// ones, see below).  Both operands are k-contiguous in memory (tokens and
// weight rows alike), so they are staged the same way: BK = 64 k-elements at a time, row-major
// tiles [rows][128 bytes] in LDS, copied there directly from HBM/L2 (global_load_lds, 16 bytes per
// lane, no registers) in a ring of two or three stages, ahead of the MFMAs.  A tile row is one
// whole 128-byte cache line, fetched by eight adjacent lanes: with 64-byte rows the same bytes
// cost twice the requests, and the L2's request rate, not its bandwidth, then bounds the kernel
// (measured: 1.1 PFLOP/s at 64 % of the L2 channels' request slots).  A lane of a copy
// instruction always fills the next 16 bytes of LDS, so the XOR swizzle that makes the later
// ds_read_b128 fragment reads conflict-free is applied on the global side: 16-byte chunk c of tile
// row r sits at chunk c ^ ((r >> 1) & 7)  (a b128 read serves 16 lanes per clock from 64 banks:
// rows r and r+1 differ in address bit 7, and rows of equal parity land on different chunks).
//
// The product is formed transposed, D[o, t] = W . X^T (A operand = weight rows, B operand =
// tokens): a lane then owns 4 consecutive output features of one token per register quad, which
// it stores as 8 (or 16) contiguous bytes.
//
// The copies and their waits are written as inline asm: the compiler does not track LDS-DMA
// per stage and would wait for every copy in flight before each LDS read.  The protocol per
// k-step kt (every wave issues the same number of copies, so the counters agree):
//   MFMAs of all but the last part of step kt (quarters of 16 k-elements, or halves of 32), each
//     with the next part's fragments on their way from LDS; then all fragments of step kt are in
//     registers
//   wait until this wave's copies of step kt+1 have landed (all but the younger steps')
//   workgroup barrier: everybody's copies of step kt+1 are in LDS, and everybody has read step
//                      kt's fragments, whose stage the next copy overwrites
//   start the copies of step kt + stages (past the end of k: the last step again, never read)
//   first fragments of step kt+1 from LDS, the last part of step kt's MFMAs, the next fragments
#include <type_traits>

#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {
namespace {

constexpr int kLinBK = 64;    // k elements per stage: one 128-byte line per tile row
constexpr int kRowBytes = kLinBK * 2;

typedef __attribute__((address_space(3))) char lin_lds_char;

// one copy instruction of a wave: 8 tile rows x 128 bytes, lane -> (row lane / 8, physical chunk lane % 8)
__device__ __forceinline__ void copy16(uint32_t lds_addr, uint32_t voffset, const char* base) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr), "v"(voffset), "s"(base)
      : "memory", "m0");
}

// Wait until at most N of this wave's copies are in flight, and for its own LDS reads: a wave
// that meets the barrier after this has the fragments it asked for in registers, so the stage
// they came from may be overwritten.
template <int N>
__device__ __forceinline__ void wait_copies_but() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(N) : "memory");
}

// BM x BN: tokens x output features per workgroup; WM x WN: per wave; kLinStages: depth of the LDS
// ring; kMfma16: 16x16x32 MFMAs and a pipeline over half steps, else 32x32x16 and quarter steps.
// Six shapes are built (which one runs, and in how many parts k is cut, is decided by linear_plan
// below):
//   256 x 256, waves 128 x 64 (8 waves, two per SIMD), 2 stages of 64 KB: many tokens, compute-bound
//   192 x 256, waves  96 x 64 (8 waves), 2 stages of 56 KB: where 256-row tiles come to just over a
//              whole number of rounds of the compute units and three quarters of a tile fill them
//   128 x 256, waves 128 x 32 (8 waves), 3 stages of 48 KB: a few hundred tokens
//      all three with 16x16x32 MFMAs: under the chip's power limit that instruction sustains a tenth
//      more flops than 32x32x16 (2.10 against 1.91 PFLOP/s in a register-resident loop on normally
//      distributed operands), and these kernels gain 3..6 %
//   128 x  64, waves  64 x 32 (4 waves), 5 stages of 24 KB: up to 256 tokens, where the pass is
//              bound by reading the weights: four times the workgroups to pull on HBM, deep prefetch
//    64 x 128 and 32 x 128, waves 64 x 32 and 32 x 32 (4 waves), 5 and 6 stages: a few tokens.  A
//              token tile is copied whole whatever the token count, and from 128 x 64 tiles on
//              two thirds of what crosses from L2 into LDS are token rows; here it is a third
//              and a fifth, and the weights can use the rest
//      these three with 32x32x16 MFMAs (bound by how fast one workgroup pulls weights, they were
//      slower in the other form)
template <int DT, typename T, int BM, int BN, int WM, int WN, int kLinStages, bool kMfma16>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void linear_kernel(const T* __restrict__ x,
                                                                           const T* __restrict__ w,
                                                                           T* __restrict__ y, int M, int N,
                                                                           int K, int tiles_m, int tiles_n,
                                                                           float* __restrict__ part, int splits) {
  constexpr int kLinBN = BN;
  constexpr int kWaves = (BM / WM) * (BN / WN);
  constexpr int kBlk = kMfma16 ? 16 : 32;    // rows (and columns) of one MFMA block
  constexpr int kGroups = 64 / kBlk;         // 8-element k-groups a block's lanes hold side by side
  constexpr int kParts = kLinBK / (8 * kGroups);  // parts of a k-step with fragments of their own: 2 halves or 4 quarters
  constexpr int MB = WM / kBlk, NB = WN / kBlk;
  constexpr int kXTile = BM * kRowBytes, kWTile = kLinBN * kRowBytes;
  constexpr int kStage = kXTile + kWTile;
  extern __shared__ __attribute__((aligned(1024))) char lin_lds[];
  lin_lds_char* lds = (lin_lds_char*)lin_lds;

  // ---- which part of k: with `splits` > 1 the k-steps are dealt to that many workgroups per tile,
  // each of which leaves an fp32 partial tile in `part` ([split][token][feature]) for the summing kernel
  const int total = tiles_m * tiles_n;
  const int split = (int)blockIdx.x / total;
  int id = (int)blockIdx.x - split * total;
  // ---- which tile: workgroups are dealt to the 8 dies in turn; give each die a compact block of
  // tiles (consecutive ids on one die), walked in groups of 4 token tiles so that the tiles
  // running together on a die share weight and token panels in its L2
  if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
  constexpr int kGroupM = 4;
  const int per_group = kGroupM * tiles_n;
  const int group = id / per_group;
  const int first_m = group * kGroupM;
  const int rows_in_group = min(tiles_m - first_m, kGroupM);
  const int tm = first_m + (id % per_group) % rows_in_group;
  const int tn = (id % per_group) / rows_in_group;
  const int m0 = tm * BM, n0 = tn * kLinBN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane % kBlk, kg = lane / kBlk;  // the lane's row of a block, and its k-group

  // ---- copies: every wave fills an equal share of the rows of both tiles, 8 rows per instruction
  // (every wave issues the same count, so the copy counters of all waves agree)
  constexpr int kXCopies = BM / 8 / kWaves;      // instructions per wave for the token tile
  constexpr int kWCopies = kLinBN / 8 / kWaves;  // ... for the weight tile
  const int crow = lane >> 3, cpc = lane & 7;
  uint32_t x_off[kXCopies], w_off[kWCopies];
#pragma unroll
  for (int j = 0; j < kXCopies; ++j) {
    const int r = wave * (8 * kXCopies) + j * 8 + crow;
    const int row = min(m0 + r, M - 1);   // rows past the last token are copies of it, never stored
    x_off[j] = (uint32_t)row * (uint32_t)K * 2u + (uint32_t)((cpc ^ ((r >> 1) & 7)) << 4);
  }
#pragma unroll
  for (int j = 0; j < kWCopies; ++j) {
    const int r = wave * (8 * kWCopies) + j * 8 + crow;
    w_off[j] = (uint32_t)(n0 + r) * (uint32_t)K * 2u + (uint32_t)((cpc ^ ((r >> 1) & 7)) << 4);
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  const int nk_all = K / kLinBK;
  const int k_first = (int)((int64_t)split * nk_all / splits);
  const int nk = (int)((int64_t)(split + 1) * nk_all / splits) - k_first;  // >= 1: the host keeps splits <= nk_all
  auto issue = [&](int kt) {  // copies of this part's k-step min(kt, nk - 1) into stage kt % kLinStages
    const int ks = k_first + min(kt, nk - 1);
    const uint32_t stage = lds0 + (uint32_t)(kt % kLinStages) * kStage;
    const char* xb = reinterpret_cast<const char*>(x) + (size_t)ks * kRowBytes;
    const char* wb = reinterpret_cast<const char*>(w) + (size_t)ks * kRowBytes;
#pragma unroll
    for (int j = 0; j < kXCopies; ++j)
      copy16(stage + (uint32_t)(wave * (8 * kXCopies) + j * 8) * kRowBytes, x_off[j], xb);
#pragma unroll
    for (int j = 0; j < kWCopies; ++j)
      copy16(stage + kXTile + (uint32_t)(wave * (8 * kWCopies) + j * 8) * kRowBytes, w_off[j], wb);
  };
  constexpr int kCopiesPerStep = kXCopies + kWCopies;

  // ---- fragments of part t of a k-step: tile row blk * kBlk + lr, logical chunk kGroups t + kg
  // (a block starts at a multiple of 16 rows, so the swizzle is that of row lr)
  const int wm = wave % (BM / WM), wn = wave / (BM / WM);
  uint32_t frag_off[kParts];
#pragma unroll
  for (int t = 0; t < kParts; ++t)
    frag_off[t] = (uint32_t)(lr * kRowBytes + (((kGroups * t + kg) ^ ((lr >> 1) & 7)) << 4));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) u32x4 lds_u32x4;

  using Acc = typename std::conditional<kMfma16, f32x4_t, f32x16_t>::type;
  constexpr int kAccRegs = kMfma16 ? 4 : 16;
  Acc acc[NB][MB];
#pragma unroll
  for (int a = 0; a < NB; ++a)
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
      for (int r = 0; r < kAccRegs; ++r) acc[a][b][r] = 0.f;

  // Fragments of one part of a k-step: NB weight and MB token fragments.
  struct Frags {
    frag8 xf[MB], wf[NB];
  };
  auto read_frags = [&](Frags& fr, int kt, int t) {
    const lin_lds_char* st = lds + (kt % kLinStages) * kStage;
#pragma unroll
    for (int b = 0; b < MB; ++b) {
      const u32x4 v = *reinterpret_cast<const lds_u32x4*>(st + (wm * WM + b * kBlk) * kRowBytes + frag_off[t]);
      fr.xf[b] = frag8{{v[0], v[1], v[2], v[3]}};
    }
#pragma unroll
    for (int a = 0; a < NB; ++a) {
      const u32x4 v = *reinterpret_cast<const lds_u32x4*>(st + kXTile + (wn * WN + a * kBlk) * kRowBytes + frag_off[t]);
      fr.wf[a] = frag8{{v[0], v[1], v[2], v[3]}};
    }
  };
  auto multiply = [&](const Frags& fr) {
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
      for (int b = 0; b < MB; ++b) {
        if constexpr (kMfma16)
          acc[a][b] = Mma<DT>::mfma16(fr.wf[a], fr.xf[b], acc[a][b]);
        else
          acc[a][b] = Mma<DT>::mfma32(fr.wf[a], fr.xf[b], acc[a][b]);
      }
  };

  // Software pipeline over the parts of a k-step: the fragments of a part are on their way from
  // LDS while the MFMAs of the part before run, and the wait for the next step's copies, the
  // barrier and the first LDS reads of the next step sit before the last part of the current
  // step's MFMAs, which hide them.  (The scheduling barriers keep the compiler from sinking the
  // LDS reads down to their first use, which would put every MFMA group behind an exposed LDS
  // round trip.)
  constexpr int kAhead = kLinStages - 1;  // k-steps whose copies are in flight or landed beyond the current one
#pragma unroll
  for (int j = 0; j < kAhead; ++j) issue(j);
  wait_copies_but<(kAhead - 1) * kCopiesPerStep>();
  __builtin_amdgcn_s_barrier();
  issue(kAhead);
  Frags fa, fb;
  read_frags(fa, 0, 0);
  read_frags(fb, 0, 1);
  __builtin_amdgcn_sched_barrier(0);
  for (int kt = 0; kt < nk; ++kt) {
    multiply(fa);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (!kMfma16) {  // quarters 2 and 3 of this step
      read_frags(fa, kt, 2);
      __builtin_amdgcn_sched_barrier(0);
      multiply(fb);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(fb, kt, 3);
      __builtin_amdgcn_sched_barrier(0);
      multiply(fa);
      __builtin_amdgcn_sched_barrier(0);
    }
    // this wave's copies of step kt+1 have landed (younger steps may be in flight); after the
    // barrier everybody's have, and everybody holds step kt's last fragments in registers, so the
    // stage of step kt can take the copies of step kt + stages
    wait_copies_but<(kAhead - 1) * kCopiesPerStep>();
    __builtin_amdgcn_s_barrier();
    issue(kt + kLinStages);
    read_frags(fa, kt + 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(fb);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(fb, kt + 1, 1);
    __builtin_amdgcn_sched_barrier(0);
  }
  wait_copies_but<0>();  // the copies past the end of k are still in flight: let them land before the workgroup ends

  // ---- store: acc[a][b][4 q + r] is output feature n0 + wn WN + kBlk a + 8 q + 4 kg + r of token
  // m0 + wm WM + kBlk b + lr  (one quad q per 16 x 16 block, four per 32 x 32 block)
#pragma unroll
  for (int b = 0; b < MB; ++b) {
    const int row = m0 + wm * WM + b * kBlk + lr;
    if (row >= M) continue;
    if (splits > 1) {
      float* prow = part + ((size_t)split * M + row) * N + n0 + wn * WN + 4 * kg;
#pragma unroll
      for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int q = 0; q < kAccRegs / 4; ++q)
          *reinterpret_cast<float4*>(prow + a * kBlk + q * 8) =
              float4{acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
      continue;
    }
    T* yrow = y + (size_t)row * N + n0 + wn * WN + 4 * kg;
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
      for (int q = 0; q < kAccRegs / 4; ++q) {
        uint2 v;
        v.x = Mma<DT>::pack2(acc[a][b][4 * q], acc[a][b][4 * q + 1]);
        v.y = Mma<DT>::pack2(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
        *reinterpret_cast<uint2*>(yrow + a * kBlk + q * 8) = v;
      }
  }
}

// y[t, o] = sum over the splits of part[split][t][o], rounded once; a thread takes 8 features.
template <int DT, typename T>
__global__ __launch_bounds__(256) void linear_sum_kernel(const float* __restrict__ part, T* __restrict__ y,
                                                         size_t elems, int splits) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= elems) return;  // elems is a multiple of 256
  float4 lo = *reinterpret_cast<const float4*>(part + i), hi = *reinterpret_cast<const float4*>(part + i + 4);
  for (int s = 1; s < splits; ++s) {
    const float4 a = *reinterpret_cast<const float4*>(part + (size_t)s * elems + i);
    const float4 b = *reinterpret_cast<const float4*>(part + (size_t)s * elems + i + 4);
    lo.x += a.x, lo.y += a.y, lo.z += a.z, lo.w += a.w;
    hi.x += b.x, hi.y += b.y, hi.z += b.z, hi.w += b.w;
  }
  uint4 v;
  v.x = Mma<DT>::pack2(lo.x, lo.y);
  v.y = Mma<DT>::pack2(lo.z, lo.w);
  v.z = Mma<DT>::pack2(hi.x, hi.y);
  v.w = Mma<DT>::pack2(hi.z, hi.w);
  *reinterpret_cast<uint4*>(y + i) = v;
}

struct LinearShape {
  int shape, bm, bn, stages;
};
constexpr LinearShape kLinearShapes[6] = {{0, 256, 256, 2}, {1, 128, 256, 3}, {2, 128, 64, 5}, {3, 64, 128, 5}, {4, 32, 128, 6}, {5, 192, 256, 2}};

struct LinearPlan {
  LinearShape sh;
  int splits;
  double cost_us;
};

// Rough time of the product with one tile shape, and in how many parts k is best cut for it.
// A tile takes what the slowest of three things takes: its flops on one compute unit's matrix
// cores, its weight rows from HBM at one unit's share of the bandwidth, its operand tiles from L2
// into LDS; the launch takes tiles x parts / units rounds (a round only begun counting for a
// little less than a whole one) of tiles of 1 / parts that length.  Cutting pays where the tiles
// alone leave compute units idle (a 5120-wide projection of up to 256 tokens is 80 tiles for 256
// units); it costs a second kernel and the fp32 partial results' way through memory, which is
// what stops it at many tokens.  (Rates fitted to
// measurements on MI355X; the model only has to rank a handful of choices.)
LinearPlan plan_shape(const LinearShape& sh, int M, int N, int K, int cus, size_t workspace_bytes) {
  const int64_t tiles = (int64_t)((M + sh.bm - 1) / sh.bm) * (N / sh.bn);
  // flops per microsecond of one unit with this shape's wave tiles (measured, every unit busy)
  const double unit_rate = sh.shape == 0 ? 5.0e6 : (sh.shape == 1 ? 4.0e6 : 4.4e6);
  // bytes per microsecond one unit pulls from HBM: bounded by the copies it keeps in flight
  const double unit_pull = (sh.shape <= 1 || sh.shape == 5) ? 45e3 : 27e3;
  const double tile_us = std::max({2.0 * sh.bm * sh.bn * K / unit_rate, 2.0 * sh.bn * K / unit_pull,
                                   2.0 * (sh.bm + sh.bn) * K / 55e3});
  const size_t per_part = (size_t)M * N * sizeof(float);
  // (tiles that fill three quarters of the units by themselves are left whole)
  const int64_t s_max = tiles * 4 > (int64_t)cus * 3
                            ? 1
                            : std::min<int64_t>({(int64_t)(K / kLinBK) / 8, 8, (int64_t)(workspace_bytes / per_part)});
  // A round that is only begun costs less than a whole one (the chip is power-limited: with part
  // of the units idle the busy ones clock higher, and the workgroups of a launch do not run in
  // lockstep): 0.6 of the missing part, fitted.
  auto rounds_us = [&](int64_t workgroups, int64_t parts) {
    const double r = (double)workgroups / cus, whole = (double)((workgroups + cus - 1) / cus);
    return (r + 0.6 * (whole - r)) / (double)parts * tile_us;
  };
  LinearPlan best{sh, 1, rounds_us(tiles, 1)};
  for (int64_t s = 2; s <= s_max; ++s) {
    const double cost = rounds_us(tiles * s, s) + 4.0 + (double)s * per_part * 2.0 / 6e6;
    if (cost < best.cost_us * 0.95) best = LinearPlan{sh, (int)s, cost};  // not for a gain the model cannot resolve
  }
  return best;
}

// Tile shapes: 256 x 256 (or 192 x 256) for many tokens; 128 x 256 up to 1024 tokens; 128 x 64 up
// to 256 (four times the workgroups to pull on HBM); 64 x 128 and 32 x 128 for a few.  Where
// several shapes are possible the model decides, the first named being kept unless another is 5 %
// better: from 64 to 256 tokens the wide tile reads the tokens a quarter as often, but needs k
// cut into parts (a workspace) to fill the chip unless the output is very wide; from 256 tokens
// on the larger tiles win where the smaller ones' count is just over a whole number of rounds.
LinearPlan linear_plan(int M, int N, int K, int cus, size_t workspace_bytes) {
  auto best_of = [&](std::initializer_list<int> shapes) {
    LinearPlan best{};
    bool first = true;
    for (int i : shapes) {
      const LinearPlan pl = plan_shape(kLinearShapes[i], M, N, K, cus, workspace_bytes);
      if (first || pl.cost_us < best.cost_us * 0.95) best = pl;  // the first named is the default
      first = false;
    }
    return best;
  };
  if (M > 1024) return best_of({0, 5});
  if (M > 256) return best_of({1, 0, 5});
  if (M > 64) return best_of({2, 1});
  if (M > 32) return best_of({2, 3});
  return best_of({2, 3, 4});
}

}  // namespace

int linear_splits(int M, int N, int K, int cus, size_t workspace_bytes) {
  return linear_plan(M, N, K, cus, workspace_bytes).splits;
}

hipError_t launch_linear(int dtype, const void* x, const void* w, void* y, int M, int N, int K, void* workspace,
                         size_t workspace_bytes, hipStream_t stream) {
  PhaseTimer timer(FSF_PHASE_LINEAR, stream);
  const LinearPlan plan = linear_plan(M, N, K, device_compute_units(), workspace ? workspace_bytes : 0);
  const int shape = plan.sh.shape, bm = plan.sh.bm, bn = plan.sh.bn, stages = plan.sh.stages;
  const int tiles_m = (M + bm - 1) / bm, tiles_n = N / bn;
  const int splits = plan.splits;
  float* part = splits > 1 ? (float*)workspace : nullptr;
  const unsigned grid = (unsigned)(tiles_m * tiles_n * splits);
  const size_t lds_bytes = (size_t)stages * (bm + bn) * kRowBytes;
#define FSF_LINEAR(DT, T, BM, BN, WM, WN, ST, M16)                                                          \
  {                                                                                                 \
    if (const hipError_t e = allow_lds_bytes<&linear_kernel<DT, T, BM, BN, WM, WN, ST, M16>>((int)lds_bytes); \
        e != hipSuccess)                                                                            \
      return e;                                                                                     \
    linear_kernel<DT, T, BM, BN, WM, WN, ST, M16><<<grid, (BM / WM) * (BN / WN) * 64, lds_bytes, stream>>>( \
        (const T*)x, (const T*)w, (T*)y, M, N, K, tiles_m, tiles_n, part, splits);                  \
    if (splits > 1) {                                                                               \
      const size_t elems = (size_t)M * N;                                                           \
      linear_sum_kernel<DT, T><<<(unsigned)((elems / 8 + 255) / 256), 256, 0, stream>>>(part, (T*)y, elems, splits); \
    }                                                                                               \
  }
#define FSF_LINEAR_SHAPES(DT, T)                                      \
  if (shape == 0) FSF_LINEAR(DT, T, 256, 256, 128, 64, 2, true)             \
  else if (shape == 1) FSF_LINEAR(DT, T, 128, 256, 128, 32, 3, true)        \
  else if (shape == 2) FSF_LINEAR(DT, T, 128, 64, 64, 32, 5, false)          \
  else if (shape == 3) FSF_LINEAR(DT, T, 64, 128, 64, 32, 5, false)          \
  else if (shape == 4) FSF_LINEAR(DT, T, 32, 128, 32, 32, 6, false)   \
  else FSF_LINEAR(DT, T, 192, 256, 96, 64, 2, true)
  if (dtype == FSF_BF16) {
    FSF_LINEAR_SHAPES(FSF_BF16, bf16_t)
  } else {
    FSF_LINEAR_SHAPES(FSF_F16, f16_t)
  }
#undef FSF_LINEAR_SHAPES
#undef FSF_LINEAR
  return hipGetLastError();
}

}  // namespace fsf
