// Linear layer over the tokens of a pass: y[t, o] = sum_k x[t, k] * w[o, k]   (bf16 / f16, fp32 accumulation).
//
// Besides attention, a forward pass applies dense projections to every token of the ragged
// batch (query/key/value and output projections, gated MLP); they are what makes a pass
// weight-bound while it holds few tokens and compute-bound once it holds many (paper Sec. 3.1),
// and so what fixes a sensible token budget.  Dense contraction: matrix cores.
//
// One workgroup of 512 threads (8 waves, two per SIMD) computes a BM x 256 tile of y; a wave owns
// WM x WN of it as 32x32x16 MFMA tiles.  Both operands are k-contiguous in memory (tokens and
// weight rows alike), so they are staged the same way: BK = 32 k-elements at a time, row-major
// tiles [rows][64 bytes] in LDS, copied there directly from HBM/L2 (global_load_lds, 16 bytes per
// lane, no registers) in a ring of four stages, three k-steps ahead of the MFMAs.  A lane of a
// copy instruction always fills the next 16 bytes of LDS, so the XOR swizzle that makes the later
// ds_read_b128 fragment reads conflict-free is applied on the global side: 16-byte chunk c of tile
// row r sits at chunk c ^ ((r >> 2) & 3)  (rows are 64 bytes = 4 chunks apart, a b128 read serves
// 16 lanes per clock from 64 banks: rows r, r+4, r+8, r+12 must land on different chunks).
//
// The product is formed transposed, D[o, t] = W . X^T (A operand = weight rows, B operand =
// tokens): a lane then owns 4 consecutive output features of one token per register quad, which
// it stores as 8 (or 16) contiguous bytes.
//
// The copies and their waits are written as inline asm: the compiler does not track LDS-DMA
// per stage and would wait for every copy in flight before each LDS read.  The protocol per
// k-step kt (every wave issues the same number of copies, so the counters agree):
//   wait until this wave's copies of step kt have landed (all but the two younger steps)
//   workgroup barrier: everybody's copies of step kt are in LDS, everybody has finished reading
//                      step kt-1, whose stage the next copy overwrites
//   start the copies of step kt+3 (past the end of k: the last step again, never read)
//   fragments of step kt from LDS, 16 MFMAs
#include "fsf_internal.h"
#include "mma.h"
#include "numeric.h"

namespace fsf {
namespace {

constexpr int kLinThreads = 512;
constexpr int kLinBN = 256;   // output features per workgroup
constexpr int kLinBK = 32;    // k elements per stage: 64 bytes per tile row
constexpr int kLinStages = 4;
constexpr int kRowBytes = kLinBK * 2;

typedef __attribute__((address_space(3))) char lin_lds_char;

// one copy instruction of a wave: 16 tile rows x 64 bytes, lane -> (row lane / 4, physical chunk lane % 4)
__device__ __forceinline__ void copy16(uint32_t lds_addr, uint32_t voffset, const char* base) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr), "v"(voffset), "s"(base)
      : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_copies_but() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// BM: tokens per workgroup (256 or 128).  Waves: (BM / WM) x (256 / WN) = 8.
template <int DT, typename T, int BM>
__global__ __launch_bounds__(kLinThreads) void linear_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                              T* __restrict__ y, int M, int N, int K, int tiles_m,
                                                              int tiles_n) {
  constexpr int WM = 128;                 // tokens per wave
  constexpr int WN = BM == 256 ? 64 : 32; // output features per wave
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr int kXTile = BM * kRowBytes, kWTile = kLinBN * kRowBytes;
  constexpr int kStage = kXTile + kWTile;
  extern __shared__ __attribute__((aligned(1024))) char lin_lds[];
  lin_lds_char* lds = (lin_lds_char*)lin_lds;

  // ---- which tile: workgroups are dealt to the 8 dies in turn; give each die a compact block of
  // tiles (consecutive ids on one die), walked in groups of 4 token tiles so that the tiles
  // running together on a die share weight and token panels in its L2
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
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
  const int l32 = lane & 31, hg = lane >> 5;

  // ---- copies: wave v fills rows [32 v, 32 v + 32) of the weight tile (256 rows) with two
  // instructions, and rows of the token tile likewise (BM = 128: waves 0..3 fill 32 rows each...
  // every wave issues the same count, so with BM = 128 each wave takes 16 rows, one instruction)
  constexpr int kXCopies = BM / 128;      // instructions per wave for the token tile
  const int crow = lane >> 2, cpc = lane & 3;
  uint32_t x_off[kXCopies], w_off[2];
#pragma unroll
  for (int j = 0; j < kXCopies; ++j) {
    const int r = wave * (16 * kXCopies) + j * 16 + crow;
    const int row = min(m0 + r, M - 1);   // rows past the last token are copies of it, never stored
    x_off[j] = (uint32_t)row * (uint32_t)K * 2u + (uint32_t)((cpc ^ ((r >> 2) & 3)) << 4);
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int r = wave * 32 + j * 16 + crow;
    w_off[j] = (uint32_t)(n0 + r) * (uint32_t)K * 2u + (uint32_t)((cpc ^ ((r >> 2) & 3)) << 4);
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  const int nk = K / kLinBK;
  auto issue = [&](int kt) {  // copies of k-step min(kt, nk - 1) into stage kt % 4
    const int ks = min(kt, nk - 1);
    const uint32_t stage = lds0 + (uint32_t)(kt % kLinStages) * kStage;
    const char* xb = reinterpret_cast<const char*>(x) + (size_t)ks * kRowBytes;
    const char* wb = reinterpret_cast<const char*>(w) + (size_t)ks * kRowBytes;
#pragma unroll
    for (int j = 0; j < kXCopies; ++j)
      copy16(stage + (uint32_t)(wave * (16 * kXCopies) + j * 16) * kRowBytes, x_off[j], xb);
#pragma unroll
    for (int j = 0; j < 2; ++j) copy16(stage + kXTile + (uint32_t)(wave * 32 + j * 16) * kRowBytes, w_off[j], wb);
  };
  constexpr int kCopiesPerStep = kXCopies + 2;

  // ---- fragments: tile row blk * 32 + l32, logical chunk 2 t + hg of k-substep t
  const int wm = wave % (BM / WM), wn = wave / (BM / WM);
  uint32_t frag_off[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) frag_off[t] = (uint32_t)(l32 * kRowBytes + (((2 * t + hg) ^ ((l32 >> 2) & 3)) << 4));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) u32x4 lds_u32x4;

  f32x16_t acc[NB][MB];
#pragma unroll
  for (int a = 0; a < NB; ++a)
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  issue(0);
  issue(1);
  issue(2);
  for (int kt = 0; kt < nk; ++kt) {
    wait_copies_but<2 * kCopiesPerStep>();
    __builtin_amdgcn_s_barrier();
    issue(kt + 3);
    const lin_lds_char* st = lds + (kt % kLinStages) * kStage;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      frag8 xf[MB], wf[NB];
#pragma unroll
      for (int b = 0; b < MB; ++b) {
        const u32x4 v = *reinterpret_cast<const lds_u32x4*>(st + (wm * WM + b * 32) * kRowBytes + frag_off[t]);
        xf[b] = frag8{{v[0], v[1], v[2], v[3]}};
      }
#pragma unroll
      for (int a = 0; a < NB; ++a) {
        const u32x4 v = *reinterpret_cast<const lds_u32x4*>(st + kXTile + (wn * WN + a * 32) * kRowBytes + frag_off[t]);
        wf[a] = frag8{{v[0], v[1], v[2], v[3]}};
      }
#pragma unroll
      for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < MB; ++b) acc[a][b] = Mma<DT>::mfma32(wf[a], xf[b], acc[a][b]);
    }
  }
  wait_copies_but<0>();  // the copies past the end of k are still in flight: let them land before the workgroup ends

  // ---- store: acc[a][b][r] is output feature n0 + wn WN + 32 a + 8 (r / 4) + 4 hg + r % 4 of token
  // m0 + wm WM + 32 b + l32
#pragma unroll
  for (int b = 0; b < MB; ++b) {
    const int row = m0 + wm * WM + b * 32 + l32;
    if (row >= M) continue;
    T* yrow = y + (size_t)row * N + n0 + wn * WN + 4 * hg;
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint2 v;
        v.x = Mma<DT>::pack2(acc[a][b][4 * q], acc[a][b][4 * q + 1]);
        v.y = Mma<DT>::pack2(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
        *reinterpret_cast<uint2*>(yrow + a * 32 + q * 8) = v;
      }
  }
}

}  // namespace

hipError_t launch_linear(int dtype, const void* x, const void* w, void* y, int M, int N, int K, hipStream_t stream) {
  PhaseTimer timer(FSF_PHASE_LINEAR, stream);
  const int tiles_n = N / kLinBN;
  // many tokens: 256-token tiles; few: 128-token tiles, so that more workgroups share the weight stream
  const bool big = M > 1024;
  const int bm = big ? 256 : 128;
  const int tiles_m = (M + bm - 1) / bm;
  const unsigned grid = (unsigned)(tiles_m * tiles_n);
  const size_t lds_bytes = (size_t)kLinStages * (bm + kLinBN) * kRowBytes;
#define FSF_LINEAR(DT, T, BM)                                                                       \
  {                                                                                                 \
    static bool attr_set = false;                                                                   \
    if (!attr_set) {                                                                                \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&linear_kernel<DT, T, BM>),                 \
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);              \
      attr_set = true;                                                                              \
    }                                                                                               \
    linear_kernel<DT, T, BM><<<grid, kLinThreads, lds_bytes, stream>>>((const T*)x, (const T*)w, (T*)y, M, N, K, \
                                                                       tiles_m, tiles_n);           \
  }
  if (dtype == FSF_BF16) {
    if (big) FSF_LINEAR(FSF_BF16, bf16_t, 256) else FSF_LINEAR(FSF_BF16, bf16_t, 128)
  } else {
    if (big) FSF_LINEAR(FSF_F16, f16_t, 256) else FSF_LINEAR(FSF_F16, f16_t, 128)
  }
#undef FSF_LINEAR
  return hipGetLastError();
}

}  // namespace fsf
