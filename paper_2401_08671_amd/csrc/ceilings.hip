// Measurement aids: what the device sustains with nothing else in the way.
//
// The roofline fractions this library reports are against published peaks (8 TB/s HBM,
// 2.5 PFLOP/s dense bf16).  Neither is reachable by any kernel: streaming reads of scattered
// 16 KB tiles (the shape of a blocked KV cache, paper Sec. 2.1) top out below the HBM figure,
// and a register-resident MFMA loop runs at the clock the chip can hold under that load,
// which depends on the operand values and on the instruction (16x16x32 sustains more than 32x32x16).  These two kernels measure both, so that a kernel's
// distance from what is achievable can be told from its distance from the data sheet.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "fsf_measure.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int kMfmaBlocks = 1024;   // x 128 threads = two waves per SIMD on 256 compute units
constexpr int kMfmaThreads = 128;
constexpr int kMfmaPerIter = 8;

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

// Each lane keeps four A and four B fragments (from `operands`, 128 bytes per lane) and two
// 32x32 (or eight 16x16) accumulators in registers; nothing but MFMAs in the loop, the same
// flops per iteration in both forms: 8 x 32x32x16, or 16 x 16x16x32.
template <bool k16>
__global__ __launch_bounds__(kMfmaThreads) void mfma_loop_kernel(const uint4* __restrict__ operands,
                                                                 int iters, float* sink,
                                                                 unsigned long long* ticks) {
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;
  bf16x8_t a[4], b[4];
  for (int i = 0; i < 4; ++i) {
    a[i] = __builtin_bit_cast(bf16x8_t, operands[(size_t)gid * 8 + i]);
    b[i] = __builtin_bit_cast(bf16x8_t, operands[(size_t)gid * 8 + 4 + i]);
  }
  float s = 0.f;
  uint64_t t0, t1, r0, r1;
  if constexpr (k16) {
    // eight independent accumulators (with four the loop waits on its own results); the
    // instruction is written out so that each accumulator stays in the registers it starts in
    // (through the builtin the compiler moved them between register files every iteration)
    auto mfma16 = [](f32x4_t& c, const bf16x8_t& x, const bf16x8_t& y) {
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(x), "v"(y));
    };
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    f32x4_t c0 = zero, c1 = zero, c2 = zero, c3 = zero, c4 = zero, c5 = zero, c6 = zero, c7 = zero;
    t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        mfma16(c0, a[0], b[2 * j]);
        mfma16(c1, a[1], b[2 * j]);
        mfma16(c2, a[2], b[2 * j]);
        mfma16(c3, a[3], b[2 * j]);
        mfma16(c4, a[0], b[2 * j + 1]);
        mfma16(c5, a[1], b[2 * j + 1]);
        mfma16(c6, a[2], b[2 * j + 1]);
        mfma16(c7, a[3], b[2 * j + 1]);
      }
    }
    t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    const f32x4_t t = c0 + c1 + c2 + c3 + c4 + c5 + c6 + c7;
    s = t[0] + t[1] + t[2] + t[3];
  } else {
    f32x16_t c0, c1;
    for (int i = 0; i < 16; ++i) c0[i] = c1[i] = 0.f;
    t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(j + 1) & 3], b[j], c1, 0, 0, 0);
      }
    }
    t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i];
  }
  if (s == 123.456f) sink[gid & 63] = s;  // keeps the loop alive; practically never true
  if (gid == 0) {
    ticks[0] = t1 - t0;  // shader clock
    ticks[1] = r1 - r0;  // constant 100 MHz counter
  }
}

constexpr int kTileBytes = 16384;
constexpr int kTilesPerWave = 32;

// Each wave reads kTilesPerWave tiles of 16 KB, 16 loads of 16 bytes per lane in flight; the
// tiles of the buffer are visited in a scattered order (multiplication by an odd constant
// modulo the power-of-two tile count).
template <bool kNonTemporal>
__global__ __launch_bounds__(64) void stream_kernel(const uint4* __restrict__ buf, uint32_t tile_mask,
                                                    uint4* sink) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const uint32_t wave = blockIdx.x, lane = threadIdx.x;
  u32x4 acc = {0, 0, 0, 0};
  for (int t = 0; t < kTilesPerWave; ++t) {
    const uint32_t tile = ((wave * kTilesPerWave + t) * 2654435761u) & tile_mask;
    const u32x4* p = reinterpret_cast<const u32x4*>(buf) + (size_t)tile * (kTileBytes / 16) + lane;
    u32x4 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = kNonTemporal ? __builtin_nontemporal_load(p + i * 64) : p[i * 64];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= v[i];
  }
  if (acc[0] == 0x12345678u && acc[1] == 0x9abcdef0u) sink[0] = uint4{acc[0], acc[1], acc[2], acc[3]};
}

int timed(hipStream_t stream, hipEvent_t& e0, hipEvent_t& e1, float& ms) {
  if (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
      hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
    return FSF_ERR_HIP;
  return FSF_OK;
}

}  // namespace

namespace {

template <bool k16>
int mfma_ceiling(const void* operands, int64_t operand_bytes, int32_t iters, void* scratch, double* tflops_out,
                 double* mhz_out, void* hip_stream) {
  const int64_t need = (int64_t)kMfmaBlocks * kMfmaThreads * 128;
  if (!operands || operand_bytes < need || iters < 1 || !scratch || !tflops_out || !mhz_out)
    return FSF_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)hip_stream;
  float* sink = (float*)scratch;
  unsigned long long* ticks = (unsigned long long*)((char*)scratch + 1024);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return FSF_ERR_HIP;
  mfma_loop_kernel<k16><<<kMfmaBlocks, kMfmaThreads, 0, stream>>>((const uint4*)operands, 64, sink, ticks);  // warm-up
  int st = hipEventRecord(e0, stream) == hipSuccess ? FSF_OK : FSF_ERR_HIP;
  mfma_loop_kernel<k16><<<kMfmaBlocks, kMfmaThreads, 0, stream>>>((const uint4*)operands, iters, sink, ticks);
  float ms = 0.f;
  if (st == FSF_OK) st = timed(stream, e0, e1, ms);
  unsigned long long h[2] = {0, 0};
  if (st == FSF_OK && hipMemcpy(h, ticks, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) st = FSF_ERR_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != FSF_OK || hipGetLastError() != hipSuccess) return FSF_ERR_HIP;
  const double flops = (double)kMfmaBlocks * (kMfmaThreads / 64) * iters * kMfmaPerIter * 2.0 * 32 * 32 * 16;
  *tflops_out = flops / (ms * 1e-3) / 1e12;
  *mhz_out = h[1] ? 100.0 * (double)h[0] / (double)h[1] : 0.0;
  return FSF_OK;
}

}  // namespace

extern "C" int fsf_ceiling_mfma_bf16(const void* operands, int64_t operand_bytes, int32_t iters,
                                     void* scratch, double* tflops_out, double* mhz_out,
                                     void* hip_stream) {
  return mfma_ceiling<false>(operands, operand_bytes, iters, scratch, tflops_out, mhz_out, hip_stream);
}

extern "C" int fsf_ceiling_mfma_bf16_16x16x32(const void* operands, int64_t operand_bytes, int32_t iters,
                                              void* scratch, double* tflops_out, double* mhz_out,
                                              void* hip_stream) {
  return mfma_ceiling<true>(operands, operand_bytes, iters, scratch, tflops_out, mhz_out, hip_stream);
}

extern "C" int fsf_ceiling_hbm_read(const void* buf, int64_t bytes, int32_t nontemporal, void* scratch,
                                    double* gbs_out, void* hip_stream) {
  // the largest power-of-two number of tiles that fits, at least one tile per wave slot
  if (!buf || !scratch || !gbs_out || bytes < (int64_t)kTileBytes * kTilesPerWave) return FSF_ERR_INVALID_ARG;
  uint64_t n_tiles = 1;
  while (n_tiles * 2 * kTileBytes <= (uint64_t)bytes && n_tiles < (1u << 30)) n_tiles *= 2;
  const unsigned grid = (unsigned)(n_tiles / kTilesPerWave);
  if (grid == 0) return FSF_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return FSF_ERR_HIP;
  const int reps = 3;
  auto launch = [&] {
    if (nontemporal)
      stream_kernel<true><<<grid, 64, 0, stream>>>((const uint4*)buf, (uint32_t)(n_tiles - 1), (uint4*)scratch);
    else
      stream_kernel<false><<<grid, 64, 0, stream>>>((const uint4*)buf, (uint32_t)(n_tiles - 1), (uint4*)scratch);
  };
  launch();  // warm-up
  int st = hipEventRecord(e0, stream) == hipSuccess ? FSF_OK : FSF_ERR_HIP;
  for (int r = 0; r < reps; ++r) launch();
  float ms = 0.f;
  if (st == FSF_OK) st = timed(stream, e0, e1, ms);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != FSF_OK || hipGetLastError() != hipSuccess) return FSF_ERR_HIP;
  *gbs_out = (double)n_tiles * kTileBytes * reps / (ms * 1e-3) / 1e9;
  return FSF_OK;
}
