// gfx950 matrix-core (MFMA) wrappers for bf16 and f16 operands with fp32 accumulation.
//
// Register layouts (wave of 64 lanes, checked on hardware):
//   16x16x32:  A: lane l holds row l%16, 8 consecutive k of k-group l/16
//              B: lane l holds col l%16, the same 8 k of k-group l/16
//              C: lane l holds col l%16, rows 4*(l/16) + r, r = 0..3
//   32x32x16:  A: lane l holds row l%32, 8 consecutive k of k-group l/32
//              B: lane l holds col l%32, same k
//              C: lane l holds col l%32, rows 8*(r/4) + 4*(l/32) + r%4, r = 0..15
// Only "A and B agree on which k sits in which (k-group, slot)" matters to a dot
// product, so kernels are free to decide which memory element plays which k.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fsf.h"

namespace fsf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

// 8 storage elements as raw bits
struct __attribute__((aligned(16))) frag8 { uint32_t w[4]; };

__device__ __forceinline__ frag8 load_frag8(const void* ptr) {
  const uint4 v = *reinterpret_cast<const uint4*>(ptr);
  return frag8{{v.x, v.y, v.z, v.w}};
}
// Same load marked non-temporal: for data that is read exactly once (the K/V stream of a
// generation row), so it does not displace reusable lines in the caches.  On MI355X this
// raises achievable HBM read bandwidth by about a tenth.
__device__ __forceinline__ frag8 load_frag8_stream(const void* ptr) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(ptr));
  return frag8{{v[0], v[1], v[2], v[3]}};
}
__device__ __forceinline__ frag8 zero_frag8() { return frag8{{0u, 0u, 0u, 0u}}; }

template <int DT> struct Mma;

template <> struct Mma<FSF_BF16> {
  static __device__ __forceinline__ f32x4_t mfma16(const frag8& a, const frag8& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ f32x16_t mfma32(const frag8& a, const frag8& b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
  // two floats -> two storage elements in one dword (lo = a, hi = b), round to nearest even
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    bf16x2_t v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
  }
};

template <> struct Mma<FSF_F16> {
  static __device__ __forceinline__ f32x4_t mfma16(const frag8& a, const frag8& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                  __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ f32x16_t mfma32(const frag8& a, const frag8& b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                  __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2_t;
    f16x2_t v;
    v[0] = (_Float16)a;
    v[1] = (_Float16)b;
    return __builtin_bit_cast(uint32_t, v);
  }
};

// In-lane transpose helpers: pick the low / high 16-bit halves of two dwords.
__device__ __forceinline__ uint32_t pack_lo16(uint32_t first, uint32_t second) {
  return __builtin_amdgcn_perm(second, first, 0x05040100u);  // {second.lo, first.lo}
}
__device__ __forceinline__ uint32_t pack_hi16(uint32_t first, uint32_t second) {
  return __builtin_amdgcn_perm(second, first, 0x07060302u);  // {second.hi, first.hi}
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace fsf
