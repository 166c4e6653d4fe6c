// Device-side helpers shared by the HERO kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;   // raw bf16 bits

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// round-to-nearest-even through the hardware conversion (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ bf16_t f32_to_bf16_hw(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(bf16_t, b);
}

__device__ __forceinline__ uint32_t pack_bf16x2_hw(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float floatx2_t __attribute__((ext_vector_type(2)));
  floatx2_t v = {lo, hi};
  bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

__device__ __forceinline__ float unpack_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float unpack_hi(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }

template <typename T> struct ResidIO;
template <> struct ResidIO<float> {
  static __device__ __forceinline__ void load8(const float* p, float* v) {
    floatx4_t a = *reinterpret_cast<const floatx4_t*>(p);
    floatx4_t b = *reinterpret_cast<const floatx4_t*>(p + 4);
    v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
    v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
  }
  static __device__ __forceinline__ void store8(float* p, const float* v) {
    floatx4_t a = {v[0], v[1], v[2], v[3]};
    floatx4_t b = {v[4], v[5], v[6], v[7]};
    *reinterpret_cast<floatx4_t*>(p) = a;
    *reinterpret_cast<floatx4_t*>(p + 4) = b;
  }
};
template <> struct ResidIO<bf16_t> {
  static __device__ __forceinline__ void load8(const bf16_t* p, float* v) {
    u32x4_t a = *reinterpret_cast<const u32x4_t*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = unpack_lo(a[i]); v[2 * i + 1] = unpack_hi(a[i]); }
  }
  static __device__ __forceinline__ void store8(bf16_t* p, const float* v) {
    u32x4_t a;
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4_t*>(p) = a;
  }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
