// Device-side helpers shared by the SVD-Cache kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svdc {

constexpr int kWave = 64;

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- element load / store for the two storage types ------------------------
__device__ __forceinline__ float ld_elem(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld_elem(const bf16_t* p, int64_t i) { return (float)p[i]; }
__device__ __forceinline__ void st_elem(float* p, int64_t i, float v) { p[i] = v; }
// float -> bf16 conversion rounds to nearest even
__device__ __forceinline__ void st_elem(bf16_t* p, int64_t i, float v) { p[i] = (bf16_t)v; }

// bf16 pair packed in a 32-bit word <-> two floats
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32, RNE
  return __builtin_bit_cast(uint32_t, b);
}

// split 8 float32 values into bf16 high and low operand words
__device__ __forceinline__ void split_operand(const float (&c)[8], u32x4* hi, u32x4* lo) {
  float rem[8];
  uint32_t h[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h[i] = pack_bf16(c[2 * i], c[2 * i + 1]);
    rem[2 * i] = c[2 * i] - bf16_lo(h[i]);
    rem[2 * i + 1] = c[2 * i + 1] - bf16_hi(h[i]);
  }
  *hi = u32x4{h[0], h[1], h[2], h[3]};
  *lo = u32x4{pack_bf16(rem[0], rem[1]), pack_bf16(rem[2], rem[3]), pack_bf16(rem[4], rem[5]),
              pack_bf16(rem[6], rem[7])};
}

// ---- wavefront reductions -----------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

}  // namespace svdc
