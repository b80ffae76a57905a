// Small device helpers shared by the gfx950 kernels: bf16 packing, wave64 reductions, vector types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rl {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;
constexpr int kPageTokens = 16;  // tokens per KV page

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f2bf(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) { return f2bf(lo) | (f2bf(hi) << 16); }

// The projections multiply on the f16 grid: the packed weights hold the f16 image of the model's bf16 weights (made
// once, when they are packed), activations are written as f16 by their producers.  f16 keeps 11 significant bits against bf16's 8, so the rounding of an
// activation entering a projection is 8 times smaller, at the same bytes and the same matrix-core rate.
//
// Two bf16 (one 32-bit word) -> two f16.  Exact for 2^-14 <= |w| <= 65504 (a bf16 significand fits an f16 one);
// smaller magnitudes are cut toward zero on the f16 subnormal grid (absolute error < 2^-24), larger ones end at
// +-65504.
__device__ __forceinline__ uint32_t bf2_to_h2(uint32_t w) {
  const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xffff0000u);
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
// fp32 -> f16 bits, round to nearest even, finite values beyond the f16 range end at +-65504 (NaN stays NaN).
__device__ __forceinline__ uint32_t f2h(float x) {
  x = x > 65504.0f ? 65504.0f : (x < -65504.0f ? -65504.0f : x);
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
}
__device__ __forceinline__ uint32_t pack2h(float lo, float hi) { return f2h(lo) | (f2h(hi) << 16); }

// Storage-type accessors used by the dtype-generic kernels.
__device__ __forceinline__ float load_as_float(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const uint16_t* p, size_t i) { return bf2f(p[i]); }
__device__ __forceinline__ void store_from_float(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_from_float(uint16_t* p, size_t i, float v) { p[i] = (uint16_t)f2bf(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

}  // namespace rl
