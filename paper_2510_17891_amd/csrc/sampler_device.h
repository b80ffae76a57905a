// Device-side arithmetic of the sampler, shared by the stand-alone sampling kernels and by the sampling epilogue of
// the output projection.  Contract (every operation in fp32 exactly as listed, so the argmax decision is
// reproducible bit for bit):
//   r    = word (i & 3) of Philox4x32-10(counter = (i >> 2, pos, seq, 0), key = (seed_lo, seed_hi))
//   u    = (2 (r >> 9) + 1) * 2^-24
//   g    = -flog(-flog(u)),  flog(x): x = m 2^e with m in [sqrt(1/2), sqrt(2)), f = m - 1,
//          p = Horner(c8..c0; f) with one fma per step, flog = fma(e, ln2, p * f)
//   y_i  = fma(z_i, 1/T, g)     token = argmax y_i, lowest index on ties
// Truncated sampling (top-k / top-p; the sampling settings of Appendix D) adds, equally exact:
//   order  tokens by descending order_key(z_i) (total order of the bit patterns), equal keys by ascending index
//   W_i    = fexp_weight(fma(z_i, 1/T, -(z_max * 1/T))): exp scaled to 2^32 and truncated to an integer --
//            t = x log2e, n = rint(t), f = fma(x, log2e, -n), 2^f by the degree-6 Taylor polynomial in f ln2
//            (one fma per step), scaled by 2^(n+32); 0 for x <= -22
//   top-k  the first min(k, V) tokens of the order;  top-p: with P = trunc(p 2^32), S = mass of those tokens,
//          T = max(1, floor(P S / 2^32)), the shortest prefix of the order whose mass reaches T
#pragma once
#include "device_utils.h"

namespace rl {

constexpr int kSamplePartFloats = 8;  // {best y, best idx bits, best z, -, running max of z/T, sum exp, -, -}

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ float flog(float x) {
  const uint32_t ix = __float_as_uint(x) - 0x3f3504f3u;
  const int e = (int)ix >> 23;
  const float m = __uint_as_float((ix & 0x007fffffu) + 0x3f3504f3u);
  const float f = __fsub_rn(m, 1.0f);
  float p = 0x1.6626eap-4f;
  p = __fmaf_rn(p, f, -0x1.26729ep-3f);
  p = __fmaf_rn(p, f, 0x1.322850p-3f);
  p = __fmaf_rn(p, f, -0x1.5329bep-3f);
  p = __fmaf_rn(p, f, 0x1.98b80ap-3f);
  p = __fmaf_rn(p, f, -0x1.0005a6p-2f);
  p = __fmaf_rn(p, f, 0x1.555790p-2f);
  p = __fmaf_rn(p, f, -0x1.fffff8p-2f);
  p = __fmaf_rn(p, f, 1.0f);
  const float r = __fmul_rn(p, f);
  return __fmaf_rn((float)e, 0x1.62e430p-1f, r);
}

__device__ __forceinline__ float gumbel(uint32_t bits) {
  const float u = __fmul_rn((float)(2u * (bits >> 9) + 1u), 0x1.0p-24f);
  const float t = -flog(u);
  return -flog(t);
}

__device__ __forceinline__ uint32_t order_key(float z) {  // ascending key = ascending value
  const uint32_t b = __float_as_uint(z);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float order_value(uint32_t key) {  // inverse of order_key
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}
__device__ __forceinline__ unsigned long long fexp_weight(float x) {
  if (!(x > -22.0f)) return 0ull;
  const float t = __fmul_rn(x, 0x1.715476p+0f);
  const float n = rintf(t);
  const float f = __fmaf_rn(x, 0x1.715476p+0f, -n);
  float p = 0x1.430912p-13f;
  p = __fmaf_rn(p, f, 0x1.5d87fep-10f);
  p = __fmaf_rn(p, f, 0x1.3b2ab6p-7f);
  p = __fmaf_rn(p, f, 0x1.c6b08ep-5f);
  p = __fmaf_rn(p, f, 0x1.ebfbe0p-3f);
  p = __fmaf_rn(p, f, 0x1.62e430p-1f);
  p = __fmaf_rn(p, f, 1.0f);
  return (unsigned long long)ldexpf(p, (int)n + 32);
}
// A cut of the order: token i with key k is kept iff it does not come after (key, idx).
struct OrderCut {
  uint32_t key;
  int32_t idx;
};
__device__ __forceinline__ bool kept_by(OrderCut c, uint32_t k, int i) { return k > c.key || (k == c.key && i <= c.idx); }

struct Best {
  float y;   // perturbed score
  int idx;   // vocabulary index, < 0 = empty
  float z;   // the raw logit at idx (needed for the log-probability)
};
__device__ __forceinline__ Best better(Best a, Best b) {
  // larger score wins; equal scores -> lower index.  idx < 0 marks "empty".
  if (b.idx < 0) return a;
  if (a.idx < 0) return b;
  if (b.y > a.y || (b.y == a.y && b.idx < a.idx)) return b;
  return a;
}
__device__ __forceinline__ void lse_merge(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  if (mn == -INFINITY) { m = mn; s = 0.f; return; }
  s = s * __expf(m - mn) + s2 * __expf(m2 - mn);
  m = mn;
}


__device__ __forceinline__ Best shfl_xor_best(Best b, int o) {
  return Best{__shfl_xor(b.y, o, kWave), __shfl_xor(b.idx, o, kWave), __shfl_xor(b.z, o, kWave)};
}

}  // namespace rl
