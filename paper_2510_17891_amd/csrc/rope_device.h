// Device code shared by every kernel that turns the QKV projection's split sums into a rotated query or key and
// that writes keys and values into KV pages.  The arithmetic is compiled with contraction off and its fused
// multiply-adds written out, so that all kernels including this file produce the same bits for the same row.
#pragma once
#include "device_utils.h"

namespace rl {

// KV page element offsets.
//   fp32 pages: plain [16 tokens][d].
//   bf16 pages (d = 128): K as [d/8][16 tokens][8] so that the 16 keys x 32 dims an MFMA step needs are
//   one coalesced 1 KiB read; V as [d/32][4 key groups][16 dims][2 x 4 keys] so that a lane's 16 bytes
//   are four keys of two dims -- the transposed operand of the P*V product with no shuffle.
__device__ __forceinline__ int k_page_offset_bf16(int t, int dd) { return ((dd >> 3) * 16 + t) * 8 + (dd & 7); }
__device__ __forceinline__ int v_page_offset_bf16(int t, int dd) {
  int dblk = dd >> 4, dl = dd & 15, jj = dblk >> 1, par = dblk & 1, g = t >> 2;
  return ((jj * 64 + g * 16 + dl) * 8) + par * 4 + (t & 3);
}

// bf16 pools: store an element that is already rounded.
__device__ __forceinline__ void kv_store_bf16_bits(void* pool_layer, int64_t page, int hk, int n_kv, int t, int dd,
                                                   uint16_t bits, bool is_v) {
  const size_t page_elems = (size_t)kPageTokens * 128;
  const size_t base = ((size_t)page * n_kv + hk) * 2 * page_elems;  // [page][kv head][K | V]; V's base pointer is one block in
  ((uint16_t*)pool_layer)[base + (is_v ? v_page_offset_bf16(t, dd) : k_page_offset_bf16(t, dd))] = bits;
}

// fp8 pages (e4m3 in the matrix cores' own encoding, no scales, d = 128): one byte per element, 2 KiB per (page, kv
// head) for K and as much for V.  K as [d/16][16 tokens][16] -- a lane's 16-byte load is one key's 16 consecutive
// dims, i.e. two matrix-core steps of 8 -- and V as [d/64][4 key groups][16 dims][2 x 2 x 4 keys]: a lane's 16 bytes
// are four keys of the four dims {dl, dl+16, dl+32, dl+48} of a 64-dim block.  After widening to bf16 in registers
// these are exactly the operands of the bf16 pages.
__device__ __forceinline__ int k_page_offset_fp8(int t, int dd) { return ((dd >> 4) * 16 + t) * 16 + (dd & 15); }
__device__ __forceinline__ int v_page_offset_fp8(int t, int dd) {
  const int jj = dd >> 5, par = (dd >> 4) & 1, dl = dd & 15, g = t >> 2;
  return (((jj >> 1) * 4 + g) * 16 + dl) * 16 + ((jj & 1) * 2 + par) * 4 + (t & 3);
}
// fp32 -> fp8 bits: nearest even in the hardware's conversion, magnitudes beyond the format's largest finite value
// (448) end there.
__device__ __forceinline__ uint32_t f2fp8(float x) {
  x = x > 448.0f ? 448.0f : (x < -448.0f ? -448.0f : x);
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x, 0.0f, 0, false) & 0xffu;
}
__device__ __forceinline__ float fp8_to_f(uint32_t b) { return __builtin_amdgcn_cvt_f32_fp8((int)b, 0); }
__device__ __forceinline__ void kv_store_fp8_bits(void* pool_layer, int64_t page, int hk, int n_kv, int t, int dd,
                                                  uint8_t bits, bool is_v) {
  const size_t page_bytes = (size_t)kPageTokens * 128;
  const size_t base = ((size_t)page * n_kv + hk) * 2 * page_bytes;  // [page][kv head][K | V]; V's base pointer is one block in
  ((uint8_t*)pool_layer)[base + (is_v ? v_page_offset_fp8(t, dd) : k_page_offset_fp8(t, dd))] = bits;
}

// KVT: 0 = fp32 pages, 1 = bf16 pages, 2 = fp8 pages (bf16 models only).
template <int KVT>
__device__ __forceinline__ void kv_store(void* pool_layer, int64_t page, int hk, int n_kv, int d, int t, int dd,
                                         float val, bool is_v) {
  if (KVT == 2) {
    kv_store_fp8_bits(pool_layer, page, hk, n_kv, t, dd, (uint8_t)f2fp8(val), is_v);
  } else if (KVT == 1) {
    kv_store_bf16_bits(pool_layer, page, hk, n_kv, t, dd, (uint16_t)f2bf(val), is_v);
  } else {
    const size_t page_elems = (size_t)kPageTokens * d;
    const size_t base = ((size_t)page * n_kv + hk) * 2 * page_elems;
    ((float*)pool_layer)[base + (size_t)t * d + dd] = val;
  }
}

// One head of one row, handled by one wave; lane i < d/2 owns the rotary pair (i, i + d/2), d <= 128.
// Two phases, so that a wave with several heads can have all their loads in flight before the arithmetic.
struct HeadPair {
  float v0, v1;  // elements i and i + d/2: sums of the split partials after load, final values after finish
  float2 cs;     // cos, sin of the pair at the row's position
  float g0, g1;  // RMSNorm gains of the two elements
};

// head_part: the head's d partial sums in split 0; consecutive splits are split_stride floats apart.
// rope_row: the table row of the position (d/2 entries); gain: d gains, or null without per-head normalisation.
// rotate: query or key (values are only summed).
template <bool BF16>
__device__ __forceinline__ HeadPair head_pair_load(const float* __restrict__ head_part, int S, size_t split_stride,
                                                   int d, int i, bool rotate, const float2* __restrict__ rope_row,
                                                   const void* __restrict__ gain) {
#pragma clang fp contract(off)
  const int half = d >> 1;
  HeadPair hp;
  hp.v0 = 0.f; hp.v1 = 0.f; hp.cs = make_float2(1.f, 0.f); hp.g0 = 1.f; hp.g1 = 1.f;
  if (i >= half) return hp;
  if (rotate) {
    hp.cs = rope_row[i];
    if (gain) {
      if (BF16) {
        const uint16_t* g = (const uint16_t*)gain;
        hp.g0 = bf2f(g[i]); hp.g1 = bf2f(g[i + half]);
      } else {
        const float* g = (const float*)gain;
        hp.g0 = g[i]; hp.g1 = g[i + half];
      }
    }
  }
#pragma unroll 4
  for (int sp = 0; sp < S; ++sp) {  // fixed order of the splits
    const float* p = head_part + sp * split_stride;
    hp.v0 += p[i];
    hp.v1 += p[i + half];
  }
  return hp;
}

// The same sums for callers that want the loads of several heads in flight at once: head_pair_issue only loads
// (S <= kHeadPairMaxS; the slots beyond S repeat the last split and are not used), head_pair_sum adds in split order.
constexpr int kHeadPairMaxS = 4;
struct HeadPairLoads { float a[kHeadPairMaxS][2]; };

__device__ __forceinline__ void head_pair_issue(HeadPairLoads& ld, const float* __restrict__ head_part, int S,
                                                size_t split_stride, int d, int i) {
  const int half = d >> 1;
#pragma unroll
  for (int sp = 0; sp < kHeadPairMaxS; ++sp) {
    const float* p = head_part + (sp < S ? sp : S - 1) * split_stride;
    ld.a[sp][0] = p[i];
    ld.a[sp][1] = p[i + half];
  }
}

__device__ __forceinline__ void head_pair_sum(HeadPair& hp, const HeadPairLoads& ld, int S) {
#pragma clang fp contract(off)
  float v0 = 0.f, v1 = 0.f;
#pragma unroll
  for (int sp = 0; sp < kHeadPairMaxS; ++sp) {
    if (sp < S) {
      v0 += ld.a[sp][0];
      v1 += ld.a[sp][1];
    }
  }
  hp.v0 = v0;
  hp.v1 = v1;
}

// Per-head RMSNorm (when normalise) and rotation of N heads side by side (their reductions overlap); must be reached
// by all 64 lanes of the wave.  Each head sees exactly the operations of N = 1.
template <int N>
__device__ __forceinline__ void head_pairs_finish(HeadPair (&hp)[N], int d, bool normalise, float eps) {
#pragma clang fp contract(off)
  if (normalise) {
    float ss[N];
#pragma unroll
    for (int n = 0; n < N; ++n) ss[n] = __builtin_fmaf(hp[n].v0, hp[n].v0, hp[n].v1 * hp[n].v1);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {  // the butterfly of wave_sum
      float other[N];
#pragma unroll
      for (int n = 0; n < N; ++n) other[n] = __shfl_xor(ss[n], o, kWave);
#pragma unroll
      for (int n = 0; n < N; ++n) ss[n] += other[n];
    }
#pragma unroll
    for (int n = 0; n < N; ++n) {
      const float mean = ss[n] / (float)d;
      const float inv = 1.0f / sqrtf(mean + eps);
      hp[n].v0 = (hp[n].v0 * inv) * hp[n].g0;
      hp[n].v1 = (hp[n].v1 * inv) * hp[n].g1;
    }
  }
#pragma unroll
  for (int n = 0; n < N; ++n) {
    const float v0 = hp[n].v0, v1 = hp[n].v1;
    const float a = v1 * hp[n].cs.y, b = v0 * hp[n].cs.y;
    hp[n].v0 = __builtin_fmaf(v0, hp[n].cs.x, -a);
    hp[n].v1 = __builtin_fmaf(v1, hp[n].cs.x, b);
  }
}

// One head; values (rotate = false) pass through.
__device__ __forceinline__ void head_pair_finish(HeadPair& hp, int d, bool rotate, bool normalise, float eps) {
  if (!rotate) return;  // wave-uniform
  HeadPair one[1] = {hp};
  head_pairs_finish<1>(one, d, normalise, eps);
  hp = one[0];
}

}  // namespace rl
