// Gumbel-max sampling with counter-based random numbers, plus the log-probability of the chosen token.
//
// Contract (every operation in fp32 exactly as listed, so the argmax decision is reproducible bit for bit):
//   r    = word (i & 3) of Philox4x32-10(counter = (i >> 2, pos, seq, 0), key = (seed_lo, seed_hi))
//   u    = (2 (r >> 9) + 1) * 2^-24
//   g    = -flog(-flog(u)),  flog(x): x = m 2^e with m in [sqrt(1/2), sqrt(2)), f = m - 1,
//          p = Horner(c8..c0; f) with one fma per step, flog = fma(e, ln2, p * f)
//   y_i  = fma(z_i, 1/T, g)     token = argmax y_i, lowest index on ties
// The log-probability log softmax(z/T)[token] is accumulated in fp32 (tolerance, not bit-exact).
#include "device_utils.h"
#include "kernels.h"

namespace rl {

namespace {

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

struct Best {
  float y;
  int idx;
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

// Stage 1: grid (tiles, rows); each block scans kSampleTile vocabulary entries of one row.
// part[row][tile] = {best y, best idx (as int bits), running max of z/T, sum exp(z/T - max)}.
__global__ __launch_bounds__(256) void sample_stage1_kernel(const float* __restrict__ logits, int V,
                                                            const RowMeta* __restrict__ rows, int pos_offset, float inv_t,
                                                            int greedy, uint32_t seed_lo, uint32_t seed_hi,
                                                            float4* __restrict__ part, int n_tiles) {
  __shared__ float sh_y[4], sh_m[4], sh_s[4];
  __shared__ int sh_i[4];
  const int tile = blockIdx.x, r = blockIdx.y;
  const RowMeta rm = rows[r];
  const uint32_t pos = (uint32_t)(rm.pos + pos_offset), seq = (uint32_t)rm.seq;
  const float* z = logits + (size_t)r * V;
  Best best{-INFINITY, -1};
  float m = -INFINITY, s = 0.f;
  const int i_end = min(V, (tile + 1) * kSampleTile);
  for (int i0 = tile * kSampleTile + threadIdx.x * 4; i0 < i_end; i0 += 256 * 4) {
    uint32_t rnd[4] = {0, 0, 0, 0};
    if (!greedy) philox4x32_10((uint32_t)i0 >> 2, pos, seq, 0u, seed_lo, seed_hi, rnd);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = i0 + e;
      if (i >= i_end) break;
      const float zi = z[i];
      const float y = greedy ? zi : __fmaf_rn(zi, inv_t, gumbel(rnd[e]));
      best = better(best, Best{y, i});
      lse_merge(m, s, zi * inv_t, 1.0f);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Best b2{__shfl_xor(best.y, o, kWave), __shfl_xor(best.idx, o, kWave)};
    best = better(best, b2);
    lse_merge(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave));
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sh_y[wave] = best.y; sh_i[wave] = best.idx; sh_m[wave] = m; sh_s[wave] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      best = better(best, Best{sh_y[w], sh_i[w]});
      lse_merge(m, s, sh_m[w], sh_s[w]);
    }
    part[(size_t)r * n_tiles + tile] = make_float4(best.y, __int_as_float(best.idx), m, s);
  }
}

// Stage 2: one wave per row merges the tiles and emits token and log-probability.
__global__ __launch_bounds__(64) void sample_stage2_kernel(const float* __restrict__ logits, int V,
                                                           const float4* __restrict__ part, int n_tiles,
                                                           const int32_t* __restrict__ forced, float inv_t,
                                                           int32_t* __restrict__ out_tok, float* __restrict__ out_lp) {
  const int r = blockIdx.x, lane = threadIdx.x;
  Best best{-INFINITY, -1};
  float m = -INFINITY, s = 0.f;
  for (int t = lane; t < n_tiles; t += 64) {
    const float4 p = part[(size_t)r * n_tiles + t];
    best = better(best, Best{p.x, __float_as_int(p.y)});
    lse_merge(m, s, p.z, p.w);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Best b2{__shfl_xor(best.y, o, kWave), __shfl_xor(best.idx, o, kWave)};
    best = better(best, b2);
    lse_merge(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave));
  }
  if (lane == 0) {
    int tok = best.idx < 0 ? 0 : best.idx;  // only when every score was NaN
    if (forced != nullptr && forced[r] >= 0) tok = min(forced[r], V - 1);
    out_tok[r] = tok;
    out_lp[r] = logits[(size_t)r * V + tok] * inv_t - (m + logf(s));
  }
}

}  // namespace

void launch_sample(hipStream_t st, const float* logits, int M, int V, const RowMeta* rows, int pos_offset,
                   const int32_t* forced, float temperature, uint64_t seed, float* part, int32_t* out_tokens,
                   float* out_logprobs) {
  const int n_tiles = (V + kSampleTile - 1) / kSampleTile;
  const int greedy = !(temperature > 0.f);
  const float inv_t = greedy ? 1.0f : 1.0f / temperature;
  dim3 grid(n_tiles, M);
  sample_stage1_kernel<<<grid, 256, 0, st>>>(logits, V, rows, pos_offset, inv_t, greedy, (uint32_t)(seed & 0xffffffffu),
                                             (uint32_t)(seed >> 32), (float4*)part, n_tiles);
  sample_stage2_kernel<<<M, 64, 0, st>>>(logits, V, (const float4*)part, n_tiles, forced, inv_t, out_tokens,
                                         out_logprobs);
}

}  // namespace rl
