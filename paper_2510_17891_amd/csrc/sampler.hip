// Stand-alone Gumbel-max sampling kernels (logits in memory) and the merge stage shared with the fused path.
// The arithmetic contract lives in sampler_device.h.  The log-probability log softmax(z/T)[token] is accumulated
// in fp32 (tolerance, not bit-exact).
#include "kernels.h"
#include "sampler_device.h"

namespace rl {

namespace {

// Stage 1: grid (tiles, rows); each block scans kSampleTile vocabulary entries of one row of fp32 logits.
__global__ __launch_bounds__(256) void sample_stage1_kernel(const float* __restrict__ logits, int V,
                                                            const RowMeta* __restrict__ rows, int pos_offset, float inv_t,
                                                            int greedy, uint32_t seed_lo, uint32_t seed_hi,
                                                            const int32_t* __restrict__ forced, float* __restrict__ forced_z,
                                                            float* __restrict__ part, int n_tiles) {
  __shared__ float sh_y[4], sh_z[4], sh_m[4], sh_s[4];
  __shared__ int sh_i[4];
  const int tile = blockIdx.x, r = blockIdx.y;
  const RowMeta rm = rows[r];
  const uint32_t pos = (uint32_t)(rm.pos + pos_offset), seq = (uint32_t)rm.seq;
  const float* z = logits + (size_t)r * V;
  const int f = forced ? forced[r] : -1;
  Best best{-INFINITY, -1, 0.f};
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
      best = better(best, Best{y, i, zi});
      lse_merge(m, s, zi * inv_t, 1.0f);
      if (i == f) forced_z[r] = zi;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    best = better(best, shfl_xor_best(best, o));
    lse_merge(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave));
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sh_y[wave] = best.y; sh_i[wave] = best.idx; sh_z[wave] = best.z; sh_m[wave] = m; sh_s[wave] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      best = better(best, Best{sh_y[w], sh_i[w], sh_z[w]});
      lse_merge(m, s, sh_m[w], sh_s[w]);
    }
    float* p = part + ((size_t)r * n_tiles + tile) * kSamplePartFloats;
    *(float4*)p = make_float4(best.y, __int_as_float(best.idx), best.z, 0.f);
    *(float4*)(p + 4) = make_float4(m, s, 0.f, 0.f);
  }
}

// Stage 2: one block of 1024 threads per row merges the tile partials and emits token and log-probability.
__global__ __launch_bounds__(1024) void sample_stage2_kernel(const float* __restrict__ part, int n_tiles, int V,
                                                             const int32_t* __restrict__ forced,
                                                             const float* __restrict__ forced_z, float inv_t,
                                                             int32_t* __restrict__ out_tok, float* __restrict__ out_lp) {
  __shared__ float sh_y[16], sh_z[16], sh_m[16], sh_s[16];
  __shared__ int sh_i[16];
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Best best{-INFINITY, -1, 0.f};
  float m = -INFINITY, s = 0.f;
  for (int t = threadIdx.x; t < n_tiles; t += 1024) {
    const float* p = part + ((size_t)r * n_tiles + t) * kSamplePartFloats;
    const float4 a = *(const float4*)p;
    const float4 b = *(const float4*)(p + 4);
    best = better(best, Best{a.x, __float_as_int(a.y), a.z});
    lse_merge(m, s, b.x, b.y);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    best = better(best, shfl_xor_best(best, o));
    lse_merge(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave));
  }
  if (lane == 0) { sh_y[wave] = best.y; sh_i[wave] = best.idx; sh_z[wave] = best.z; sh_m[wave] = m; sh_s[wave] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w) {
      best = better(best, Best{sh_y[w], sh_i[w], sh_z[w]});
      lse_merge(m, s, sh_m[w], sh_s[w]);
    }
    int tok = best.idx < 0 ? 0 : best.idx;  // idx < 0 only when every score was NaN
    float zt = best.z;
    if (forced != nullptr && forced[r] >= 0 && forced[r] < V) { tok = forced[r]; zt = forced_z[r]; }
    out_tok[r] = tok;
    out_lp[r] = zt * inv_t - (m + logf(s));
  }
}

}  // namespace

void launch_sample(hipStream_t st, const float* logits, int M, int V, const RowMeta* rows, int pos_offset,
                   const int32_t* forced, float temperature, uint64_t seed, float* part, float* forced_z,
                   int32_t* out_tokens, float* out_logprobs) {
  const int n_tiles = (V + kSampleTile - 1) / kSampleTile;
  const int greedy = !(temperature > 0.f);
  const float inv_t = greedy ? 1.0f : 1.0f / temperature;
  dim3 grid(n_tiles, M);
  sample_stage1_kernel<<<grid, 256, 0, st>>>(logits, V, rows, pos_offset, inv_t, greedy, (uint32_t)(seed & 0xffffffffu),
                                             (uint32_t)(seed >> 32), forced, forced_z, part, n_tiles);
  sample_stage2_kernel<<<M, 1024, 0, st>>>(part, n_tiles, V, forced, forced_z, inv_t, out_tokens, out_logprobs);
}

void launch_sample_merge(hipStream_t st, const float* part, int n_tiles, int M, int V, const int32_t* forced,
                         const float* forced_z, float temperature, int32_t* out_tokens, float* out_logprobs) {
  const float inv_t = temperature > 0.f ? 1.0f / temperature : 1.0f;
  sample_stage2_kernel<<<M, 1024, 0, st>>>(part, n_tiles, V, forced, forced_z, inv_t, out_tokens, out_logprobs);
}

}  // namespace rl
