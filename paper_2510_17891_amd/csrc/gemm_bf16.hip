// Weight-streaming bf16 GEMM for decode-sized batches:  Y[M x N] = X[M x K] * W[N x K]^T.
//
// At M <= 256 the projection is bound by reading W once from HBM (M flop per weight byte), so the kernel is
// organised around that stream: both operands are stored fragment-major (see frag_offset), which makes every
// global load a fully coalesced 1 KiB wave access that lands directly in MFMA 32x32x16 operand registers -- no
// LDS staging, no shuffles.  A wave owns a 64 x (32*MB) output tile over a slice of K; the four waves of a
// block take four K slices and add their accumulators through LDS in a fixed order; further K splits across
// blocks (to put >= 256 blocks on the chip for the small matrices) leave fp32 partials that the consumer sums.
#include "device_utils.h"
#include "kernels.h"
#include "sampler_device.h"

namespace rl {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <int MB>
struct Frags {
  u32x4_t a[2][4];
  u32x4_t b[MB][4];
};

template <int MB>
__device__ __forceinline__ void load_frags(Frags<MB>& f, const u32x4_t* __restrict__ w0, const u32x4_t* __restrict__ w1,
                                           const u32x4_t* const* __restrict__ xb, int kb, int lane) {
  // block (rb, kb) = 256 uint4; sub-load t is [t*64 + lane]
  const int o = kb * 256 + lane;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    f.a[0][t] = __builtin_nontemporal_load(w0 + o + t * 64);
    f.a[1][t] = __builtin_nontemporal_load(w1 + o + t * 64);
  }
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int t = 0; t < 4; ++t) f.b[mb][t] = xb[mb][o + t * 64];
}

template <int MB>
__device__ __forceinline__ void mma_frags(const Frags<MB>& f, f32x16_t (&acc)[2][MB]) {
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, f.a[nb][t]),
                                                              __builtin_bit_cast(bf16x8_t, f.b[mb][t]), acc[nb][mb], 0,
                                                              0, 0);
}

// grid: x = N tile, y = K split, z = M tile of 32*MB rows.
//   EPI == kEpiPartial: tile = 64 output columns (row blocks 2x, 2x+1 of W); out fp32 [S][M][N].
//   EPI == kEpiSwiGLU : tile = 32 output columns (gate block x, up block x + N/32); out bf16 fragment-major [M x N].
//   EPI == kEpiSample : tile = 64 vocabulary entries; the logits stay in registers: temperature, Gumbel noise, running
//                       arg-max and log-sum-exp are taken per (row, tile) and only those partials are written
//                       (plus the logits themselves when the caller asked for them).
// ST = k blocks a wave keeps in flight.  HBM latency is ~10x the MFMA time of a block, so the loop is a ring of
// ST register buffers: compute block i, immediately re-issue its buffer for block i + ST.  The scheduling
// barriers keep the compiler from sinking the loads below the next block's MFMAs.
template <int MB, int EPI, int ST>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                        void* __restrict__ out, int M, int N, int K, int kb_per_wave,
                                                        SampleEpilogue se) {
  __shared__ float red[4][16][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int KB = K >> 6;
  const int m_blk0 = blockIdx.z * MB;
  const int n_blocks_m = (M + 31) >> 5;

  int rb0, rb1;
  if (EPI == kEpiSwiGLU) { rb0 = blockIdx.x; rb1 = blockIdx.x + (N >> 5); }
  else                   { rb0 = blockIdx.x * 2; rb1 = rb0 + 1; }
  const u32x4_t* w0 = W + (size_t)rb0 * KB * 256;
  const u32x4_t* w1 = W + (size_t)rb1 * KB * 256;
  const u32x4_t* xb[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    int b = m_blk0 + mb;
    if (b >= n_blocks_m) b = n_blocks_m - 1;  // clamp: surplus column blocks are computed but never stored
    xb[mb] = X + (size_t)b * KB * 256;
  }

  f32x16_t acc[2][MB];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nb][mb][r] = 0.f;

  const int kb0 = (blockIdx.y * 4 + wave) * kb_per_wave;
  const int n = kb_per_wave;
  Frags<MB> f[ST];
#pragma unroll
  for (int s = 0; s < ST; ++s) load_frags<MB>(f[s], w0, w1, xb, kb0 + s, lane);  // the launcher guarantees ST <= n
  const int full = n / ST, rem = n - full * ST;
  int b = 0;
  for (int r = 0; r + 1 < full; ++r) {  // steady state: every buffer is refilled
#pragma unroll
    for (int s = 0; s < ST; ++s) {
      mma_frags<MB>(f[s], acc);
      __builtin_amdgcn_sched_barrier(0);
      load_frags<MB>(f[s], w0, w1, xb, kb0 + b + s + ST, lane);
      __builtin_amdgcn_sched_barrier(0);
    }
    b += ST;
  }
  if (full > 0) {  // last full round: refill only what the remainder round will use
#pragma unroll
    for (int s = 0; s < ST; ++s) {
      mma_frags<MB>(f[s], acc);
      __builtin_amdgcn_sched_barrier(0);
      if (s < rem) load_frags<MB>(f[s], w0, w1, xb, kb0 + b + s + ST, lane);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int s = 0; s < ST; ++s)
    if (s < rem) mma_frags<MB>(f[s], acc);

  // ---- add the four waves' accumulators (fixed order) and write --------------------------------
  // Output block mb is finished by wave mb % 4, which takes both row blocks (needed by SwiGLU).
  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float sum[2][16];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      __syncthreads();
#pragma unroll
      for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[nb][mb][r];
      __syncthreads();
      if (wave == (mb & 3)) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          sum[nb][r] = (red[0][r][lane] + red[1][r][lane]) + (red[2][r][lane] + red[3][r][lane]);
      }
    }
    if (wave != (mb & 3)) continue;
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
    if (EPI == kEpiPartial) {
      float* o = (float*)out + ((size_t)blockIdx.y * M + m) * N;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = (nb ? rb1 : rb0) * 32 + 8 * q + 4 * hb;
          *(float4*)(o + n) = make_float4(sum[nb][4 * q], sum[nb][4 * q + 1], sum[nb][4 * q + 2], sum[nb][4 * q + 3]);
        }
    } else if (EPI == kEpiSwiGLU) {
      uint16_t* o = (uint16_t*)out;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float a[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float gte = sum[0][4 * q + e], up = sum[1][4 * q + e];
          a[e] = gte / (1.0f + __expf(-gte)) * up;
        }
        const int n = rb0 * 32 + 8 * q + 4 * hb;
        *(uint2*)(o + frag_offset(m, n, N >> 6)) = make_uint2(pack2bf(a[0], a[1]), pack2bf(a[2], a[3]));
      }
    } else {
      // lane (col, hb) holds 32 logits of row m: vocabulary ids (rb*32 + 8q + 4hb + e), in aligned groups of four,
      // i.e. one Philox block per group.
      const RowMeta rm = se.rows[m];
      const uint32_t pos = (uint32_t)(rm.pos + se.pos_offset), seq = (uint32_t)rm.seq;
      const int f = se.forced ? se.forced[m] : -1;
      Best best{-INFINITY, -1, 0.f};
      float lm = -INFINITY, ls = 0.f;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n0 = (nb ? rb1 : rb0) * 32 + 8 * q + 4 * hb;
          uint32_t rnd[4] = {0, 0, 0, 0};
          if (!se.greedy) philox4x32_10((uint32_t)n0 >> 2, pos, seq, 0u, se.seed_lo, se.seed_hi, rnd);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float zi = sum[nb][4 * q + e];
            const float y = se.greedy ? zi : __fmaf_rn(zi, se.inv_t, gumbel(rnd[e]));
            best = better(best, Best{y, n0 + e, zi});
            lse_merge(lm, ls, zi * se.inv_t, 1.0f);
            if (n0 + e == f) se.forced_z[m] = zi;
          }
          if (se.logits_out)
            *(float4*)(se.logits_out + (size_t)m * N + n0) =
                make_float4(sum[nb][4 * q], sum[nb][4 * q + 1], sum[nb][4 * q + 2], sum[nb][4 * q + 3]);
        }
      best = better(best, shfl_xor_best(best, 32));  // the other half of this row's 64 entries
      lse_merge(lm, ls, __shfl_xor(lm, 32, kWave), __shfl_xor(ls, 32, kWave));
      if (hb == 0) {
        float* p = se.part + ((size_t)m * (N >> 6) + blockIdx.x) * kSamplePartFloats;
        *(float4*)p = make_float4(best.y, __int_as_float(best.idx), best.z, 0.f);
        *(float4*)(p + 4) = make_float4(lm, ls, 0.f, 0.f);
      }
    }
  }
}

struct Plan {
  int splits;       // K splits across blocks
  int kb_per_wave;  // 64-wide k blocks per wave
};

Plan make_plan(int N, int K, int epi, bool allow_split) {
  const int KB = K >> 6;
  const int tiles = epi == kEpiSwiGLU ? (N >> 5) : (N >> 6);
  int S = 1;
  // Split K across blocks until about one block per CU exists; each wave keeps >= 2 k blocks.
  while (tiles * S < 256 && (KB % (S * 2 * 4) == 0) && KB / (S * 2 * 4) >= 2 && epi == kEpiPartial && allow_split) S *= 2;
  return Plan{S, KB / (S * 4)};
}

template <int MB, int ST>
void launch_mb(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
               const SampleEpilogue& se) {
  Plan p = make_plan(N, K, epi, allow_split);
  const int m_tiles = (M + 32 * MB - 1) / (32 * MB);
  if (epi == kEpiSwiGLU) {
    dim3 grid(N >> 5, 1, m_tiles);
    gemm_bf16_kernel<MB, kEpiSwiGLU, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else if (epi == kEpiSample) {
    dim3 grid(N >> 6, 1, m_tiles);
    gemm_bf16_kernel<MB, kEpiSample, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else {
    dim3 grid(N >> 6, p.splits, m_tiles);
    gemm_bf16_kernel<MB, kEpiPartial, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  }
}

}  // namespace

int gemm_bf16_splits(int N, int K, int epi) { return make_plan(N, K, epi, true).splits; }

template <int MB>
void launch_st(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
               int stages, const SampleEpilogue& se) {
  const int n = make_plan(N, K, epi, allow_split).kb_per_wave;
  if (stages > n) stages = n;  // the kernel's prologue fills all of its buffers unconditionally
  switch (stages) {
    case 1: launch_mb<MB, 1>(s, X, W, out, M, N, K, epi, allow_split, se); break;
    case 2: launch_mb<MB, 2>(s, X, W, out, M, N, K, epi, allow_split, se); break;
    case 3: launch_mb<MB, 3>(s, X, W, out, M, N, K, epi, allow_split, se); break;
    default: launch_mb<MB, 4>(s, X, W, out, M, N, K, epi, allow_split, se); break;
  }
}

// Requirements (checked at model init): K % 256 == 0, N % 64 == 0 (N % 32 for SwiGLU).
void launch_gemm_bf16(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi,
                      bool allow_split, const SampleEpilogue* se) {
  static const SampleEpilogue none{};
  const SampleEpilogue& e = se ? *se : none;
  if (epi == kEpiSample) allow_split = false;
  if (M <= 32) launch_st<1>(s, X, W, out, M, N, K, epi, allow_split, 4, e);
  else if (M <= 64) launch_st<2>(s, X, W, out, M, N, K, epi, allow_split, 2, e);
  else launch_st<4>(s, X, W, out, M, N, K, epi, allow_split, 2, e);
}

}  // namespace rl
