// fp32 kernels for models stored in fp32 (any dimensions that are multiples of 8): projections on the vector
// ALUs and single-pass paged attention.  These serve the small full-precision configuration, where every
// tensor fits in cache and launches dominate; they are written for exactness and generality, not bandwidth.
#include "device_utils.h"
#include "kernels.h"

namespace rl {

namespace {

constexpr int kRowsPerPass = 8;

// One wave per output column n (4 waves per block), all M rows in passes of 8.
// kEpiSwiGLU: W has 2N rows (gate then up); out[m][n] = silu(gate)*up.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                       float* __restrict__ out, int M, int N, int K) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + wave;
  if (n >= N) return;
  const float* w0 = W + (size_t)n * K;
  const float* w1 = W + (size_t)(n + N) * K;  // only read for SwiGLU
  for (int m0 = 0; m0 < M; m0 += kRowsPerPass) {
    float a0[kRowsPerPass], a1[kRowsPerPass];
#pragma unroll
    for (int i = 0; i < kRowsPerPass; ++i) a0[i] = a1[i] = 0.f;
    for (int k = lane; k < K; k += 64) {
      const float wv0 = w0[k];
      const float wv1 = (EPI == kEpiSwiGLU) ? w1[k] : 0.f;
#pragma unroll
      for (int i = 0; i < kRowsPerPass; ++i) {
        const int m = min(m0 + i, M - 1);
        const float xv = X[(size_t)m * K + k];
        a0[i] = fmaf(wv0, xv, a0[i]);
        if (EPI == kEpiSwiGLU) a1[i] = fmaf(wv1, xv, a1[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < kRowsPerPass; ++i) {
      const float s0 = wave_sum(a0[i]);
      const float s1 = (EPI == kEpiSwiGLU) ? wave_sum(a1[i]) : 0.f;
      if (lane == 0 && m0 + i < M) {
        if (EPI == kEpiSwiGLU)
          out[(size_t)(m0 + i) * N + n] = s0 / (1.0f + expf(-s0)) * s1;
        else
          out[(size_t)(m0 + i) * N + n] = s0;
      }
    }
  }
}

// One wave per (row, q head); keys in blocks of 64 (one key per lane for the scores, one dim per lane for
// the weighted sum), online softmax across blocks.  head_dim <= 256.
__global__ __launch_bounds__(64) void attn_f32_kernel(const float* __restrict__ q, const RowMeta* __restrict__ rows,
                                                      const int32_t* __restrict__ block_table, int max_blocks,
                                                      const float* __restrict__ k_pool, const float* __restrict__ v_pool,
                                                      float* __restrict__ o_out, int n_q, int n_kv, int d, float scale) {
  __shared__ float qs[256];
  __shared__ float ps[64];
  __shared__ int32_t pg[4];
  const int h = blockIdx.x, r = blockIdx.y, lane = threadIdx.x;
  const RowMeta rm = rows[r];
  const int ctx = rm.pos + 1;
  const int hk = h / (n_q / n_kv);
  for (int i = lane; i < d; i += 64) qs[i] = q[((size_t)r * n_q + h) * d + i];
  __syncthreads();
  const size_t page_elems = (size_t)kPageTokens * d;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};  // dims lane, lane+64, lane+128, lane+192
  float m_run = -INFINITY, l_run = 0.f;
  for (int kb = 0; kb < ctx; kb += 64) {
    if (lane < 4) {
      int blk = (kb >> 4) + lane;
      const int last = (ctx - 1) >> 4;
      pg[lane] = block_table[(size_t)rm.seq * max_blocks + (blk > last ? last : blk)];
    }
    __syncthreads();
    const int key = kb + lane;
    float sc = -INFINITY;
    if (key < ctx) {
      const float* kp = k_pool + ((size_t)pg[lane >> 4] * n_kv + hk) * 2 * page_elems + (size_t)(key & 15) * d;
      float dot = 0.f;
      for (int i = 0; i < d; ++i) dot = fmaf(qs[i], kp[i], dot);
      sc = dot * scale;
    }
    const float m_new = fmaxf(m_run, wave_max(sc));
    const float alpha = expf(m_run - m_new);
    const float p = expf(sc - m_new);
    l_run = l_run * alpha + wave_sum(p);
    m_run = m_new;
    ps[lane] = p;
    __syncthreads();
    const int nk = min(64, ctx - kb);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int i = lane + 64 * c;
      if (i < d) {
        float a = acc[c] * alpha;
        for (int t = 0; t < nk; ++t) {
          const float* vp = v_pool + ((size_t)pg[t >> 4] * n_kv + hk) * 2 * page_elems + (size_t)(t & 15) * d;
          a = fmaf(ps[t], vp[i], a);
        }
        acc[c] = a;
      }
    }
    __syncthreads();
  }
  const float inv = 1.0f / l_run;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int i = lane + 64 * c;
    if (i < d) o_out[((size_t)r * n_q + h) * d + i] = acc[c] * inv;
  }
}

}  // namespace

void launch_gemm_f32(hipStream_t s, const float* X, const float* W, float* out, int M, int N, int K, int epi) {
  dim3 grid((N + 3) / 4);
  if (epi == kEpiSwiGLU)
    gemm_f32_kernel<kEpiSwiGLU><<<grid, 256, 0, s>>>(X, W, out, M, N, K);
  else
    gemm_f32_kernel<kEpiPartial><<<grid, 256, 0, s>>>(X, W, out, M, N, K);
}

void launch_attn_f32(hipStream_t s, const Geometry& g, const float* q, const RowMeta* rows, const int32_t* block_table,
                     const void* k_pool_layer, const void* v_pool_layer, float* o_out, int M) {
  dim3 grid(g.n_q, M);
  attn_f32_kernel<<<grid, 64, 0, s>>>(q, rows, block_table, g.max_blocks, (const float*)k_pool_layer,
                                      (const float*)v_pool_layer, o_out, g.n_q, g.n_kv, g.head_dim,
                                      1.0f / sqrtf((float)g.head_dim));
}

}  // namespace rl
