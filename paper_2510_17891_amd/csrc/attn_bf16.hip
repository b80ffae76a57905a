// GQA decode attention over a paged bf16 KV cache, head_dim 128, split over the context.
//
// The step reads ctx * n_kv * 2 * 256 bytes per row and does ~4 flop per byte: a pure HBM stream.  The kernel
// is therefore built so that every K/V byte is loaded exactly once, with fully coalesced 1 KiB wave loads, straight
// into the registers that feed the matrix cores (the page layouts are chosen for that; see small_kernels.hip):
//
//   scores  S[key][head]  = sum_d K[key][d] q[head][d]   MFMA 16x16x32, A = K page (16 keys), B = q (<= 8 heads
//                                                        of the group, remaining columns zero); q is split into
//                                                        a bf16 high and low part so q keeps ~16 mantissa bits
//   O^T[d][head]          += V^T[d][key] P[key][head]    MFMA 16x16x32 over two pages (32 keys); the P operand is
//                                                        exactly the registers the score MFMA produced
//
// One wave handles one (row, kv head, 256-key chunk) and leaves (max, sum, unnormalised O) per head; a second
// small kernel merges the chunks of a row in index order, which makes the result independent of the batch.
#include "device_utils.h"
#include "kernels.h"

namespace rl {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kD = 128;
constexpr int kPageElems = kPageTokens * kD;  // 2048 bf16 = 4 KiB per (page, kv head), K or V
constexpr int kPartStride = kD + 2;           // floats per (row, head, chunk): O[128], max, sum

struct PagePair {
  u32x4_t k[2][4];  // [page a|b][mfma step s]: keys x dims 32s..32s+31
  u32x4_t v[2][4];  // [page a|b][jj]: dims 32jj..32jj+31 (two 16-dim blocks) x this lane's 4 keys
};

__device__ __forceinline__ void load_pair(PagePair& pp, const u32x4_t* __restrict__ kbase,
                                          const u32x4_t* __restrict__ vbase, int64_t page_a, int64_t page_b, int n_kv,
                                          int lane) {
  const size_t oa = (size_t)page_a * n_kv * (kPageElems / 8) + lane;
  const size_t ob = (size_t)page_b * n_kv * (kPageElems / 8) + lane;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    pp.k[0][s] = __builtin_nontemporal_load(kbase + oa + s * 64);
    pp.k[1][s] = __builtin_nontemporal_load(kbase + ob + s * 64);
  }
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    pp.v[0][s] = __builtin_nontemporal_load(vbase + oa + s * 64);
    pp.v[1][s] = __builtin_nontemporal_load(vbase + ob + s * 64);
  }
}

// grid: x = chunk, y = kv head, z = row.  block = one wave.
__global__ __launch_bounds__(64) void attn_decode_bf16_kernel(const float* __restrict__ q, const RowMeta* __restrict__ rows,
                                                              const int32_t* __restrict__ block_table, int max_blocks,
                                                              const u32x4_t* __restrict__ k_pool,
                                                              const u32x4_t* __restrict__ v_pool, float* __restrict__ part,
                                                              int max_chunks, int n_q, int n_kv, float scale) {
  const int chunk = blockIdx.x, hk = blockIdx.y, r = blockIdx.z, lane = threadIdx.x;
  const RowMeta rm = rows[r];
  const int ctx = rm.pos + 1;  // keys 0..pos (the row's own key was appended before this kernel)
  const int key0 = chunk * kAttnChunk;
  if (key0 >= ctx) return;
  const int group = n_q / n_kv;  // <= 8
  const int j = lane & 15, g = lane >> 4;

  // ---- q operand: column j < group holds head hk*group + j; hi/lo bf16 split ---------------------
  u32x4_t q_hi[4], q_lo[4];
  {
    const float* qh = q + ((size_t)r * n_q + (size_t)hk * group + (j < group ? j : 0)) * kD;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        float x0 = 0.f, x1 = 0.f;
        if (j < group) { x0 = qh[32 * s + 8 * g + e]; x1 = qh[32 * s + 8 * g + e + 1]; }
        const uint32_t h0 = f2bf(x0), h1 = f2bf(x1);
        hi[e >> 1] = h0 | (h1 << 16);
        lo[e >> 1] = pack2bf(x0 - bf2f(h0), x1 - bf2f(h1));
      }
      q_hi[s] = (u32x4_t){hi[0], hi[1], hi[2], hi[3]};
      q_lo[s] = (u32x4_t){lo[0], lo[1], lo[2], lo[3]};
    }
  }

  // ---- page ids of this chunk (16 pages), lane i < 16 holds page i -------------------------------
  const int last_blk = (ctx - 1) >> 4;
  int my_blk = (key0 >> 4) + (lane & 15);
  if (my_blk > last_blk) my_blk = last_blk;  // never dereference unallocated entries
  const int32_t my_page = block_table[(size_t)rm.seq * max_blocks + my_blk];

  const u32x4_t* kb = k_pool + (size_t)hk * (kPageElems / 8);
  const u32x4_t* vb = v_pool + (size_t)hk * (kPageElems / 8);

  f32x4_t o_acc[8];
#pragma unroll
  for (int b = 0; b < 8; ++b) o_acc[b] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  const int keys_here = min(kAttnChunk, ctx - key0);
  const int n_iter = (keys_here + 31) >> 5;

  PagePair cur, nxt;
  load_pair(cur, kb, vb, __shfl(my_page, 0, kWave), __shfl(my_page, 1, kWave), n_kv, lane);
  for (int it = 0; it < n_iter; ++it) {
    if (it + 1 < n_iter)
      load_pair(nxt, kb, vb, __shfl(my_page, 2 * it + 2, kWave), __shfl(my_page, 2 * it + 3, kWave), n_kv, lane);

    // scores for 32 keys: lane (g, j) gets keys 4g..4g+3 of page a (sa) and of page b (sb) for column j
    f32x4_t sa = (f32x4_t){0.f, 0.f, 0.f, 0.f}, sb = sa;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const bf16x8_t qa = __builtin_bit_cast(bf16x8_t, q_hi[s]), ql = __builtin_bit_cast(bf16x8_t, q_lo[s]);
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur.k[0][s]), qa, sa, 0, 0, 0);
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur.k[0][s]), ql, sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur.k[1][s]), qa, sb, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur.k[1][s]), ql, sb, 0, 0, 0);
    }
    const int kbase = key0 + it * 32 + 4 * g;
    float sc[8];
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sc[e] = (kbase + e < ctx) ? sa[e] * scale : -INFINITY;
      sc[4 + e] = (kbase + 16 + e < ctx) ? sb[e] * scale : -INFINITY;
      mx = fmaxf(mx, fmaxf(sc[e], sc[4 + e]));
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float m_new = fmaxf(m_run, mx);  // finite: key0 + it*32 < ctx always holds for lane group 0
    const float alpha = __expf(m_run - m_new);
    m_run = m_new;
    uint32_t pw[4];
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const uint32_t b0 = f2bf(__expf(sc[e] - m_new)), b1 = f2bf(__expf(sc[e + 1] - m_new));
      psum += bf2f(b0) + bf2f(b1);  // the sum uses the rounded weights the product uses
      pw[e >> 1] = b0 | (b1 << 16);
    }
    l_run = l_run * alpha + psum;
    const bf16x8_t p_op = __builtin_bit_cast(bf16x8_t, (u32x4_t){pw[0], pw[1], pw[2], pw[3]});
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const int jj = b >> 1, par = b & 1;
      u32x4_t vop;
      vop[0] = cur.v[0][jj][2 * par];
      vop[1] = cur.v[0][jj][2 * par + 1];
      vop[2] = cur.v[1][jj][2 * par];
      vop[3] = cur.v[1][jj][2 * par + 1];
      o_acc[b] *= alpha;
      o_acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vop), p_op, o_acc[b], 0, 0, 0);
    }
    cur = nxt;
  }

  // ---- write the chunk's partial: lanes with j < group hold head hk*group + j --------------------
  l_run += __shfl_xor(l_run, 16, kWave);
  l_run += __shfl_xor(l_run, 32, kWave);
  if (j < group) {
    float* p = part + (((size_t)r * n_q + (size_t)hk * group + j) * max_chunks + chunk) * kPartStride;
#pragma unroll
    for (int b = 0; b < 8; ++b)
      *(float4*)(p + 16 * b + 4 * g) = make_float4(o_acc[b][0], o_acc[b][1], o_acc[b][2], o_acc[b][3]);
    if (g == 0) { p[kD] = m_run; p[kD + 1] = l_run; }
  }
}

// One wave per (row, head): combine chunks in index order; lane owns dims 2*lane, 2*lane+1.
__global__ __launch_bounds__(64) void attn_merge_bf16_kernel(const float* __restrict__ part, const RowMeta* __restrict__ rows,
                                                             int max_chunks, uint16_t* __restrict__ o_out, int n_q) {
  const int h = blockIdx.x, r = blockIdx.y, lane = threadIdx.x;
  const int ctx = rows[r].pos + 1;
  const int n_chunks = (ctx + kAttnChunk - 1) / kAttnChunk;
  const float* p = part + ((size_t)r * n_q + h) * max_chunks * kPartStride;
  float M = -INFINITY;
  for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, p[(size_t)c * kPartStride + kD]);
  float o0 = 0.f, o1 = 0.f, den = 0.f;
  for (int c = 0; c < n_chunks; ++c) {
    const float* pc = p + (size_t)c * kPartStride;
    const float w = __expf(pc[kD] - M);
    den += w * pc[kD + 1];
    const float2 v = *(const float2*)(pc + 2 * lane);
    o0 += w * v.x;
    o1 += w * v.y;
  }
  const float inv = 1.0f / den;
  const int k = h * kD + 2 * lane;
  *(uint32_t*)(o_out + frag_offset(r, k, (n_q * kD) >> 6)) = pack2bf(o0 * inv, o1 * inv);
}

}  // namespace

void launch_attn_decode_bf16(hipStream_t s, const Geometry& g, const float* q, const RowMeta* rows,
                             const int32_t* block_table, const void* k_pool_layer, const void* v_pool_layer,
                             float* part, int max_chunks_alloc, int grid_chunks, int M) {
  dim3 grid(grid_chunks, g.n_kv, M);
  attn_decode_bf16_kernel<<<grid, 64, 0, s>>>(q, rows, block_table, g.max_blocks, (const u32x4_t*)k_pool_layer,
                                              (const u32x4_t*)v_pool_layer, part, max_chunks_alloc, g.n_q, g.n_kv,
                                              1.0f / sqrtf((float)g.head_dim));
}

void launch_attn_merge_bf16(hipStream_t s, const Geometry& g, const float* part, const RowMeta* rows,
                            int max_chunks_alloc, void* o_out, int M) {
  dim3 grid(g.n_q, M);
  attn_merge_bf16_kernel<<<grid, 64, 0, s>>>(part, rows, max_chunks_alloc, (uint16_t*)o_out, g.n_q);
}

}  // namespace rl
