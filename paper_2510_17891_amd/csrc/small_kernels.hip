// Embedding gather, residual + RMSNorm, per-head norm + rotary + KV append, KV import, weight packing.
// These move little data per step; they are written for few launches and simple indexing.
#include "device_utils.h"
#include "kernels.h"
#include "rope_device.h"

namespace rl {

// ------------------------------------------------------------------------------------------------
// Embedding gather (rollout step "x = E[token]").
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tok,
                                                    float* __restrict__ x, int H, int V, const RowMeta* __restrict__ rows,
                                                    const int32_t* __restrict__ last_tok) {
  const int r = blockIdx.x;
  const int fed = tok != nullptr ? tok[r] : last_tok[rows[r].seq];
  const int t = min(max(fed, 0), V - 1);  // ids come from device memory the host cannot inspect
  const size_t base = (size_t)t * H;
  for (int i = threadIdx.x; i < H; i += 256) x[(size_t)r * H + i] = load_as_float(E, base + i);
}

void launch_embed(hipStream_t s, int dtype, const void* embed, const int32_t* tokens, float* x, int M, int H, int V,
                  const RowMeta* rows, const int32_t* last_tok) {
  if (dtype == kBF16)
    embed_kernel<uint16_t><<<M, 256, 0, s>>>((const uint16_t*)embed, tokens, x, H, V, rows, last_tok);
  else
    embed_kernel<float><<<M, 256, 0, s>>>((const float*)embed, tokens, x, H, V, rows, last_tok);
}

// ------------------------------------------------------------------------------------------------
// Residual update + RMSNorm.  One block per row, one float4 per thread and pass (H/4 threads, at most 1024), so
// that the few dependent memory round trips of this latency-bound step are as short as possible.  The split
// partials of the preceding projection are summed in a fixed order, so results do not depend on the batch.
// ------------------------------------------------------------------------------------------------
// gain: H gains; without a norm (has_gain = 0) any readable H-element array of the model's dtype.
template <bool BF16>
__global__ __launch_bounds__(1024) void residual_norm_kernel(float* __restrict__ x, const float* __restrict__ part,
                                                             int S, size_t split_stride, const void* __restrict__ gain,
                                                             int has_gain, void* __restrict__ h_out,
                                                             float* __restrict__ capture, int H, float eps) {
  __shared__ float red[16];
  const int r = blockIdx.x, nthr = blockDim.x;
  float* xr = x + (size_t)r * H;
  float ss = 0.f;
  constexpr int kMaxPass = 2;  // H <= 1024 threads * 4 * kMaxPass, checked by the host
  float4 keep[kMaxPass];
  // Gains are requested together with the data, as stored (bf16: two words per thread), and first touched after the
  // sums: converting them here would make the compiler wait for them before it even asks for the data.
  uint4 graw[kMaxPass];
#pragma unroll
  for (int pass = 0; pass < kMaxPass; ++pass) {
    const int i0 = (pass * nthr + threadIdx.x) * 4;
    const int ig = i0 < H ? i0 : 0;  // unconditional loads (a branch here costs a wait); `gain` is always readable
    if (BF16) {
      const uint2 gb = *(const uint2*)((const uint16_t*)gain + ig);
      graw[pass] = make_uint4(gb.x, gb.y, 0u, 0u);
    } else {
      graw[pass] = *(const uint4*)((const float*)gain + ig);
    }
  }
#pragma unroll
  for (int pass = 0; pass < kMaxPass; ++pass) {
    const int i0 = (pass * nthr + threadIdx.x) * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i0 < H) {
      v = *(const float4*)(xr + i0);
#pragma unroll 4
      for (int sp = 0; sp < S; ++sp) {
        const float4 p = *(const float4*)(part + sp * split_stride + (size_t)r * H + i0);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
      }
      if (S > 0) *(float4*)(xr + i0) = v;
      if (capture) *(float4*)(capture + (size_t)r * H + i0) = v;
    }
    keep[pass] = v;
    ss += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
  }
  if (!has_gain) return;
#pragma unroll
  for (int pass = 0; pass < kMaxPass; ++pass)
    asm volatile("" : "+v"(graw[pass].x), "+v"(graw[pass].y), "+v"(graw[pass].z), "+v"(graw[pass].w));
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = 0.f;
  for (int w = 0; w < (nthr >> 6); ++w) ss += red[w];
  const float inv = 1.0f / sqrtf(ss / (float)H + eps);
#pragma unroll
  for (int pass = 0; pass < kMaxPass; ++pass) {
    const int i0 = (pass * nthr + threadIdx.x) * 4;
    if (i0 >= H) continue;
    const float4 v = keep[pass];
    float4 g;
    if (BF16) {
      g = make_float4(bf2f(graw[pass].x & 0xffffu), bf2f(graw[pass].x >> 16), bf2f(graw[pass].y & 0xffffu), bf2f(graw[pass].y >> 16));
    } else {
      g = make_float4(__uint_as_float(graw[pass].x), __uint_as_float(graw[pass].y), __uint_as_float(graw[pass].z),
                      __uint_as_float(graw[pass].w));
    }
    if (BF16) {
      *(uint2*)((uint16_t*)h_out + frag_offset(r, i0, H >> 6)) =
          make_uint2(pack2h(v.x * inv * g.x, v.y * inv * g.y), pack2h(v.z * inv * g.z, v.w * inv * g.w));
    } else {
      *(float4*)((float*)h_out + (size_t)r * H + i0) = make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w);
    }
  }
}

void launch_residual_norm(hipStream_t s, int dtype, float* x, const float* part, int S, const void* gain,
                          void* h_out, float* capture, int M, int H, float eps) {
  size_t stride = (size_t)M * H;
  int threads = ((H / 4 + 63) / 64) * 64;
  if (threads > 1024) threads = 1024;
  const int has_gain = gain != nullptr;
  const void* g = has_gain ? gain : x;  // read and ignored without a norm
  if (dtype == kBF16)
    residual_norm_kernel<true><<<M, threads, 0, s>>>(x, part, S, stride, g, has_gain, h_out, capture, H, eps);
  else
    residual_norm_kernel<false><<<M, threads, 0, s>>>(x, part, S, stride, g, has_gain, h_out, capture, H, eps);
}

// One wave per (row, head), four heads per block.  Lane i < d/2 owns the rotary pair (i, i + d/2).
template <bool BF16, int KVT>
__global__ __launch_bounds__(256) void qk_rope_append_kernel(const float* __restrict__ part, int S, size_t split_stride,
                                                            const void* __restrict__ q_gain,
                                                            const void* __restrict__ k_gain,
                                                            const float2* __restrict__ rope, const RowMeta* __restrict__ rows,
                                                            void* __restrict__ k_pool, void* __restrict__ v_pool,
                                                            float* __restrict__ q_out, int n_q, int n_kv, int d,
                                                            int qk_norm, float eps) {
  const int hh = blockIdx.x * 4 + (threadIdx.x >> 6), r = blockIdx.y, lane = threadIdx.x & 63;
  if (hh >= n_q + 2 * n_kv) return;  // wave-uniform; no barriers in this kernel
  const int half = d >> 1;
  const int n_tot = (n_q + 2 * n_kv) * d;
  const RowMeta rm = rows[r];
  const bool is_q = hh < n_q, is_k = !is_q && hh < n_q + n_kv;
  // Everything that depends only on the row's (seq, pos) is requested first, so that it travels together with the
  // partial sums instead of after them.
  const int64_t page = rm.page;
  const bool rotate = is_q || is_k;
  const float* head_part = part + (size_t)r * n_tot + (size_t)hh * d;
  const void* gain = qk_norm ? (is_q ? q_gain : k_gain) : nullptr;
  // lanes may own more than one pair when d/2 > 64 (without per-head normalisation only: the host rejects wider
  // normalised heads for this kernel)
  for (int i = lane; i < ((half + 63) & ~63); i += 64) {
    HeadPair hp = head_pair_load<BF16>(head_part, S, split_stride, d, i, rotate, rope + (size_t)rm.pos * half, gain);
    head_pair_finish(hp, d, rotate, qk_norm != 0, eps);
    if (i >= half) continue;
    if (is_q) {
      float* q = q_out + ((size_t)r * n_q + hh) * d;
      q[i] = hp.v0;
      q[i + half] = hp.v1;
    } else {
      const int hk = is_k ? hh - n_q : hh - n_q - n_kv;
      const int t = rm.pos & 15;
      kv_store<KVT>(is_k ? k_pool : v_pool, page, hk, n_kv, d, t, i, hp.v0, !is_k);
      kv_store<KVT>(is_k ? k_pool : v_pool, page, hk, n_kv, d, t, i + half, hp.v1, !is_k);
    }
  }
}

void launch_qk_rope_append(hipStream_t s, const Geometry& g, const float* qkv_part, int S, const void* q_gain,
                           const void* k_gain, const float2* rope_table, const RowMeta* rows, void* k_pool_layer,
                           void* v_pool_layer, float* q_out, int M) {
  dim3 grid((g.n_q + 2 * g.n_kv + 3) / 4, M);
  size_t stride = (size_t)M * (g.n_q + 2 * g.n_kv) * g.head_dim;
  if (g.dtype == kBF16 && g.kv_fp8)
    qk_rope_append_kernel<true, 2><<<grid, 256, 0, s>>>(qkv_part, S, stride, q_gain, k_gain, rope_table, rows,
                                                       k_pool_layer, v_pool_layer, q_out, g.n_q, g.n_kv,
                                                       g.head_dim, g.qk_norm, g.rms_eps);
  else if (g.dtype == kBF16)
    qk_rope_append_kernel<true, 1><<<grid, 256, 0, s>>>(qkv_part, S, stride, q_gain, k_gain, rope_table, rows,
                                                       k_pool_layer, v_pool_layer, q_out, g.n_q, g.n_kv,
                                                       g.head_dim, g.qk_norm, g.rms_eps);
  else
    qk_rope_append_kernel<false, 0><<<grid, 256, 0, s>>>(qkv_part, S, stride, q_gain, k_gain, rope_table, rows,
                                                        k_pool_layer, v_pool_layer, q_out, g.n_q, g.n_kv,
                                                        g.head_dim, g.qk_norm, g.rms_eps);
}

// ------------------------------------------------------------------------------------------------
// KV import: contiguous [n_tokens][n_kv][d] -> positions first_pos .. first_pos + n_tokens - 1 of one sequence.
// ------------------------------------------------------------------------------------------------
template <typename T, int KVT>
__global__ __launch_bounds__(256) void kv_import_kernel(const T* __restrict__ k_src, const T* __restrict__ v_src,
                                                        int first_pos, const int32_t* __restrict__ bt_row,
                                                        void* __restrict__ k_pool, void* __restrict__ v_pool, int n_kv,
                                                        int d) {
  const int tok = first_pos + blockIdx.x;  // position in the sequence; source token blockIdx.x
  const int64_t page = bt_row[tok >> 4];
  const int t = tok & 15;
  for (int i = threadIdx.x; i < n_kv * d; i += 256) {
    int hk = i / d, dd = i - hk * d;
    size_t src = (size_t)blockIdx.x * n_kv * d + i;
    kv_store<KVT>(k_pool, page, hk, n_kv, d, t, dd, load_as_float(k_src, src), false);
    kv_store<KVT>(v_pool, page, hk, n_kv, d, t, dd, load_as_float(v_src, src), true);
  }
}

void launch_kv_import(hipStream_t s, const Geometry& g, const void* k_src, const void* v_src, int first_pos, int n_tokens,
                      const int32_t* block_table_row, void* k_pool_layer, void* v_pool_layer) {
  if (n_tokens <= 0) return;
  if (g.dtype == kBF16 && g.kv_fp8)
    kv_import_kernel<uint16_t, 2><<<n_tokens, 256, 0, s>>>((const uint16_t*)k_src, (const uint16_t*)v_src, first_pos,
                                                           block_table_row, k_pool_layer, v_pool_layer, g.n_kv,
                                                           g.head_dim);
  else if (g.dtype == kBF16)
    kv_import_kernel<uint16_t, 1><<<n_tokens, 256, 0, s>>>((const uint16_t*)k_src, (const uint16_t*)v_src, first_pos,
                                                           block_table_row, k_pool_layer, v_pool_layer, g.n_kv,
                                                           g.head_dim);
  else
    kv_import_kernel<float, 0><<<n_tokens, 256, 0, s>>>((const float*)k_src, (const float*)v_src, first_pos,
                                                            block_table_row, k_pool_layer, v_pool_layer, g.n_kv,
                                                            g.head_dim);
}

// ------------------------------------------------------------------------------------------------
// Weight packing: row-major [N][K] bf16 -> fragment-major, each weight as its f16 image (the grid the matrix cores
// multiply on; see bf2_to_h2: exact from 2^-14 up, smaller magnitudes cut toward zero, same bytes per weight), so
// that no kernel spends an instruction on it.  One thread per 8 consecutive k.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_weight_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int N,
                                                          int K, int seg) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // over N * K/8
  const int kg = K >> 3;
  if (idx >= (size_t)N * kg) return;
  const int n = (int)(idx / kg), k = (int)(idx - (size_t)n * kg) * 8;
  const uint4 w = src[idx];
  dst[weight_offset(n, k, K >> 6, seg) >> 3] = make_uint4(bf2_to_h2(w.x), bf2_to_h2(w.y), bf2_to_h2(w.z), bf2_to_h2(w.w));
}

void launch_pack_weight_bf16(hipStream_t s, const void* src, void* dst, int N, int K, int seg) {
  size_t total = (size_t)N * (K >> 3);
  pack_weight_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint4*)src, (uint4*)dst, N, K, seg);
}

}  // namespace rl

namespace rl {

__global__ void table_update_kernel(int32_t* __restrict__ bt, int max_blocks, const int32_t* __restrict__ upd, int n) {
  const int i = blockIdx.x * 64 + threadIdx.x;
  if (i < n) bt[(size_t)upd[3 * i] * max_blocks + upd[3 * i + 1]] = upd[3 * i + 2];
}

void launch_table_update(hipStream_t s, int32_t* block_table, int max_blocks, const int32_t* upd, int n) {
  if (n <= 0) return;
  table_update_kernel<<<(n + 63) / 64, 64, 0, s>>>(block_table, max_blocks, upd, n);
}

// The same with the number of entries read on the device (rows[0].pad), for launches whose shape must not depend
// on it: a grid for n_max entries, of which the first rows[0].pad are applied.
__global__ void table_update_counted_kernel(int32_t* __restrict__ bt, int max_blocks, const int32_t* __restrict__ upd,
                                            const RowMeta* __restrict__ rows) {
  const int i = blockIdx.x * 64 + threadIdx.x;
  if (i < rows[0].pad) bt[(size_t)upd[3 * i] * max_blocks + upd[3 * i + 1]] = upd[3 * i + 2];
}

void launch_table_update_counted(hipStream_t s, int32_t* block_table, int max_blocks, const int32_t* upd,
                                 const RowMeta* rows, int n_max) {
  table_update_counted_kernel<<<(n_max + 63) / 64, 64, 0, s>>>(block_table, max_blocks, upd, rows);
}

}  // namespace rl

namespace rl {

// grid: x = layer, y = pair.  Copies one page (all kv heads, K and V: contiguous inside a layer) with 16-byte accesses.
__global__ __launch_bounds__(256) void page_copy_kernel(char* __restrict__ pool, size_t layer_bytes, size_t page_bytes,
                                                        const int32_t* __restrict__ pairs) {
  const int32_t src = pairs[2 * blockIdx.y], dst = pairs[2 * blockIdx.y + 1];
  char* base = pool + (size_t)blockIdx.x * layer_bytes;
  const uint4* s = (const uint4*)(base + (size_t)src * page_bytes);
  uint4* d = (uint4*)(base + (size_t)dst * page_bytes);
  for (size_t i = threadIdx.x; i < page_bytes / 16; i += 256) d[i] = s[i];
}

void launch_page_copy(hipStream_t s, void* kv_pool, size_t layer_bytes, size_t page_bytes, int n_layers,
                      const int32_t* pairs, int n_pairs) {
  if (n_pairs <= 0) return;
  dim3 grid(n_layers, n_pairs);
  page_copy_kernel<<<grid, 256, 0, s>>>((char*)kv_pool, layer_bytes, page_bytes, pairs);
}

}  // namespace rl

namespace rl {

__global__ void scatter_f32_kernel(const float* __restrict__ src, const int32_t* __restrict__ idx, float* __restrict__ out, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n && idx[i] >= 0) out[idx[i]] = src[i];
}

void launch_scatter_f32(hipStream_t s, const float* src, const int32_t* idx, float* out, int n) {
  if (n <= 0) return;
  scatter_f32_kernel<<<(n + 255) / 256, 256, 0, s>>>(src, idx, out, n);
}

}  // namespace rl
