// Launchers of the gfx950 kernels.  Host orchestration (model.hip) calls these; each enqueues on the
// given stream and returns.  Shapes are validated by the caller against what each kernel assumes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_plan.h"
#include "weight_order.h"

namespace rl {

// Records the message that rl_last_error() returns on this thread and hands back `status` (an rl_status value), so
// that every entry point, whichever source file it lives in, reports failures the same way.
int set_error(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// One batch row = one (sequence, position) pair being pushed through the decoder.
struct RowMeta {
  int32_t seq;   // sequence id (row of the block table, RNG stream)
  int32_t pos;   // absolute position of the token fed in this row
  int32_t page;  // KV page that holds position pos (the host knows it; saves the append kernel a dependent load)
  int32_t pad;   // row 0 of a decode call: number of page grants uploaded with the rows; otherwise 0
};

enum Dtype : int { kF32 = 0, kBF16 = 1 };

// Geometry of the decoder, fixed at init and passed by value to launchers.
struct Geometry {
  int n_layers, hidden, n_q, n_kv, head_dim, ffn, vocab;
  int qk_norm;
  float rms_eps;
  int dtype;
  int max_blocks;   // block-table row length = max_ctx / 16
  int64_t n_pages;  // pages in the pool
  int kv_fp8;       // bf16 models: keys and values are cached as fp8 (e4m3), one byte per element
};

// "Fragment-major" order of a [rows x K] bf16 operand of the MFMA GEMM: 32-row blocks, 64-wide k
// blocks, inside a block [t(4)][hb(2)][row(32)][e(8)] with k = 64 kb + 32 hb + 8 t + e.  A wave reads
// block (rb, kb) as four fully coalesced 1 KiB loads, each already in MFMA 32x32x16 operand order.
__host__ __device__ inline size_t frag_offset(int r, int k, int k_blocks) {
  int rb = r >> 5, row = r & 31, kb = k >> 6, hb = (k >> 5) & 1, t = (k >> 3) & 3, e = k & 7;
  return ((((size_t)(rb * (size_t)k_blocks + kb) * 4 + t) * 2 + hb) * 32 + row) * 8 + e;
}

// Offset of weight element (r, k) in the packed matrix: frag_offset with the k block moved to its slot.
__host__ __device__ inline size_t weight_offset(int r, int k, int k_blocks, int seg) {
  const int kb = k >> 6;
  return frag_offset(r, (weight_kb_slot(kb, seg) << 6) | (k & 63), k_blocks);
}

// ---- elementwise / small kernels (both dtypes) -------------------------------------------------
// x[r][:] = E[tok[r]][:] widened to fp32 (ids clamped to [0, V)).
// tokens == null: row r is fed last_tok[rows[r].seq] (the token the sampler recorded for that sequence).
void launch_embed(hipStream_t s, int dtype, const void* embed, const int32_t* tokens, float* x, int M, int H, int V,
                  const RowMeta* rows = nullptr, const int32_t* last_tok = nullptr);

// x[r] += sum_{s<S} part[s][r][:] (part may be null);  capture (may be null) gets x;  if gain != null,
// h = x * rsqrt(mean(x^2)+eps) * gain written as fp32 row-major (kF32) or f16 fragment-major (kBF16 models).
void launch_residual_norm(hipStream_t s, int dtype, float* x, const float* part, int S, const void* gain,
                          void* h_out, float* capture, int M, int H, float eps);

// Sum the split partials of the QKV projection, apply per-head RMSNorm (q,k) and the rotation (q,k) at
// each row's position, write q as fp32 [M][n_q][d] and append k,v to the row's KV page (rows[r].page).
void launch_qk_rope_append(hipStream_t s, const Geometry& g, const float* qkv_part, int S, const void* q_gain,
                           const void* k_gain, const float2* rope_table, const RowMeta* rows, void* k_pool_layer,
                           void* v_pool_layer, float* q_out, int M);

// Scatter contiguous [n_tokens][n_kv][d] K and V (model dtype) into the pages of one sequence, as its positions
// first_pos .. first_pos + n_tokens - 1 (the block-table row must already name their pages).
void launch_kv_import(hipStream_t s, const Geometry& g, const void* k_src, const void* v_src, int first_pos, int n_tokens,
                      const int32_t* block_table_row, void* k_pool_layer, void* v_pool_layer);

// Copy whole KV pages (all layers): pool byte layout [layer][page][page_bytes]; pairs = n x (src page, dst page)
// in device memory.
void launch_page_copy(hipStream_t s, void* kv_pool, size_t layer_bytes, size_t page_bytes, int n_layers,
                      const int32_t* pairs, int n_pairs);

// ---- attention -----------------------------------------------------------------------------------
// bf16, head_dim 128: decode attention over paged KV (MFMA), one block per (row, kv head), context cut into
// segments that depend on the context length only and merged in index order; writes f16 fragment-major
// [M x n_q*d].  part: fp32, per (row, head) max_segs rows of d floats followed by max_segs (max, sum) pairs, with
// max_segs = attn_bf16_max_segments(max_ctx).
int attn_bf16_max_segments(int max_ctx);
// skip_segs (per row, may be null): leading segments of the row that a set in `shared` covers; every row with a
// non-zero entry must belong to exactly one set with that n_segs.  max_shared_segs = largest n_segs.
// append (may be null): the kernel forms the rows' queries, new keys and new values from the QKV projection's split
// sums itself and writes the keys and values into the pages (RowMeta::page); `q` is then unused and
// launch_qk_rope_append is not called.  Only for batches with one row per sequence: the block of a row is then the
// only one that needs the row's new key, and it takes it from registers, not from the page.  The arithmetic is the
// one of launch_qk_rope_append, bit for bit.
// segs_per_block (1..16): segments one block takes of a context of more than 16 segments (> 4096 keys); results do
// not depend on it.
constexpr int kAttnAppendMaxSplits = 4;
struct AttnAppend {
  const float* qkv_part;  // [S][M][(n_q + 2 n_kv) * d]
  int S;                  // <= kAttnAppendMaxSplits
  const void* q_gain;     // per-head RMSNorm gains: both set, or both null
  const void* k_gain;
  const float2* rope_table;
};
// Returns true when the partials of some rows were left in the workspace, i.e. launch_attn_merge_bf16 (same arguments)
// has to follow; the two launches are separate calls so that a caller can time them separately.
bool launch_attn_decode_bf16(hipStream_t s, const Geometry& g, const float* q, const RowMeta* rows,
                             const int32_t* block_table, void* k_pool_layer, void* v_pool_layer,
                             float* part, int max_segs_alloc, int max_ctx_in_batch, void* o_out, int M,
                             const int32_t* skip_segs = nullptr, const AttnShared* shared = nullptr, int n_shared = 0,
                             int max_shared_segs = 0, const AttnAppend* append = nullptr, int segs_per_block = 16);
void launch_attn_merge_bf16(hipStream_t s, const Geometry& g, const RowMeta* rows, float* part, int max_segs_alloc,
                            void* o_out, int M, const int32_t* skip_segs, int n_shared);
// fp32, any head_dim <= 256: one wave per (row, q head), whole context, output fp32 row-major [M][n_q*d].
void launch_attn_f32(hipStream_t s, const Geometry& g, const float* q, const RowMeta* rows,
                     const int32_t* block_table, const void* k_pool_layer, const void* v_pool_layer,
                     float* o_out, int M);

// ---- projections ---------------------------------------------------------------------------------
enum Epilogue : int { kEpiPartial = 0, kEpiSwiGLU = 1, kEpiSample = 2 };

// Arguments of the sampling epilogue of the output projection (ignored by the other epilogues).
struct SampleEpilogue {
  const RowMeta* rows = nullptr;  // RNG stream (seq) and position (pos + pos_offset) per row
  int pos_offset = 0;
  float inv_t = 1.f;
  int greedy = 1;
  uint32_t seed_lo = 0, seed_hi = 0;
  const int32_t* forced = nullptr;  // per row, or null
  float* forced_z = nullptr;        // [M] logit of the forced token
  float* part = nullptr;            // [M][N/64][8] per-tile partials for launch_sample_merge
  float* logits_out = nullptr;      // optional [M][N] copy of the logits
};

// Number of K splits the bf16 GEMM uses for (N, K); partial outputs are [S][M][N] fp32.
int gemm_bf16_splits(int N, int K, int epi);
// MFMA GEMM of the bf16 models: X f16 fragment-major [M x K], W bf16 fragment-major [N x K] (2N rows for SwiGLU: gate
// and up rows interleaved in groups of 16).
// kEpiPartial: out = fp32 [S][M][N];  kEpiSwiGLU: out = f16 fragment-major [M x N] = silu(gate)*up;
// kEpiSample: out unused, results go through *se.  allow_split = false forces S = 1 (finished [M][N] product).
void launch_gemm_bf16(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi,
                      bool allow_split = true, const SampleEpilogue* se = nullptr);
// fp32 GEMM on vector ALUs, row-major everything; kEpiPartial writes [M][N] (one split).
void launch_gemm_f32(hipStream_t s, const float* X, const float* W, float* out, int M, int N, int K, int epi);

// Row-major [N x K] bf16 -> fragment-major with the k blocks in weight_kb_slot order for segments of `seg` k blocks
// (N % 32 == 0, K % 64 == 0, (K / 64) % (4 seg) == 0).
void launch_pack_weight_bf16(hipStream_t s, const void* src, void* dst, int N, int K, int seg);
// Segment length (k blocks per wave) of the plan that launch_gemm_bf16 uses for an [N x K] weight matrix: split_k says
// whether the product may be split along K over several blocks (QKV, O, down) or never is (gate/up, output projection).
int gemm_bf16_weight_segment(int N, int K, bool split_k);

// ---- sampler ---------------------------------------------------------------------------------------
constexpr int kSampleTile = 2048;  // vocabulary entries per first-stage block of the stand-alone sampler
// Gumbel-max sampling with log-probabilities from fp32 logits [M][V] in memory (two stages).
// part: [M][ceil(V/2048)][8] floats; forced may be null; forced_z: [M] floats.
// The RNG position of row r is rows[r].pos + pos_offset.
// top_k / top_p cut the distribution first (0 / outside (0,1): no cut; ignored when greedy); cut_buf: scratch of
// M * sample_cut_bytes_per_row() bytes (256-byte aligned), needed when sample_is_truncated().  V % 4 == 0, V < 2^22.
size_t sample_cut_bytes_per_row();
inline bool sample_is_truncated(int V, int top_k, float top_p) {
  return (top_k > 0 && top_k < V) || (top_p > 0.0f && top_p < 1.0f);
}
void launch_sample(hipStream_t s, const float* logits, int M, int V, const RowMeta* rows, int pos_offset,
                   const int32_t* forced, float temperature, uint64_t seed, float* part, float* forced_z,
                   int32_t* out_tokens, float* out_logprobs, int top_k = 0, float top_p = 0.f, void* cut_buf = nullptr,
                   int32_t* last_tok = nullptr);
// Second stage alone, over the [M][n_tiles][8] partials the sampling epilogue of the bf16 projection left.
// last_tok (may be null): [max_seqs] table that also receives each row's token at index rows[r].seq (both samplers).
void launch_sample_merge(hipStream_t s, const float* part, int n_tiles, int M, int V, const int32_t* forced,
                         const float* forced_z, float temperature, int32_t* out_tokens, float* out_logprobs,
                         const RowMeta* rows = nullptr, int32_t* last_tok = nullptr);

// out[idx[i]] = src[i] for idx[i] >= 0.
void launch_scatter_f32(hipStream_t s, const float* src, const int32_t* idx, float* out, int n);

// block_table[upd[3i]][upd[3i+1]] = upd[3i+2] for i < n (device-side mirror update of newly granted pages).
void launch_table_update(hipStream_t s, int32_t* block_table, int max_blocks, const int32_t* upd, int n);
// The same for at most n_max entries, of which the first rows[0].pad (read on the device) are applied.
void launch_table_update_counted(hipStream_t s, int32_t* block_table, int max_blocks, const int32_t* upd,
                                 const RowMeta* rows, int n_max);

}  // namespace rl
