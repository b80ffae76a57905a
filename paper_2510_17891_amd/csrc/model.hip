// Host side of the rollout library: C boundary, sequence table, per-call metadata, kernel sequencing.
//
// A "row" is one (sequence, position) pair pushed through the decoder.  A decode step is one row per
// sequence; prefill pushes every prompt token as a row, in chunks of max_rows, so both share one code path
// (the KV append of a layer runs for all rows of a chunk before that layer's attention, and a row only
// attends to keys at or before its own position).
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <chrono>
#include <cmath>
#include <string>
#include <vector>

#include "../../include/rl.h"
#include "kernels.h"
#include "seq_table.h"

using namespace rl;

namespace rl {

thread_local std::string g_err = "";

int set_error(int st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return st;
}

}  // namespace rl

#define fail(st, ...) ((rl_status)rl::set_error((int)(st), __VA_ARGS__))

namespace {

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) return fail(RL_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr int kRing = 64;  // per-call metadata slots in the workspace
constexpr int kRingCalls = kRing - 2;  // slots that ordinary calls cycle through; the last two belong to a decode graph
constexpr int T_MAX_SCORE = 4096;  // sequences per scoring call

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Layout {
  size_t block_table, rope, ring, x, x_last, h, part, q, attn_part, o, a, logits, samp_part, forced_z, tmp_tok, tmp_lp, cuts, last_tok, total;
  size_t slot_bytes, slot_upd, slot_tok, slot_skip, slot_sets;
  int max_segs, n_tiles;
};

size_t elem_size(uint32_t dtype) { return dtype == RL_BF16 ? 2 : 4; }
size_t kv_elem_size(const rl_model_config& c) { return c.kv_dtype == RL_KV_FP8 ? 1 : elem_size(c.dtype); }

rl_status check_config(const rl_model_config* c) {
  if (!c) return fail(RL_ERR_INVALID_ARG, "config is NULL");
  if (c->struct_size != sizeof(rl_model_config)) return fail(RL_ERR_INVALID_ARG, "struct_size mismatch");
  if (c->dtype != RL_F32 && c->dtype != RL_BF16) return fail(RL_ERR_INVALID_ARG, "unknown dtype");
  if (c->kv_dtype != RL_KV_SAME && c->kv_dtype != RL_KV_FP8) return fail(RL_ERR_INVALID_ARG, "unknown kv_dtype");
  if (c->kv_dtype == RL_KV_FP8 && c->dtype != RL_BF16) return fail(RL_ERR_UNSUPPORTED, "fp8 keys and values need a bf16 model");
  if (c->reserved != 0) return fail(RL_ERR_INVALID_ARG, "reserved must be 0");
  if (c->kv_block != 16) return fail(RL_ERR_UNSUPPORTED, "kv_block must be 16");
  if (!c->n_layers || !c->hidden || !c->n_q_heads || !c->n_kv_heads || !c->head_dim || !c->ffn)
    return fail(RL_ERR_INVALID_ARG, "zero dimension");
  if (c->n_q_heads % c->n_kv_heads) return fail(RL_ERR_INVALID_ARG, "n_q_heads %% n_kv_heads != 0");
  if (c->max_seqs == 0 || c->max_rows == 0 || c->max_rows > 1024) return fail(RL_ERR_INVALID_ARG, "max_rows must be in [1,1024]");
  if (c->max_ctx == 0 || c->max_ctx % 16) return fail(RL_ERR_INVALID_ARG, "max_ctx must be a positive multiple of 16");
  if (c->hidden % 8 || c->hidden > 8192 || c->head_dim % 2 || c->head_dim > 128 || c->ffn % 8 || c->vocab % 4)
    return fail(RL_ERR_UNSUPPORTED, "need hidden %% 8 == 0, hidden <= 8192, even head_dim <= 128, ffn %% 8 == 0, vocab %% 4 == 0");
  if (c->vocab >= (1u << 22)) return fail(RL_ERR_UNSUPPORTED, "vocab must be below 2^22");
  if (c->dtype == RL_BF16) {
    const uint32_t qd = c->n_q_heads * c->head_dim, nqkv = (c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
    if (c->head_dim != 128 || c->n_q_heads / c->n_kv_heads > 8) return fail(RL_ERR_UNSUPPORTED, "bf16 needs head_dim 128 and group <= 8");
    if (c->hidden % 256 || qd % 256 || c->ffn % 256) return fail(RL_ERR_UNSUPPORTED, "bf16 needs hidden, n_q*head_dim, ffn multiples of 256");
    if (nqkv % 64 || c->hidden % 64 || c->ffn % 64 || c->vocab % 64) return fail(RL_ERR_UNSUPPORTED, "bf16 needs projection widths multiples of 64");
    if (c->max_ctx > 65536) return fail(RL_ERR_UNSUPPORTED, "bf16 attention merges at most 256 segments: max_ctx <= 65536");
  }
  return RL_OK;
}

void compute_layout(const rl_model_config& c, Layout* L) {
  const size_t R = c.max_rows, Rp = (R + 31) / 32 * 32, H = c.hidden, d = c.head_dim;
  const size_t nq = c.n_q_heads, nkv = c.n_kv_heads, F = c.ffn, V = c.vocab;
  const size_t act = elem_size(c.dtype);
  const size_t nqkv = (nq + 2 * nkv) * d;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L->max_segs = attn_bf16_max_segments((int)c.max_ctx);
  L->n_tiles = (int)((V + kSampleTile - 1) / kSampleTile);
  L->slot_upd = align_up(R * sizeof(RowMeta));
  L->slot_tok = L->slot_upd + align_up(R * 3 * sizeof(int32_t));
  L->slot_skip = L->slot_tok + align_up(R * sizeof(int32_t));
  L->slot_sets = L->slot_skip + align_up(R * sizeof(int32_t));
  L->slot_bytes = L->slot_sets + align_up(R / 2 * sizeof(AttnShared) + sizeof(AttnShared));
  L->block_table = take((size_t)c.max_seqs * (c.max_ctx / 16) * 4);
  L->rope = take((size_t)c.max_ctx * (d / 2) * sizeof(float2));
  L->ring = take(kRing * L->slot_bytes);
  L->x = take(R * H * 4);
  L->x_last = take(R * H * 4);
  L->h = take(Rp * H * act);
  size_t part_elems;
  if (c.dtype == RL_BF16) {
    size_t a1 = (size_t)gemm_bf16_splits((int)nqkv, (int)H, kEpiPartial) * R * nqkv;
    size_t a2 = (size_t)gemm_bf16_splits((int)H, (int)(nq * d), kEpiPartial) * R * H;
    size_t a3 = (size_t)gemm_bf16_splits((int)H, (int)F, kEpiPartial) * R * H;
    part_elems = a1 > a2 ? a1 : a2;
    if (a3 > part_elems) part_elems = a3;
  } else {
    part_elems = R * (nqkv > H ? nqkv : H);
  }
  L->part = take(part_elems * 4);
  L->q = take(R * nq * d * 4);
  L->attn_part = take(c.dtype == RL_BF16 ? R * nq * (size_t)L->max_segs * (d + 2) * 4 : 256);
  L->o = take(Rp * nq * d * act);
  L->a = take(Rp * F * act);
  // bf16: logits never reach memory (sampling happens in the projection's epilogue, 64 entries per partial) unless
  // the distribution is truncated (top-k / top-p need the whole row before any token can be drawn);
  // fp32: logits are written and scanned by the stand-alone sampler (2048 entries per partial).  rl_sample_logits
  // uses the stand-alone sampler in both cases.
  L->logits = take(V ? R * V * 4 : 256);
  const size_t tiles_fused = V / 64 + 1;
  L->samp_part = take(V ? R * (tiles_fused > (size_t)L->n_tiles ? tiles_fused : (size_t)L->n_tiles) * 32 : 256);
  L->forced_z = take(R * 4);
  L->tmp_tok = take(R * 4);
  L->tmp_lp = take(R * 4);
  L->cuts = take(V ? R * sample_cut_bytes_per_row() : 256);
  L->last_tok = take((size_t)c.max_seqs * 4);  // per sequence id: the token its last prefill / decode call returned
  L->total = off;
}

enum Kind { K_META, K_EMBED, K_NORM, K_QKV, K_ROPE_APPEND, K_ATTN, K_ATTN_MERGE, K_OPROJ, K_GATEUP, K_DOWN, K_LMHEAD, K_SAMPLE, K_COUNT };
const char* const kKindNames[K_COUNT] = {"meta", "embed", "residual_norm", "gemm_qkv", "qk_rope_append", "attn_decode", "attn_merge",
                                        "gemm_o", "gemm_gate_up_swiglu", "gemm_down", "gemm_lm_head", "sample"};

}  // namespace

struct rl_model {
  rl_model_config cfg;
  Geometry geo;
  Layout lay;
  SeqTable* table = nullptr;
  // weights (device pointers)
  const void *embed, *lm_head, *final_norm;
  std::vector<const void*> attn_norm, wqkv, q_norm, k_norm, wo, mlp_norm, w_gate_up, w_down;
  char* kv_pool;
  char* ws;
  size_t layer_kv_bytes, kv_block_bytes;  // one layer of the pool; one K (or V) block of a (page, kv head)
  // pinned host ring for per-call metadata
  char* host_ring = nullptr;
  hipEvent_t ring_ev[kRing];
  bool ring_used[kRing];
  int ring_next = 0;
  float* capture = nullptr;
  bool graph_alive = false;     // a decode graph owns the last two metadata slots
  int attn_segs_per_block = 4;  // segments per attention block of contexts beyond 4096 keys (one per wave)
  int share_attention = 1;  // compute segments inside shared prompt pages once per set of rows (0: off, 2 / 3: wide sets always / never)
  bool attention_appends = true;  // decode steps: the attention kernel forms q and appends k, v itself
  // profiling
  bool prof_on = false;
  std::vector<hipEvent_t> ev_pool;
  struct Pending { int kind; hipEvent_t a, b; };
  std::vector<Pending> pending;
  double prof_ms[K_COUNT];
  int64_t prof_n[K_COUNT];
  // host time of rl_decode_step since the last read: admission checks, metadata build + upload, kernel launches
  double host_us[4] = {0.0, 0.0, 0.0, 0.0};  // admission, metadata, enqueue, wait for a metadata slot
  int64_t host_calls = 0;

  template <typename T> T* wsp(size_t off) const { return reinterpret_cast<T*>(ws + off); }
  void* k_pool(int l) const { return kv_pool + (size_t)l * layer_kv_bytes; }
  void* v_pool(int l) const { return kv_pool + (size_t)l * layer_kv_bytes + kv_block_bytes; }
};

namespace {

struct Timer {
  rl_model* m;
  hipStream_t st;
  hipEvent_t b = nullptr;
  int kind;
  Timer(rl_model* m_, hipStream_t st_, int kind_) : m(m_), st(st_), kind(kind_) {
    if (!m->prof_on) return;
    hipEvent_t a = take();
    b = take();
    if (a && b) {
      (void)hipEventRecord(a, st);
      m->pending.push_back({kind, a, b});
    } else {
      b = nullptr;
    }
  }
  ~Timer() {
    if (b) (void)hipEventRecord(b, st);
  }
  hipEvent_t take() {
    if (!m->ev_pool.empty()) { hipEvent_t e = m->ev_pool.back(); m->ev_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};

// Reserve a metadata slot: wait (practically never) until its previous upload has been consumed.
rl_status ring_acquire(rl_model* m, int* slot_out) {
  int s = m->ring_next;
  m->ring_next = (s + 1) % kRingCalls;
  if (m->ring_used[s]) {  // the device is kRingCalls calls behind: the host has nothing better to do than wait
    const auto t0 = std::chrono::steady_clock::now();
    HIP_TRY(hipEventSynchronize(m->ring_ev[s]));
    m->host_us[3] += std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
  }
  *slot_out = s;
  return RL_OK;
}

// Run all decoder layers on the M rows whose residual stream sits in ws.x.  Leaves the last down-projection's
// split partials pending; returns their count so that the caller's final residual_norm adds them.
struct SharedAttn {  // device pointers into the metadata slot of the call (empty: every row on its own)
  const int32_t* skip = nullptr;
  const AttnShared* sets = nullptr;
  int n_sets = 0, max_segs = 0;
};

// one_row_per_seq: the batch is a decode step, which lets the bf16 attention kernel take over the rotation and the
// KV append (a row's block is then the only reader of the key it writes).
int run_layers(rl_model* m, hipStream_t st, int M, const RowMeta* rows, int max_ctx_in_batch,
               const SharedAttn& sa = SharedAttn(), bool one_row_per_seq = false) {
  const Geometry& g = m->geo;
  const bool bf = g.dtype == kBF16;
  const int H = g.hidden, nqd = g.n_q * g.head_dim, nqkv = (g.n_q + 2 * g.n_kv) * g.head_dim, F = g.ffn;
  float* x = m->wsp<float>(m->lay.x);
  void* h = m->wsp<void>(m->lay.h);
  float* part = m->wsp<float>(m->lay.part);
  float* q = m->wsp<float>(m->lay.q);
  float* apart = m->wsp<float>(m->lay.attn_part);
  void* o = m->wsp<void>(m->lay.o);
  void* a = m->wsp<void>(m->lay.a);
  const float2* rope = m->wsp<float2>(m->lay.rope);
  const int32_t* bt = m->wsp<int32_t>(m->lay.block_table);
  int pend = 0;
  for (int l = 0; l < g.n_layers; ++l) {
    float* cap = m->capture ? m->capture + (size_t)l * m->cfg.max_rows * H : nullptr;
    { Timer t(m, st, K_NORM);
      launch_residual_norm(st, g.dtype, x, pend ? part : nullptr, pend, m->attn_norm[l], h, cap, M, H, g.rms_eps); }
    int s_qkv = 1;
    { Timer t(m, st, K_QKV);
      if (bf) { launch_gemm_bf16(st, h, m->wqkv[l], part, M, nqkv, H, kEpiPartial); s_qkv = gemm_bf16_splits(nqkv, H, kEpiPartial); }
      else launch_gemm_f32(st, (const float*)h, (const float*)m->wqkv[l], part, M, nqkv, H, kEpiPartial); }
    const void* q_gain = g.qk_norm ? m->q_norm[l] : nullptr;
    const void* k_gain = g.qk_norm ? m->k_norm[l] : nullptr;
    const bool fused = bf && one_row_per_seq && m->attention_appends && s_qkv <= kAttnAppendMaxSplits;
    if (!fused) {
      Timer t(m, st, K_ROPE_APPEND);
      launch_qk_rope_append(st, g, part, s_qkv, q_gain, k_gain, rope, rows, m->k_pool(l), m->v_pool(l), q, M);
    }
    if (bf) {
      bool merge;
      { Timer t(m, st, K_ATTN);
        const AttnAppend ap = {part, s_qkv, q_gain, k_gain, rope};
        merge = launch_attn_decode_bf16(st, g, q, rows, bt, m->k_pool(l), m->v_pool(l), apart, m->lay.max_segs, max_ctx_in_batch,
                                        o, M, sa.skip, sa.sets, sa.n_sets, sa.max_segs, fused ? &ap : nullptr,
                                        m->attn_segs_per_block); }
      if (merge) {
        Timer t(m, st, K_ATTN_MERGE);
        launch_attn_merge_bf16(st, g, rows, apart, m->lay.max_segs, o, M, sa.skip, sa.n_sets);
      }
    } else {
      Timer t(m, st, K_ATTN);
      launch_attn_f32(st, g, q, rows, bt, m->k_pool(l), m->v_pool(l), (float*)o, M);
    }
    int s_o = 1;
    { Timer t(m, st, K_OPROJ);
      if (bf) { launch_gemm_bf16(st, o, m->wo[l], part, M, H, nqd, kEpiPartial); s_o = gemm_bf16_splits(H, nqd, kEpiPartial); }
      else launch_gemm_f32(st, (const float*)o, (const float*)m->wo[l], part, M, H, nqd, kEpiPartial); }
    { Timer t(m, st, K_NORM);
      launch_residual_norm(st, g.dtype, x, part, s_o, m->mlp_norm[l], h, nullptr, M, H, g.rms_eps); }
    { Timer t(m, st, K_GATEUP);
      if (bf) launch_gemm_bf16(st, h, m->w_gate_up[l], a, M, F, H, kEpiSwiGLU);
      else launch_gemm_f32(st, (const float*)h, (const float*)m->w_gate_up[l], (float*)a, M, F, H, kEpiSwiGLU); }
    { Timer t(m, st, K_DOWN);
      if (bf) { launch_gemm_bf16(st, a, m->w_down[l], part, M, H, F, kEpiPartial); pend = gemm_bf16_splits(H, F, kEpiPartial); }
      else { launch_gemm_f32(st, (const float*)a, (const float*)m->w_down[l], part, M, H, F, kEpiPartial); pend = 1; } }
  }
  return pend;
}

// Final norm, output projection and sampling for M rows whose residual is in `xbuf` (pending partials added).
void run_head(rl_model* m, hipStream_t st, int M, float* xbuf, int pend, const RowMeta* rows, int pos_offset,
              const int32_t* forced, const rl_sampling* sp, int32_t* out_tokens, float* out_lp, float* debug_logits,
              bool score_only = false) {
  int32_t* last_tok = score_only ? nullptr : m->wsp<int32_t>(m->lay.last_tok);
  const Geometry& g = m->geo;
  void* h = m->wsp<void>(m->lay.h);
  float* part = m->wsp<float>(m->lay.part);
  float* logits = m->wsp<float>(m->lay.logits);
  float* cap = m->capture ? m->capture + (size_t)g.n_layers * m->cfg.max_rows * g.hidden : nullptr;
  { Timer t(m, st, K_NORM);
    launch_residual_norm(st, g.dtype, xbuf, pend ? part : nullptr, pend, m->final_norm, h, cap, M, g.hidden, g.rms_eps); }
  float* spart = m->wsp<float>(m->lay.samp_part);
  float* fz = m->wsp<float>(m->lay.forced_z);
  const int top_k = sp->top_k > (uint32_t)g.vocab ? 0 : (int)sp->top_k;
  const bool truncated = !score_only && sp->temperature > 0.f && sample_is_truncated(g.vocab, top_k, sp->top_p);
  if (g.dtype == kBF16 && !truncated) {
    SampleEpilogue se;
    se.rows = rows; se.pos_offset = pos_offset;
    se.greedy = !(sp->temperature > 0.f);
    se.inv_t = se.greedy ? 1.0f : 1.0f / sp->temperature;
    if (score_only) se.greedy = 1;  // every row is forced: skip the random numbers, keep the temperature
    se.seed_lo = (uint32_t)(sp->seed & 0xffffffffu); se.seed_hi = (uint32_t)(sp->seed >> 32);
    se.forced = forced; se.forced_z = fz; se.part = spart; se.logits_out = debug_logits;
    { Timer t(m, st, K_LMHEAD);
      launch_gemm_bf16(st, h, m->lm_head, nullptr, M, g.vocab, g.hidden, kEpiSample, false, &se); }
    { Timer t(m, st, K_SAMPLE);
      launch_sample_merge(st, spart, g.vocab >> 6, M, g.vocab, forced, fz, sp->temperature, out_tokens, out_lp, rows, last_tok); }
  } else {
    // logits to memory (a truncated distribution needs the whole row first), then the stand-alone sampler
    { Timer t(m, st, K_LMHEAD);
      if (g.dtype == kBF16) launch_gemm_bf16(st, h, m->lm_head, logits, M, g.vocab, g.hidden, kEpiPartial, false);
      else launch_gemm_f32(st, (const float*)h, (const float*)m->lm_head, logits, M, g.vocab, g.hidden, kEpiPartial); }
    { Timer t(m, st, K_SAMPLE);
      launch_sample(st, logits, M, g.vocab, rows, pos_offset, forced, sp->temperature, sp->seed, spart, fz, out_tokens, out_lp,
                    truncated ? top_k : 0, truncated ? sp->top_p : 0.f, m->wsp<void>(m->lay.cuts), last_tok); }
    if (debug_logits)
      (void)hipMemcpyAsync(debug_logits, logits, (size_t)M * g.vocab * 4, hipMemcpyDeviceToDevice, st);
  }
}

// Checks shared by decode calls; on success `grants` holds the pages handed out and lens are NOT yet advanced.
rl_status admit_decode(rl_model* m, int32_t n, const int32_t* seq_ids, std::vector<PageGrant>* grants) {
  if (n < 1 || n > (int32_t)m->cfg.max_rows) return fail(RL_ERR_INVALID_ARG, "n_seqs %d outside [1, max_rows=%u]", n, m->cfg.max_rows);
  if (!seq_ids) return fail(RL_ERR_INVALID_ARG, "seq_ids is NULL");
  SeqTable& T = *m->table;
  std::vector<char> seen(T.max_seqs(), 0);
  int64_t need = 0;
  for (int i = 0; i < n; ++i) {
    int32_t s = seq_ids[i];
    if (!T.active(s)) return fail(RL_ERR_BAD_SEQ, "sequence %d is not active", s);
    if (seen[s]) return fail(RL_ERR_INVALID_ARG, "sequence %d appears twice", s);
    seen[s] = 1;
    if (T.len(s) + 1 > T.max_ctx()) return fail(RL_ERR_CTX_OVERFLOW, "sequence %d would exceed max_ctx %d", s, T.max_ctx());
    need += T.pages_missing(s, T.len(s) + 1);
  }
  if (need > T.free_pages()) return fail(RL_ERR_KV_FULL, "need %lld pages, %lld free", (long long)need, (long long)T.free_pages());
  for (int i = 0; i < n; ++i) T.reserve(seq_ids[i], T.len(seq_ids[i]) + 1, grants);
  return RL_OK;
}

// Copy a plan of shared attention into the metadata slot (host side hs, device side ds) and describe it in *sa.
rl_status upload_attn_plan(rl_model* m, hipStream_t st, char* hs, char* ds, int n, const AttnPlan& plan, SharedAttn* sa) {
  *sa = SharedAttn();
  if (plan.sets.empty()) return RL_OK;
  memcpy(hs + m->lay.slot_skip, plan.skip.data(), (size_t)n * 4);
  memcpy(hs + m->lay.slot_sets, plan.sets.data(), plan.sets.size() * sizeof(AttnShared));
  HIP_TRY(hipMemcpyAsync(ds + m->lay.slot_skip, hs + m->lay.slot_skip, (size_t)n * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(hipMemcpyAsync(ds + m->lay.slot_sets, hs + m->lay.slot_sets, plan.sets.size() * sizeof(AttnShared), hipMemcpyHostToDevice, st));
  sa->skip = (const int32_t*)(ds + m->lay.slot_skip);
  sa->sets = (const AttnShared*)(ds + m->lay.slot_sets);
  sa->n_sets = (int)plan.sets.size();
  sa->max_segs = plan.max_shared_segs;
  return RL_OK;
}

// Rows per set for a call of n rows (the test switch can ask for the wide sets always or never, whatever the size).
int rows_per_set(const rl_model* m, int n) {
  if (m->share_attention == 2) n = 1 << 20;
  if (m->share_attention == 3) n = 0;
  return attn_rows_per_set(m->geo.n_q / m->geo.n_kv, m->geo.kv_fp8, n, m->geo.n_kv);
}

// Sets of neighbouring rows of one sequence for a chunk of prefill or scoring rows (bf16 only).
rl_status upload_window_plan(rl_model* m, hipStream_t st, char* hs, char* ds, int n, const RowMeta* hr, SharedAttn* sa) {
  *sa = SharedAttn();
  if (m->geo.dtype != kBF16 || !m->share_attention) return RL_OK;
  std::vector<int32_t> seq(n), pos(n);
  for (int i = 0; i < n; ++i) { seq[i] = hr[i].seq; pos[i] = hr[i].pos; }
  AttnPlan plan;
  plan_window_sets(n, seq.data(), pos.data(), rows_per_set(m, n), &plan);
  return upload_attn_plan(m, st, hs, ds, n, plan, sa);
}

// Write the rows, page grants and shared-attention plan of one decode call into the host slot hs and describe them
// (device pointers relative to the device slot ds).  Returns the bytes of the slot in use.
size_t build_decode_meta(rl_model* m, int32_t n, const int32_t* seq_ids, const std::vector<PageGrant>& grants, char* hs,
                         char* ds, int* max_ctx_out, SharedAttn* sa) {
  RowMeta* hr = (RowMeta*)hs;
  int max_ctx = 0;
  for (int i = 0; i < n; ++i) {
    hr[i].seq = seq_ids[i];
    hr[i].pos = m->table->len(seq_ids[i]);
    hr[i].page = m->table->pages(seq_ids[i])[hr[i].pos >> 4];  // reserved by admit_decode
    hr[i].pad = 0;
    if (hr[i].pos + 1 > max_ctx) max_ctx = hr[i].pos + 1;
  }
  int32_t* hu = (int32_t*)(hs + m->lay.slot_upd);
  for (size_t i = 0; i < grants.size(); ++i) { hu[3 * i] = grants[i].seq; hu[3 * i + 1] = grants[i].block; hu[3 * i + 2] = grants[i].page; }
  // rows of sequences that hold prompt pages in common and stand at the same position share those segments
  *sa = SharedAttn();
  AttnPlan plan;
  if (m->geo.dtype == kBF16 && m->share_attention) {
    std::vector<int64_t> fam(n);
    std::vector<int32_t> fam_blocks(n), pos(n);
    bool any = false;
    for (int i = 0; i < n; ++i) {
      fam[i] = m->table->prefix_id(seq_ids[i]);
      fam_blocks[i] = m->table->prefix_blocks(seq_ids[i]);
      pos[i] = hr[i].pos;
      any |= fam[i] != 0;
    }
    if (any) plan_shared_attention(n, fam.data(), fam_blocks.data(), pos.data(), rows_per_set(m, n), &plan);
  }
  hr[0].pad = (int32_t)grants.size();
  // One upload for everything the step needs: the slot's regions lie at fixed offsets, so the copy runs from the rows
  // to the end of the last region in use (a few KB; what lies between is not read).
  size_t used = (size_t)n * sizeof(RowMeta);
  if (!grants.empty()) used = m->lay.slot_upd + grants.size() * 12;
  if (!plan.sets.empty()) {
    memcpy(hs + m->lay.slot_skip, plan.skip.data(), (size_t)n * 4);
    memcpy(hs + m->lay.slot_sets, plan.sets.data(), plan.sets.size() * sizeof(AttnShared));
    used = m->lay.slot_sets + plan.sets.size() * sizeof(AttnShared);
    sa->skip = (const int32_t*)(ds + m->lay.slot_skip);
    sa->sets = (const AttnShared*)(ds + m->lay.slot_sets);
    sa->n_sets = (int)plan.sets.size();
    sa->max_segs = plan.max_shared_segs;
  }
  *max_ctx_out = max_ctx;
  return used;
}

// Build and upload the rows (and page grants) of one decode call; returns device pointers into the slot.
rl_status upload_decode_meta(rl_model* m, hipStream_t st, int32_t n, const int32_t* seq_ids,
                             const std::vector<PageGrant>& grants, const RowMeta** rows_dev, int* max_ctx_out,
                             SharedAttn* sa) {
  int slot;
  rl_status rs = ring_acquire(m, &slot);
  if (rs != RL_OK) return rs;
  char* hs = m->host_ring + (size_t)slot * m->lay.slot_bytes;
  char* ds = m->ws + m->lay.ring + (size_t)slot * m->lay.slot_bytes;
  const size_t used = build_decode_meta(m, n, seq_ids, grants, hs, ds, max_ctx_out, sa);
  Timer t(m, st, K_META);
  HIP_TRY(hipMemcpyAsync(ds, hs, used, hipMemcpyHostToDevice, st));
  if (!grants.empty())
    launch_table_update(st, m->wsp<int32_t>(m->lay.block_table), m->geo.max_blocks, (const int32_t*)(ds + m->lay.slot_upd), (int)grants.size());
  HIP_TRY(hipEventRecord(m->ring_ev[slot], st));
  m->ring_used[slot] = true;
  *rows_dev = (const RowMeta*)ds;
  return RL_OK;
}

// The kernels of one decode step for n rows whose metadata is on the device: embedding, layers, head.
void decode_enqueue(rl_model* m, hipStream_t st, int n, const RowMeta* rows, int max_ctx_in_batch, const SharedAttn& sa,
                    const int32_t* in_tokens, const int32_t* forced_next, const rl_sampling* sp, int32_t* out_tokens,
                    float* out_logprobs, float* debug_logits) {
  float* x = m->wsp<float>(m->lay.x);
  { Timer t(m, st, K_EMBED);
    launch_embed(st, m->geo.dtype, m->embed, in_tokens, x, n, m->geo.hidden, m->geo.vocab, rows, m->wsp<int32_t>(m->lay.last_tok)); }
  int pend = run_layers(m, st, n, rows, max_ctx_in_batch, sa, true);
  run_head(m, st, n, x, pend, rows, 1, forced_next, sp, out_tokens, out_logprobs, debug_logits);
}

}  // namespace

// A decode step of a fixed batch as a HIP graph.  What changes from step to step is data (rows, page grants, the
// shared-attention plan: one upload from a pinned buffer that the graph's copy node reads at every launch) except for
// three launch shapes, which form the key of the captured graph: the 1024-key bracket of the longest context (block
// count and shared-memory size of the attention launch), the number of row sets, and the blocks the sets need.  When
// the key changes -- once per 1024 steps for a batch in lock step -- the step is captured again.  Two buffers and two
// graphs alternate, so the host may prepare step k + 1 while step k runs.
struct rl_decode_graph {
  rl_model* m = nullptr;
  std::vector<int32_t> ids;
  rl_sampling sp;
  int32_t* out_tokens = nullptr;
  float* out_logprobs = nullptr;
  char* host[2] = {nullptr, nullptr};  // pinned copies of the metadata slot
  hipEvent_t ev[2] = {nullptr, nullptr};
  bool ev_used[2] = {false, false};
  hipGraphExec_t exec[2] = {nullptr, nullptr};
  struct Key { int ctx_bracket, n_sets, set_blocks; } key[2] = {{-1, -1, -1}, {-1, -1, -1}};
  int next = 0;
  int64_t captures = 0;
};

extern "C" {

const char* rl_last_error(void) { return g_err.c_str(); }

uint64_t rl_kv_page_bytes(const rl_model_config* c) {
  if (check_config(c) != RL_OK) return 0;
  return (uint64_t)c->n_layers * 2 * c->n_kv_heads * 16 * c->head_dim * kv_elem_size(*c);
}

rl_status rl_query_workspace(const rl_model_config* c, uint64_t* bytes_out) {
  rl_status rs = check_config(c);
  if (rs != RL_OK) return rs;
  if (!bytes_out) return fail(RL_ERR_INVALID_ARG, "bytes_out is NULL");
  Layout L;
  compute_layout(*c, &L);
  *bytes_out = L.total;
  return RL_OK;
}

rl_status rl_init_model(const rl_model_config* c, const rl_weights* w, rl_model** out) {
  rl_status rs = check_config(c);
  if (rs != RL_OK) return rs;
  if (!w || !out) return fail(RL_ERR_INVALID_ARG, "weights or out is NULL");
  if (!w->final_norm || !w->attn_norm || !w->wqkv || !w->wo || !w->mlp_norm || !w->w_gate_up || !w->w_down || !w->kv_pool || !w->workspace)
    return fail(RL_ERR_INVALID_ARG, "a required weight pointer is NULL");
  if (c->vocab && (!w->embed || !w->lm_head)) return fail(RL_ERR_INVALID_ARG, "embed/lm_head is NULL with vocab > 0");
  if (c->qk_norm && (!w->q_norm || !w->k_norm)) return fail(RL_ERR_INVALID_ARG, "q_norm/k_norm is NULL with qk_norm = 1");
  Layout L;
  compute_layout(*c, &L);
  if (c->workspace_bytes < L.total) return fail(RL_ERR_INVALID_ARG, "workspace_bytes %llu < required %llu", (unsigned long long)c->workspace_bytes, (unsigned long long)L.total);
  const uint64_t page_bytes = rl_kv_page_bytes(c);
  const int64_t n_pages = (int64_t)(c->kv_pool_bytes / page_bytes);
  if (n_pages < 1 || n_pages > 0x7fffffff) return fail(RL_ERR_INVALID_ARG, "kv_pool_bytes gives %lld pages", (long long)n_pages);

  rl_model* m = new rl_model();
  m->cfg = *c;
  m->lay = L;
  m->geo = Geometry{(int)c->n_layers, (int)c->hidden, (int)c->n_q_heads, (int)c->n_kv_heads, (int)c->head_dim, (int)c->ffn,
                    (int)c->vocab, (int)c->qk_norm, c->rms_eps, (int)c->dtype, (int)(c->max_ctx / 16), n_pages,
                    c->kv_dtype == RL_KV_FP8 ? 1 : 0};
  m->embed = w->embed; m->lm_head = w->lm_head; m->final_norm = w->final_norm;
  auto copy = [&](std::vector<const void*>& dst, const void* const* src) {
    dst.assign(c->n_layers, nullptr);
    if (src) for (uint32_t l = 0; l < c->n_layers; ++l) dst[l] = src[l];
  };
  copy(m->attn_norm, w->attn_norm); copy(m->wqkv, w->wqkv); copy(m->q_norm, w->q_norm); copy(m->k_norm, w->k_norm);
  copy(m->wo, w->wo); copy(m->mlp_norm, w->mlp_norm); copy(m->w_gate_up, w->w_gate_up); copy(m->w_down, w->w_down);
  for (uint32_t l = 0; l < c->n_layers; ++l)
    if (!m->attn_norm[l] || !m->wqkv[l] || !m->wo[l] || !m->mlp_norm[l] || !m->w_gate_up[l] || !m->w_down[l] ||
        (c->qk_norm && (!m->q_norm[l] || !m->k_norm[l]))) {
      delete m;
      return fail(RL_ERR_INVALID_ARG, "layer %u has a NULL weight pointer", l);
    }
  m->kv_pool = (char*)w->kv_pool;
  m->ws = (char*)w->workspace;
  m->kv_block_bytes = (size_t)16 * c->head_dim * kv_elem_size(*c);
  m->layer_kv_bytes = (size_t)n_pages * c->n_kv_heads * 2 * m->kv_block_bytes;
  m->table = new SeqTable((int)c->max_seqs, (int)c->max_ctx, n_pages);
  for (int i = 0; i < K_COUNT; ++i) { m->prof_ms[i] = 0; m->prof_n[i] = 0; }
  for (int i = 0; i < kRing; ++i) { m->ring_ev[i] = nullptr; m->ring_used[i] = false; }

  auto bail = [&](hipError_t e, const char* what) {
    rl_status r = fail(RL_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    rl_destroy_model(m);
    return r;
  };
  hipError_t e;
  if ((e = hipHostMalloc((void**)&m->host_ring, kRing * L.slot_bytes, hipHostMallocDefault)) != hipSuccess) return bail(e, "hipHostMalloc");
  for (int i = 0; i < kRing; ++i)
    if ((e = hipEventCreateWithFlags(&m->ring_ev[i], hipEventDisableTiming)) != hipSuccess) return bail(e, "hipEventCreate");
  // Stale slots of recycled pages are multiplied by zero weights, so the pool must never hold NaN/Inf patterns.
  if ((e = hipMemset(m->kv_pool, 0, (size_t)n_pages * page_bytes)) != hipSuccess) return bail(e, "hipMemset(kv_pool)");
  if ((e = hipMemset(m->ws + L.block_table, 0, (size_t)c->max_seqs * (c->max_ctx / 16) * 4)) != hipSuccess) return bail(e, "hipMemset(block_table)");
  {
    const int half = (int)c->head_dim / 2;
    std::vector<float2> tab((size_t)c->max_ctx * half);
    for (int i = 0; i < half; ++i) {
      const double freq = std::pow((double)c->rope_base, -2.0 * i / (double)c->head_dim);
      for (uint32_t p = 0; p < c->max_ctx; ++p) {
        const double ang = (double)p * freq;
        tab[(size_t)p * half + i] = make_float2((float)std::cos(ang), (float)std::sin(ang));
      }
    }
    if ((e = hipMemcpy(m->ws + L.rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice)) != hipSuccess) return bail(e, "hipMemcpy(rope)");
  }
  if ((e = hipDeviceSynchronize()) != hipSuccess) return bail(e, "hipDeviceSynchronize");
  *out = m;
  return RL_OK;
}

void rl_destroy_model(rl_model* m) {
  if (!m) return;
  for (auto& p : m->pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  for (auto ev : m->ev_pool) (void)hipEventDestroy(ev);
  for (int i = 0; i < kRing; ++i) if (m->ring_ev[i]) (void)hipEventDestroy(m->ring_ev[i]);
  if (m->host_ring) (void)hipHostFree(m->host_ring);
  delete m->table;
  delete m;
}

rl_status rl_kv_stats(const rl_model* m, uint64_t* free_pages, uint64_t* total_pages) {
  if (!m) return fail(RL_ERR_INVALID_ARG, "model is NULL");
  if (free_pages) *free_pages = (uint64_t)m->table->free_pages();
  if (total_pages) *total_pages = (uint64_t)m->table->n_pages();
  return RL_OK;
}

rl_status rl_seq_len(const rl_model* m, int32_t seq_id, int32_t* len_out) {
  if (!m || !len_out) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  if (!m->table->active(seq_id)) return fail(RL_ERR_BAD_SEQ, "sequence %d is not active", seq_id);
  *len_out = m->table->len(seq_id);
  return RL_OK;
}

rl_status rl_free_seqs(rl_model* m, int32_t n, const int32_t* seq_ids) {
  if (!m || (n > 0 && !seq_ids) || n < 0) return fail(RL_ERR_INVALID_ARG, "bad arguments");
  SeqTable& T = *m->table;
  std::vector<char> seen(T.max_seqs(), 0);
  for (int i = 0; i < n; ++i) {
    if (!T.active(seq_ids[i])) return fail(RL_ERR_BAD_SEQ, "sequence %d is not active", seq_ids[i]);
    if (seen[seq_ids[i]]) return fail(RL_ERR_INVALID_ARG, "sequence %d appears twice", seq_ids[i]);
    seen[seq_ids[i]] = 1;
  }
  for (int i = 0; i < n; ++i) T.release(seq_ids[i]);
  return RL_OK;
}

rl_status rl_debug_shuffle_free_pages(rl_model* m, uint64_t seed) {
  if (!m) return fail(RL_ERR_INVALID_ARG, "model is NULL");
  m->table->shuffle_free(seed);
  return RL_OK;
}

rl_status rl_debug_share_attention(rl_model* m, int32_t on) {
  if (!m) return fail(RL_ERR_INVALID_ARG, "model is NULL");
  m->share_attention = (on == 2 || on == 3) ? on : on != 0;
  return RL_OK;
}

rl_status rl_debug_attention_split(rl_model* m, int32_t segs_per_block) {
  if (!m) return fail(RL_ERR_INVALID_ARG, "model is NULL");
  if (segs_per_block < 1 || segs_per_block > 16) return fail(RL_ERR_INVALID_ARG, "segs_per_block %d outside [1, 16]", segs_per_block);
  m->attn_segs_per_block = segs_per_block;
  return RL_OK;
}

rl_status rl_debug_attention_appends(rl_model* m, int32_t on) {
  if (!m) return fail(RL_ERR_INVALID_ARG, "model is NULL");
  m->attention_appends = on != 0;
  return RL_OK;
}

rl_status rl_set_capture(rl_model* m, float* buf) {
  if (!m) return fail(RL_ERR_INVALID_ARG, "model is NULL");
  m->capture = buf;
  return RL_OK;
}

rl_status rl_decode_step(rl_model* m, void* stream, int32_t n, const int32_t* seq_ids, const int32_t* in_tokens,
                         const int32_t* forced_next, const rl_sampling* sp, int32_t* out_tokens, float* out_logprobs,
                         float* debug_logits) {
  if (!m || !sp || !out_tokens || !out_logprobs) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  if (m->geo.vocab == 0) return fail(RL_ERR_UNSUPPORTED, "model has no vocabulary");
  hipStream_t st = (hipStream_t)stream;
  const auto t0 = std::chrono::steady_clock::now();
  std::vector<PageGrant> grants;
  rl_status rs = admit_decode(m, n, seq_ids, &grants);
  if (rs != RL_OK) return rs;
  const auto t1 = std::chrono::steady_clock::now();
  const double waited = m->host_us[3];
  const RowMeta* rows;
  int max_ctx_in_batch;
  SharedAttn sa;
  rs = upload_decode_meta(m, st, n, seq_ids, grants, &rows, &max_ctx_in_batch, &sa);
  if (rs != RL_OK) return rs;
  const auto t2 = std::chrono::steady_clock::now();
  decode_enqueue(m, st, n, rows, max_ctx_in_batch, sa, in_tokens, forced_next, sp, out_tokens, out_logprobs, debug_logits);
  HIP_TRY(hipGetLastError());
  for (int i = 0; i < n; ++i) m->table->set_len(seq_ids[i], m->table->len(seq_ids[i]) + 1);
  const auto t3 = std::chrono::steady_clock::now();
  m->host_us[0] += std::chrono::duration<double, std::micro>(t1 - t0).count();
  m->host_us[1] += std::chrono::duration<double, std::micro>(t2 - t1).count() - (m->host_us[3] - waited);
  m->host_us[2] += std::chrono::duration<double, std::micro>(t3 - t2).count();
  m->host_calls += 1;
  return RL_OK;
}

rl_status rl_profile_host_read(rl_model* m, double* admit_us, double* meta_us, double* launch_us, double* wait_us,
                               int64_t* calls) {
  if (!m || !admit_us || !meta_us || !launch_us || !wait_us || !calls) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  *admit_us = m->host_us[0]; *meta_us = m->host_us[1]; *launch_us = m->host_us[2]; *wait_us = m->host_us[3];
  *calls = m->host_calls;
  m->host_us[0] = m->host_us[1] = m->host_us[2] = m->host_us[3] = 0.0;
  m->host_calls = 0;
  return RL_OK;
}

rl_status rl_decode_graph_create(rl_model* m, int32_t n, const int32_t* seq_ids, const rl_sampling* sp,
                                 int32_t* out_tokens, float* out_logprobs, rl_decode_graph** out) {
  if (!m || !seq_ids || !sp || !out_tokens || !out_logprobs || !out) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  if (m->geo.vocab == 0) return fail(RL_ERR_UNSUPPORTED, "model has no vocabulary");
  if (n < 1 || n > (int32_t)m->cfg.max_rows) return fail(RL_ERR_INVALID_ARG, "n_seqs %d outside [1, max_rows=%u]", n, m->cfg.max_rows);
  if (m->graph_alive) return fail(RL_ERR_UNSUPPORTED, "one decode graph per model at a time");
  rl_decode_graph* g = new rl_decode_graph();
  g->m = m;
  g->ids.assign(seq_ids, seq_ids + n);
  g->sp = *sp;
  g->out_tokens = out_tokens;
  g->out_logprobs = out_logprobs;
  for (int b = 0; b < 2; ++b) {
    hipError_t e = hipHostMalloc((void**)&g->host[b], m->lay.slot_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&g->ev[b], hipEventDisableTiming);
    if (e != hipSuccess) {
      rl_decode_graph_destroy(g);
      return fail(RL_ERR_DEVICE, "rl_decode_graph_create: %s", hipGetErrorString(e));
    }
    memset(g->host[b], 0, m->lay.slot_bytes);
  }
  m->graph_alive = true;
  *out = g;
  return RL_OK;
}

void rl_decode_graph_destroy(rl_decode_graph* g) {
  if (!g) return;
  for (int b = 0; b < 2; ++b) {
    if (g->ev[b]) { if (g->ev_used[b]) (void)hipEventSynchronize(g->ev[b]); (void)hipEventDestroy(g->ev[b]); }
    if (g->exec[b]) (void)hipGraphExecDestroy(g->exec[b]);
    if (g->host[b]) (void)hipHostFree(g->host[b]);
  }
  if (g->m) g->m->graph_alive = false;
  delete g;
}

rl_status rl_decode_graph_step(rl_decode_graph* g, void* stream, int64_t* captures_out) {
  if (!g) return fail(RL_ERR_INVALID_ARG, "graph is NULL");
  if (!stream) return fail(RL_ERR_INVALID_ARG, "the null stream cannot be captured: pass a stream created by the caller");
  rl_model* m = g->m;
  hipStream_t st = (hipStream_t)stream;
  const int n = (int)g->ids.size();
  std::vector<PageGrant> grants;
  rl_status rs = admit_decode(m, n, g->ids.data(), &grants);
  if (rs != RL_OK) return rs;
  const int b = g->next;
  if (g->ev_used[b]) HIP_TRY(hipEventSynchronize(g->ev[b]));  // the launch that read this buffer last has finished
  char* hs = g->host[b];
  char* ds = m->ws + m->lay.ring + (size_t)(kRingCalls + b) * m->lay.slot_bytes;
  int max_ctx = 0;
  SharedAttn sa;
  build_decode_meta(m, n, g->ids.data(), grants, hs, ds, &max_ctx, &sa);
  const rl_decode_graph::Key key = {(max_ctx + 1023) / 1024, sa.n_sets, (sa.max_segs + 3) / 4};
  if (!g->exec[b] || key.ctx_bracket != g->key[b].ctx_bracket || key.n_sets != g->key[b].n_sets ||
      key.set_blocks != g->key[b].set_blocks) {
    if (g->exec[b]) { (void)hipGraphExecDestroy(g->exec[b]); g->exec[b] = nullptr; }
    const bool prof = m->prof_on;
    m->prof_on = false;  // no event pairs inside a captured step
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal);
    if (e == hipSuccess) {
      e = hipMemcpyAsync(ds, hs, m->lay.slot_bytes, hipMemcpyHostToDevice, st);
      launch_table_update_counted(st, m->wsp<int32_t>(m->lay.block_table), m->geo.max_blocks,
                                  (const int32_t*)(ds + m->lay.slot_upd), (const RowMeta*)ds, n);
      SharedAttn sa_cap = sa;
      sa_cap.max_segs = key.set_blocks * 4;  // the attention grid only takes its block count from it
      decode_enqueue(m, st, n, (const RowMeta*)ds, key.ctx_bracket * 1024, sa_cap, nullptr, nullptr, &g->sp, g->out_tokens,
                     g->out_logprobs, nullptr);
      const hipError_t e_end = hipStreamEndCapture(st, &graph);  // always ends the capture
      if (e == hipSuccess) e = e_end;
    }
    if (e == hipSuccess) e = hipGraphInstantiate(&g->exec[b], graph, nullptr, nullptr, 0);
    if (graph) (void)hipGraphDestroy(graph);
    m->prof_on = prof;
    if (e != hipSuccess) { g->exec[b] = nullptr; return fail(RL_ERR_DEVICE, "rl_decode_graph_step: capture: %s", hipGetErrorString(e)); }
    g->key[b] = key;
    g->captures += 1;
  }
  HIP_TRY(hipGraphLaunch(g->exec[b], st));
  HIP_TRY(hipEventRecord(g->ev[b], st));
  g->ev_used[b] = true;
  for (int i = 0; i < n; ++i) m->table->set_len(g->ids[i], m->table->len(g->ids[i]) + 1);
  g->next = b ^ 1;
  if (captures_out) *captures_out = g->captures;
  return RL_OK;
}

rl_status rl_decode_hidden(rl_model* m, void* stream, int32_t n, const int32_t* seq_ids, const float* hidden_in,
                           float* hidden_out) {
  if (!m || !hidden_in || !hidden_out) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  hipStream_t st = (hipStream_t)stream;
  std::vector<PageGrant> grants;
  rl_status rs = admit_decode(m, n, seq_ids, &grants);
  if (rs != RL_OK) return rs;
  const RowMeta* rows;
  int max_ctx_in_batch;
  SharedAttn sa;
  rs = upload_decode_meta(m, st, n, seq_ids, grants, &rows, &max_ctx_in_batch, &sa);
  if (rs != RL_OK) return rs;
  float* x = m->wsp<float>(m->lay.x);
  const size_t bytes = (size_t)n * m->geo.hidden * 4;
  HIP_TRY(hipMemcpyAsync(x, hidden_in, bytes, hipMemcpyDeviceToDevice, st));
  int pend = run_layers(m, st, n, rows, max_ctx_in_batch, sa, true);
  float* cap = m->capture ? m->capture + (size_t)m->geo.n_layers * m->cfg.max_rows * m->geo.hidden : nullptr;
  { Timer t(m, st, K_NORM);
    launch_residual_norm(st, m->geo.dtype, x, m->wsp<float>(m->lay.part), pend, nullptr, nullptr, cap, n, m->geo.hidden, m->geo.rms_eps); }
  HIP_TRY(hipMemcpyAsync(hidden_out, x, bytes, hipMemcpyDeviceToDevice, st));
  HIP_TRY(hipGetLastError());
  for (int i = 0; i < n; ++i) m->table->set_len(seq_ids[i], m->table->len(seq_ids[i]) + 1);
  return RL_OK;
}

// Make each `dst` (valid id, inactive) a continuation of `src` (active) at `len` tokens: the pages that `len`
// tokens fill completely are shared, a partial last page is copied into a page of dst's own.  The caller has
// checked ids and free pages (one per dst when len % 16 != 0) and sets the lengths.  At most max_rows forks.
struct Fork { int32_t src, dst, len; };
static rl_status fork_seqs(rl_model* m, hipStream_t st, const std::vector<Fork>& forks) {
  SeqTable& T = *m->table;
  int32_t* bt = m->wsp<int32_t>(m->lay.block_table);
  std::vector<int32_t> pairs;  // (src page, dst page)
  for (const Fork& f : forks) {
    const int full = f.len / SeqTable::kBlock;
    T.activate(f.dst);
    T.share_prefix(f.dst, f.src, full);
    if (f.len % SeqTable::kBlock) {
      T.reserve(f.dst, f.len, nullptr);
      pairs.push_back(T.pages(f.src)[full]);
      pairs.push_back(T.pages(f.dst)[full]);
    }
    // pageable source: the runtime stages it before returning, so the vector may change afterwards
    if (!T.pages(f.dst).empty())
      HIP_TRY(hipMemcpyAsync(bt + (size_t)f.dst * m->geo.max_blocks, T.pages(f.dst).data(), T.pages(f.dst).size() * 4, hipMemcpyHostToDevice, st));
  }
  if (!pairs.empty()) {
    int slot;
    rl_status rs = ring_acquire(m, &slot);
    if (rs != RL_OK) return rs;
    char* hs = m->host_ring + (size_t)slot * m->lay.slot_bytes;
    char* ds = m->ws + m->lay.ring + (size_t)slot * m->lay.slot_bytes;
    memcpy(hs + m->lay.slot_upd, pairs.data(), pairs.size() * 4);  // at most 2 * max_rows ints
    HIP_TRY(hipMemcpyAsync(ds + m->lay.slot_upd, hs + m->lay.slot_upd, pairs.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipEventRecord(m->ring_ev[slot], st));
    m->ring_used[slot] = true;
    launch_page_copy(st, m->kv_pool, m->layer_kv_bytes, (size_t)m->geo.n_kv * 2 * m->kv_block_bytes, m->geo.n_layers,
                     (const int32_t*)(ds + m->lay.slot_upd), (int)(pairs.size() / 2));
  }
  return RL_OK;
}

// Prefill of n_prompts prompts, each followed by `group` sequences (seq_ids[i*group + j]).  Member 0 of a group
// runs the prompt; the others share every page the prompt fills completely and get a private copy of the partial
// last page, so the prompt's KV is computed and stored once per group.
static rl_status prefill_impl(rl_model* m, hipStream_t st, int32_t n_prompts, int32_t group, const int32_t* seq_ids,
                              const int32_t* prompt_tokens, const int32_t* prompt_lens, const rl_sampling* sp,
                              int32_t* out_tokens, float* out_logprobs) {
  if (m->geo.vocab == 0) return fail(RL_ERR_UNSUPPORTED, "model has no vocabulary");
  if (n_prompts < 1 || group < 1 || (int64_t)n_prompts * group > (int64_t)m->cfg.max_rows)
    return fail(RL_ERR_INVALID_ARG, "n_prompts %d x group %d outside [1, max_rows=%u]", n_prompts, group, m->cfg.max_rows);
  SeqTable& T = *m->table;
  const int n_all = n_prompts * group;
  const int R = (int)m->cfg.max_rows, H = m->geo.hidden;
  std::vector<char> seen(T.max_seqs(), 0);
  int64_t need = 0, total = 0;
  for (int i = 0; i < n_all; ++i) {
    const int32_t s = seq_ids[i];
    if (!T.valid_id(s)) return fail(RL_ERR_BAD_SEQ, "sequence id %d out of range", s);
    if (T.active(s)) return fail(RL_ERR_BAD_SEQ, "sequence %d is already active", s);
    if (seen[s]) return fail(RL_ERR_INVALID_ARG, "sequence %d appears twice", s);
    seen[s] = 1;
  }
  for (int i = 0; i < n_prompts; ++i) {
    if (prompt_lens[i] < 1) return fail(RL_ERR_INVALID_ARG, "prompt %d is empty", i);
    if (prompt_lens[i] > T.max_ctx() - 1) return fail(RL_ERR_CTX_OVERFLOW, "prompt %d has %d tokens, max_ctx is %d", i, prompt_lens[i], T.max_ctx());
    need += SeqTable::blocks_for(prompt_lens[i]) + (int64_t)(group - 1) * ((prompt_lens[i] % SeqTable::kBlock) ? 1 : 0);
    total += prompt_lens[i];
  }
  for (int64_t i = 0; i < total; ++i)
    if (prompt_tokens[i] < 0 || prompt_tokens[i] >= m->geo.vocab) return fail(RL_ERR_INVALID_ARG, "token %d at %lld outside the vocabulary", prompt_tokens[i], (long long)i);
  if (need > T.free_pages()) return fail(RL_ERR_KV_FULL, "need %lld pages, %lld free", (long long)need, (long long)T.free_pages());

  // Everything below changes sequence state; if a HIP call fails half way, the ids this call activated are released
  // again (their pages return to the pool) before the error is reported.
  auto run = [&]() -> rl_status {
  int32_t* bt = m->wsp<int32_t>(m->lay.block_table);
  for (int i = 0; i < n_prompts; ++i) {
    const int32_t s = seq_ids[i * group];
    T.activate(s);
    T.reserve(s, prompt_lens[i], nullptr);
    // pageable source: the runtime stages it before returning, so the vector may change afterwards
    HIP_TRY(hipMemcpyAsync(bt + (size_t)s * m->geo.max_blocks, T.pages(s).data(), T.pages(s).size() * 4, hipMemcpyHostToDevice, st));
  }

  float* x = m->wsp<float>(m->lay.x);
  float* x_last = m->wsp<float>(m->lay.x_last);
  // rows in (prompt, position) order, cut into chunks of R
  int pi = 0, pos = 0;
  int64_t done = 0, tok_off = 0;
  std::vector<int64_t> tok_base(n_prompts);
  for (int i = 0; i < n_prompts; ++i) { tok_base[i] = tok_off; tok_off += prompt_lens[i]; }
  while (done < total) {
    const int M = (int)std::min<int64_t>(R, total - done);
    int slot;
    rl_status rs = ring_acquire(m, &slot);
    if (rs != RL_OK) return rs;
    char* hs = m->host_ring + (size_t)slot * m->lay.slot_bytes;
    char* ds = m->ws + m->lay.ring + (size_t)slot * m->lay.slot_bytes;
    RowMeta* hr = (RowMeta*)hs;
    int32_t* ht = (int32_t*)(hs + m->lay.slot_tok);
    int max_ctx = 0;
    struct Last { int row, prompt; };
    std::vector<Last> lasts;
    for (int r = 0; r < M; ++r) {
      hr[r].seq = seq_ids[pi * group];
      hr[r].pos = pos;
      hr[r].page = T.pages(hr[r].seq)[pos >> 4];
      hr[r].pad = 0;
      ht[r] = prompt_tokens[tok_base[pi] + pos];
      if (pos + 1 > max_ctx) max_ctx = pos + 1;
      if (pos + 1 == prompt_lens[pi]) { lasts.push_back({r, pi}); ++pi; pos = 0; }
      else ++pos;
    }
    SharedAttn sa;
    { Timer t(m, st, K_META);
      HIP_TRY(hipMemcpyAsync(ds, hs, (size_t)M * sizeof(RowMeta), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(ds + m->lay.slot_tok, ht, (size_t)M * 4, hipMemcpyHostToDevice, st));
      rs = upload_window_plan(m, st, hs, ds, M, hr, &sa);
      if (rs != RL_OK) return rs;
      HIP_TRY(hipEventRecord(m->ring_ev[slot], st));
      m->ring_used[slot] = true; }
    const RowMeta* rows = (const RowMeta*)ds;
    { Timer t(m, st, K_EMBED);
      launch_embed(st, m->geo.dtype, m->embed, (const int32_t*)(ds + m->lay.slot_tok), x, M, H, m->geo.vocab); }
    int pend = run_layers(m, st, M, rows, max_ctx, sa);
    // fold the pending partials into x, then keep the rows that end a prompt (one copy per group member)
    float* cap = m->capture ? m->capture + (size_t)m->geo.n_layers * m->cfg.max_rows * H : nullptr;
    { Timer t(m, st, K_NORM);
      launch_residual_norm(st, m->geo.dtype, x, m->wsp<float>(m->lay.part), pend, nullptr, nullptr, cap, M, H, m->geo.rms_eps); }
    for (const Last& l : lasts)
      for (int j = 0; j < group; ++j)
        HIP_TRY(hipMemcpyAsync(x_last + (size_t)(l.prompt * group + j) * H, x + (size_t)l.row * H, (size_t)H * 4, hipMemcpyDeviceToDevice, st));
    done += M;
  }

  // ---- the other members of each group: shared full pages, private copy of the partial page ---------------
  if (group > 1) {
    std::vector<Fork> forks;
    for (int i = 0; i < n_prompts; ++i)
      for (int j = 1; j < group; ++j) forks.push_back({seq_ids[i * group], seq_ids[i * group + j], prompt_lens[i]});
    rl_status rs = fork_seqs(m, st, forks);
    if (rs != RL_OK) return rs;
  }

  // logits at the last prompt position of every sequence; the sampled token sits at position prompt_len
  {
    int slot;
    rl_status rs = ring_acquire(m, &slot);
    if (rs != RL_OK) return rs;
    char* hs = m->host_ring + (size_t)slot * m->lay.slot_bytes;
    char* ds = m->ws + m->lay.ring + (size_t)slot * m->lay.slot_bytes;
    RowMeta* hr = (RowMeta*)hs;
    for (int i = 0; i < n_all; ++i) { hr[i].seq = seq_ids[i]; hr[i].pos = prompt_lens[i / group]; hr[i].page = 0; hr[i].pad = 0; }
    HIP_TRY(hipMemcpyAsync(ds, hs, (size_t)n_all * sizeof(RowMeta), hipMemcpyHostToDevice, st));
    HIP_TRY(hipEventRecord(m->ring_ev[slot], st));
    m->ring_used[slot] = true;
    float* keep = m->capture;
    m->capture = nullptr;  // slot n_layers was already written per chunk
    run_head(m, st, n_all, x_last, 0, (const RowMeta*)ds, 0, nullptr, sp, out_tokens, out_logprobs, nullptr);
    m->capture = keep;
  }
  HIP_TRY(hipGetLastError());
  for (int i = 0; i < n_all; ++i) T.set_len(seq_ids[i], prompt_lens[i / group]);
  return RL_OK;
  };
  const rl_status rs = run();
  if (rs != RL_OK)
    for (int i = 0; i < n_all; ++i)
      if (T.active(seq_ids[i])) T.release(seq_ids[i]);  // all were inactive on entry
  return rs;
}

rl_status rl_prefill(rl_model* m, void* stream, int32_t n, const int32_t* seq_ids, const int32_t* prompt_tokens,
                     const int32_t* prompt_lens, const rl_sampling* sp, int32_t* out_tokens, float* out_logprobs) {
  if (!m || !seq_ids || !prompt_tokens || !prompt_lens || !sp || !out_tokens || !out_logprobs)
    return fail(RL_ERR_INVALID_ARG, "NULL argument");
  return prefill_impl(m, (hipStream_t)stream, n, 1, seq_ids, prompt_tokens, prompt_lens, sp, out_tokens, out_logprobs);
}

rl_status rl_prefill_groups(rl_model* m, void* stream, int32_t n_prompts, int32_t group_size, const int32_t* seq_ids,
                            const int32_t* prompt_tokens, const int32_t* prompt_lens, const rl_sampling* sp,
                            int32_t* out_tokens, float* out_logprobs) {
  if (!m || !seq_ids || !prompt_tokens || !prompt_lens || !sp || !out_tokens || !out_logprobs)
    return fail(RL_ERR_INVALID_ARG, "NULL argument");
  return prefill_impl(m, (hipStream_t)stream, n_prompts, group_size, seq_ids, prompt_tokens, prompt_lens, sp, out_tokens,
                      out_logprobs);
}

rl_status rl_seq_fork(rl_model* m, void* stream, int32_t src_seq, int32_t n, const int32_t* new_seq_ids) {
  if (!m || !new_seq_ids) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  if (n < 1 || n > (int32_t)m->cfg.max_rows) return fail(RL_ERR_INVALID_ARG, "n %d outside [1, max_rows=%u]", n, m->cfg.max_rows);
  SeqTable& T = *m->table;
  if (!T.active(src_seq)) return fail(RL_ERR_BAD_SEQ, "sequence %d is not active", src_seq);
  std::vector<char> seen(T.max_seqs(), 0);
  for (int i = 0; i < n; ++i) {
    const int32_t s = new_seq_ids[i];
    if (!T.valid_id(s)) return fail(RL_ERR_BAD_SEQ, "sequence id %d out of range", s);
    if (T.active(s)) return fail(RL_ERR_BAD_SEQ, "sequence %d is already active", s);
    if (seen[s]) return fail(RL_ERR_INVALID_ARG, "sequence %d appears twice", s);
    seen[s] = 1;
  }
  const int32_t len = T.len(src_seq);
  const int64_t need = (len % SeqTable::kBlock) ? n : 0;
  if (need > T.free_pages()) return fail(RL_ERR_KV_FULL, "need %lld pages, %lld free", (long long)need, (long long)T.free_pages());
  std::vector<Fork> forks;
  for (int i = 0; i < n; ++i) forks.push_back({src_seq, new_seq_ids[i], len});
  rl_status rs = fork_seqs(m, (hipStream_t)stream, forks);
  if (rs == RL_OK && hipGetLastError() != hipSuccess) rs = fail(RL_ERR_DEVICE, "rl_seq_fork: kernel launch failed");
  if (rs != RL_OK) {  // release what was activated (all new ids were inactive on entry)
    for (int i = 0; i < n; ++i)
      if (T.active(new_seq_ids[i])) T.release(new_seq_ids[i]);
    return rs;
  }
  for (int i = 0; i < n; ++i) T.set_len(new_seq_ids[i], len);
  return RL_OK;
}

rl_status rl_score(rl_model* m, void* stream, int32_t n, const int32_t* seq_ids, const int32_t* tokens,
                   const int32_t* lens, float temperature, float* out_logprobs) {
  if (!m || !seq_ids || !tokens || !lens || !out_logprobs) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  if (m->geo.vocab == 0) return fail(RL_ERR_UNSUPPORTED, "model has no vocabulary");
  if (n < 1 || n > T_MAX_SCORE) return fail(RL_ERR_INVALID_ARG, "n_seqs %d outside [1, %d]", n, T_MAX_SCORE);
  hipStream_t st = (hipStream_t)stream;
  SeqTable& T = *m->table;
  const int R = (int)m->cfg.max_rows, H = m->geo.hidden;
  std::vector<char> seen(T.max_seqs(), 0);
  int64_t need = 0, total = 0;
  for (int i = 0; i < n; ++i) {
    const int32_t s = seq_ids[i];
    if (!T.valid_id(s)) return fail(RL_ERR_BAD_SEQ, "sequence id %d out of range", s);
    if (T.active(s)) return fail(RL_ERR_BAD_SEQ, "sequence %d is already active", s);
    if (seen[s]) return fail(RL_ERR_INVALID_ARG, "sequence %d appears twice", s);
    seen[s] = 1;
    if (lens[i] < 2) return fail(RL_ERR_INVALID_ARG, "sequence %d has fewer than 2 tokens", i);
    if (lens[i] > T.max_ctx()) return fail(RL_ERR_CTX_OVERFLOW, "sequence %d has %d tokens, max_ctx is %d", i, lens[i], T.max_ctx());
    need += SeqTable::blocks_for(lens[i]);
    total += lens[i];
  }
  for (int64_t i = 0; i < total; ++i)
    if (tokens[i] < 0 || tokens[i] >= m->geo.vocab) return fail(RL_ERR_INVALID_ARG, "token %d at %lld outside the vocabulary", tokens[i], (long long)i);
  if (need > T.free_pages()) return fail(RL_ERR_KV_FULL, "need %lld pages, %lld free", (long long)need, (long long)T.free_pages());

  int32_t* bt = m->wsp<int32_t>(m->lay.block_table);
  rl_status result = RL_OK;
  for (int i = 0; i < n; ++i) {
    const int32_t s = seq_ids[i];
    T.activate(s);
    T.reserve(s, lens[i], nullptr);
    const hipError_t e = hipMemcpyAsync(bt + (size_t)s * m->geo.max_blocks, T.pages(s).data(), T.pages(s).size() * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) {  // give back what was taken so far: the ids were only scratch
      for (int k = 0; k <= i; ++k) T.release(seq_ids[k]);
      return fail(RL_ERR_DEVICE, "rl_score: block table upload: %s", hipGetErrorString(e));
    }
  }
  float* x = m->wsp<float>(m->lay.x);
  int32_t* tmp_tok = m->wsp<int32_t>(m->lay.tmp_tok);
  float* tmp_lp = m->wsp<float>(m->lay.tmp_lp);
  rl_sampling sp{temperature, 0u, 0ull, 0.f, 0u};
  int si = 0, pos = 0;
  int64_t done = 0, tok_off = 0, out_off = 0;
  std::vector<int64_t> tok_base(n), out_base(n);
  for (int i = 0; i < n; ++i) { tok_base[i] = tok_off; tok_off += lens[i]; out_base[i] = out_off; out_off += lens[i] - 1; }
  while (done < total && result == RL_OK) {
    const int M = (int)std::min<int64_t>(R, total - done);
    int slot;
    result = ring_acquire(m, &slot);
    if (result != RL_OK) break;
    char* hs = m->host_ring + (size_t)slot * m->lay.slot_bytes;
    char* ds = m->ws + m->lay.ring + (size_t)slot * m->lay.slot_bytes;
    RowMeta* hr = (RowMeta*)hs;
    int32_t* ht = (int32_t*)(hs + m->lay.slot_tok);
    int32_t* hf = (int32_t*)(hs + m->lay.slot_upd);  // [0,R): token to score, [R,2R): output index or -1
    int max_ctx = 0;
    for (int r = 0; r < M; ++r) {
      hr[r].seq = seq_ids[si];
      hr[r].pos = pos;
      hr[r].page = T.pages(hr[r].seq)[pos >> 4];
      hr[r].pad = 0;
      ht[r] = tokens[tok_base[si] + pos];
      if (pos + 1 > max_ctx) max_ctx = pos + 1;
      if (pos + 1 == lens[si]) { hf[r] = 0; hf[R + r] = -1; ++si; pos = 0; }
      else { hf[r] = tokens[tok_base[si] + pos + 1]; hf[R + r] = (int32_t)(out_base[si] + pos); ++pos; }
    }
    SharedAttn sa;
    { Timer t(m, st, K_META);
      hipError_t e = hipMemcpyAsync(ds, hs, (size_t)M * sizeof(RowMeta), hipMemcpyHostToDevice, st);
      if (e == hipSuccess) e = hipMemcpyAsync(ds + m->lay.slot_tok, ht, (size_t)M * 4, hipMemcpyHostToDevice, st);
      if (e == hipSuccess) e = hipMemcpyAsync(ds + m->lay.slot_upd, hf, (size_t)2 * R * 4, hipMemcpyHostToDevice, st);
      if (e != hipSuccess) { result = fail(RL_ERR_DEVICE, "rl_score: metadata upload: %s", hipGetErrorString(e)); break; }
      if (upload_window_plan(m, st, hs, ds, M, hr, &sa) != RL_OK) { result = RL_ERR_DEVICE; break; }
      e = hipEventRecord(m->ring_ev[slot], st);
      if (e != hipSuccess) { result = fail(RL_ERR_DEVICE, "rl_score: hipEventRecord: %s", hipGetErrorString(e)); break; }
      m->ring_used[slot] = true; }
    const RowMeta* rows = (const RowMeta*)ds;
    const int32_t* forced = (const int32_t*)(ds + m->lay.slot_upd);
    { Timer t(m, st, K_EMBED);
      launch_embed(st, m->geo.dtype, m->embed, (const int32_t*)(ds + m->lay.slot_tok), x, M, H, m->geo.vocab); }
    int pend = run_layers(m, st, M, rows, max_ctx, sa);
    run_head(m, st, M, x, pend, rows, 1, forced, &sp, tmp_tok, tmp_lp, nullptr, true);
    launch_scatter_f32(st, tmp_lp, forced + R, out_logprobs, M);
    done += M;
  }
  if (result == RL_OK && hipGetLastError() != hipSuccess) result = fail(RL_ERR_DEVICE, "kernel launch failed");
  // the sequences were only scratch: later work on this stream is ordered after the kernels above
  for (int i = 0; i < n; ++i) T.release(seq_ids[i]);
  return result;
}

// Append n_tokens positions of given K/V to the active sequence seq_id (length `len` >= 0): pages, block table,
// scatter kernels.  The caller has validated ids, sizes and free pages.
static rl_status append_kv(rl_model* m, hipStream_t st, int32_t seq_id, int32_t n_tokens, const void* const* k_layers,
                           const void* const* v_layers) {
  SeqTable& T = *m->table;
  const int32_t len = T.len(seq_id);
  const size_t have = T.pages(seq_id).size();
  T.reserve(seq_id, len + n_tokens, nullptr);
  int32_t* bt_row = m->wsp<int32_t>(m->lay.block_table) + (size_t)seq_id * m->geo.max_blocks;
  if (n_tokens > 0) {
    const size_t now = T.pages(seq_id).size();
    // pageable source: the runtime stages it before returning, so the vector may change afterwards
    if (now > have)
      HIP_TRY(hipMemcpyAsync(bt_row + have, T.pages(seq_id).data() + have, (now - have) * 4, hipMemcpyHostToDevice, st));
    for (int l = 0; l < m->geo.n_layers; ++l)
      launch_kv_import(st, m->geo, k_layers[l], v_layers[l], len, n_tokens, bt_row, m->k_pool(l), m->v_pool(l));
  }
  HIP_TRY(hipGetLastError());
  T.set_len(seq_id, len + n_tokens);
  return RL_OK;
}

rl_status rl_seq_import_kv(rl_model* m, void* stream, int32_t seq_id, int32_t n_tokens, const void* const* k_layers,
                           const void* const* v_layers) {
  if (!m || !k_layers || !v_layers) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  SeqTable& T = *m->table;
  if (!T.valid_id(seq_id)) return fail(RL_ERR_BAD_SEQ, "sequence id %d out of range", seq_id);
  if (T.active(seq_id)) return fail(RL_ERR_BAD_SEQ, "sequence %d is already active", seq_id);
  if (n_tokens < 0 || n_tokens > T.max_ctx() - 1) return fail(RL_ERR_CTX_OVERFLOW, "n_tokens %d outside [0, max_ctx)", n_tokens);
  for (int l = 0; l < m->geo.n_layers; ++l)
    if (n_tokens > 0 && (!k_layers[l] || !v_layers[l])) return fail(RL_ERR_INVALID_ARG, "layer %d KV pointer is NULL", l);
  if (SeqTable::blocks_for(n_tokens) > T.free_pages()) return fail(RL_ERR_KV_FULL, "need %d pages, %lld free", SeqTable::blocks_for(n_tokens), (long long)T.free_pages());
  T.activate(seq_id);
  const rl_status rs = append_kv(m, (hipStream_t)stream, seq_id, n_tokens, k_layers, v_layers);
  if (rs != RL_OK) T.release(seq_id);
  return rs;
}

rl_status rl_seq_append_kv(rl_model* m, void* stream, int32_t seq_id, int32_t n_tokens, const void* const* k_layers,
                           const void* const* v_layers) {
  if (!m || !k_layers || !v_layers) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  SeqTable& T = *m->table;
  if (!T.active(seq_id)) return fail(RL_ERR_BAD_SEQ, "sequence %d is not active", seq_id);
  if (n_tokens < 1) return fail(RL_ERR_INVALID_ARG, "n_tokens %d < 1", n_tokens);
  if ((int64_t)T.len(seq_id) + n_tokens > T.max_ctx() - 1)
    return fail(RL_ERR_CTX_OVERFLOW, "sequence %d would hold %lld tokens, max_ctx is %d", seq_id, (long long)T.len(seq_id) + n_tokens, T.max_ctx());
  for (int l = 0; l < m->geo.n_layers; ++l)
    if (!k_layers[l] || !v_layers[l]) return fail(RL_ERR_INVALID_ARG, "layer %d KV pointer is NULL", l);
  const int missing = T.pages_missing(seq_id, T.len(seq_id) + n_tokens);
  if (missing > T.free_pages()) return fail(RL_ERR_KV_FULL, "need %d pages, %lld free", missing, (long long)T.free_pages());
  return append_kv(m, (hipStream_t)stream, seq_id, n_tokens, k_layers, v_layers);
}

rl_status rl_sample_logits(rl_model* m, void* stream, int32_t n, const float* logits, const int32_t* seq_ids,
                           const int32_t* positions, const int32_t* forced, const rl_sampling* sp, int32_t* out_tokens,
                           float* out_logprobs) {
  if (!m || !logits || !seq_ids || !positions || !sp || !out_tokens || !out_logprobs) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  if (m->geo.vocab == 0) return fail(RL_ERR_UNSUPPORTED, "model has no vocabulary");
  if (n < 1 || n > (int32_t)m->cfg.max_rows) return fail(RL_ERR_INVALID_ARG, "n %d outside [1, max_rows]", n);
  hipStream_t st = (hipStream_t)stream;
  int slot;
  rl_status rs = ring_acquire(m, &slot);
  if (rs != RL_OK) return rs;
  char* hs = m->host_ring + (size_t)slot * m->lay.slot_bytes;
  char* ds = m->ws + m->lay.ring + (size_t)slot * m->lay.slot_bytes;
  RowMeta* hr = (RowMeta*)hs;
  for (int i = 0; i < n; ++i) { hr[i].seq = seq_ids[i]; hr[i].pos = positions[i]; hr[i].page = 0; hr[i].pad = 0; }
  HIP_TRY(hipMemcpyAsync(ds, hs, (size_t)n * sizeof(RowMeta), hipMemcpyHostToDevice, st));
  HIP_TRY(hipEventRecord(m->ring_ev[slot], st));
  m->ring_used[slot] = true;
  launch_sample(st, logits, n, m->geo.vocab, (const RowMeta*)ds, 0, forced, sp->temperature, sp->seed,
                m->wsp<float>(m->lay.samp_part), m->wsp<float>(m->lay.forced_z), out_tokens, out_logprobs,
                sp->top_k > (uint32_t)m->geo.vocab ? 0 : (int)sp->top_k, sp->top_p, m->wsp<void>(m->lay.cuts));
  HIP_TRY(hipGetLastError());
  return RL_OK;
}

rl_status rl_pack_weight(void* stream, uint32_t dtype, uint32_t kind, const void* src, void* dst, int64_t rows, int64_t cols) {
  if (!src || !dst || rows < 1 || cols < 1) return fail(RL_ERR_INVALID_ARG, "bad arguments");
  if (kind != RL_W_SPLIT_K && kind != RL_W_WHOLE_K) return fail(RL_ERR_INVALID_ARG, "unknown weight kind %u", kind);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == RL_F32) {
    HIP_TRY(hipMemcpyAsync(dst, src, (size_t)rows * cols * 4, hipMemcpyDeviceToDevice, st));
    return RL_OK;
  }
  if (dtype != RL_BF16) return fail(RL_ERR_INVALID_ARG, "unknown dtype");
  if (rows % 64 || cols % 256 || rows > 0x7fffffff || cols > 0x7fffffff) return fail(RL_ERR_UNSUPPORTED, "bf16 packing needs rows %% 64 == 0 and cols %% 256 == 0");
  launch_pack_weight_bf16(st, src, dst, (int)rows, (int)cols, gemm_bf16_weight_segment((int)rows, (int)cols, kind == RL_W_SPLIT_K));
  HIP_TRY(hipGetLastError());
  return RL_OK;
}

rl_status rl_profile_enable(rl_model* m, int32_t on) {
  if (!m) return fail(RL_ERR_INVALID_ARG, "model is NULL");
  m->prof_on = on != 0;
  return RL_OK;
}

rl_status rl_profile_read(rl_model* m, int32_t n_max, const char** names_out, double* ms_out, int64_t* counts_out,
                          int32_t* n_out) {
  if (!m || !names_out || !ms_out || !counts_out || !n_out) return fail(RL_ERR_INVALID_ARG, "NULL argument");
  for (auto& p : m->pending) {
    HIP_TRY(hipEventSynchronize(p.b));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, p.a, p.b));
    m->prof_ms[p.kind] += ms;
    m->prof_n[p.kind] += 1;
    m->ev_pool.push_back(p.a);
    m->ev_pool.push_back(p.b);
  }
  m->pending.clear();
  int k = 0;
  for (int i = 0; i < K_COUNT && k < n_max; ++i) {
    names_out[k] = kKindNames[i];
    ms_out[k] = m->prof_ms[i];
    counts_out[k] = m->prof_n[i];
    m->prof_ms[i] = 0;
    m->prof_n[i] = 0;
    ++k;
  }
  *n_out = k;
  return RL_OK;
}

}  // extern "C"
