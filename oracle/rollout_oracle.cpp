// CPU oracle for rollout generation (TEST INFRASTRUCTURE ONLY).
//
// This file is the slow, plain definition of what the rollout hot path
// computes: ancestral sampling of responses o ~ pi_theta_old(. | q) from a
// decoder-only policy (rollout workflow of Section 2.3; the expectation
// subscript of J(theta) in the HRD objective; Appendix C), together with the
// per-token probability pi_theta_old(o_t | q, o_<t) that the ratio s_{i,j,t}
// of the HRD objective needs in its denominator.
//
// The paper names the policy (an 8B decoder, Section 3.1) but does not spell
// out its arithmetic; the decoder here is the standard pre-norm GQA decoder
// with rotary embeddings and a SwiGLU MLP, every reading listed in the design
// notes of the repository.
//
// Rules this file keeps:
//   * storage fp32, accumulation in double; no blocking, fusion or reordering;
//   * shares no code, header, table or constant generator with the GPU path;
//   * only tests, the smoke check and the CPU-baseline leg of the benchmark may
//     load it.  The product never routes through it.
//
// Parity pins (tests/test_oracle_*.py): softmax rows sum to one, one-key
// attention returns V, RoPE keeps norms and is relative, RMSNorm scale
// invariance, SiLU identities, brute-force matvec, prefill-vs-decode
// consistency, zero-layer model = one matvec, the whole-model step against its own composition from the pinned parts, published known-answer vectors
// of the counter generator, log accuracy against libm, Gumbel-max frequencies
// against softmax on a tiny vocabulary; for the objective: ratio-one closed form, zero-sum advantages, clip
// cases worked by hand, class weights, both printed forms of the clipped term.  No function here is
// "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

// ---------------------------------------------------------------------------
// Dimensions of one decoder layer.
// ---------------------------------------------------------------------------
struct orc_dims {
  int32_t hidden;     // H
  int32_t n_q;        // query heads
  int32_t n_kv;       // key/value heads (n_q % n_kv == 0)
  int32_t head_dim;   // d (even)
  int32_t ffn;        // F
  int32_t qk_norm;    // 1: per-head RMSNorm on q and k before the rotation
  float rms_eps;
  float rope_base;
};

// Weights of one layer, row-major [out][in], fp32 (already rounded to the
// storage precision under test by the caller).
struct orc_layer {
  const float* attn_norm;  // [H]
  const float* wq;         // [n_q*d][H]
  const float* wk;         // [n_kv*d][H]
  const float* wv;         // [n_kv*d][H]
  const float* q_norm;     // [d]   (ignored when qk_norm == 0)
  const float* k_norm;     // [d]
  const float* wo;         // [H][n_q*d]
  const float* mlp_norm;   // [H]
  const float* w_gate;     // [F][H]
  const float* w_up;       // [F][H]
  const float* w_down;     // [H][F]
};

// Threads the row-parallel matvec uses (reported next to timings of this oracle).
int32_t orc_num_threads() {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// Round-to-nearest-even of an fp32 value to bfloat16, widened back to fp32.
// Used by tests to put weights / KV on the bf16 grid before both sides see them.
float orc_bf16_round(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return x;  // inf / nan unchanged
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  float y;
  std::memcpy(&y, &u, 4);
  return y;
}

void orc_bf16_round_array(float* x, int64_t n) {
  for (int64_t i = 0; i < n; ++i) x[i] = orc_bf16_round(x[i]);
}

// ---------------------------------------------------------------------------
// RMSNorm: out_i = x_i / sqrt(mean(x^2) + eps) * g_i
// ---------------------------------------------------------------------------
void orc_rmsnorm(const float* x, const float* g, int32_t n, float eps, float* out) {
  double ss = 0.0;
  for (int32_t i = 0; i < n; ++i) ss += (double)x[i] * (double)x[i];
  double inv = 1.0 / std::sqrt(ss / (double)n + (double)eps);
  for (int32_t i = 0; i < n; ++i) out[i] = (float)((double)x[i] * inv * (double)g[i]);
}

// ---------------------------------------------------------------------------
// y = W x, W row-major [n_out][n_in], double accumulation, no bias.
// ---------------------------------------------------------------------------
void orc_matvec(const float* W, const float* x, int32_t n_out, int32_t n_in, float* y) {
#pragma omp parallel for schedule(static)
  for (int32_t o = 0; o < n_out; ++o) {
    const float* w = W + (int64_t)o * n_in;
    double acc = 0.0;
    for (int32_t i = 0; i < n_in; ++i) acc += (double)w[i] * (double)x[i];
    y[o] = (float)acc;
  }
}

// ---------------------------------------------------------------------------
// Rotary embedding, rotate-half pairing (i, i + d/2), angle pos * base^(-2i/d),
// applied in place to one head vector of length d.
// ---------------------------------------------------------------------------
void orc_rope(float* u, int32_t d, int32_t pos, float base) {
  int32_t half = d / 2;
  for (int32_t i = 0; i < half; ++i) {
    double freq = std::pow((double)base, -2.0 * (double)i / (double)d);
    double ang = (double)pos * freq;
    double c = std::cos(ang), s = std::sin(ang);
    double a = u[i], b = u[i + half];
    u[i] = (float)(a * c - b * s);
    u[i + half] = (float)(b * c + a * s);
  }
}

double orc_silu(double z) { return z / (1.0 + std::exp(-z)); }

// ---------------------------------------------------------------------------
// Attention of ONE query position over n_keys cached positions.
//   q      [n_q][d]
//   kcache [n_keys][n_kv][d],  vcache likewise (contiguous, no paging)
//   out    [n_q][d]
//   probs  optional [n_q][n_keys] softmax weights (may be null)
// Query head h reads key/value head h / (n_q / n_kv).
// ---------------------------------------------------------------------------
void orc_attention(const float* q, const float* kcache, const float* vcache, int32_t n_keys,
                   int32_t n_q, int32_t n_kv, int32_t d, float* out, double* probs) {
  int32_t group = n_q / n_kv;
  double scale = 1.0 / std::sqrt((double)d);
  std::vector<double> s(n_keys), acc(d);
  for (int32_t h = 0; h < n_q; ++h) {
    int32_t hk = h / group;
    const float* qh = q + (int64_t)h * d;
    double m = -INFINITY;
    for (int32_t j = 0; j < n_keys; ++j) {
      const float* kj = kcache + ((int64_t)j * n_kv + hk) * d;
      double dot = 0.0;
      for (int32_t i = 0; i < d; ++i) dot += (double)qh[i] * (double)kj[i];
      s[j] = dot * scale;
      if (s[j] > m) m = s[j];
    }
    double denom = 0.0;
    for (int32_t j = 0; j < n_keys; ++j) {
      s[j] = std::exp(s[j] - m);
      denom += s[j];
    }
    for (int32_t i = 0; i < d; ++i) acc[i] = 0.0;
    for (int32_t j = 0; j < n_keys; ++j) {
      const float* vj = vcache + ((int64_t)j * n_kv + hk) * d;
      double w = s[j] / denom;
      if (probs) probs[(int64_t)h * n_keys + j] = w;
      for (int32_t i = 0; i < d; ++i) acc[i] += w * (double)vj[i];
    }
    for (int32_t i = 0; i < d; ++i) out[(int64_t)h * d + i] = (float)acc[i];
  }
}

// ---------------------------------------------------------------------------
// One decoder layer for the token at position `pos` of one sequence.
//   x       [H]   residual stream, updated in place
//   kcache  [>=pos+1][n_kv][d]  this layer's keys of this sequence; row `pos`
//           is written here, rows < pos must already hold earlier positions
//   vcache  same for values
// Steps: pre-norm -> q,k,v -> optional per-head norm -> rotation of q and k ->
// append -> causal attention over 0..pos -> output projection + residual ->
// pre-norm -> SwiGLU MLP + residual.
// ---------------------------------------------------------------------------
void orc_layer_forward(const orc_dims* dm, const orc_layer* w, float* x, int32_t pos,
                       float* kcache, float* vcache) {
  const int32_t H = dm->hidden, nq = dm->n_q, nkv = dm->n_kv, d = dm->head_dim, F = dm->ffn;
  std::vector<float> h(H), q((size_t)nq * d), k((size_t)nkv * d), v((size_t)nkv * d);
  orc_rmsnorm(x, w->attn_norm, H, dm->rms_eps, h.data());
  orc_matvec(w->wq, h.data(), nq * d, H, q.data());
  orc_matvec(w->wk, h.data(), nkv * d, H, k.data());
  orc_matvec(w->wv, h.data(), nkv * d, H, v.data());
  if (dm->qk_norm) {
    for (int32_t a = 0; a < nq; ++a) orc_rmsnorm(&q[(size_t)a * d], w->q_norm, d, dm->rms_eps, &q[(size_t)a * d]);
    for (int32_t a = 0; a < nkv; ++a) orc_rmsnorm(&k[(size_t)a * d], w->k_norm, d, dm->rms_eps, &k[(size_t)a * d]);
  }
  for (int32_t a = 0; a < nq; ++a) orc_rope(&q[(size_t)a * d], d, pos, dm->rope_base);
  for (int32_t a = 0; a < nkv; ++a) orc_rope(&k[(size_t)a * d], d, pos, dm->rope_base);
  std::memcpy(kcache + (int64_t)pos * nkv * d, k.data(), sizeof(float) * (size_t)nkv * d);
  std::memcpy(vcache + (int64_t)pos * nkv * d, v.data(), sizeof(float) * (size_t)nkv * d);

  std::vector<float> o((size_t)nq * d), t(H);
  orc_attention(q.data(), kcache, vcache, pos + 1, nq, nkv, d, o.data(), nullptr);
  orc_matvec(w->wo, o.data(), H, nq * d, t.data());
  for (int32_t i = 0; i < H; ++i) x[i] += t[i];

  std::vector<float> h2(H), g(F), u(F), a(F);
  orc_rmsnorm(x, w->mlp_norm, H, dm->rms_eps, h2.data());
  orc_matvec(w->w_gate, h2.data(), F, H, g.data());
  orc_matvec(w->w_up, h2.data(), F, H, u.data());
  for (int32_t i = 0; i < F; ++i) a[i] = (float)(orc_silu((double)g[i]) * (double)u[i]);
  orc_matvec(w->w_down, a.data(), H, F, t.data());
  for (int32_t i = 0; i < H; ++i) x[i] += t[i];
}

// ---------------------------------------------------------------------------
// Counter-based generator Philox4x32 with 10 rounds, as published by Salmon,
// Moraes, Dror and Shaw (SC'11): two 32x32->64 multiplies per round, the
// Weyl key schedule, and the word permutation of the 4-word variant.
// ---------------------------------------------------------------------------
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    uint64_t p0 = (uint64_t)M0 * (uint64_t)c0;
    uint64_t p1 = (uint64_t)M1 * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The whole decoder for one token of one sequence: x = E[token]; the n_layers blocks in order, each appending its
// key and value at `pos` of its own contiguous cache (kcaches[l], vcaches[l]: [max_ctx][n_kv][head_dim]); logits =
// W_lm rmsnorm(x, g_final) over the untied output matrix.  hidden_out (may be null) receives the residual stream
// that leaves the last block.  This is the function a rollout iterates: feed a token, read the next-token logits.
void orc_model_forward_token(const orc_dims* dm, int32_t n_layers, const orc_layer* layers, const float* embed,
                             const float* lm_head, const float* final_norm, int32_t vocab, int32_t token, int32_t pos,
                             float* const* kcaches, float* const* vcaches, float* logits, float* hidden_out) {
  const int32_t H = dm->hidden;
  std::vector<float> x(embed + (int64_t)token * H, embed + (int64_t)(token + 1) * H), h(H);
  for (int32_t l = 0; l < n_layers; ++l) orc_layer_forward(dm, &layers[l], x.data(), pos, kcaches[l], vcaches[l]);
  if (hidden_out) std::memcpy(hidden_out, x.data(), sizeof(float) * (size_t)H);
  orc_rmsnorm(x.data(), final_norm, H, dm->rms_eps, h.data());
  orc_matvec(lm_head, h.data(), vocab, H, logits);
}


// Random word for vocabulary index i of the token generated at absolute
// position `pos` of sequence `seq`: counter (i >> 2, pos, seq, 0), key = the
// two halves of the seed, word i & 3 of the block.
uint32_t orc_token_bits(uint64_t seed, uint32_t seq, uint32_t pos, uint32_t i) {
  uint32_t ctr[4] = {i >> 2, pos, seq, 0u};
  uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  return out[i & 3u];
}

// ---------------------------------------------------------------------------
// Sampler arithmetic.  Everything from the random word to the perturbed score
// is specified operation by operation in fp32, so that any conforming
// implementation takes the same argmax decision bit for bit.
//
// flog(x), x a positive normal fp32: write x = m * 2^e with m in
// [sqrt(1/2), sqrt(2)) by integer arithmetic on the bit pattern, f = m - 1
// (exact), p = Horner of the degree-8 polynomial below with one fused
// multiply-add per step, r = p * f (one rounding),
// flog = fma((float)e, LN2, r).
// ---------------------------------------------------------------------------
#pragma STDC FP_CONTRACT OFF
float orc_flog(float x) {
  uint32_t bits;
  std::memcpy(&bits, &x, 4);
  uint32_t ix = bits - 0x3f3504f3u;
  int32_t e = (int32_t)ix >> 23;  // arithmetic shift
  uint32_t mb = (ix & 0x007fffffu) + 0x3f3504f3u;
  float m;
  std::memcpy(&m, &mb, 4);
  float f = m - 1.0f;
  float p = 0x1.6626eap-4f;
  p = fmaf(p, f, -0x1.26729ep-3f);
  p = fmaf(p, f, 0x1.322850p-3f);
  p = fmaf(p, f, -0x1.5329bep-3f);
  p = fmaf(p, f, 0x1.98b80ap-3f);
  p = fmaf(p, f, -0x1.0005a6p-2f);
  p = fmaf(p, f, 0x1.555790p-2f);
  p = fmaf(p, f, -0x1.fffff8p-2f);
  p = fmaf(p, f, 1.0f);
  volatile float r = p * f;  // volatile: one rounding, never contracted
  return fmaf((float)e, 0x1.62e430p-1f, r);
}

// Uniform in (0,1) from the top 23 bits: u = (2k+1) * 2^-24, exact in fp32.
float orc_uniform(uint32_t bits) {
  uint32_t k = bits >> 9;
  return (float)(2u * k + 1u) * 0x1.0p-24f;
}

// Standard Gumbel variate g = -log(-log(u)) with the project log above.
float orc_gumbel(uint32_t bits) {
  float u = orc_uniform(bits);
  float t = -orc_flog(u);
  return -orc_flog(t);
}

// ---------------------------------------------------------------------------
// Sample one token from softmax(z / T) by the Gumbel-max construction and
// report its log-probability under that distribution.
//   temperature == 0 : greedy, tok = argmax z (lowest index on ties), lp is the
//                      log-softmax at T = 1.
//   forced >= 0      : teacher forcing, tok = forced, lp = its log-probability.
// Score y_i = fma(z_i, invT, g_i) with invT = 1.0f / T rounded once in fp32;
// ties go to the lowest index.  The log-probability is computed in double.
// ---------------------------------------------------------------------------
void orc_sample(const float* z, int32_t vocab, float temperature, uint64_t seed, uint32_t seq,
                uint32_t pos, int32_t forced, int32_t* tok_out, double* lp_out) {
  float invT = (temperature > 0.0f) ? (1.0f / temperature) : 1.0f;
  int32_t best = 0;
  if (forced >= 0) {
    best = forced;
  } else if (temperature > 0.0f) {
    float best_y = -INFINITY;
    best = -1;
    for (int32_t i = 0; i < vocab; ++i) {
      float g = orc_gumbel(orc_token_bits(seed, seq, pos, (uint32_t)i));
      float y = fmaf(z[i], invT, g);
      if (best < 0 || y > best_y) { best_y = y; best = i; }
    }
  } else {
    float best_z = z[0];
    for (int32_t i = 1; i < vocab; ++i)
      if (z[i] > best_z) { best_z = z[i]; best = i; }
  }
  double M = -INFINITY;
  for (int32_t i = 0; i < vocab; ++i) {
    double s = (double)z[i] * (double)invT;
    if (s > M) M = s;
  }
  double sum = 0.0;
  for (int32_t i = 0; i < vocab; ++i) sum += std::exp((double)z[i] * (double)invT - M);
  *tok_out = best;
  *lp_out = (double)z[best] * (double)invT - (M + std::log(sum));
}

// Full log-softmax row (double), for the "probabilities sum to one" pin.
void orc_log_softmax(const float* z, int32_t vocab, float invT, double* out) {
  double M = -INFINITY;
  for (int32_t i = 0; i < vocab; ++i) {
    double s = (double)z[i] * (double)invT;
    if (s > M) M = s;
  }
  double sum = 0.0;
  for (int32_t i = 0; i < vocab; ++i) sum += std::exp((double)z[i] * (double)invT - M);
  double lse = M + std::log(sum);
  for (int32_t i = 0; i < vocab; ++i) out[i] = (double)z[i] * (double)invT - lse;
}

// Draw `n_draws` tokens from fixed logits at positions pos0, pos0+1, ... and
// count them; brute-force check of the sampler's distribution on tiny vocabs.
void orc_sample_histogram(const float* z, int32_t vocab, float temperature, uint64_t seed,
                          uint32_t seq, uint32_t pos0, int64_t n_draws, int64_t* counts) {
  for (int32_t i = 0; i < vocab; ++i) counts[i] = 0;
  for (int64_t t = 0; t < n_draws; ++t) {
    int32_t tok;
    double lp;
    orc_sample(z, vocab, temperature, seed, seq, pos0 + (uint32_t)t, -1, &tok, &lp);
    counts[tok] += 1;
  }
}

// ---------------------------------------------------------------------------
// Truncated sampling (top-k, top-p): the sampling settings Appendix D states for the data-generating models
// (temperature 0.6 / top-p 0.95, 0.7 / 0.8).  The paper gives no definition; this is the usual one, made exactly
// reproducible by integer probability masses.
//
//   order     tokens by descending logit, equal logits by ascending index; "descending" is the total order of the
//             bit patterns (orc_order_key), so -0 comes after +0.
//   mass      W_i = orc_fexp_weight(fma(z_i, invT, -(z_max * invT))): a project-defined fp32 exp scaled to 2^32 and
//             truncated to an integer, so that sums are exact and independent of their order.
//   top-k     keep the first K = min(k, V) tokens of the order (k = 0: all).
//   top-p     P = trunc(p * 2^32), S = mass of those K tokens, T = max(1, floor(P * S / 2^32)); keep the shortest
//             prefix of the order whose mass reaches T (p <= 0 or p >= 1: no top-p cut).
//   draw      Gumbel-max over the kept tokens with the same per-token noise as orc_sample; the log-probability is
//             that of the renormalised distribution over the kept tokens (double here).
//   T = 0     greedy: the cuts are ignored (the argmax is always kept), lp as in orc_sample.
//   forced    lp of the forced token under the truncated distribution, -inf if it was cut.
// ---------------------------------------------------------------------------
uint32_t orc_order_key(float z) {  // ascending key = ascending value
  uint32_t b;
  std::memcpy(&b, &z, 4);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

uint64_t orc_fexp_weight(float x) {
  if (!(x > -22.0f)) return 0;  // below 2^-31.7 (and -inf)
  const float t = x * 0x1.715476p+0f;  // log2(e)
  const float n = std::nearbyintf(t);  // ties to even
  const float f = fmaf(x, 0x1.715476p+0f, -n);
  float p = 0x1.430912p-13f;           // 2^f = sum (f ln2)^k / k!, k = 6 .. 0
  p = fmaf(p, f, 0x1.5d87fep-10f);
  p = fmaf(p, f, 0x1.3b2ab6p-7f);
  p = fmaf(p, f, 0x1.c6b08ep-5f);
  p = fmaf(p, f, 0x1.ebfbe0p-3f);
  p = fmaf(p, f, 0x1.62e430p-1f);
  p = fmaf(p, f, 1.0f);
  return (uint64_t)std::ldexp(p, (int)n + 32);  // power-of-two scaling is exact; conversion truncates
}

// Number of tokens kept; keep[i] (optional) is set to 1 for kept tokens.
int32_t orc_truncation(const float* z, int32_t vocab, float invT, int32_t top_k, float top_p, uint8_t* keep) {
  std::vector<int32_t> order(vocab);
  for (int32_t i = 0; i < vocab; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(),
                   [&](int32_t a, int32_t b) { return orc_order_key(z[a]) > orc_order_key(z[b]); });
  const float s_max = z[order[0]] * invT;
  const int32_t K = (top_k > 0 && top_k < vocab) ? top_k : vocab;
  int32_t n = K;
  if (top_p > 0.0f && top_p < 1.0f) {
    unsigned __int128 S = 0;
    for (int32_t j = 0; j < K; ++j) S += orc_fexp_weight(fmaf(z[order[j]], invT, -s_max));
    const uint64_t P = (uint64_t)(top_p * 4294967296.0f);
    unsigned __int128 T = (S * P) >> 32;
    if (T < 1) T = 1;
    unsigned __int128 c = 0;
    for (n = 0; n < K;) {
      c += orc_fexp_weight(fmaf(z[order[n]], invT, -s_max));
      ++n;
      if (c >= T) break;
    }
  }
  if (keep) {
    std::memset(keep, 0, vocab);
    for (int32_t j = 0; j < n; ++j) keep[order[j]] = 1;
  }
  return n;
}

void orc_sample_truncated(const float* z, int32_t vocab, float temperature, int32_t top_k, float top_p, uint64_t seed,
                          uint32_t seq, uint32_t pos, int32_t forced, int32_t* tok_out, double* lp_out,
                          int32_t* kept_out) {
  if (!(temperature > 0.0f)) {
    orc_sample(z, vocab, temperature, seed, seq, pos, forced, tok_out, lp_out);
    if (kept_out) *kept_out = vocab;
    return;
  }
  const float invT = 1.0f / temperature;
  std::vector<uint8_t> keep(vocab);
  const int32_t n = orc_truncation(z, vocab, invT, top_k, top_p, keep.data());
  if (kept_out) *kept_out = n;
  int32_t best = forced;
  if (forced < 0) {
    float best_y = -INFINITY;
    for (int32_t i = 0; i < vocab; ++i) {
      if (!keep[i]) continue;
      const float y = fmaf(z[i], invT, orc_gumbel(orc_token_bits(seed, seq, pos, (uint32_t)i)));
      if (best < 0 || y > best_y) { best_y = y; best = i; }
    }
  }
  double M = -INFINITY;
  for (int32_t i = 0; i < vocab; ++i)
    if (keep[i]) M = std::fmax(M, (double)z[i] * (double)invT);
  double sum = 0.0;
  for (int32_t i = 0; i < vocab; ++i)
    if (keep[i]) sum += std::exp((double)z[i] * (double)invT - M);
  *tok_out = best;
  *lp_out = keep[best] ? (double)z[best] * (double)invT - (M + std::log(sum)) : -INFINITY;
}

// ---------------------------------------------------------------------------
// Policy objective with Hierarchical Reward Decomposition (Section 2.3) and its uniform-reward GRPO counterpart
// (Appendix C), forward value only, for a batch of n_prompts groups of G sampled outputs.
//
// Output (i,j) has |o| = off[k+1]-off[k] tokens (k = i*G+j); its first n_plan[k] tokens are the plan class T^plan,
// the rest the code class T^code.  Per token t: s_t = exp(lp_new[t] - lp_old[t]).
//   mode 0 (HRD):     A^c = r^c - mean_j r^c with r^plan = r_speedup, r^code = r_correct;
//                     J_i^c = 1/G sum_j 1/|o| sum_{t in T^c} min(A^c s_t, A^c clip(s_t, 1-eps, 1+eps));
//                     J = mean_i [alpha J_i^plan + J_i^code].
//   mode 1 (uniform): r = beta r_correct + (1-beta) r_speedup, A = r - mean_j r;
//                     L_i = 1/G sum_j 1/|o| sum_t A min(s_t, clip(s_t, 1-eps, 1+eps));  J = mean_i L_i
//                     (the advantage multiplies the min, as the appendix writes it).
// seq_term[k] (optional) receives the 1/|o| sum of output k before the 1/G and 1/n_prompts factors.
// ---------------------------------------------------------------------------
double orc_hrd_objective(int32_t n_prompts, int32_t G, const int32_t* off, const int32_t* n_plan,
                         const float* lp_new, const float* lp_old, const float* r_speedup, const float* r_correct,
                         double alpha, double eps, double beta, int32_t mode, double* seq_term) {
  double J = 0.0;
  for (int32_t i = 0; i < n_prompts; ++i) {
    double mean_s = 0.0, mean_c = 0.0, mean_u = 0.0;
    for (int32_t j = 0; j < G; ++j) {
      const int32_t k = i * G + j;
      mean_s += r_speedup[k];
      mean_c += r_correct[k];
      mean_u += beta * r_correct[k] + (1.0 - beta) * r_speedup[k];
    }
    mean_s /= G; mean_c /= G; mean_u /= G;
    double Ji = 0.0;
    for (int32_t j = 0; j < G; ++j) {
      const int32_t k = i * G + j;
      const int32_t len = off[k + 1] - off[k];
      double acc = 0.0;
      for (int32_t t = 0; t < len; ++t) {
        const double s = std::exp((double)lp_new[off[k] + t] - (double)lp_old[off[k] + t]);
        const double sc = s < 1.0 - eps ? 1.0 - eps : (s > 1.0 + eps ? 1.0 + eps : s);
        if (mode == 0) {
          const bool plan = t < n_plan[k];
          const double A = plan ? (double)r_speedup[k] - mean_s : (double)r_correct[k] - mean_c;
          const double term = std::fmin(A * s, A * sc);
          acc += plan ? alpha * term : term;
        } else {
          const double A = beta * r_correct[k] + (1.0 - beta) * r_speedup[k] - mean_u;
          acc += A * std::fmin(s, sc);
        }
      }
      const double term = len > 0 ? acc / (double)len : 0.0;
      if (seq_term) seq_term[k] = term;
      Ji += term;
    }
    J += Ji / G;
  }
  return J / n_prompts;
}

// Number of plan tokens of one output: everything up to and including the first occurrence of the delimiter
// token that closes the reasoning trace; an output without it is all plan.
int32_t orc_plan_length(const int32_t* tokens, int32_t len, int32_t delimiter) {
  for (int32_t t = 0; t < len; ++t)
    if (tokens[t] == delimiter) return t + 1;
  return len;
}

}  // extern "C"
