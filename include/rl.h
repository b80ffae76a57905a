/*
 * rl.h -- C boundary of the rollout-generation library for MI355X (gfx950).
 *
 * What the calls compute.  In each RL iteration the policy pi_theta_old
 * generates, for every prompt q_i, a group of G sampled responses o_{i,j}
 * (workflow paragraph of Section 2.3; subscript of the expectation in the
 * objective J(theta); Appendix C), each up to 16384 tokens after a prompt of
 * up to 2048 (Appendix D).  The optimiser later needs, per generated token,
 * pi_theta_old(o_{i,j,t} | q_i, o_{i,j,<t}) -- the denominator of the ratios
 * s^plan, s^code of the HRD objective.  This library is that generator: a
 * decoder-only policy (the 8B model named in Section 3.1) run autoregressively
 * over a paged KV cache, returning sampled token ids and their log-probabilities
 * under the sampling distribution.
 *
 * General conventions
 *   - Every function returns rl_status; on any error other than RL_ERR_DEVICE
 *     no sequence state has changed (after RL_ERR_DEVICE the model should be
 *     destroyed).  rl_last_error() gives a message for the last failing call
 *     on the calling thread.
 *   - "host" / "device" on a pointer says where the memory lives.  The library
 *     allocates no device memory: weights, KV pool, workspace and outputs are
 *     caller-owned device buffers that must outlive the model.
 *   - `stream` is a hipStream_t passed as void*.  Calls enqueue work on it and
 *     return; outputs are valid once the stream has been synchronised.  Host
 *     arrays passed to a call may be reused as soon as the call returns.
 *   - A sequence is named by a caller-chosen id in [0, max_seqs).  The id is
 *     also the stream id of the sampler's random numbers.  Group member j of
 *     prompt i is simply a distinct id (e.g. i*G + j).
 *   - Results for a sequence depend only on the weights, its own tokens, the
 *     seed and its id -- not on which other sequences share the batch nor on
 *     which physical pages it was given.
 *
 * Tensor layouts (row-major, "rows x cols"; element type = rl_model_config.dtype)
 *   embed, lm_head  vocab x hidden               (not tied)
 *   wqkv            (n_q+2*n_kv)*head_dim x hidden, rows ordered q heads, k heads, v heads
 *   wo              hidden x n_q*head_dim
 *   w_gate_up       2*ffn x hidden.  RL_F32: the ffn gate rows followed by the ffn up rows.  RL_BF16: gate and up rows
 *                   alternate in groups of 16 -- rows 32j .. 32j+15 are gate rows 16j .. 16j+15, rows 32j+16 .. 32j+31
 *                   the up rows of the same outputs -- so that one 32-row block of the streamed matrix holds both
 *                   factors of 16 outputs (then packed like the other matrices)
 *   w_down          hidden x ffn
 *   *_norm          RMSNorm gains: hidden (attn_norm, mlp_norm, final_norm), head_dim (q_norm, k_norm)
 *   kv_pool         opaque; n_pages = kv_pool_bytes / rl_kv_page_bytes(cfg); one page holds
 *                   kv_block tokens of K and V for all layers and kv heads
 * For RL_BF16 the five projection matrices (wqkv, wo, w_gate_up, w_down, lm_head) are handed over in the
 * library's tiled order, produced from the row-major form by rl_pack_weight(); embed and the gains stay
 * row-major.  For RL_F32 everything is row-major (rl_pack_weight is then a copy).
 *
 * The decoder: pre-norm blocks  x += Wo * attn(rope(norm_q(Wq h)), ...),  x += Wd (silu(Wg h') * Wu h'),
 * h = rmsnorm(x).  Rotary pairing is (i, i + head_dim/2) with angle pos * rope_base^(-2i/head_dim);
 * positions count from 0 at the first prompt token.  No biases.
 *
 * Sampler (bit-exact contract): for vocabulary index i of the token generated at absolute
 * position pos of sequence seq, a 32-bit word r is word (i & 3) of Philox4x32-10 with counter
 * (i >> 2, pos, seq, 0) and key (seed low, seed high); u = (2 (r >> 9) + 1) 2^-24;
 * g = -flog(-flog(u)) with the fp32 log fixed in the library's design notes;
 * y_i = fma(z_i, 1/T, g) in fp32; token = argmax_i y_i, lowest index on ties.  The reported
 * log-probability is log softmax(z / T)[token].  temperature == 0 means greedy (argmax z_i) and the
 * log-probability is then taken at T = 1.
 */
#ifndef RL_ROLLOUT_H_
#define RL_ROLLOUT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rl_model rl_model; /* opaque, owned by the library (host memory only) */

typedef enum {
  RL_OK = 0,
  RL_ERR_INVALID_ARG = -1,  /* null pointer, size out of range, duplicate id in one call */
  RL_ERR_KV_FULL = -2,      /* not enough free pages for the whole call; nothing was allocated */
  RL_ERR_BAD_SEQ = -3,      /* id out of range, not active (decode/free) or already active (prefill) */
  RL_ERR_CTX_OVERFLOW = -4, /* a sequence would exceed max_ctx */
  RL_ERR_DEVICE = -5,       /* a HIP call failed */
  RL_ERR_UNSUPPORTED = -6   /* dimensions the kernels of the chosen dtype do not cover */
} rl_status;

typedef enum { RL_F32 = 0, RL_BF16 = 1 } rl_dtype;

/*
 * How keys and values are cached.  RL_KV_SAME: in the model's dtype.  RL_KV_FP8 (bf16 models only): one byte per
 * element, e4m3 as the matrix cores of the device encode it (nearest even, no scales, magnitudes above 448 end at
 * 448): half the bytes per cached token, which is what a decode step at long contexts mostly reads.  A performance
 * option outside the default path: the cached values then carry 4 significant bits, and results agree with the
 * unrounded definition only to about that (a layer's output to a few per cent of its change to the residual
 * stream on unit-variance keys and values; the tests bound it by 1e-1 per layer).  rl_seq_import_kv still takes
 * bf16 arrays and rounds them.
 */
typedef enum { RL_KV_SAME = 0, RL_KV_FP8 = 2 } rl_kv_dtype;

typedef struct {
  uint32_t struct_size; /* sizeof(rl_model_config), checked */
  uint32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab; /* vocab % 4 == 0, < 2^22; 0: no head */
  float rms_eps, rope_base;
  uint32_t qk_norm;  /* 1: per-head RMSNorm of q and k before the rotation */
  uint32_t dtype;    /* rl_dtype of weights and KV; RL_BF16 needs head_dim 128 and 8B-like multiples */
  uint32_t kv_block; /* tokens per page; must be 16 */
  uint32_t max_seqs; /* ids are in [0, max_seqs) */
  uint32_t max_ctx;  /* longest prompt + response, multiple of kv_block; bf16: at most 65536 */
  uint32_t max_rows; /* most sequences per decode call (<= 1024); prefill and scoring push their tokens through
                        the layers in chunks of this many rows (workspace grows with it) */
  uint32_t kv_dtype; /* rl_kv_dtype */
  uint32_t reserved; /* 0 */
  uint64_t kv_pool_bytes;   /* size of rl_weights.kv_pool */
  uint64_t workspace_bytes; /* size of rl_weights.workspace, >= rl_query_workspace() */
} rl_model_config;

typedef struct {
  /* device pointers */
  const void* embed;
  const void* lm_head;
  const void* final_norm;
  /* host arrays of n_layers device pointers */
  const void* const* attn_norm;
  const void* const* wqkv;
  const void* const* q_norm; /* may be NULL when qk_norm == 0 */
  const void* const* k_norm;
  const void* const* wo;
  const void* const* mlp_norm;
  const void* const* w_gate_up;
  const void* const* w_down;
  /* device buffers the library manages the contents of */
  void* kv_pool;
  void* workspace;
} rl_weights;

/*
 * Sampling settings.  The RL rollouts of the paper draw from the untruncated policy (the ratios of Section 2.3
 * need pi_theta_old of the token that was drawn); top_k / top_p serve the truncated settings Appendix D lists
 * for data generation (temperature 0.6 / top-p 0.95, 0.7 / 0.8).  With a cut the tokens are ordered by descending
 * logit (ties: lower id first), top_k keeps the first top_k of them, top_p then the shortest prefix whose
 * probability mass (under temperature, renormalised over the top_k set) reaches top_p; the draw and the returned
 * log-probability refer to the renormalised distribution over the kept tokens (a forced token outside it has
 * log-probability -inf).  Masses are exact integers, so the kept set is reproducible bit for bit.  Greedy
 * (temperature 0) ignores both cuts.  rl_score never truncates.
 */
typedef struct {
  float temperature; /* 0 => greedy */
  uint32_t top_k;    /* 0 (or > vocab) => no top-k cut */
  uint64_t seed;
  float top_p;       /* outside (0, 1) => no top-p cut */
  uint32_t reserved; /* 0 */
} rl_sampling;

/* Bytes of one KV page (kv_block tokens, all layers, K and V) for this configuration; 0 on bad config. */
uint64_t rl_kv_page_bytes(const rl_model_config* cfg);

/* Smallest workspace_bytes rl_init_model accepts for this configuration (ignores cfg->workspace_bytes). */
rl_status rl_query_workspace(const rl_model_config* cfg, uint64_t* bytes_out);

/*
 * Build a model over caller-owned device buffers on the current HIP device.  Validates the
 * configuration, zero-fills the KV pool, builds the rotary table in the workspace (synchronous).
 * *out is set only on RL_OK.  Errors: INVALID_ARG, UNSUPPORTED, DEVICE.
 */
rl_status rl_init_model(const rl_model_config* cfg, const rl_weights* w, rl_model** out);

/* Releases host state.  Sequences and pages die with the model; device buffers stay the caller's. */
void rl_destroy_model(rl_model* m);

/*
 * Prefill: run the whole prompt of each new sequence through the decoder, fill its KV pages, and
 * sample the first response token from the logits at the last prompt position (its RNG position is
 * the prompt length).
 *   seq_ids        host  [n_seqs]       fresh ids (not active)
 *   prompt_tokens  host  [sum lens]     concatenated prompts, ids in [0, vocab)
 *   prompt_lens    host  [n_seqs]       each in [1, max_ctx - 1]
 *   out_tokens     device[n_seqs] int32 sampled first tokens
 *   out_logprobs   device[n_seqs] fp32  their log-probabilities
 * Errors: INVALID_ARG, BAD_SEQ, KV_FULL, CTX_OVERFLOW, DEVICE.
 */
rl_status rl_prefill(rl_model* m, void* stream, int32_t n_seqs, const int32_t* seq_ids,
                     const int32_t* prompt_tokens, const int32_t* prompt_lens, const rl_sampling* sp,
                     int32_t* out_tokens, float* out_logprobs);

/*
 * Prefill for grouped sampling: prompt i is followed by group_size sequences seq_ids[i*group_size + j], the G
 * samples that the RL loop draws from the same prompt (Section 2.3).  The prompt is run once; the members share
 * every KV page the prompt fills completely (those pages are never written again) and own a private copy of the
 * partial last page, so later calls treat them as ordinary independent sequences.  Each member's first token is
 * sampled from the same logits with its own random stream.  Results are identical to rl_prefill of the prompt
 * repeated group_size times.
 *   seq_ids        host  [n_prompts * group_size]   fresh ids;  n_prompts * group_size <= max_rows
 *   prompt_tokens  host  [sum lens], prompt_lens host [n_prompts]
 *   out_tokens / out_logprobs  device [n_prompts * group_size]
 * Errors as rl_prefill.
 */
rl_status rl_prefill_groups(rl_model* m, void* stream, int32_t n_prompts, int32_t group_size, const int32_t* seq_ids,
                            const int32_t* prompt_tokens, const int32_t* prompt_lens, const rl_sampling* sp,
                            int32_t* out_tokens, float* out_logprobs);

/*
 * Teacher-forced scoring: log pi_theta(tok[t+1] | tok[0..t]) under softmax(z / T) for t = 0 .. len-2 of every
 * sequence -- the numerator of the ratios s^plan, s^code of the HRD objective (Section 2.3) and, with the rollout
 * weights, a recomputation of their denominator.  The sequences are scratch: seq_ids must be fresh ids, their
 * pages are taken for the duration of the call and given back before it returns (work enqueued later on the
 * same stream is ordered after this call's kernels).
 *   seq_ids host [n_seqs];  tokens host [sum lens];  lens host [n_seqs], each in [2, max_ctx]
 *   temperature   T > 0; T = 0 is read as T = 1
 *   out_logprobs  device [sum (len_i - 1)] fp32, sequence after sequence
 * Errors: INVALID_ARG, BAD_SEQ, KV_FULL, CTX_OVERFLOW, DEVICE.
 */
rl_status rl_score(rl_model* m, void* stream, int32_t n_seqs, const int32_t* seq_ids, const int32_t* tokens,
                   const int32_t* lens, float temperature, float* out_logprobs);

/*
 * One decode step for n_seqs active sequences (1 <= n_seqs <= max_rows): feed in_tokens[b] at the
 * sequence's next position, append its K/V, and sample the following token.
 *   seq_ids       host  [n_seqs]
 *   in_tokens     device[n_seqs] int32 (normally the previous call's out_tokens), or NULL: every sequence is then
 *                 fed the token that its last rl_prefill / rl_prefill_groups / rl_decode_step call returned for it
 *                 (the library keeps one per sequence id), so a caller whose batch changes from step to step --
 *                 sequences retire, new groups join -- needs no gather of its own.  Only for sequences that have
 *                 sampled before (not for ones made by rl_seq_import_kv or rl_seq_fork and never stepped)
 *   forced_next   device[n_seqs] int32 or NULL; entries in [0, vocab) replace the sampled token (teacher
 *                 forcing) and the log-probability reported is that of the forced token; any other
 *                 value leaves that row sampled
 *   out_tokens    device[n_seqs] int32;  out_logprobs device[n_seqs] fp32
 *   debug_logits  device[n_seqs x vocab] fp32 or NULL: a copy of the logits z (otherwise the bf16
 *                 path never writes logits to memory: sampling runs in the output projection)
 * No host synchronisation happens inside.  Errors: INVALID_ARG, BAD_SEQ, KV_FULL, CTX_OVERFLOW, DEVICE.
 */
rl_status rl_decode_step(rl_model* m, void* stream, int32_t n_seqs, const int32_t* seq_ids,
                         const int32_t* in_tokens, const int32_t* forced_next, const rl_sampling* sp,
                         int32_t* out_tokens, float* out_logprobs, float* debug_logits);

/*
 * The decode step of a batch that stays the same from step to step, launched as a HIP graph: one graph launch per
 * step instead of several hundred kernel launches.  Every step is rl_decode_step(m, stream, n_seqs, seq_ids, NULL,
 * NULL, sp, out_tokens, out_logprobs, NULL) -- each sequence is fed the token it sampled last -- and gives the same
 * bits.  The step is captured on first use and again whenever a launch shape changes (the longest context crosses
 * a multiple of 1024 tokens, or the sets of samples that share prompt pages change); *captures_out (may be NULL)
 * counts the captures so far.  Every step reads the sequences' state afresh, so other calls (also rl_decode_step on
 * the same sequences) may come between two steps.  One graph per model at a time; destroy it before the model;
 * out_tokens / out_logprobs must stay valid until then.  rl_decode_graph_step captures on `stream` itself: it must
 * not be the null stream (RL_ERR_INVALID_ARG), and no other thread may enqueue on it during the call.
 * Errors of rl_decode_graph_step: as rl_decode_step.
 */
typedef struct rl_decode_graph rl_decode_graph;
rl_status rl_decode_graph_create(rl_model* m, int32_t n_seqs, const int32_t* seq_ids, const rl_sampling* sp,
                                 int32_t* out_tokens, float* out_logprobs, rl_decode_graph** out);
rl_status rl_decode_graph_step(rl_decode_graph* g, void* stream, int64_t* captures_out);
void rl_decode_graph_destroy(rl_decode_graph* g);

/* Retire sequences and return their pages to the pool.  Errors: INVALID_ARG, BAD_SEQ. */
rl_status rl_free_seqs(rl_model* m, int32_t n_seqs, const int32_t* seq_ids);

/* ---- helpers ------------------------------------------------------------------------------- */

/* Message of the last failing call on this thread (never NULL). */
const char* rl_last_error(void);

rl_status rl_kv_stats(const rl_model* m, uint64_t* free_pages, uint64_t* total_pages);

/* Tokens currently cached for a sequence; BAD_SEQ if not active. */
rl_status rl_seq_len(const rl_model* m, int32_t seq_id, int32_t* len_out);

/*
 * Sampler alone, on logits the caller supplies (used to check the bit-exact sampling contract).
 *   logits  device[n x vocab] fp32;  seq_ids, positions  host[n];  forced device[n] or NULL.
 */
rl_status rl_sample_logits(rl_model* m, void* stream, int32_t n, const float* logits,
                           const int32_t* seq_ids, const int32_t* positions, const int32_t* forced,
                           const rl_sampling* sp, int32_t* out_tokens, float* out_logprobs);

/*
 * rl_sample_logits for callers that cannot allocate device memory or hold a model: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same kernels and bits as rl_sample_logits without a cut,
 * but the scratch they need (row metadata, forced-token logits, per-tile partials) lives in a static device array
 * of 660 480 bytes inside the library (one copy per GPU, held until the process ends) instead of a model's
 * workspace, and the call allocates nothing.
 *   logits  device[n x vocab] fp32, rows 16-byte aligned (vocab % 4 == 0, 4 <= vocab < 2^22)
 *   seq_ids, positions  DEVICE[n] int32 (stream id and absolute position of the random numbers of each row)
 *   forced  device[n] or NULL;  out_tokens device[n] int32;  out_logprobs device[n] fp32
 * Limits: n <= 256 and n * ceil(vocab / 2048) <= 20480 (a 151 936-entry vocabulary at 256 rows needs 19 200);
 * beyond them RL_ERR_INVALID_ARG.  top_k / top_p cuts are not available here (RL_ERR_UNSUPPORTED): they need
 * 164 KB of histograms per row.  All calls on one GPU share that GPU's array: calls that overlap on one GPU
 * (different streams or threads) race; calls on one stream are ordered.  Nothing in the array has to be cleared
 * between calls.
 */
rl_status rl_sample_logits_static(void* stream, int32_t n, int32_t vocab, const float* logits,
                                  const int32_t* seq_ids, const int32_t* positions, const int32_t* forced,
                                  const rl_sampling* sp, int32_t* out_tokens, float* out_logprobs);

/*
 * Create a sequence whose first n_tokens positions of KV are given instead of computed.
 *   k_layers, v_layers  host arrays of n_layers device pointers, each [n_tokens][n_kv][head_dim] in
 *   the model dtype (keys as they are stored, i.e. after norm and rotation).
 * Errors as rl_prefill.
 */
rl_status rl_seq_import_kv(rl_model* m, void* stream, int32_t seq_id, int32_t n_tokens,
                           const void* const* k_layers, const void* const* v_layers);

/*
 * Append n_tokens (>= 1) positions of given KV to an active sequence, behind the tokens it already caches (its own
 * tokens, a prompt it shares with the other samples of its group, or imported ones); arrays as for
 * rl_seq_import_kv.  Measurement and test aid: it places sequences at a stated context length (e.g. the shared
 * 2048-token prompt of Appendix D plus several thousand private response tokens) without running that many decode
 * steps.  The sequence may hold at most max_ctx - 1 tokens afterwards.
 * Errors: INVALID_ARG, BAD_SEQ, KV_FULL, CTX_OVERFLOW (state untouched), DEVICE.
 */
rl_status rl_seq_append_kv(rl_model* m, void* stream, int32_t seq_id, int32_t n_tokens,
                           const void* const* k_layers, const void* const* v_layers);

/*
 * Decoder layers alone: like rl_decode_step but the residual stream entering layer 0 is given
 * (hidden_in, device [n_seqs x hidden] fp32) instead of looked up from a token, and the residual
 * stream leaving the last layer is returned (hidden_out, same shape) instead of being normalised,
 * projected and sampled.  K/V are appended and the sequences advance by one position.
 */
rl_status rl_decode_hidden(rl_model* m, void* stream, int32_t n_seqs, const int32_t* seq_ids,
                           const float* hidden_in, float* hidden_out);

/*
 * While `buf` (device, (n_layers+1) x max_rows x hidden fp32) is non-NULL, every decode call also
 * stores the residual stream entering each layer (slot l) and leaving the last one (slot n_layers),
 * row b at buf[(l*max_rows + b)*hidden].  NULL switches it off.
 */
rl_status rl_set_capture(rl_model* m, float* buf);

/*
 * Forward value of the policy objective (no model needed; all arrays on the device).
 *   mode 0  Hierarchical Reward Decomposition (Section 2.3): tokens of an output are split into the plan class (the
 *           reasoning trace, up to and including the delimiter that closes it) and the code class; advantages are
 *           group-mean-baselined per class, A^plan from r_speedup and A^code from r_correct;
 *           J = mean_i [ alpha J_i^plan + J_i^code ],
 *           J_i^c = 1/G sum_j 1/|o_ij| sum_{t in T^c} min(A^c s_t, A^c clip(s_t, 1-eps, 1+eps)),
 *           s_t = exp(lp_new[t] - lp_old[t]).
 *   mode 1  uniform-reward GRPO (Appendix C): r = beta r_correct + (1-beta) r_speedup, A = r - mean_j r,
 *           L_i = 1/G sum_j 1/|o_ij| sum_t A min(s_t, clip(s_t, 1-eps, 1+eps)).
 *   offsets    [n_prompts*G + 1] int32: output k (= i*G + j) owns tokens offsets[k] .. offsets[k+1]-1 of lp_new/lp_old
 *   n_plan     [n_prompts*G] int32 plan-token counts (a count below 0 or above the output's length is clamped to that
 *              range), or NULL: then tokens (response token ids, same indexing as lp_*) are scanned for
 *              delimiter_token (an output without it is all plan)
 *   r_speedup, r_correct  [n_prompts*G] fp32 rewards
 *   seq_terms  [n_prompts*G] fp32 out: the 1/|o| sum of each output (before the 1/G and 1/n_prompts factors)
 *   n_plan_out [n_prompts*G] int32 out or NULL: the plan lengths used
 *   out_value  [1] fp32 out: the objective
 * Sums run in a fixed order (reproducible bits).  Errors: INVALID_ARG, DEVICE.
 */
typedef struct {
  float alpha;    /* weight of the plan class, 0.1 in the paper's main runs */
  float eps_clip; /* clip range, 0.2 */
  float beta;     /* mode 1 only: share of the correctness reward */
  int32_t mode;   /* 0 = HRD, 1 = uniform */
} rl_objective_params;

rl_status rl_hrd_objective(void* stream, int32_t n_prompts, int32_t group_size, const int32_t* offsets,
                           const int32_t* n_plan, const int32_t* tokens, int32_t delimiter_token, const float* lp_new,
                           const float* lp_old, const float* r_speedup, const float* r_correct,
                           const rl_objective_params* p, float* seq_terms, int32_t* n_plan_out, float* out_value);

/*
 * Reorder a row-major [rows x cols] matrix (device) into the order the projection kernels stream
 * (device, same size, must not overlap src).  RL_BF16: 32-row x 64-column tiles, each stored so that a
 * wavefront reads it as four contiguous 1 KiB pieces in matrix-core operand order, the tiles of a 32-row block
 * ordered so that what the four wavefronts of a block read together is contiguous, and every weight stored as its
 * f16 image, the grid on which the matrix cores multiply (exact for 2^-14 <= |w| <= 65504; smaller magnitudes are cut
 * toward zero on the f16 subnormal grid, absolute error < 2^-24; same two bytes per weight); needs rows % 64 == 0 and
 * cols % 256 == 0.  That order depends on how the product is cut along the columns, hence `kind`:
 * RL_W_SPLIT_K for wqkv, wo and w_down, RL_W_WHOLE_K for w_gate_up and lm_head.  RL_F32: plain copy.  No model
 * is needed.
 */
typedef enum { RL_W_SPLIT_K = 0, RL_W_WHOLE_K = 1 } rl_weight_kind;
rl_status rl_pack_weight(void* stream, uint32_t dtype, uint32_t kind, const void* src, void* dst, int64_t rows,
                         int64_t cols);

/*
 * Continue one sequence as several (the G outputs sampled for one prompt, Section 2.3, from a state that is
 * already in the cache): each new_seq_ids[i] (host [n], inactive ids, n <= max_rows) becomes a sequence of the same
 * length as src_seq whose KV is that of src_seq.  Pages that src_seq has filled completely are shared (never
 * written again, returned to the pool with their last holder); a partial last page is copied, one new page per
 * new sequence.  Later decode steps of the new sequences and of src_seq are independent and give, bit for bit,
 * what sequences prefilled one by one give.  RL_ERR_BAD_SEQ, RL_ERR_KV_FULL, RL_ERR_INVALID_ARG leave the state
 * untouched.  The page copy is enqueued on `stream`.
 */
rl_status rl_seq_fork(rl_model* m, void* stream, int32_t src_seq, int32_t n, const int32_t* new_seq_ids);

/*
 * Test aid: permute the free-page list with a seeded shuffle, so that later allocations scatter over
 * the pool.  Results of every other call must not change.
 */
rl_status rl_debug_shuffle_free_pages(rl_model* m, uint64_t seed);

/*
 * Test aid: switch off (on = 0) or on again (the default) the decode-step treatment of the samples of one
 * prompt (Section 2.3): sequences made by rl_prefill_groups hold the prompt's full pages in common, and rows
 * of such sequences that stand at the same position have the attention over those pages computed once per set
 * of rows instead of once per row.  Results of every other call must not change by a single bit.
 */
rl_status rl_debug_share_attention(rl_model* m, int32_t on);
/* on = 2: as on = 1, and the sets are as large as the kernel allows (bf16 pages: two 16-column operands side by
 * side, i.e. up to 32 / (query heads per kv head) rows) in every call; on = 3: a single operand in every call.
 * By default the size of the call decides.  No bit of any result depends on the choice. */

/*
 * Test aid: switch off (on = 0) or on again (the default) the fused form of a bf16 decode step in which the
 * attention kernel itself forms the rotated queries and writes the new keys and values into their pages, instead
 * of a separate kernel before it.  Results of every other call must not change by a single bit.  No effect on
 * fp32 models and on calls that feed several positions of one sequence (prefill, scoring).
 */
rl_status rl_debug_attention_appends(rl_model* m, int32_t on);

/*
 * Test and tuning aid: how many 256-key segments one attention block takes of a context beyond 4096 keys (1..16).
 * Smaller blocks balance better at the end of a launch, larger ones amortise their prologue.  Results of every
 * other call must not change by a single bit.  Not to be changed while a decode graph exists.
 */
rl_status rl_debug_attention_split(rl_model* m, int32_t segs_per_block);

/*
 * Per-kernel timing.  While enabled, every kernel launch of decode/prefill calls is bracketed by
 * HIP events on the caller's stream.  rl_profile_read synchronises those events, returns per kernel
 * class the number of launches and their total milliseconds since the last read, and clears them.
 *   names_out  host[n_max] pointers to static strings;  ms_out host[n_max];  counts_out host[n_max]
 *   *n_out     number of classes written
 */
rl_status rl_profile_enable(rl_model* m, int32_t on);
/* Host microseconds that rl_decode_step spent since the last read (always collected): admission checks (ids, pages),
 * building and uploading the rows / page grants / shared-attention plan, enqueueing the kernels, and -- apart from
 * those -- waiting for a metadata slot that the device has not consumed yet (the device is then 62 calls behind the
 * host; calls of other entry points that take a slot add to this figure too); and the number of calls. */
rl_status rl_profile_host_read(rl_model* m, double* admit_us, double* meta_us, double* launch_us, double* wait_us,
                               int64_t* calls);
rl_status rl_profile_read(rl_model* m, int32_t n_max, const char** names_out, double* ms_out,
                          int64_t* counts_out, int32_t* n_out);

#ifdef __cplusplus
}
#endif
#endif /* RL_ROLLOUT_H_ */
