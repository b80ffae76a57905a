"""ctypes binding of the rollout library (argument marshalling only).

Every step of the path runs in the HIP kernels behind the C boundary declared in include/rl.h; PyTorch is
used here for device allocations and the current stream.  The binding fails loudly when the shared
library has not been built -- there is no fallback.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librl_rollout.so")

RL_OK = 0
RL_ERR_INVALID_ARG, RL_ERR_KV_FULL, RL_ERR_BAD_SEQ = -1, -2, -3
RL_ERR_CTX_OVERFLOW, RL_ERR_DEVICE, RL_ERR_UNSUPPORTED = -4, -5, -6
RL_F32, RL_BF16 = 0, 1
RL_KV_SAME, RL_KV_FP8 = 0, 2
RL_W_SPLIT_K, RL_W_WHOLE_K = 0, 1

EXPORTS = [
    "rl_kv_page_bytes", "rl_query_workspace", "rl_init_model", "rl_destroy_model", "rl_prefill", "rl_prefill_groups", "rl_score", "rl_hrd_objective",
    "rl_decode_step", "rl_decode_graph_create", "rl_decode_graph_step", "rl_decode_graph_destroy", "rl_free_seqs", "rl_last_error", "rl_kv_stats", "rl_seq_len", "rl_sample_logits", "rl_sample_logits_static",
    "rl_seq_import_kv", "rl_seq_append_kv", "rl_decode_hidden", "rl_set_capture", "rl_pack_weight",
    "rl_debug_shuffle_free_pages", "rl_debug_share_attention", "rl_debug_attention_appends", "rl_debug_attention_split", "rl_seq_fork", "rl_profile_enable", "rl_profile_read", "rl_profile_host_read",
]


class rl_model_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_layers", C.c_uint32), ("hidden", C.c_uint32),
                ("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("ffn", C.c_uint32), ("vocab", C.c_uint32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("qk_norm", C.c_uint32), ("dtype", C.c_uint32),
                ("kv_block", C.c_uint32), ("max_seqs", C.c_uint32), ("max_ctx", C.c_uint32),
                ("max_rows", C.c_uint32), ("kv_dtype", C.c_uint32), ("reserved", C.c_uint32),
                ("kv_pool_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64)]


_pp = C.POINTER(C.c_void_p)


class rl_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", _pp), ("wqkv", _pp), ("q_norm", _pp), ("k_norm", _pp), ("wo", _pp),
                ("mlp_norm", _pp), ("w_gate_up", _pp), ("w_down", _pp),
                ("kv_pool", C.c_void_p), ("workspace", C.c_void_p)]


class rl_sampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_k", C.c_uint32), ("seed", C.c_uint64), ("top_p", C.c_float),
                ("reserved", C.c_uint32)]


class rl_objective_params(C.Structure):
    _fields_ = [("alpha", C.c_float), ("eps_clip", C.c_float), ("beta", C.c_float), ("mode", C.c_int32)]


class RLError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"rl_status {status}: {message}")
        self.status = status


_lib = None
_i32p = C.POINTER(C.c_int32)


def lib():
    """Load librl_rollout.so; raises if it has not been built (python -m paper_2510_17891_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2510_17891_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.rl_last_error.restype = C.c_char_p
        L.rl_kv_page_bytes.restype = C.c_uint64
        L.rl_kv_page_bytes.argtypes = [C.POINTER(rl_model_config)]
        L.rl_query_workspace.argtypes = [C.POINTER(rl_model_config), C.POINTER(C.c_uint64)]
        L.rl_init_model.argtypes = [C.POINTER(rl_model_config), C.POINTER(rl_weights), C.POINTER(C.c_void_p)]
        L.rl_destroy_model.restype = None
        L.rl_destroy_model.argtypes = [C.c_void_p]
        L.rl_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _i32p, _i32p, _i32p,
                                 C.POINTER(rl_sampling), C.c_void_p, C.c_void_p]
        L.rl_prefill_groups.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, _i32p, _i32p, _i32p,
                                        C.POINTER(rl_sampling), C.c_void_p, C.c_void_p]
        L.rl_score.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _i32p, _i32p, _i32p, C.c_float, C.c_void_p]
        L.rl_hrd_objective.argtypes = [C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 3 + [C.c_int32] + \
            [C.c_void_p] * 4 + [C.POINTER(rl_objective_params)] + [C.c_void_p] * 3
        L.rl_decode_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _i32p, C.c_void_p, C.c_void_p,
                                     C.POINTER(rl_sampling), C.c_void_p, C.c_void_p, C.c_void_p]
        L.rl_decode_graph_create.argtypes = [C.c_void_p, C.c_int32, _i32p, C.POINTER(rl_sampling), C.c_void_p, C.c_void_p,
                                             C.POINTER(C.c_void_p)]
        L.rl_decode_graph_step.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int64)]
        L.rl_decode_graph_destroy.restype = None
        L.rl_decode_graph_destroy.argtypes = [C.c_void_p]
        L.rl_free_seqs.argtypes = [C.c_void_p, C.c_int32, _i32p]
        L.rl_kv_stats.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.rl_seq_len.argtypes = [C.c_void_p, C.c_int32, _i32p]
        L.rl_sample_logits.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, _i32p, _i32p,
                                       C.c_void_p, C.POINTER(rl_sampling), C.c_void_p, C.c_void_p]
        L.rl_sample_logits_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.POINTER(rl_sampling), C.c_void_p, C.c_void_p]
        L.rl_seq_import_kv.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, _pp, _pp]
        L.rl_seq_append_kv.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, _pp, _pp]
        L.rl_decode_hidden.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _i32p, C.c_void_p, C.c_void_p]
        L.rl_set_capture.argtypes = [C.c_void_p, C.c_void_p]
        L.rl_pack_weight.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64]
        L.rl_debug_shuffle_free_pages.argtypes = [C.c_void_p, C.c_uint64]
        L.rl_debug_share_attention.argtypes = [C.c_void_p, C.c_int32]
        L.rl_debug_attention_appends.argtypes = [C.c_void_p, C.c_int32]
        L.rl_debug_attention_split.argtypes = [C.c_void_p, C.c_int32]
        L.rl_seq_fork.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, _i32p]
        L.rl_profile_enable.argtypes = [C.c_void_p, C.c_int32]
        L.rl_profile_read.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                      C.POINTER(C.c_int64), _i32p]
        L.rl_profile_host_read.argtypes = [C.c_void_p] + [C.POINTER(C.c_double)] * 4 + [C.POINTER(C.c_int64)]
        _lib = L
    return _lib


def check(status):
    if status != RL_OK:
        raise RLError(status, lib().rl_last_error().decode())


def _i32(values):
    return (C.c_int32 * len(values))(*[int(v) for v in values])


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def make_config(shape, dtype, max_seqs, max_ctx, max_rows, kv_pool_bytes=0, workspace_bytes=0, kv_dtype=RL_KV_SAME):
    """rl_model_config from a shape dict (keys as in rollout_inputs.SHAPES)."""
    c = rl_model_config()
    c.struct_size = C.sizeof(rl_model_config)
    c.n_layers, c.hidden = shape["n_layers"], shape["hidden"]
    c.n_q_heads, c.n_kv_heads, c.head_dim = shape["n_q"], shape["n_kv"], shape["head_dim"]
    c.ffn, c.vocab = shape["ffn"], shape["vocab"]
    c.rms_eps, c.rope_base, c.qk_norm = shape["rms_eps"], shape["rope_base"], shape["qk_norm"]
    c.dtype = dtype
    c.kv_block = 16
    c.max_seqs, c.max_ctx, c.max_rows = max_seqs, max_ctx, max_rows
    c.kv_dtype, c.reserved = kv_dtype, 0
    c.kv_pool_bytes, c.workspace_bytes = kv_pool_bytes, workspace_bytes
    return c


def rl_pack_weight(w, kind):
    """Row-major device matrix -> the order the projection kernels stream (new tensor, same shape).
    kind: RL_W_SPLIT_K for wqkv, wo, w_down; RL_W_WHOLE_K for w_gate_up, lm_head."""
    assert w.is_cuda and w.is_contiguous() and w.dim() == 2
    dt = RL_BF16 if w.dtype == torch.bfloat16 else RL_F32
    out = torch.empty_like(w)
    check(lib().rl_pack_weight(_stream(), dt, kind, _ptr(w), _ptr(out), w.shape[0], w.shape[1]))
    return out


def rl_hrd_objective(n_prompts, group_size, offsets, lp_new, lp_old, r_speedup, r_correct, alpha=0.1, eps_clip=0.2,
                     beta=0.0, mode=0, n_plan=None, tokens=None, delimiter_token=-1):
    """Objective value (device scalar), per-output terms and plan lengths; all inputs are device tensors."""
    n = n_prompts * group_size
    dev = lp_new.device
    seq = torch.empty(n, dtype=torch.float32, device=dev)
    npl = torch.empty(n, dtype=torch.int32, device=dev)
    out = torch.empty(1, dtype=torch.float32, device=dev)
    p = rl_objective_params(alpha, eps_clip, beta, mode)
    st = lib().rl_hrd_objective(_stream(), n_prompts, group_size, _ptr(offsets), _ptr(n_plan), _ptr(tokens),
                                delimiter_token, _ptr(lp_new), _ptr(lp_old), _ptr(r_speedup), _ptr(r_correct),
                                C.byref(p), _ptr(seq), _ptr(npl), _ptr(out))
    check(st)
    return out, seq, npl


def rl_sample_logits_static(logits, seq_ids, positions, temperature, seed, forced=None, out_tokens=None,
                            out_logprobs=None, top_k=0, top_p=0.0):
    """The plain sampler without a model; seq_ids / positions are device int32 tensors.  The call itself allocates
    nothing when out_tokens / out_logprobs are given."""
    n, vocab = logits.shape
    out_t = out_tokens if out_tokens is not None else torch.empty(n, dtype=torch.int32, device=logits.device)
    out_lp = out_logprobs if out_logprobs is not None else torch.empty(n, dtype=torch.float32, device=logits.device)
    sp = rl_sampling(temperature, top_k, seed, top_p, 0)
    check(lib().rl_sample_logits_static(_stream(), n, vocab, _ptr(logits), _ptr(seq_ids), _ptr(positions), _ptr(forced),
                                        C.byref(sp), _ptr(out_t), _ptr(out_lp)))
    return out_t, out_lp


class Rollout:
    """Owns the device buffers of one model and forwards calls to the C boundary.

    `weights` are the logical tensors (dict: embed, lm_head, final_norm, layers[...] with wq, wk, wv, wo,
    w_gate, w_up, w_down and the gains), on the GPU, in the model dtype.  They are concatenated / packed into
    the layouts rl.h prescribes; the logical tensors are not kept.
    """

    def __init__(self, shape, weights, max_seqs, max_ctx, max_rows, kv_pages, device="cuda:0", consume_weights=False,
                 kv_slack_bytes=2 << 30, kv_fp8=False):
        """kv_pages: pages in the KV pool, or None for as many as the card holds once the packed weights and the
        workspace are placed (less kv_slack_bytes).  consume_weights: the entries of `weights` are removed as they are
        packed, so that a model of 16 GB does not exist twice on the card at any time.  kv_fp8: cache keys and values as
        fp8 (bf16 models only; a performance option, see rl.h)."""
        L = lib()
        self.shape = dict(shape)
        self.device = torch.device(device)
        self.tdtype = weights["final_norm"].dtype
        self.dtype = RL_BF16 if self.tdtype == torch.bfloat16 else RL_F32
        cfg = make_config(shape, self.dtype, max_seqs, max_ctx, max_rows, kv_dtype=RL_KV_FP8 if kv_fp8 else RL_KV_SAME)
        page = L.rl_kv_page_bytes(C.byref(cfg))
        if page == 0:
            raise RLError(RL_ERR_UNSUPPORTED, L.rl_last_error().decode())
        need = C.c_uint64()
        check(L.rl_query_workspace(C.byref(cfg), C.byref(need)))
        self._keep = []
        n_layers = shape["n_layers"]

        def arr(tensors):
            a = (C.c_void_p * n_layers)(*[t.data_ptr() for t in tensors])
            self._keep.append((a, tensors))
            return C.cast(a, _pp)

        def take(d, k):
            return d.pop(k) if consume_weights else d[k]

        def packed(d, keys, kind=RL_W_SPLIT_K):
            parts = [take(d, k) for k in keys]
            src = parts[0].contiguous() if len(parts) == 1 else torch.cat(parts, 0)
            del parts
            out = rl_pack_weight(src, kind)
            del src
            return out

        def packed_gate_up(d):
            g, u = take(d, "w_gate"), take(d, "w_up")
            if self.dtype == RL_BF16:   # rl.h: gate and up rows alternate in groups of 16
                F, H = g.shape
                src = torch.stack([g.view(F // 16, 16, H), u.view(F // 16, 16, H)], 1).reshape(2 * F, H)
            else:
                src = torch.cat([g, u], 0)
            del g, u
            out = rl_pack_weight(src, RL_W_WHOLE_K)
            del src
            return out

        lay = weights["layers"]
        w = rl_weights()
        if shape["vocab"] > 0:
            self.embed = take(weights, "embed").contiguous()
            self.lm_head = packed(weights, ["lm_head"], RL_W_WHOLE_K)
            w.embed, w.lm_head = self.embed.data_ptr(), self.lm_head.data_ptr()
        self.final_norm = take(weights, "final_norm").contiguous()
        w.final_norm = self.final_norm.data_ptr()
        w.attn_norm = arr([take(l, "attn_norm").contiguous() for l in lay])
        w.mlp_norm = arr([take(l, "mlp_norm").contiguous() for l in lay])
        w.q_norm = arr([take(l, "q_norm").contiguous() for l in lay])
        w.k_norm = arr([take(l, "k_norm").contiguous() for l in lay])
        w.wqkv = arr([packed(l, ["wq", "wk", "wv"]) for l in lay])
        w.wo = arr([packed(l, ["wo"]) for l in lay])
        w.w_gate_up = arr([packed_gate_up(l) for l in lay])
        w.w_down = arr([packed(l, ["w_down"]) for l in lay])
        if kv_pages is None:
            torch.cuda.synchronize(self.device)
            torch.cuda.empty_cache()
            free_b, _ = torch.cuda.mem_get_info(self.device)
            kv_pages = int((free_b - need.value - kv_slack_bytes) // page)
            if kv_pages < 1:
                raise RLError(RL_ERR_KV_FULL, "no room for a KV pool beside the weights")
        cfg.kv_pool_bytes = page * kv_pages
        cfg.workspace_bytes = need.value
        self.cfg = cfg
        self.kv_pool = torch.empty(cfg.kv_pool_bytes, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(cfg.workspace_bytes, dtype=torch.uint8, device=self.device)
        w.kv_pool, w.workspace = self.kv_pool.data_ptr(), self.workspace.data_ptr()
        torch.cuda.synchronize(self.device)
        h = C.c_void_p()
        check(L.rl_init_model(C.byref(cfg), C.byref(w), C.byref(h)))
        self.h = h
        self._capture = None

    def close(self):
        if self.h:
            torch.cuda.synchronize(self.device)
            lib().rl_destroy_model(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the four calls of the boundary --------------------------------------------------------
    def rl_prefill(self, seq_ids, prompts, temperature, seed, top_k=0, top_p=0.0):
        """prompts: list of int sequences.  Returns (tokens int32[n], logprobs fp32[n]) on the device."""
        n = len(seq_ids)
        flat = [int(t) for p in prompts for t in p]
        out_t = torch.empty(n, dtype=torch.int32, device=self.device)
        out_lp = torch.empty(n, dtype=torch.float32, device=self.device)
        sp = rl_sampling(temperature, top_k, seed, top_p, 0)
        check(lib().rl_prefill(self.h, _stream(), n, _i32(seq_ids), _i32(flat), _i32([len(p) for p in prompts]),
                               C.byref(sp), _ptr(out_t), _ptr(out_lp)))
        return out_t, out_lp

    def rl_prefill_groups(self, seq_ids, group_size, prompts, temperature, seed, top_k=0, top_p=0.0):
        """prompts: one int sequence per group; seq_ids: len(prompts) * group_size ids, group-major."""
        n = len(seq_ids)
        assert n == len(prompts) * group_size
        flat = [int(t) for p in prompts for t in p]
        out_t = torch.empty(n, dtype=torch.int32, device=self.device)
        out_lp = torch.empty(n, dtype=torch.float32, device=self.device)
        sp = rl_sampling(temperature, top_k, seed, top_p, 0)
        check(lib().rl_prefill_groups(self.h, _stream(), len(prompts), group_size, _i32(seq_ids), _i32(flat),
                                      _i32([len(p) for p in prompts]), C.byref(sp), _ptr(out_t), _ptr(out_lp)))
        return out_t, out_lp

    def rl_score(self, seq_ids, sequences, temperature):
        """Teacher-forced log-probs of tokens 1.. of each int sequence; returns one device fp32 tensor (concatenated)."""
        flat = [int(t) for q in sequences for t in q]
        out = torch.empty(len(flat) - len(sequences), dtype=torch.float32, device=self.device)
        check(lib().rl_score(self.h, _stream(), len(sequences), _i32(seq_ids), _i32(flat),
                             _i32([len(q) for q in sequences]), temperature, _ptr(out)))
        return out

    def rl_decode_step(self, seq_ids, in_tokens, temperature, seed, forced_next=None, debug_logits=None,
                       out_tokens=None, out_logprobs=None, top_k=0, top_p=0.0):
        n = len(seq_ids)
        out_t = out_tokens if out_tokens is not None else torch.empty(n, dtype=torch.int32, device=self.device)
        out_lp = out_logprobs if out_logprobs is not None else torch.empty(n, dtype=torch.float32, device=self.device)
        sp = rl_sampling(temperature, top_k, seed, top_p, 0)
        ids = seq_ids if isinstance(seq_ids, C.Array) else _i32(seq_ids)
        check(lib().rl_decode_step(self.h, _stream(), n, ids, _ptr(in_tokens), _ptr(forced_next), C.byref(sp),
                                   _ptr(out_t), _ptr(out_lp), _ptr(debug_logits)))
        return out_t, out_lp

    def decode_graph(self, seq_ids, temperature, seed):
        """DecodeGraph over a fixed batch: .step() runs one decode step (fed the last sampled tokens) as a graph launch
        and returns (out_tokens, out_logprobs), the same two device tensors every step."""
        return DecodeGraph(self, seq_ids, temperature, seed)

    def rl_free_seqs(self, seq_ids):
        check(lib().rl_free_seqs(self.h, len(seq_ids), _i32(seq_ids)))

    # ---- helpers -----------------------------------------------------------------------------------
    def rl_kv_stats(self):
        f, t = C.c_uint64(), C.c_uint64()
        check(lib().rl_kv_stats(self.h, C.byref(f), C.byref(t)))
        return f.value, t.value

    def rl_seq_len(self, seq_id):
        n = C.c_int32()
        check(lib().rl_seq_len(self.h, seq_id, C.byref(n)))
        return n.value

    def rl_sample_logits(self, logits, seq_ids, positions, temperature, seed, forced=None, top_k=0, top_p=0.0):
        n = logits.shape[0]
        out_t = torch.empty(n, dtype=torch.int32, device=self.device)
        out_lp = torch.empty(n, dtype=torch.float32, device=self.device)
        sp = rl_sampling(temperature, top_k, seed, top_p, 0)
        check(lib().rl_sample_logits(self.h, _stream(), n, _ptr(logits), _i32(seq_ids), _i32(positions),
                                     _ptr(forced), C.byref(sp), _ptr(out_t), _ptr(out_lp)))
        return out_t, out_lp

    def rl_seq_import_kv(self, seq_id, k_layers, v_layers):
        """k_layers/v_layers: per layer a device tensor [n_tokens, n_kv, head_dim] in the model dtype."""
        n_tokens = k_layers[0].shape[0]
        n_layers = self.shape["n_layers"]
        ka = (C.c_void_p * n_layers)(*[t.data_ptr() for t in k_layers])
        va = (C.c_void_p * n_layers)(*[t.data_ptr() for t in v_layers])
        check(lib().rl_seq_import_kv(self.h, _stream(), seq_id, n_tokens, C.cast(ka, _pp), C.cast(va, _pp)))

    def rl_seq_append_kv(self, seq_id, k_layers, v_layers):
        """Append [n_tokens, n_kv, head_dim] K/V per layer behind what the active sequence already caches."""
        n_tokens = k_layers[0].shape[0]
        n_layers = self.shape["n_layers"]
        ka = (C.c_void_p * n_layers)(*[t.data_ptr() for t in k_layers])
        va = (C.c_void_p * n_layers)(*[t.data_ptr() for t in v_layers])
        check(lib().rl_seq_append_kv(self.h, _stream(), seq_id, n_tokens, C.cast(ka, _pp), C.cast(va, _pp)))

    def rl_decode_hidden(self, seq_ids, hidden_in, hidden_out=None):
        out = hidden_out if hidden_out is not None else torch.empty_like(hidden_in)
        ids = seq_ids if isinstance(seq_ids, C.Array) else _i32(seq_ids)
        check(lib().rl_decode_hidden(self.h, _stream(), len(seq_ids), ids, _ptr(hidden_in), _ptr(out)))
        return out

    def rl_set_capture(self, on):
        """Returns the capture buffer [(n_layers+1), max_rows, hidden] fp32 (or None when switched off)."""
        if on:
            self._capture = torch.zeros(self.shape["n_layers"] + 1, self.cfg.max_rows, self.shape["hidden"],
                                        dtype=torch.float32, device=self.device)
            check(lib().rl_set_capture(self.h, _ptr(self._capture)))
        else:
            check(lib().rl_set_capture(self.h, None))
            self._capture = None
        return self._capture

    def rl_debug_shuffle_free_pages(self, seed):
        check(lib().rl_debug_shuffle_free_pages(self.h, seed))

    def rl_seq_fork(self, src_seq, new_seq_ids):
        check(lib().rl_seq_fork(self.h, _stream(), src_seq, len(new_seq_ids), _i32(new_seq_ids)))

    def rl_debug_share_attention(self, on):
        check(lib().rl_debug_share_attention(self.h, int(on)))

    def rl_debug_attention_split(self, segs_per_block):
        check(lib().rl_debug_attention_split(self.h, int(segs_per_block)))

    def rl_debug_attention_appends(self, on):
        check(lib().rl_debug_attention_appends(self.h, int(on)))

    def rl_profile_enable(self, on):
        check(lib().rl_profile_enable(self.h, 1 if on else 0))

    def rl_profile_host_read(self):
        """Host microseconds inside rl_decode_step since the last read: dict(admit, meta, launch, wait, calls)."""
        a, b, c, w, n = C.c_double(), C.c_double(), C.c_double(), C.c_double(), C.c_int64()
        check(lib().rl_profile_host_read(self.h, C.byref(a), C.byref(b), C.byref(c), C.byref(w), C.byref(n)))
        return {"admit_us": a.value, "meta_us": b.value, "launch_us": c.value, "wait_us": w.value, "calls": n.value}

    def rl_profile_read(self):
        """{kernel class: (launches, total ms)} since the last read."""
        n_max = 32
        names = (C.c_char_p * n_max)()
        ms = (C.c_double * n_max)()
        cnt = (C.c_int64 * n_max)()
        n = C.c_int32()
        check(lib().rl_profile_read(self.h, n_max, names, ms, cnt, C.byref(n)))
        return {names[i].decode(): (cnt[i], ms[i]) for i in range(n.value)}


class DecodeGraph:
    """rl_decode_graph_create / _step / _destroy for a fixed batch of sequences of one Rollout."""

    def __init__(self, ro, seq_ids, temperature, seed):
        n = len(seq_ids)
        self.ro = ro
        self.out_tokens = torch.empty(n, dtype=torch.int32, device=ro.device)
        self.out_logprobs = torch.empty(n, dtype=torch.float32, device=ro.device)
        self.captures = 0
        sp = rl_sampling(temperature, 0, seed, 0.0, 0)
        h = C.c_void_p()
        check(lib().rl_decode_graph_create(ro.h, n, _i32(seq_ids), C.byref(sp), _ptr(self.out_tokens),
                                           _ptr(self.out_logprobs), C.byref(h)))
        self.h = h

    def step(self):
        c = C.c_int64()
        check(lib().rl_decode_graph_step(self.h, _stream(), C.byref(c)))
        self.captures = c.value
        return self.out_tokens, self.out_logprobs

    def close(self):
        if self.h:
            torch.cuda.synchronize(self.ro.device)
            lib().rl_decode_graph_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
