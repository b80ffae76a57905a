"""ctypes front end of the C++ oracle (test infrastructure only).

`OracleModel` strings the per-layer oracle into the full decoder of the
rollout definition (Section 2.3 workflow; Appendix C): embedding lookup,
L decoder layers with a contiguous per-sequence KV history, final RMSNorm,
untied output projection, then the sampler.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)


class _Dims(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q", C.c_int32), ("n_kv", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("qk_norm", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float)]


class _Layer(C.Structure):
    _fields_ = [(n, _f32p) for n in ("attn_norm", "wq", "wk", "wv", "q_norm", "k_norm",
                                     "wo", "mlp_norm", "w_gate", "w_up", "w_down")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = C.CDLL(path)
        L.orc_num_threads.restype = C.c_int32
        L.orc_bf16_round.restype = C.c_float
        L.orc_bf16_round.argtypes = [C.c_float]
        L.orc_bf16_round_array.argtypes = [_f32p, C.c_int64]
        L.orc_rmsnorm.argtypes = [_f32p, _f32p, C.c_int32, C.c_float, _f32p]
        L.orc_matvec.argtypes = [_f32p, _f32p, C.c_int32, C.c_int32, _f32p]
        L.orc_rope.argtypes = [_f32p, C.c_int32, C.c_int32, C.c_float]
        L.orc_silu.restype = C.c_double
        L.orc_silu.argtypes = [C.c_double]
        L.orc_attention.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int32, C.c_int32,
                                    C.c_int32, _f32p, _f64p]
        L.orc_layer_forward.argtypes = [C.POINTER(_Dims), C.POINTER(_Layer), _f32p, C.c_int32,
                                        _f32p, _f32p]
        L.orc_model_forward_token.restype = None
        L.orc_model_forward_token.argtypes = [C.POINTER(_Dims), C.c_int32, C.POINTER(_Layer), _f32p, _f32p, _f32p, C.c_int32,
                                              C.c_int32, C.c_int32, C.POINTER(_f32p), C.POINTER(_f32p), _f32p, _f32p]
        L.orc_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                        C.POINTER(C.c_uint32)]
        L.orc_token_bits.restype = C.c_uint32
        L.orc_token_bits.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_flog.restype = C.c_float
        L.orc_flog.argtypes = [C.c_float]
        L.orc_uniform.restype = C.c_float
        L.orc_uniform.argtypes = [C.c_uint32]
        L.orc_gumbel.restype = C.c_float
        L.orc_gumbel.argtypes = [C.c_uint32]
        L.orc_sample.argtypes = [_f32p, C.c_int32, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                 C.c_int32, C.POINTER(C.c_int32), _f64p]
        L.orc_log_softmax.argtypes = [_f32p, C.c_int32, C.c_float, _f64p]
        L.orc_order_key.restype = C.c_uint32
        L.orc_order_key.argtypes = [C.c_float]
        L.orc_fexp_weight.restype = C.c_uint64
        L.orc_fexp_weight.argtypes = [C.c_float]
        L.orc_truncation.restype = C.c_int32
        L.orc_truncation.argtypes = [_f32p, C.c_int32, C.c_float, C.c_int32, C.c_float, C.POINTER(C.c_uint8)]
        L.orc_sample_truncated.argtypes = [_f32p, C.c_int32, C.c_float, C.c_int32, C.c_float, C.c_uint64, C.c_uint32,
                                           C.c_uint32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                           C.POINTER(C.c_int32)]
        L.orc_sample_histogram.argtypes = [_f32p, C.c_int32, C.c_float, C.c_uint64, C.c_uint32,
                                           C.c_uint32, C.c_int64, C.POINTER(C.c_int64)]
        _i32p = C.POINTER(C.c_int32)
        L.orc_hrd_objective.restype = C.c_double
        L.orc_hrd_objective.argtypes = [C.c_int32, C.c_int32, _i32p, _i32p, _f32p, _f32p, _f32p, _f32p,
                                        C.c_double, C.c_double, C.c_double, C.c_int32, _f64p]
        L.orc_plan_length.restype = C.c_int32
        L.orc_plan_length.argtypes = [_i32p, C.c_int32, C.c_int32]
        _lib = L
    return _lib


def _p(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_f32p)


def f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def num_threads():
    return int(lib().orc_num_threads())


def bf16_round(a):
    """Round an array to the bfloat16 grid (nearest even), returned as fp32."""
    out = f32(a).copy()
    lib().orc_bf16_round_array(_p(out), out.size)
    return out


def rmsnorm(x, g, eps):
    x, g = f32(x), f32(g)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), x.size, eps, _p(out))
    return out


def matvec(W, x):
    W, x = f32(W), f32(x)
    y = np.empty(W.shape[0], dtype=np.float32)
    lib().orc_matvec(_p(W), _p(x), W.shape[0], W.shape[1], _p(y))
    return y


def rope(u, pos, base):
    out = f32(u).copy()
    lib().orc_rope(_p(out), out.size, pos, base)
    return out


def silu(z):
    return lib().orc_silu(float(z))


def attention(q, kcache, vcache, want_probs=False):
    """q [n_q,d]; kcache/vcache [n_keys,n_kv,d] -> out [n_q,d] (and probs [n_q,n_keys])."""
    q, kcache, vcache = f32(q), f32(kcache), f32(vcache)
    n_q, d = q.shape
    n_keys, n_kv, _ = kcache.shape
    out = np.empty_like(q)
    probs = np.empty((n_q, n_keys), dtype=np.float64) if want_probs else None
    lib().orc_attention(_p(q), _p(kcache), _p(vcache), n_keys, n_q, n_kv, d, _p(out),
                        probs.ctypes.data_as(_f64p) if want_probs else None)
    return (out, probs) if want_probs else out


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def token_bits(seed, seq, pos, i):
    return int(lib().orc_token_bits(seed, seq, pos, i))


def flog(x):
    return float(lib().orc_flog(float(x)))


def uniform(bits):
    return float(lib().orc_uniform(bits))


def gumbel(bits):
    return float(lib().orc_gumbel(bits))


def sample(z, temperature, seed, seq, pos, forced=-1):
    z = f32(z)
    tok = C.c_int32()
    lp = C.c_double()
    lib().orc_sample(_p(z), z.size, temperature, seed, seq, pos, forced, C.byref(tok), C.byref(lp))
    return int(tok.value), float(lp.value)


def order_key(z):
    return int(lib().orc_order_key(float(z)))


def fexp_weight(x):
    return int(lib().orc_fexp_weight(float(x)))


def truncation(z, invT, top_k, top_p):
    """Mask (uint8 [V]) of the tokens that top-k / top-p keep."""
    z = f32(z)
    keep = np.zeros(z.size, dtype=np.uint8)
    n = lib().orc_truncation(_p(z), z.size, invT, top_k, top_p, keep.ctypes.data_as(C.POINTER(C.c_uint8)))
    assert int(keep.sum()) == n
    return keep


def sample_truncated(z, temperature, top_k, top_p, seed, seq, pos, forced=-1):
    """(token, log-probability under the truncated distribution, number of kept tokens)."""
    z = f32(z)
    tok, lp, kept = C.c_int32(), C.c_double(), C.c_int32()
    lib().orc_sample_truncated(_p(z), z.size, temperature, top_k, top_p, seed, seq, pos, forced, C.byref(tok),
                               C.byref(lp), C.byref(kept))
    return int(tok.value), float(lp.value), int(kept.value)


def log_softmax(z, invT=1.0):
    z = f32(z)
    out = np.empty(z.size, dtype=np.float64)
    lib().orc_log_softmax(_p(z), z.size, invT, out.ctypes.data_as(_f64p))
    return out


def sample_histogram(z, temperature, seed, seq, pos0, n_draws):
    z = f32(z)
    counts = np.zeros(z.size, dtype=np.int64)
    lib().orc_sample_histogram(_p(z), z.size, temperature, seed, seq, pos0, n_draws,
                               counts.ctypes.data_as(C.POINTER(C.c_int64)))
    return counts


LAYER_KEYS = ("attn_norm", "wq", "wk", "wv", "q_norm", "k_norm", "wo", "mlp_norm",
              "w_gate", "w_up", "w_down")


def layer_forward(dims, layer, x, pos, kcache, vcache):
    """One decoder layer at position `pos`; `x` [H] is updated in place.

    dims: dict(hidden,n_q,n_kv,head_dim,ffn,qk_norm,rms_eps,rope_base);
    layer: dict of fp32 arrays keyed by LAYER_KEYS;
    kcache/vcache: fp32 [max_pos,n_kv,d], row `pos` is written.
    """
    dm = _Dims(dims["hidden"], dims["n_q"], dims["n_kv"], dims["head_dim"], dims["ffn"],
               int(dims["qk_norm"]), dims["rms_eps"], dims["rope_base"])
    lw = _Layer(*[_p(layer[k]) for k in LAYER_KEYS])
    assert x.dtype == np.float32 and x.flags["C_CONTIGUOUS"]
    assert kcache.dtype == np.float32 and kcache.flags["C_CONTIGUOUS"]
    assert vcache.dtype == np.float32 and vcache.flags["C_CONTIGUOUS"]
    assert pos < kcache.shape[0]
    lib().orc_layer_forward(C.byref(dm), C.byref(lw), _p(x), pos, _p(kcache), _p(vcache))


class OracleModel:
    """Whole decoder with per-sequence contiguous KV histories; the arithmetic is orc_model_forward_token (C++), this
    class only keeps the arrays and the per-sequence positions.

    weights: dict with 'embed' [V,H], 'lm_head' [V,H], 'final_norm' [H] and
    'layers' = list of per-layer dicts (LAYER_KEYS), all fp32 numpy arrays that
    the caller has already put on the storage grid under test.
    """

    def __init__(self, dims, weights, max_ctx):
        self.dims = dict(dims)
        self.w = weights
        self.max_ctx = max_ctx
        self.n_layers = len(weights["layers"])
        self.seqs = {}
        self._dm = _Dims(dims["hidden"], dims["n_q"], dims["n_kv"], dims["head_dim"], dims["ffn"],
                         int(dims["qk_norm"]), dims["rms_eps"], dims["rope_base"])
        for l in weights["layers"]:
            for k in LAYER_KEYS:
                assert l[k].dtype == np.float32 and l[k].flags["C_CONTIGUOUS"]
        self._layers = (_Layer * max(1, self.n_layers))(*[_Layer(*[_p(l[k]) for k in LAYER_KEYS])
                                                          for l in weights["layers"]])
        for k in ("embed", "lm_head", "final_norm"):
            assert weights[k].dtype == np.float32 and weights[k].flags["C_CONTIGUOUS"]
        self.vocab = weights["lm_head"].shape[0]

    def _cache(self, seq):
        if seq not in self.seqs:
            shape = (self.max_ctx, self.dims["n_kv"], self.dims["head_dim"])
            k = [np.zeros(shape, np.float32) for _ in range(self.n_layers)]
            v = [np.zeros(shape, np.float32) for _ in range(self.n_layers)]
            fpp = C.POINTER(C.c_float) * max(1, self.n_layers)
            self.seqs[seq] = dict(len=0, k=k, v=v, kp=fpp(*[_p(a) for a in k]), vp=fpp(*[_p(a) for a in v]))
        return self.seqs[seq]

    def free(self, seq):
        self.seqs.pop(seq, None)

    def forward_token(self, seq, tok, want_hidden=False):
        """Feed one token, extend the history, return the next-token logits [V] (and the last residual stream)."""
        st = self._cache(seq)
        pos = st["len"]
        assert pos < self.max_ctx and 0 <= int(tok) < self.w["embed"].shape[0]
        logits = np.empty(self.vocab, np.float32)
        hidden = np.empty(self.dims["hidden"], np.float32)
        lib().orc_model_forward_token(C.byref(self._dm), self.n_layers, self._layers, _p(self.w["embed"]),
                                      _p(self.w["lm_head"]), _p(self.w["final_norm"]), self.vocab, int(tok), pos,
                                      st["kp"], st["vp"], _p(logits), _p(hidden))
        st["len"] = pos + 1
        return (logits, hidden) if want_hidden else logits

    def prefill(self, seq, tokens):
        z = None
        for t in tokens:
            z = self.forward_token(seq, int(t))
        return z


def _ip(a):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def hrd_objective(n_prompts, G, off, n_plan, lp_new, lp_old, r_speedup, r_correct, alpha=0.1, eps=0.2, beta=0.0,
                  mode=0):
    """(J, per-output terms) of the HRD objective (mode 0) or the uniform-reward GRPO objective (mode 1)."""
    off = np.ascontiguousarray(off, np.int32)
    n_plan = np.ascontiguousarray(n_plan, np.int32)
    seq = np.zeros(n_prompts * G, np.float64)
    J = lib().orc_hrd_objective(n_prompts, G, _ip(off), _ip(n_plan), _p(f32(lp_new)), _p(f32(lp_old)),
                                _p(f32(r_speedup)), _p(f32(r_correct)), alpha, eps, beta, mode,
                                seq.ctypes.data_as(_f64p))
    return float(J), seq


def plan_length(tokens, delimiter):
    t = np.ascontiguousarray(tokens, np.int32)
    return int(lib().orc_plan_length(_ip(t), t.size, delimiter))
