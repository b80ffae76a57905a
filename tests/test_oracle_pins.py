"""Pins of the CPU oracle against what mathematics and published vectors fix.

The paper prints no worked numeric example of a forward pass or of a sampled
token, so every pin here is a closed form, an invariant, a special case that
reduces to a library routine, a published known-answer vector, or brute force.
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import rollout_inputs as ri
from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)


# --------------------------------------------------------------------------- RNG
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert orc.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_token_bits_keying():
    # word i&3 of block (i>>2, pos, seq, 0) under key (seed_lo, seed_hi)
    seed = 0x299f31d0a4093822
    blk = orc.philox4x32_10([0x243f6a88, 0x85a308d3, 0x13198a2e, 0], [0xa4093822, 0x299f31d0])
    for w in range(4):
        assert orc.token_bits(seed, 0x13198a2e, 0x85a308d3, 4 * 0x243f6a88 + w) == blk[w]
    # distinct positions / sequences / seeds give distinct streams
    a = [orc.token_bits(1, 0, 0, i) for i in range(64)]
    assert a != [orc.token_bits(1, 0, 1, i) for i in range(64)]
    assert a != [orc.token_bits(1, 1, 0, i) for i in range(64)]
    assert a != [orc.token_bits(2, 0, 0, i) for i in range(64)]


def test_bits_uniformity_chi2():
    n, bins = 1 << 16, 64
    h = np.zeros(bins)
    for i in range(n):
        h[orc.token_bits(99, 3, 5, i) >> 26] += 1
    chi2 = ((h - n / bins) ** 2 / (n / bins)).sum()
    assert chi2 < 63 + 6 * math.sqrt(2 * 63)


# ----------------------------------------------------------------- sampler maths
def test_uniform_exact_grid():
    assert orc.uniform(0) == 2.0 ** -24
    assert orc.uniform(0xffffffff) == 1.0 - 2.0 ** -24
    assert orc.uniform(0x1ff) == 2.0 ** -24            # low 9 bits are dropped
    assert orc.uniform(0x200) == 3 * 2.0 ** -24
    assert orc.uniform(0x80000000) == 0.5 + 2.0 ** -24


def test_flog_against_libm():
    xs = np.concatenate([
        np.exp(rng.uniform(math.log(5e-8), math.log(20.0), 20000)),
        1.0 - np.arange(1, 2000, 2) * 2.0 ** -24,
        np.array([2.0 ** -24, 0.5, 1.0, 2.0, 16.635532, math.sqrt(0.5), math.sqrt(2.0)]),
    ]).astype(np.float32)
    worst = 0.0
    for x in xs:
        ref = math.log(float(x))
        got = orc.flog(float(x))
        tol = max(abs(ref) * 2.0 ** -22, 1.2e-7)
        worst = max(worst, abs(got - ref) / tol)
    assert worst <= 1.0
    assert orc.flog(1.0) == 0.0
    assert orc.flog(1.0 - 2.0 ** -24) < 0.0            # keeps -log(u) strictly positive


def test_gumbel_range_and_moments():
    assert abs(orc.gumbel(0) - (-math.log(24 * math.log(2)))) < 1e-5
    assert abs(orc.gumbel(0xffffffff) - (-math.log(-math.log1p(-2.0 ** -24)))) < 1e-4
    g = np.array([orc.gumbel(orc.token_bits(5, 0, 0, i)) for i in range(100000)])
    assert abs(g.mean() - 0.5772157) < 4.5 * math.sqrt(math.pi ** 2 / 6 / g.size)
    assert abs(g.var() - math.pi ** 2 / 6) < 0.03
    # Gumbel CDF exp(-exp(-x)) at a few points
    for x in (-1.0, 0.0, 1.0, 2.5):
        p = math.exp(-math.exp(-x))
        assert abs((g <= x).mean() - p) < 4.5 * math.sqrt(p * (1 - p) / g.size)


@pytest.mark.parametrize("T", [1.0, 0.5, 2.0])
def test_sampler_frequencies_match_softmax(T):
    z = np.array([0.3, -1.2, 2.0, 0.0, 1.1, -0.4, 0.9, -3.0], dtype=np.float32)
    n = 200000
    counts = orc.sample_histogram(z, T, seed=1234, seq=2, pos0=0, n_draws=n)
    p = np.exp(z.astype(np.float64) / T)
    p /= p.sum()
    sigma = np.sqrt(n * p * (1 - p))
    assert counts.sum() == n
    assert np.all(np.abs(counts - n * p) < 4.5 * sigma)


def test_sampler_permutation_equivariance_in_distribution():
    z = np.array([1.5, -0.5, 0.2, 0.7], dtype=np.float32)
    perm = np.array([2, 0, 3, 1])
    n = 100000
    c1 = orc.sample_histogram(z, 1.0, 11, 0, 0, n)
    c2 = orc.sample_histogram(z[perm], 1.0, 12, 0, 0, n)
    p = np.exp(z.astype(np.float64))
    p /= p.sum()
    sigma = np.sqrt(2 * n * p * (1 - p))
    assert np.all(np.abs(c1[perm] - c2) < 4.5 * sigma[perm])


def test_sampler_greedy_ties_and_low_temperature():
    z = np.array([0.1, 3.0, 3.0, -1.0], dtype=np.float32)
    tok, lp = orc.sample(z, 0.0, 1, 0, 0)
    assert tok == 1                                     # lowest index on ties
    assert abs(lp - (3.0 - math.log(np.exp(z.astype(np.float64)).sum()))) < 1e-12
    z2 = np.array([0.0, 1.0, 5.0, 2.0], dtype=np.float32)
    c = orc.sample_histogram(z2, 0.02, 3, 0, 0, 2000)   # T -> 0 concentrates on argmax
    assert c[2] == 2000
    zi = np.array([-np.inf, 0.0, -np.inf], dtype=np.float32)
    assert orc.sample(zi, 1.0, 5, 0, 0)[0] == 1        # -inf never wins


def test_logprob_is_log_softmax_entry_and_sums_to_one():
    z = rng.normal(0, 1.3, 4096).astype(np.float32)
    for T in (1.0, 0.7):
        invT = float(np.float32(1.0) / np.float32(T))
        ls = orc.log_softmax(z, invT)
        assert abs(np.exp(ls).sum() - 1.0) < 1e-12
        assert np.allclose(orc.log_softmax(z + np.float32(8.0), invT), ls, atol=2e-6)
        tok, lp = orc.sample(z, T, 77, 1, 9)
        assert abs(lp - ls[tok]) < 1e-12
        tok_f, lp_f = orc.sample(z, T, 77, 1, 9, forced=123)
        assert tok_f == 123 and abs(lp_f - ls[123]) < 1e-12
    ref = torch.log_softmax(torch.from_numpy(z).double(), 0).numpy()
    assert np.allclose(orc.log_softmax(z, 1.0), ref, atol=1e-12)


def test_sample_is_deterministic_in_its_key():
    z = rng.normal(0, 1.0, 512).astype(np.float32)
    a = [orc.sample(z, 1.0, 42, 3, p)[0] for p in range(50)]
    b = [orc.sample(z, 1.0, 42, 3, p)[0] for p in range(50)]
    assert a == b and len(set(a)) > 10


# ------------------------------------------------------------------ bf16 rounding
def test_bf16_round_matches_torch():
    x = rng.normal(0, 1, 10000).astype(np.float32)
    x = np.concatenate([x, np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.3895314e38], np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert np.array_equal(orc.bf16_round(x), ref)


# ------------------------------------------------------------------ building blocks
def test_rmsnorm_properties():
    x = rng.normal(0, 3, 256).astype(np.float32)
    g1 = np.ones(256, np.float32)
    y = orc.rmsnorm(x, g1, 0.0)
    assert abs(np.mean(y.astype(np.float64) ** 2) - 1.0) < 1e-6
    assert np.allclose(orc.rmsnorm(7.5 * x, g1, 0.0), y, rtol=1e-6)
    g = rng.normal(1, 0.1, 256).astype(np.float32)
    assert np.allclose(orc.rmsnorm(x, g, 1e-6), orc.rmsnorm(x, g1, 1e-6) * g, rtol=1e-6)
    ref = F.rms_norm(torch.from_numpy(x).double(), (256,), torch.from_numpy(g).double(), 1e-6)
    assert np.allclose(orc.rmsnorm(x, g, 1e-6), ref.numpy(), rtol=1e-6)
    # eps matters for tiny inputs: x = 0 -> 0, and |x| << sqrt(eps) is damped
    assert np.all(orc.rmsnorm(np.zeros(8, np.float32), np.ones(8, np.float32), 1e-6) == 0)
    t = orc.rmsnorm(np.full(4, 1e-4, np.float32), np.ones(4, np.float32), 1e-6)
    assert np.allclose(t, 1e-4 / math.sqrt(1e-8 + 1e-6), rtol=1e-5)


def test_silu_identities():
    assert orc.silu(0.0) == 0.0
    for z in (-7.0, -1.3, 0.4, 2.0, 11.0):
        assert abs(orc.silu(z) - orc.silu(-z) - z) < 1e-12
        assert abs(orc.silu(z) - F.silu(torch.tensor(z, dtype=torch.float64)).item()) < 1e-12
    assert abs(orc.silu(40.0) - 40.0) < 1e-12 and abs(orc.silu(-40.0)) < 1e-12


def test_matvec_brute_force_and_identity():
    W = rng.normal(0, 1, (37, 53)).astype(np.float32)
    x = rng.normal(0, 1, 53).astype(np.float32)
    brute = np.array([sum(float(W[o, i]) * float(x[i]) for i in range(53)) for o in range(37)])
    assert np.allclose(orc.matvec(W, x), brute, rtol=1e-6, atol=1e-6)
    assert np.array_equal(orc.matvec(np.eye(53, dtype=np.float32), x), x)
    E = np.zeros((3, 53), np.float32)
    E[0, 5] = E[1, 0] = E[2, 52] = 1
    assert np.array_equal(orc.matvec(E, x), x[[5, 0, 52]])   # not transposed


def test_rope_properties():
    d, base = 64, 1e6
    u = rng.normal(0, 1, d).astype(np.float32)
    assert np.array_equal(orc.rope(u, 0, base), u)
    for pos in (1, 17, 4097):
        r = orc.rope(u, pos, base)
        assert abs(np.linalg.norm(r) - np.linalg.norm(u)) < 1e-5 * np.linalg.norm(u)
        pn = np.hypot(r[:d // 2], r[d // 2:])
        assert np.allclose(pn, np.hypot(u[:d // 2], u[d // 2:]), rtol=1e-5)
    # one-hot on pair i rotates by pos * base^(-2i/d), counter-clockwise, partner at i + d/2
    for i in (0, 1, 5, 31):
        e = np.zeros(d, np.float32)
        e[i] = 1
        r = orc.rope(e, 3, base)
        th = 3 * base ** (-2.0 * i / d)
        assert abs(r[i] - math.cos(th)) < 1e-6 and abs(r[i + d // 2] - math.sin(th)) < 1e-6
        assert np.count_nonzero(r) <= 2
    # relative property: <rope(q,m), rope(k,n)> depends on m-n only
    q = rng.normal(0, 1, d).astype(np.float32)
    k = rng.normal(0, 1, d).astype(np.float32)
    a = np.dot(orc.rope(q, 9, base).astype(np.float64), orc.rope(k, 4, base))
    b = np.dot(orc.rope(q, 1005, base).astype(np.float64), orc.rope(k, 1000, base))
    assert abs(a - b) < 1e-4
    # complex-number formulation: (u_i + j u_{i+d/2}) * exp(j theta_i)
    zc = (u[:d // 2] + 1j * u[d // 2:]) * np.exp(1j * 21 * base ** (-2.0 * np.arange(d // 2) / d))
    r = orc.rope(u, 21, base)
    assert np.allclose(r[:d // 2], zc.real, atol=1e-6) and np.allclose(r[d // 2:], zc.imag, atol=1e-6)


def test_attention_special_cases():
    n_q, n_kv, d = 4, 2, 16
    q = rng.normal(0, 1, (n_q, d)).astype(np.float32)
    K = rng.normal(0, 1, (9, n_kv, d)).astype(np.float32)
    V = rng.normal(0, 1, (9, n_kv, d)).astype(np.float32)
    # one key -> V of the mapped kv head, exactly
    o = orc.attention(q, K[:1], V[:1])
    assert np.array_equal(o, V[0][[0, 0, 1, 1]])
    # identical keys -> mean of V; zero query -> mean of V
    Ksame = np.repeat(K[:1], 9, axis=0)
    assert np.allclose(orc.attention(q, Ksame, V), V.mean(0)[[0, 0, 1, 1]], atol=1e-6)
    assert np.allclose(orc.attention(np.zeros_like(q), K, V), V.mean(0)[[0, 0, 1, 1]], atol=1e-6)
    # GQA mapping: constant V per kv head
    Vc = np.zeros_like(V)
    Vc[:, 0, :] = 3.0
    Vc[:, 1, :] = -5.0
    o = orc.attention(q, K, Vc)
    assert np.allclose(o[:2], 3.0) and np.allclose(o[2:], -5.0)
    # rows of the softmax sum to one, and are shift-invariant in the scores
    _, p = orc.attention(q, K, V, want_probs=True)
    assert np.allclose(p.sum(1), 1.0, atol=1e-12)
    # library routine: scaled_dot_product_attention with repeated kv heads
    tq = torch.from_numpy(q).double()[:, None, :]                       # [n_q,1,d]
    tk = torch.from_numpy(K).double().permute(1, 0, 2).repeat_interleave(2, 0)
    tv = torch.from_numpy(V).double().permute(1, 0, 2).repeat_interleave(2, 0)
    ref = F.scaled_dot_product_attention(tq, tk, tv)[:, 0, :].numpy()
    assert np.allclose(orc.attention(q, K, V), ref, atol=1e-6)
    # a dominant key takes all the weight
    Kd = K.copy()
    Kd[4] = 0
    Kd[4, 0] = 50 * q[0] / np.linalg.norm(q[0])
    _, p = orc.attention(q, Kd, V, want_probs=True)
    assert p[0, 4] > 0.999


# ------------------------------------------------------------------------- layer
def _tiny(qk_norm=1, seed=5):
    s = dict(ri.SHAPES["tiny"])
    s.update(hidden=32, n_q=4, n_kv=2, head_dim=8, ffn=24, vocab=50, qk_norm=qk_norm)
    w = ri.make_weights(s, seed, std=0.3)
    wn = {k: (v.numpy() if k != "layers" else [{a: b.numpy() for a, b in l.items()} for l in v])
          for k, v in w.items()}
    dims = {k: s[k] for k in ("hidden", "n_q", "n_kv", "head_dim", "ffn", "qk_norm", "rms_eps",
                              "rope_base")}
    return s, dims, w, wn


def _torch_layer_fullseq(s, lw, X):
    """Whole-sequence layer from library routines in float64 (matrix form, causal mask)."""
    T = X.shape[0]
    d, nq, nkv = s["head_dim"], s["n_q"], s["n_kv"]
    W = {k: v.double() for k, v in lw.items()}
    h = F.rms_norm(X, (X.shape[1],), W["attn_norm"], s["rms_eps"])
    q = F.linear(h, W["wq"]).view(T, nq, d)
    k = F.linear(h, W["wk"]).view(T, nkv, d)
    v = F.linear(h, W["wv"]).view(T, nkv, d)
    if s["qk_norm"]:
        q = F.rms_norm(q, (d,), W["q_norm"], s["rms_eps"])
        k = F.rms_norm(k, (d,), W["k_norm"], s["rms_eps"])
    ang = torch.arange(T, dtype=torch.float64)[:, None] * \
        s["rope_base"] ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]

    def rope(u):
        c = torch.complex(u[..., :d // 2], u[..., d // 2:]) * rot
        return torch.cat([c.real, c.imag], -1)
    q, k = rope(q), rope(k)
    o = F.scaled_dot_product_attention(q.permute(1, 0, 2), k.permute(1, 0, 2).repeat_interleave(nq // nkv, 0),
                                       v.permute(1, 0, 2).repeat_interleave(nq // nkv, 0), is_causal=True)
    X = X + F.linear(o.permute(1, 0, 2).reshape(T, nq * d), W["wo"])
    h2 = F.rms_norm(X, (X.shape[1],), W["mlp_norm"], s["rms_eps"])
    return X + F.linear(F.silu(F.linear(h2, W["w_gate"])) * F.linear(h2, W["w_up"]), W["w_down"])


@pytest.mark.parametrize("qk_norm", [0, 1])
def test_layer_incremental_equals_full_sequence_library_form(qk_norm):
    s, dims, w, wn = _tiny(qk_norm)
    T = 11
    X = ri.normal((T, s["hidden"]), 1.0, 3, 50)
    ref = _torch_layer_fullseq(s, w["layers"][0], X.double()).numpy()
    kc = np.zeros((T, s["n_kv"], s["head_dim"]), np.float32)
    vc = np.zeros_like(kc)
    for p in range(T):
        x = X[p].numpy().copy()
        orc.layer_forward(dims, wn["layers"][0], x, p, kc, vc)
        assert np.allclose(x, ref[p], rtol=2e-5, atol=2e-5), p


def test_layer_causality_and_residual_structure():
    s, dims, w, wn = _tiny()
    lw = wn["layers"][0]
    T = 6
    X = ri.normal((T, s["hidden"]), 1.0, 4, 51).numpy()
    kc = np.zeros((T, s["n_kv"], s["head_dim"]), np.float32)
    vc = np.zeros_like(kc)
    outs = []
    for p in range(T):
        x = X[p].copy()
        orc.layer_forward(dims, lw, x, p, kc, vc)
        outs.append(x)
    # garbage in cache rows beyond pos never changes the result at pos
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[3:] = 1e3
    vc2[3:] = -1e3
    x = X[2].copy()
    orc.layer_forward(dims, lw, x, 2, kc2, vc2)
    assert np.array_equal(x, outs[2])
    # zero output projections -> identity layer
    lz = dict(lw)
    lz["wo"] = np.zeros_like(lw["wo"])
    lz["w_down"] = np.zeros_like(lw["w_down"])
    x = X[0].copy()
    orc.layer_forward(dims, lz, x, 0, kc.copy(), vc.copy())
    assert np.array_equal(x, X[0])
    # position 0, MLP switched off: x + Wo * (v repeated per query group), v = Wv rmsnorm(x)
    lz = dict(lw)
    lz["w_down"] = np.zeros_like(lw["w_down"])
    x = X[0].copy()
    orc.layer_forward(dims, lz, x, 0, kc.copy(), vc.copy())
    h = F.rms_norm(torch.from_numpy(X[0]).double(), (s["hidden"],),
                   torch.from_numpy(lw["attn_norm"]).double(), s["rms_eps"]).numpy()
    v = (lw["wv"].astype(np.float64) @ h).reshape(s["n_kv"], s["head_dim"])
    o = np.repeat(v, s["n_q"] // s["n_kv"], axis=0).reshape(-1)
    assert np.allclose(x, X[0] + lw["wo"].astype(np.float64) @ o, atol=1e-5)


def test_model_zero_layers_is_one_matvec_and_batch_invariance():
    s, dims, w, wn = _tiny()
    m0 = orc.OracleModel(dims, dict(wn, layers=[]), max_ctx=8)
    z = m0.forward_token(0, 17)
    h = F.rms_norm(w["embed"][17].double(), (s["hidden"],), w["final_norm"].double(), s["rms_eps"])
    assert np.allclose(z, (w["lm_head"].double() @ h).numpy(), atol=1e-5)
    # a sequence's logits do not depend on other sequences being decoded in between
    toks = ri.tokens((2, 7), s["vocab"], 9, 60).numpy()
    ma = orc.OracleModel(dims, wn, max_ctx=8)
    za = [ma.forward_token(0, int(t)) for t in toks[0]]
    mb = orc.OracleModel(dims, wn, max_ctx=8)
    zb = []
    for t0, t1 in zip(toks[0], toks[1]):
        mb.forward_token(1, int(t1))
        zb.append(mb.forward_token(0, int(t0)))
    assert all(np.array_equal(a, b) for a, b in zip(za, zb))
    # prefill() is the same chain
    mc = orc.OracleModel(dims, wn, max_ctx=8)
    assert np.array_equal(mc.prefill(0, toks[0]), za[-1])


def test_model_step_is_the_composition_of_its_pinned_parts():
    """orc_model_forward_token (embedding row, the layers in order with their own caches, final norm, output matrix)
    against the same chain assembled here from the separately pinned functions: equal bits, logits and last residual
    stream, over several positions of two interleaved sequences; a wrong layer order, cache or position would show."""
    s, dims, w, wn = _tiny()
    m = orc.OracleModel(dims, wn, max_ctx=8)
    toks = ri.tokens((2, 6), s["vocab"], 9, 61).numpy()
    caches = {q: ([np.zeros((8, s["n_kv"], s["head_dim"]), np.float32) for _ in wn["layers"]],
                  [np.zeros((8, s["n_kv"], s["head_dim"]), np.float32) for _ in wn["layers"]]) for q in (0, 1)}
    for pos in range(6):
        for q in (1, 0):
            tok = int(toks[q, pos])
            z, hid = m.forward_token(q, tok, want_hidden=True)
            x = wn["embed"][tok].copy()
            for l, lw in enumerate(wn["layers"]):
                orc.layer_forward(dims, lw, x, pos, caches[q][0][l], caches[q][1][l])
            assert np.array_equal(hid, x)
            assert np.array_equal(z, orc.matvec(wn["lm_head"], orc.rmsnorm(x, wn["final_norm"], s["rms_eps"])))
    # swapping two layers changes the result (the order is observable)
    swapped = orc.OracleModel(dims, dict(wn, layers=wn["layers"][::-1]), max_ctx=8)
    assert not np.array_equal(swapped.forward_token(0, int(toks[0, 0])), orc.OracleModel(dims, wn, max_ctx=8).forward_token(0, int(toks[0, 0])))
