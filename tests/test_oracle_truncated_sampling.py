"""CPU pins of the oracle's truncated sampling (top-k / top-p; settings of Appendix D: 0.6 / 0.95 and 0.7 / 0.8).

The oracle's cuts are checked against what the definition fixes, computed here with Python integers and numpy in
double precision: exact integer masses, minimality of the kept prefix, the k largest logits with ties by index,
draw frequencies against the renormalised softmax, and the special cases that reduce to plain sampling / argmax."""
import math

import numpy as np
import pytest

import rollout_inputs as ri
from oracle import oracle as orc


def _logits(n, seed, scale=3.0):
    return (ri.normal((n,), scale, ri.BASE_SEED, seed).numpy()).astype(np.float32)


def test_order_key_is_the_total_order_of_the_values():
    vals = np.array([-np.inf, -3.5, -1e-30, -0.0, 0.0, 1e-30, 1.0, 1.0000001, 7e37, np.inf], np.float32)
    keys = [orc.order_key(v) for v in vals]
    assert keys == sorted(keys) and len(set(keys)) == len(keys)          # strictly increasing, -0 before +0
    r = _logits(2000, 501)
    k = np.array([orc.order_key(v) for v in r], np.uint64)
    assert np.array_equal(np.argsort(k, kind="stable"), np.argsort(r, kind="stable"))


def test_fexp_weight_against_libm():
    assert orc.fexp_weight(0.0) == 2 ** 32
    assert orc.fexp_weight(-22.0) == 0 and orc.fexp_weight(-1e30) == 0 and orc.fexp_weight(-math.inf) == 0
    assert orc.fexp_weight(-21.99) in (0, 1)                              # 2^32 e^-21.99 = 1.2
    worst = 0.0
    for x in np.concatenate([np.linspace(-21.99, 0.0, 40001), -np.logspace(-8, 1.3, 2000)]).astype(np.float32):
        w = orc.fexp_weight(x)
        exact = math.exp(float(x)) * 2 ** 32
        assert w <= exact * (1 + 5e-7) and w > exact * (1 - 5e-7) - 1, (x, w, exact)   # truncation: at most one below
        worst = max(worst, abs(w + 0.5 - exact) / exact if exact > 1e8 else 0.0)
    assert worst < 4e-7
    # one ulp above zero (the maximum's product may round down): still close to 2^32 and representable
    assert abs(orc.fexp_weight(np.float32(1e-6)) / 2 ** 32 - 1) < 2e-6


def _masses(z, invT):
    s_max = np.float32(np.float32(z.max()) * np.float32(invT))
    x = (z.astype(np.float64) * float(np.float32(invT)) - float(s_max)).astype(np.float32)   # exact in double, one rounding
    return [orc.fexp_weight(v) for v in x]


def _order(z):
    keys = np.array([orc.order_key(v) for v in z], np.int64)
    return np.lexsort((np.arange(z.size), -keys))                            # descending value, ascending index


@pytest.mark.parametrize("T,top_k,top_p", [(1.0, 0, 0.9), (0.6, 0, 0.95), (0.7, 0, 0.8), (1.0, 20, 0.5), (1.3, 7, 0.999),
                                           (1.0, 0, 1e-4), (0.25, 0, 0.3)])
def test_kept_set_is_the_minimal_prefix(T, top_k, top_p):
    for seed in range(6):
        z = _logits(300, 510 + seed)
        z[17] = z[5]                                                         # a tie in the order
        invT = float(np.float32(1.0) / np.float32(T))
        keep = orc.truncation(z, invT, top_k, top_p).astype(bool)
        order = _order(z)
        n = int(keep.sum())
        assert keep[order[:n]].all() and n >= 1                              # a prefix of the order
        w = _masses(z, invT)
        K = top_k if 0 < top_k < z.size else z.size
        assert n <= K
        S = sum(w[i] for i in order[:K])
        P = int(float(np.float32(top_p)) * 2 ** 32)
        Tm = max(1, (P * S) >> 32)
        got = sum(w[i] for i in order[:n])
        assert got >= Tm and got - w[order[n - 1]] < Tm                      # reaches the target, and not without its last token
        # the same statement in double precision about probabilities
        pr = np.exp(z[order[:K]].astype(np.float64) * invT)
        pr /= pr.sum()
        assert pr[:n].sum() >= top_p - 1e-6 and pr[:n - 1].sum() < top_p + 1e-6


def test_top_k_keeps_the_k_largest_with_ties_by_index():
    z = _logits(500, 520)
    z[[3, 40, 41, 300]] = 1.25                                               # four equal logits straddling the cut
    order = _order(z)
    rank = int(np.where(order == 40)[0][0])                                  # 3 then 40, 41, 300 in the order
    assert list(order[rank - 1:rank + 3]) == [3, 40, 41, 300]
    for k in (rank, rank + 1, rank + 2, rank + 3, 1, 499, 500, 0, 10 ** 6):
        keep = orc.truncation(z, 1.0, k, 0.0).astype(bool)
        kk = k if 0 < k < 500 else 500
        assert keep.sum() == kk and keep[order[:kk]].all()
    zz = np.zeros(64, np.float32)                                            # all equal: the lowest indices win
    assert list(np.nonzero(orc.truncation(zz, 1.0, 5, 0.0))[0]) == [0, 1, 2, 3, 4]
    zz[10] = -0.0                                                            # -0 sorts after +0
    assert orc.truncation(zz, 1.0, 63, 0.0)[10] == 0
    keep = orc.truncation(zz, 1.0, 0, 0.5)                                   # mass: 32 of 64 equal tokens reach one half
    assert keep.sum() == 32 and keep[:33].sum() == 32 and keep[10] == 0      # indices 0..32 without the -0 at 10


def test_truncated_draws_follow_the_renormalised_distribution():
    z = _logits(12, 530, scale=1.5)
    for T, k, p in [(1.0, 5, 0.0), (0.6, 0, 0.95), (0.7, 0, 0.8), (1.0, 8, 0.7)]:
        invT = float(np.float32(1.0) / np.float32(T))
        keep = orc.truncation(z, invT, k, p).astype(bool)
        pr = np.where(keep, np.exp(z.astype(np.float64) * invT), 0.0)
        pr /= pr.sum()
        n = 20000
        cnt = np.zeros(12)
        for t in range(n):
            tok, lp, kept = orc.sample_truncated(z, T, k, p, 77, 3, t)
            assert keep[tok] and kept == keep.sum()
            assert abs(lp - math.log(pr[tok])) < 1e-9
            cnt[tok] += 1
        assert np.all(np.abs(cnt / n - pr) < 4.5 * np.sqrt(pr * (1 - pr) / n) + 1e-9), (T, k, p)
        assert cnt[~keep].sum() == 0


def test_truncation_special_cases():
    z = _logits(4096, 540)
    am = int(np.argmax(z))
    for pos in range(20):
        assert orc.sample_truncated(z, 1.0, 1, 0.0, 5, 1, pos)[:2] == (am, 0.0)          # top-1: the argmax, probability one
        assert orc.sample_truncated(z, 0.8, 0, 1e-9, 5, 1, pos)[0] == am                 # a vanishing p keeps one token
        tok, lp = orc.sample(z, 0.9, 5, 1, pos)                                          # no cut: plain sampling
        assert orc.sample_truncated(z, 0.9, 0, 1.0, 5, 1, pos) == (tok, lp, 4096)
        assert orc.sample_truncated(z, 0.9, 0, 0.0, 5, 1, pos) == (tok, lp, 4096)
        assert orc.sample_truncated(z, 0.9, 4096, 0.0, 5, 1, pos) == (tok, lp, 4096)
        g, lpg = orc.sample(z, 0.0, 5, 1, pos)
        assert orc.sample_truncated(z, 0.0, 3, 0.5, 5, 1, pos) == (g, lpg, 4096)         # greedy ignores the cuts
    # forced tokens: inside the kept set the renormalised log-probability, outside minus infinity
    keep = orc.truncation(z, 1.0, 50, 0.0).astype(bool)
    inside, outside = int(np.nonzero(keep)[0][7]), int(np.nonzero(~keep)[0][0])
    pr = np.where(keep, np.exp(z.astype(np.float64)), 0.0)
    tok, lp, _ = orc.sample_truncated(z, 1.0, 50, 0.0, 5, 1, 0, forced=inside)
    assert tok == inside and abs(lp - math.log(pr[inside] / pr.sum())) < 1e-9
    tok, lp, _ = orc.sample_truncated(z, 1.0, 50, 0.0, 5, 1, 0, forced=outside)
    assert tok == outside and lp == -math.inf
    # a draw with a cut equals the plain draw whenever the plain draw falls inside the kept set
    same = 0
    for pos in range(200):
        t0, _ = orc.sample(z, 1.0, 9, 2, pos)
        t1, _, _ = orc.sample_truncated(z, 1.0, 50, 0.0, 9, 2, pos)
        assert keep[t1] and (t1 == t0 or not keep[t0])
        same += t1 == t0
    assert 0 < same < 200
