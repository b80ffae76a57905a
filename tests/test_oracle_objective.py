"""Pins of the oracle's policy objective (HRD and uniform-reward GRPO) against closed forms and hand-worked cases.

The paper prints no numeric example of the objective; the pins are its algebra: ratio one, zero-sum group
advantages, the four clip cases, class weights, the 1/|o| normalisation over the whole output.
"""
import math

import numpy as np

from oracle import oracle as orc

rng = np.random.default_rng(3)


def _batch(n_prompts=3, G=4, max_len=12):
    lens = rng.integers(1, max_len, n_prompts * G)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n_plan = np.array([rng.integers(0, l + 1) for l in lens], np.int32)
    lp_old = rng.normal(-2, 1, off[-1]).astype(np.float32)
    lp_new = (lp_old + rng.normal(0, 0.3, off[-1])).astype(np.float32)
    rs = rng.uniform(0, 2, n_prompts * G).astype(np.float32)
    rc = rng.integers(0, 2, n_prompts * G).astype(np.float32)
    return n_prompts, G, off, n_plan, lp_new, lp_old, rs, rc, lens


def test_ratio_one_closed_form_and_zero_sum_advantages():
    n, G, off, n_plan, lp_new, lp_old, rs, rc, lens = _batch()
    J, seq = orc.hrd_objective(n, G, off, n_plan, lp_old, lp_old, rs, rc, alpha=0.1)
    rs64, rc64 = rs.astype(np.float64), rc.astype(np.float64)
    As = rs64.reshape(n, G) - rs64.reshape(n, G).mean(1, keepdims=True)
    Ac = rc64.reshape(n, G) - rc64.reshape(n, G).mean(1, keepdims=True)
    assert np.allclose(As.sum(1), 0, atol=1e-6) and np.allclose(Ac.sum(1), 0, atol=1e-6)
    want = (0.1 * n_plan * As.ravel() + (lens - n_plan) * Ac.ravel()) / lens   # s = 1: every term is A
    assert np.allclose(seq, want, atol=1e-9)
    assert abs(J - want.reshape(n, G).mean(1).mean()) < 1e-12
    # identical rewards inside every group -> no signal at all
    J0, _ = orc.hrd_objective(n, G, off, n_plan, lp_new, lp_old, np.ones(n * G), np.ones(n * G))
    assert J0 == 0.0


def test_clip_cases_worked_by_hand():
    # one prompt, two outputs of one code token each (n_plan = 0), rewards (1, 0) -> A = (+0.5, -0.5), eps = 0.2
    off, n_plan = [0, 1, 2], [0, 0]
    rc, rs = [1.0, 0.0], [0.0, 0.0]

    def J(s0, s1):
        lp_new = np.log(np.array([s0, s1], np.float64)).astype(np.float32)
        return orc.hrd_objective(1, 2, off, n_plan, lp_new, np.zeros(2, np.float32), rs, rc, eps=0.2)[0]
    assert abs(J(1.5, 1.0) - 0.5 * (0.5 * 1.2 - 0.5 * 1.0)) < 1e-7     # A>0, s above the clip: capped at 1+eps
    assert abs(J(0.5, 1.0) - 0.5 * (0.5 * 0.5 - 0.5 * 1.0)) < 1e-7     # A>0, s below: not clipped (min takes A*s)
    assert abs(J(1.0, 0.5) - 0.5 * (0.5 * 1.0 - 0.5 * 0.8)) < 1e-7     # A<0, s below the clip: capped at 1-eps
    assert abs(J(1.0, 1.5) - 0.5 * (0.5 * 1.0 - 0.5 * 1.5)) < 1e-7     # A<0, s above: not clipped
    assert abs(J(1.1, 0.7) - 0.5 * (0.5 * 1.1 - 0.5 * 0.8)) < 1e-7     # just inside / just outside the band
    assert abs(J(1.3, 0.9) - 0.5 * (0.5 * 1.2 - 0.5 * 0.9)) < 1e-7


def test_class_split_weights_and_length_normalisation():
    # one prompt, G = 2; output 0 has 4 tokens (3 plan, 1 code), output 1 has 2 tokens (all code)
    off, n_plan = [0, 4, 6], [3, 0]
    rs, rc = [2.0, 0.0], [1.0, 0.0]           # A^plan = (+1, -1), A^code = (+0.5, -0.5)
    z = np.zeros(6, np.float32)
    for alpha in (0.0, 0.1, 1.0):
        J, seq = orc.hrd_objective(1, 2, off, n_plan, z, z, rs, rc, alpha=alpha)
        # 1/|o| runs over the whole output even for the class-restricted sums
        assert abs(seq[0] - (alpha * 3 * 1.0 + 1 * 0.5) / 4) < 1e-12
        assert abs(seq[1] - (2 * -0.5) / 2) < 1e-12
        assert abs(J - 0.5 * (seq[0] + seq[1])) < 1e-12
    # speedup reward only reaches plan tokens, correctness reward only code tokens
    J_a, _ = orc.hrd_objective(1, 2, off, [0, 0], z, z, rs, [0.0, 0.0])
    J_b, _ = orc.hrd_objective(1, 2, off, [4, 2], z, z, [0.0, 0.0], rc)
    assert J_a == 0.0 and J_b == 0.0


def test_uniform_mode_matches_its_printed_form():
    n, G, off, n_plan, lp_new, lp_old, rs, rc, lens = _batch(2, 3)
    beta, eps = 0.9, 0.2
    J, seq = orc.hrd_objective(n, G, off, n_plan, lp_new, lp_old, rs, rc, eps=eps, beta=beta, mode=1)
    r = beta * rc.astype(np.float64) + (1 - beta) * rs.astype(np.float64)
    A = (r.reshape(n, G) - r.reshape(n, G).mean(1, keepdims=True)).ravel()
    s = np.exp(lp_new.astype(np.float64) - lp_old)
    m = np.minimum(s, np.clip(s, 1 - eps, 1 + eps))          # the appendix puts the advantage outside the min
    want = np.array([A[k] * m[off[k]:off[k + 1]].mean() for k in range(n * G)])
    assert np.allclose(seq, want, atol=1e-9) and abs(J - want.mean()) < 1e-9
    # the class split plays no role in uniform mode
    J2, _ = orc.hrd_objective(n, G, off, np.zeros_like(n_plan), lp_new, lp_old, rs, rc, eps=eps, beta=beta, mode=1)
    assert J2 == J
    # with a single class, alpha = 1 and positive advantages only the two objectives coincide
    rs1 = np.tile(np.array([1.0, 0.0, 0.0], np.float32), n)
    Jh, seqh = orc.hrd_objective(n, G, off, np.diff(off), lp_new, lp_old, rs1, rs1, alpha=1.0, eps=eps)
    Ju, sequ = orc.hrd_objective(n, G, off, n_plan, lp_new, lp_old, rs1, rs1, eps=eps, beta=0.5, mode=1)
    assert np.allclose(seqh[0::3], sequ[0::3], atol=1e-12)   # outputs with A > 0


def test_objective_is_linear_in_rewards_and_shift_invariant():
    n, G, off, n_plan, lp_new, lp_old, rs, rc, lens = _batch()
    J1, _ = orc.hrd_objective(n, G, off, n_plan, lp_new, lp_old, rs, rc)
    J2, _ = orc.hrd_objective(n, G, off, n_plan, lp_new, lp_old, rs + 5.0, rc - 3.0)   # group baseline removes shifts
    assert abs(J1 - J2) < 1e-5
    J3, _ = orc.hrd_objective(n, G, off, n_plan, lp_new, lp_old, 2 * rs, 2 * rc)
    assert abs(J3 - 2 * J1) < 1e-6
    # adding the same constant to lp_new and lp_old leaves the ratio unchanged
    J4, _ = orc.hrd_objective(n, G, off, n_plan, lp_new - 1.0, lp_old - 1.0, rs, rc)
    assert abs(J4 - J1) < 1e-5


def test_plan_length_from_delimiter():
    assert orc.plan_length([5, 9, 7, 9, 1], 9) == 2          # up to and including the first delimiter
    assert orc.plan_length([5, 1, 7], 9) == 3                # no delimiter: everything is plan
    assert orc.plan_length([9], 9) == 1
    assert orc.plan_length([], 9) == 0
