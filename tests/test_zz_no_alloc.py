"""rl_sample_logits_static -- the sampler entry point that allocates nothing (its scratch is a static device array
inside the library) -- against rl_sample_logits, whose scratch comes from a model's workspace.

Two calls in a row on one stream, the second with a smaller input (fewer rows, smaller vocabulary), so that what the
first call left in the shared array must not leak into the second.  Bars: token ids bit-exact, log-probabilities
within 1e-5 (here they are the same kernels, so the bits are equal too); the ids are also checked against the oracle.
"""
import numpy as np
import pytest
import torch

import rollout_inputs as ri
from helpers import make_both, to_device
from oracle import oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _model(amd, vocab):
    shape = dict(ri.SHAPES["tiny"], n_layers=1, vocab=vocab)
    w, _ = make_both(shape, 11)
    return amd.Rollout(shape, to_device(w), max_seqs=64, max_ctx=64, max_rows=16, kv_pages=8)


def test_static_sampler_equals_workspace_sampler_twice_in_a_row():
    import paper_2510_17891_amd as amd
    B = amd.binding
    big_v, small_v = 151936, 4096
    z_big = ri.normal((7, big_v), 1.3, 5, 70)
    z_big[1, 17] = z_big[1, 900] = 9.0
    z_big[3, 5] = float("-inf")
    z_small = ri.normal((3, small_v), 1.3, 5, 71)
    seq_big, pos_big = [3, 0, 7, 63, 1, 2, 9], [0, 1, 65535, 77, 2048, 16383, 5]
    seq_small, pos_small = [4, 8, 1], [12, 0, 300]
    forced_big = torch.tensor([5, -1, 0, big_v - 1, -1, 3, -1], dtype=torch.int32, device=DEV)
    zb, zs = z_big.to(DEV), z_small.to(DEV)
    i32 = lambda v: torch.tensor(v, dtype=torch.int32, device=DEV)
    sb, pb, ss, ps = i32(seq_big), i32(pos_big), i32(seq_small), i32(pos_small)
    ro_big, ro_small = _model(amd, big_v), _model(amd, small_v)
    for T, seed, forced in [(1.0, 1234, None), (0.7, 99, forced_big), (0.0, 5, None)]:
        # the two static calls back to back, nothing between them
        tb, lb = B.rl_sample_logits_static(zb, sb, pb, T, seed, forced=forced)
        ts, ls = B.rl_sample_logits_static(zs, ss, ps, T, seed)
        torch.cuda.synchronize()
        rb_t, rb_l = ro_big.rl_sample_logits(zb, seq_big, pos_big, T, seed, forced=forced)
        rs_t, rs_l = ro_small.rl_sample_logits(zs, seq_small, pos_small, T, seed)
        torch.cuda.synchronize()
        assert torch.equal(tb, rb_t) and torch.equal(ts, rs_t), (T, seed)
        assert torch.equal(lb, rb_l) and torch.equal(ls, rs_l), (T, seed)
        for r in range(3):                                   # and the oracle agrees on the smaller call
            t_ref, lp_ref = orc.sample(z_small[r].numpy(), T, seed, seq_small[r], pos_small[r])
            assert int(ts[r]) == t_ref and abs(float(ls[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref))
        for r in range(7):
            f = -1 if forced is None else int(forced[r])
            t_ref, lp_ref = orc.sample(z_big[r].numpy(), T, seed, seq_big[r], pos_big[r], forced=f)
            assert int(tb[r]) == t_ref
            assert abs(float(lb[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref))
    # limits and unsupported settings are refused with a message, before anything is launched
    with pytest.raises(B.RLError) as e:
        B.rl_sample_logits_static(torch.zeros(257, 8, device=DEV), i32([0] * 257), i32([0] * 257), 1.0, 1)
    assert e.value.status == B.RL_ERR_INVALID_ARG and "static scratch" in str(e.value)
    with pytest.raises(B.RLError) as e:
        B.rl_sample_logits_static(zs, ss, ps, 1.0, 1, top_p=0.9)
    assert e.value.status == B.RL_ERR_UNSUPPORTED
    with pytest.raises(B.RLError) as e:
        B.rl_sample_logits_static(torch.zeros(2, 6, device=DEV), i32([0, 1]), i32([0, 0]), 1.0, 1)
    assert e.value.status == B.RL_ERR_INVALID_ARG
    ro_big.close()
    ro_small.close()
