"""GPU parity of the HRD / uniform GRPO objective kernel against the CPU oracle (through the C boundary)."""
import numpy as np
import pytest
import torch

import rollout_inputs as ri
from oracle import oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(n_prompts, G, lo, hi, seed, vocab=1000, delim=7):
    n = n_prompts * G
    lens = ri.lengths(n, lo, hi, seed, 1).numpy()
    lens[0] = lo                                        # shortest and longest outputs are present
    lens[-1] = hi
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(off[-1])
    toks = ri.tokens((total,), vocab, seed, 2).numpy()
    toks[toks == delim] = delim + 1
    n_plan = np.zeros(n, np.int32)
    for k in range(n):                                  # one delimiter somewhere, except in every fifth output
        if k % 5 != 4 and lens[k] > 0:
            p = int(ri.lengths(1, 0, int(lens[k]) - 1, seed, 100 + k))
            toks[off[k] + p] = delim
            n_plan[k] = p + 1
        else:
            n_plan[k] = lens[k]
    lp_old = (-ri.normal((total,), 1.0, seed, 3).abs() - 0.1).numpy()
    lp_new = lp_old + ri.normal((total,), 0.25, seed, 4).numpy()
    rs = ri.normal((n,), 0.6, seed, 5).abs().clamp(max=2.0).numpy()       # speedup reward, clipped at 2
    rc = (ri.normal((n,), 1.0, seed, 6) > 0).float().numpy()              # correctness reward in {0, 1}
    return off, toks, n_plan, lp_new.astype(np.float32), lp_old.astype(np.float32), rs, rc


@pytest.mark.parametrize("n_prompts,G,lo,hi", [(3, 4, 1, 40), (32, 8, 64, 16384), (1, 1, 1, 1), (2, 2, 0, 300)])
def test_objective_matches_oracle(n_prompts, G, lo, hi):
    from paper_2510_17891_amd import binding as B
    off, toks, n_plan, lp_new, lp_old, rs, rc = _case(n_prompts, G, lo, hi, seed=n_prompts * 10 + G)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    for mode, alpha, beta in [(0, 0.1, 0.0), (0, 1.0, 0.0), (1, 0.1, 0.9), (1, 0.1, 0.0)]:
        J_ref, seq_ref = orc.hrd_objective(n_prompts, G, off, n_plan, lp_new, lp_old, rs, rc, alpha, 0.2, beta, mode)
        for given in (True, False):
            out, seq, npl = B.rl_hrd_objective(n_prompts, G, d(off), d(lp_new), d(lp_old), d(rs), d(rc), alpha, 0.2,
                                               beta, mode, n_plan=d(n_plan) if given else None,
                                               tokens=None if given else d(toks), delimiter_token=7)
            torch.cuda.synchronize()
            assert np.array_equal(npl.cpu().numpy(), n_plan)               # integer work: exact
            scale = max(1e-6, np.abs(seq_ref).max())
            assert np.abs(seq.cpu().numpy() - seq_ref).max() < 2e-5 * scale, (mode, given)
            assert abs(float(out) - J_ref) < 2e-5 * scale
    # plan lengths agree with the oracle's scan of the token ids
    for k in range(0, n_prompts * G, max(1, n_prompts * G // 7)):
        assert orc.plan_length(toks[off[k]:off[k + 1]], 7) == n_plan[k]
    # reproducible bits
    a = B.rl_hrd_objective(n_prompts, G, d(off), d(lp_new), d(lp_old), d(rs), d(rc), n_plan=d(n_plan))[0]
    b = B.rl_hrd_objective(n_prompts, G, d(off), d(lp_new), d(lp_old), d(rs), d(rc), n_plan=d(n_plan))[0]
    assert torch.equal(a, b)


def test_objective_on_a_real_rollout_is_the_ratio_one_closed_form():
    """Rollout with grouped sampling, rescoring with the same weights: s = 1, so J reduces to the reward algebra."""
    import paper_2510_17891_amd as amd
    from helpers import make_both, to_device
    shape = ri.SHAPES["tiny"]
    w, _ = make_both(shape, 81)
    ro = amd.Rollout(shape, to_device(w), max_seqs=8, max_ctx=64, max_rows=16, kv_pages=24)
    G, n_new, seed = 4, 12, 3
    prompts = [ri.tokens((9,), shape["vocab"], 81, 1).tolist(), ri.tokens((20,), shape["vocab"], 81, 2).tolist()]
    ids = list(range(2 * G))
    tok, lp = ro.rl_prefill_groups(ids, G, prompts, 1.0, seed)
    toks, lps = [tok], [lp]
    for _ in range(n_new - 1):
        tok, lp = ro.rl_decode_step(ids, tok, 1.0, seed)
        toks.append(tok)
        lps.append(lp)
    toks, lp_old = torch.stack(toks, 1).contiguous(), torch.stack(lps, 1).contiguous()   # [8, n_new]
    ro.rl_free_seqs(ids)
    full = [prompts[i // G] + toks[i].tolist() for i in ids]
    sc = ro.rl_score(ids, full, 1.0)
    lp_new = torch.stack([sc[sum(len(f) - 1 for f in full[:i]) + len(prompts[i // G]) - 1:][:n_new] for i in ids]).contiguous()
    off = torch.arange(0, (2 * G + 1) * n_new, n_new, dtype=torch.int32, device=DEV)
    n_plan = torch.tensor([5, 12, 0, 7, 1, 2, 3, 4], dtype=torch.int32, device=DEV)
    rs = torch.tensor([2.0, 0.5, 0.0, 1.0, 0.0, 0.0, 1.5, 0.3], device=DEV)
    rc = torch.tensor([1.0, 0.0, 0.0, 1.0, 0.0, 1.0, 1.0, 0.0], device=DEV)
    out, seq, _ = amd.binding.rl_hrd_objective(2, G, off, lp_new.view(-1), lp_old.view(-1), rs, rc, alpha=0.1, n_plan=n_plan)
    As = (rs.view(2, G) - rs.view(2, G).mean(1, keepdim=True)).view(-1)
    Ac = (rc.view(2, G) - rc.view(2, G).mean(1, keepdim=True)).view(-1)
    want = (0.1 * n_plan * As + (n_new - n_plan) * Ac) / n_new
    assert torch.allclose(seq, want, atol=1e-5)
    assert abs(float(out) - float(want.mean())) < 1e-5
    ro.close()


def test_objective_plan_counts_outside_the_output_are_clamped_and_errors_carry_text():
    """A plan count below zero or above the output's length reads as "no plan token" / "all plan": the same value the
    oracle gives (its test `t < n_plan` treats them so).  Failing calls leave a message for rl_last_error."""
    from paper_2510_17891_amd import binding as B
    off, toks, n_plan, lp_new, lp_old, rs, rc = _case(3, 4, 1, 40, seed=7)
    lens = np.diff(off)
    wild = n_plan.copy()
    wild[0], wild[1], wild[2] = -5, lens[1] + 1000, 2 ** 31 - 1
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    J_ref, seq_ref = orc.hrd_objective(3, 4, off, wild, lp_new, lp_old, rs, rc, 0.1, 0.2, 0.0, 0)
    out, seq, npl = B.rl_hrd_objective(3, 4, d(off), d(lp_new), d(lp_old), d(rs), d(rc), n_plan=d(wild))
    torch.cuda.synchronize()
    assert np.array_equal(npl.cpu().numpy(), np.clip(wild, 0, lens))
    scale = max(1e-6, np.abs(seq_ref).max())
    assert np.abs(seq.cpu().numpy() - seq_ref).max() < 2e-5 * scale and abs(float(out) - J_ref) < 2e-5 * scale
    with pytest.raises(B.RLError) as e:
        B.rl_hrd_objective(3, 4, d(off), d(lp_new), d(lp_old), d(rs), d(rc), mode=2, n_plan=d(n_plan))
    assert e.value.status == B.RL_ERR_INVALID_ARG and "mode 2" in str(e.value)
    with pytest.raises(B.RLError) as e:
        B.rl_hrd_objective(3, 4, d(off), d(lp_new), d(lp_old), d(rs), d(rc))
    assert e.value.status == B.RL_ERR_INVALID_ARG and "neither n_plan nor tokens" in str(e.value)
