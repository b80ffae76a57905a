"""GPU parity: the HIP path, called through the C boundary, against the CPU oracle on the same seeded inputs.

Bars: sampled ids bit-exact given the same logits and RNG counters; fp32 logits within 1e-4 (max |diff| over
max |ref| per row); bf16 logits / layer outputs within 3e-2 on the same bf16-rounded weights with >= 99 %
argmax agreement; log-probabilities within 1e-5 (fp32 logits).
"""
import numpy as np
import pytest
import torch

import rollout_inputs as ri
from helpers import ArgmaxCount, dims_of, make_both, rel_inf, to_device
from oracle import oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def amd():
    import paper_2510_17891_amd as pkg
    pkg.lib()
    return pkg


# ------------------------------------------------------------------------------------------------ sampler
def _sampler_model(amd, vocab, bf16):
    if bf16:
        shape = dict(ri.SHAPES["layer8b"], n_layers=1, hidden=256, n_q=2, n_kv=1, ffn=256, vocab=vocab)
    else:
        shape = dict(ri.SHAPES["tiny"], n_layers=1, vocab=vocab)
    w, _ = make_both(shape, 11)
    return amd.Rollout(shape, to_device(w), max_seqs=64, max_ctx=64, max_rows=16, kv_pages=8)


@pytest.mark.parametrize("vocab,bf16", [(4096, False), (151936, True), (1000, False)])
def test_sampler_bit_exact_and_logprob(amd, vocab, bf16):
    ro = _sampler_model(amd, vocab, bf16)
    n = 6
    z = ri.normal((n, vocab), 1.3, 5, 70)
    z[1, 17] = z[1, 900] = 9.0           # an exact tie far above the rest (greedy must take the lower index)
    z[2, :] = 0.25                       # all equal: only the noise decides
    z[3, 5] = float("-inf")
    zd = z.to(DEV)
    seqs, poss = [3, 0, 7, 63, 1, 2], [0, 1, 65535, 77, 2048, 16383]
    for T, seed in [(1.0, 1234), (0.7, 99), (0.0, 5), (1.0, 2 ** 63 + 12345)]:
        tok, lp = ro.rl_sample_logits(zd, seqs, poss, T, seed)
        torch.cuda.synchronize()
        for r in range(n):
            t_ref, lp_ref = orc.sample(z[r].numpy(), T, seed, seqs[r], poss[r])
            assert int(tok[r]) == t_ref, (T, seed, r)
            assert abs(float(lp[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref)), (T, r, float(lp[r]), lp_ref)
    forced = torch.tensor([5, -1, 0, vocab - 1, -1, 3], dtype=torch.int32, device=DEV)
    tok, lp = ro.rl_sample_logits(zd, seqs, poss, 1.0, 1234, forced=forced)
    torch.cuda.synchronize()
    for r in range(n):
        t_ref, lp_ref = orc.sample(z[r].numpy(), 1.0, 1234, seqs[r], poss[r], forced=int(forced[r]))
        assert int(tok[r]) == t_ref
        if np.isfinite(lp_ref):
            assert abs(float(lp[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref))
        else:
            assert float(lp[r]) == lp_ref
    ro.close()


# ------------------------------------------------------------------------------- fp32 tiny model, end to end
def test_tiny_fp32_greedy_rollout_matches_oracle(amd):
    """4 prompts x 64 tokens, greedy decode of 32 tokens: every token identical, logits within 1e-4."""
    shape = ri.SHAPES["tiny"]
    w, wn = make_both(shape, ri.BASE_SEED + 1)
    ro = amd.Rollout(shape, to_device(w), max_seqs=8, max_ctx=128, max_rows=64, kv_pages=40)
    ro.rl_debug_shuffle_free_pages(3)
    om = orc.OracleModel(dims_of(shape), wn, max_ctx=128)
    prompts = ri.tokens((4, 64), shape["vocab"], ri.BASE_SEED + 1, 900).tolist()
    seqs = [5, 0, 2, 7]
    tok, lp = ro.rl_prefill(seqs, prompts, 0.0, 0)        # prefill is chunked: 256 rows > max_rows = 64
    torch.cuda.synchronize()
    z0 = [om.prefill(s, p) for s, p in zip(seqs, prompts)]
    for i, s in enumerate(seqs):
        t_ref, lp_ref = orc.sample(z0[i], 0.0, 0, s, 64)
        assert int(tok[i]) == t_ref and abs(float(lp[i]) - lp_ref) < 2e-5
    logits = torch.empty(4, shape["vocab"], device=DEV)
    worst = 0.0
    for step in range(32):
        cur = tok
        tok, lp = ro.rl_decode_step(seqs, cur, 0.0, 0, debug_logits=logits)
        torch.cuda.synchronize()
        zg = logits.cpu().numpy()
        for i, s in enumerate(seqs):
            z = om.forward_token(s, int(cur[i]))
            worst = max(worst, float(rel_inf(zg[i], z)))
            t_ref, lp_ref = orc.sample(z, 0.0, 0, s, 65 + step)
            assert int(tok[i]) == t_ref, (step, i)
            assert abs(float(lp[i]) - lp_ref) < 2e-5
    assert worst < 1e-4, worst
    assert ro.rl_seq_len(5) == 96
    ro.rl_free_seqs(seqs)
    assert ro.rl_kv_stats() == (40, 40)
    ro.close()


def test_tiny_fp32_sampled_rollout_ids_bit_exact_given_logits(amd):
    """T = 1 sampling: with the GPU's own logits the oracle sampler reproduces every id; ragged prompts."""
    shape = dict(ri.SHAPES["tiny"], qk_norm=0)
    w, wn = make_both(shape, ri.BASE_SEED + 2)
    ro = amd.Rollout(shape, to_device(w), max_seqs=4, max_ctx=64, max_rows=4, kv_pages=12)
    om = orc.OracleModel(dims_of(shape), wn, max_ctx=64)
    lens = [1, 17, 16]
    prompts = [ri.tokens((n,), shape["vocab"], 3, 910 + i).tolist() for i, n in enumerate(lens)]
    seqs = [0, 1, 3]
    seed = 20251017
    tok, lp = ro.rl_prefill(seqs, prompts, 1.0, seed)
    torch.cuda.synchronize()
    for i, s in enumerate(seqs):
        z = om.prefill(s, prompts[i])
        t_ref, lp_ref = orc.sample(z, 1.0, seed, s, lens[i])
        assert int(tok[i]) == t_ref and abs(float(lp[i]) - lp_ref) < 2e-5
    logits = torch.empty(3, shape["vocab"], device=DEV)
    for step in range(20):
        cur = tok
        tok, lp = ro.rl_decode_step(seqs, cur, 1.0, seed, debug_logits=logits)
        torch.cuda.synchronize()
        zg = logits.cpu().numpy()
        for i, s in enumerate(seqs):
            z = om.forward_token(s, int(cur[i]))
            assert rel_inf(zg[i], z) < 1e-4
            t_ref, lp_ref = orc.sample(zg[i], 1.0, seed, s, lens[i] + step + 1)
            assert int(tok[i]) == t_ref
            assert abs(float(lp[i]) - lp_ref) < 1e-5
    ro.close()


@pytest.mark.parametrize("vocab,bf16", [(4096, False), (151936, True), (1000, False)])
def test_truncated_sampler_cut_and_draw_bit_exact(amd, vocab, bf16):
    """Top-k / top-p (Appendix D's sampling settings): the kept set is probed through forced tokens on both sides of
    the oracle's cut (finite log-probability inside, -inf outside), and the drawn ids equal the oracle's."""
    ro = _sampler_model(amd, vocab, bf16)
    n = 8
    z = ri.normal((n, vocab), 2.0, 6, 71)
    z[1, 17] = z[1, 900] = z[1, 333] = z[1, 4]          # equal logits that a cut can fall between
    z[2, :] = 0.25                                        # all equal: the lowest ids are kept
    z[3, 5] = float("-inf")
    z[4] *= 4.0                                           # peaked: top-p keeps a handful
    z[5] *= 0.05                                          # flat: top-p keeps almost everything
    z[6, 100:140] = z[6, 99]                              # a long run of ties
    z[7, 7] = -0.0
    z[7, 8] = 0.0
    zd = z.to(DEV)
    seqs, poss = [3, 0, 7, 63, 1, 2, 9, 11], [0, 1, 65535, 77, 2048, 16383, 5, 6]
    settings = [(0.6, 0, 0.95), (0.7, 0, 0.8), (1.0, 50, 0.0), (1.0, 1, 0.0), (1.3, 40, 0.9), (1.0, 0, 1e-6),
                (0.5, vocab - 1, 0.999), (1.0, 3, 0.5)]
    for T, k, p in settings:
        seed = 1000 + k
        tok, lp = ro.rl_sample_logits(zd, seqs, poss, T, seed, top_k=k, top_p=p)
        torch.cuda.synchronize()
        inside, outside = [], []
        for r in range(n):
            t_ref, lp_ref, kept = orc.sample_truncated(z[r].numpy(), T, k, p, seed, seqs[r], poss[r])
            assert int(tok[r]) == t_ref, (T, k, p, r, kept)
            assert abs(float(lp[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref)), (T, k, p, r, float(lp[r]), lp_ref)
            keep = orc.truncation(z[r].numpy(), float(np.float32(1.0) / np.float32(T)), k, p).astype(bool)
            keys = np.array([orc.order_key(v) for v in z[r].numpy()], np.int64)
            order = np.lexsort((np.arange(vocab), -keys))
            assert keep[order[:kept]].all() and kept == keep.sum()
            inside.append(int(order[kept - 1]))                          # last kept token
            outside.append(int(order[kept]) if kept < vocab else -1)     # first one cut
        for forced in (inside, outside):
            f = torch.tensor(forced, dtype=torch.int32, device=DEV)
            tok, lp = ro.rl_sample_logits(zd, seqs, poss, T, seed, forced=f, top_k=k, top_p=p)
            torch.cuda.synchronize()
            for r in range(n):
                t_ref, lp_ref, _ = orc.sample_truncated(z[r].numpy(), T, k, p, seed, seqs[r], poss[r], forced=forced[r])
                assert int(tok[r]) == t_ref
                if np.isfinite(lp_ref):
                    assert abs(float(lp[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref)), (T, k, p, r)
                else:
                    assert float(lp[r]) == lp_ref, (T, k, p, r, forced[r], float(lp[r]))
    # no cut requested, or greedy: exactly the plain sampler
    for T, k, p in [(0.9, 0, 1.0), (0.9, vocab, 0.0), (0.0, 5, 0.5)]:
        a = ro.rl_sample_logits(zd, seqs, poss, T, 77, top_k=k, top_p=p)
        b = ro.rl_sample_logits(zd, seqs, poss, T, 77)
        torch.cuda.synchronize()
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    ro.close()


def test_fork_errors_and_long_run_of_steps(amd):
    """rl_seq_fork's error paths leave the pool untouched; a forked sequence continues exactly like its source
    (fp32: same logits at the same position); 200 steps run through the 64-slot metadata ring several times."""
    B = amd.binding
    shape = ri.SHAPES["tiny"]
    w, wn = make_both(shape, 52)
    ro = amd.Rollout(shape, to_device(w), max_seqs=6, max_ctx=256, max_rows=6, kv_pages=48)
    p = ri.tokens((21,), shape["vocab"], 52, 941).tolist()
    tok, _ = ro.rl_prefill([0], [p], 0.0, 0)
    free0 = ro.rl_kv_stats()[0]
    for bad, status in [((1, [2]), B.RL_ERR_BAD_SEQ),        # source not active
                        ((0, [0]), B.RL_ERR_BAD_SEQ),        # target already active
                        ((0, [6]), B.RL_ERR_BAD_SEQ),        # id out of range
                        ((0, [2, 2]), B.RL_ERR_INVALID_ARG)]:
        with pytest.raises(B.RLError) as e:
            ro.rl_seq_fork(*bad)
        assert e.value.status == status and ro.rl_kv_stats()[0] == free0
    small = amd.Rollout(shape, to_device(w), max_seqs=6, max_ctx=64, max_rows=6, kv_pages=3)
    small.rl_prefill([0], [p], 0.0, 0)                        # 2 pages, 1 free; a fork needs one page per member
    with pytest.raises(B.RLError) as e:
        small.rl_seq_fork(0, [1, 2])
    assert e.value.status == B.RL_ERR_KV_FULL and small.rl_kv_stats() == (1, 3)
    small.rl_seq_fork(0, [1])
    assert small.rl_kv_stats() == (0, 3) and small.rl_seq_len(1) == 21
    small.close()
    ro.rl_seq_fork(0, [3, 5])
    assert ro.rl_kv_stats()[0] == free0 - 2 and ro.rl_seq_len(5) == 21
    ids = [0, 3, 5]
    cur = torch.cat([tok, tok, tok])
    z = torch.empty(3, shape["vocab"], device=DEV)
    om = orc.OracleModel(dims_of(shape), wn, max_ctx=256)
    zo = om.prefill(0, p)
    for step in range(200):
        feed = cur
        cur, lp = ro.rl_decode_step(ids, feed, 1.0, 7, debug_logits=z)
        if step < 3 or step == 199:
            torch.cuda.synchronize()
            zc = z.cpu().numpy()
            if step == 0:                                     # same history, same token: the three rows are equal
                assert np.array_equal(zc[0], zc[1]) and np.array_equal(zc[0], zc[2])
                zo = om.forward_token(0, int(feed[0]))
                assert rel_inf(zc[0], zo) < 1e-4
            for r in range(3):
                t_ref, lp_ref = orc.sample(zc[r], 1.0, 7, ids[r], 22 + step)
                assert int(cur[r]) == t_ref and abs(float(lp[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref))
    torch.cuda.synchronize()
    assert [ro.rl_seq_len(i) for i in ids] == [221, 221, 221]
    assert len({int(t) for t in cur}) > 1                     # different random streams: the samples have diverged
    ro.rl_free_seqs(ids)
    assert ro.rl_kv_stats() == (48, 48)
    ro.close()


# ------------------------------------------------------------------------- bf16, one layer at 8B dimensions
def _layer_case(amd, ctxs, seed, max_rows=None, shuffle=None, extra_pages=0, max_seqs=None, **shape_over):
    """Import random N(0,1) bf16 KV of the given lengths, run one decode step on N(0,1) hidden rows."""
    shape = dict(ri.SHAPES["layer8b"], **shape_over)
    w, wn = make_both(shape, seed)
    B = len(ctxs)
    max_ctx = (max(ctxs) + 1 + 15) // 16 * 16 + 16
    pages = sum((c + 1 + 15) // 16 for c in ctxs) + 4 + extra_pages
    ro = amd.Rollout(shape, to_device(w), max_seqs=max_seqs or B, max_ctx=max_ctx, max_rows=max_rows or B, kv_pages=pages)
    if shuffle is not None:
        ro.rl_debug_shuffle_free_pages(shuffle)
    nkv, d, H = shape["n_kv"], shape["head_dim"], shape["hidden"]
    ks, vs = [], []
    for b, c in enumerate(ctxs):
        k = ri.normal((c, nkv, d), 1.0, seed, 2000 + 2 * b, dtype=torch.bfloat16)
        v = ri.normal((c, nkv, d), 1.0, seed, 2001 + 2 * b, dtype=torch.bfloat16)
        ks.append(k)
        vs.append(v)
        ro.rl_seq_import_kv(b, [k.to(DEV)], [v.to(DEV)])
    x = ri.normal((B, H), 1.0, seed, 1999).to(torch.bfloat16).float()
    return shape, wn, ro, ks, vs, x


def _oracle_layer_row(shape, wn, k, v, x_row, ctx):
    kc = np.zeros((ctx + 1, shape["n_kv"], shape["head_dim"]), np.float32)
    vc = np.zeros_like(kc)
    kc[:ctx] = k.float().numpy()
    vc[:ctx] = v.float().numpy()
    xo = np.ascontiguousarray(x_row.numpy().copy())
    orc.layer_forward(dims_of(shape), wn["layers"][0], xo, ctx, kc, vc)
    return xo


@pytest.mark.parametrize("ctxs", [
    [0, 1, 15, 16, 17, 255, 256, 257, 700],            # page and chunk boundaries, empty history
    [300 + 7 * i for i in range(37)],                  # 37 rows: two column blocks with a ragged tail
    [33],                                              # a single row
    [16383, 8191, 4096, 4095, 1024, 1023],             # longest context; both sides of the LDS/workspace merge switch
    [65519, 40000],                                    # the largest context the bf16 path accepts: 256 segments
])
def test_bf16_layer_decode_matches_oracle(amd, ctxs):
    shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=31, shuffle=9)
    out = ro.rl_decode_hidden(list(range(len(ctxs))), x.to(DEV))
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    assert np.isfinite(out).all()
    for b, c in enumerate(ctxs):
        ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[b], c)
        err = rel_inf(out[b] - x[b].numpy(), ref - x[b].numpy())
        assert err < 3e-2, (b, c, err)
        assert ro.rl_seq_len(b) == c + 1
    ro.close()


def test_bf16_layer_bits_do_not_depend_on_attention_block_size(amd):
    """Contexts beyond 4096 keys are cut over several attention blocks per (row, kv head); how many segments a block
    takes is a launch parameter.  Outputs are bit-equal for every choice (also one that leaves a block a single
    segment), with rows on both sides of the switch and a forked pair that shares its prompt pages."""
    ctxs = [16383, 5000, 4097, 4096, 300, 9000]
    outs = []
    for spb in (16, 8, 5, 4, 1):
        shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=40, shuffle=5, max_rows=8, extra_pages=8, max_seqs=8)
        ro.rl_debug_attention_split(spb)
        ro.rl_seq_fork(5, [6])
        xin = torch.cat([x, x[5:6]])
        outs.append(ro.rl_decode_hidden(list(range(7)), xin.to(DEV)).cpu())
        ro.close()
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
    assert torch.equal(outs[0][5], outs[0][6])


def test_bf16_layer_pages_far_into_a_large_pool(amd):
    """A 5.2 GB pool (80 000 pages of 64 KiB per layer) with the free list shuffled: the sequences' pages lie all
    over it, most of them beyond 4 GiB from its start, which 32-bit offset arithmetic anywhere would not survive."""
    ctxs = [700, 33, 1500, 260]
    shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=39, shuffle=11, extra_pages=80000)
    out = ro.rl_decode_hidden(list(range(len(ctxs))), x.to(DEV)).cpu().numpy()
    for b, c in enumerate(ctxs):
        ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[b], c)
        err = rel_inf(out[b] - x[b].numpy(), ref - x[b].numpy())
        assert err < 3e-2, (b, c, err)
    ro.close()


def test_bf16_layer_eight_query_heads_per_kv_head_long_contexts(amd):
    """The widest query group the bf16 path accepts (8 heads per kv head: the largest per-block merge area), at
    contexts on both sides of the switch between the merge inside the block and the one through the workspace."""
    ctxs = [4000, 3000, 100, 5000, 4096]
    shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=37, shuffle=3, hidden=1024, n_q=16, n_kv=2, ffn=1536)
    B = len(ctxs)
    out = ro.rl_decode_hidden(list(range(B)), x.to(DEV)).cpu().numpy()
    for b, c in enumerate(ctxs):
        ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[b], c)
        err = rel_inf(out[b] - x[b].numpy(), ref - x[b].numpy())
        assert err < 3e-2, (b, c, err)
    ro.close()


@pytest.mark.parametrize("ctxs,G", [([2100, 5000, 700], 6), ([1024] * 4, 8)])
def test_bf16_layer_forked_rows_share_prompt_attention_and_match_oracle(amd, ctxs, G):
    """8B-dimension layer: cached contexts are each continued as G sequences (shared full pages, copied partial
    page).  The step computes the attention over the common pages once per set of rows; every row still matches
    the oracle run on that row alone, and the bits equal those with the sharing switched off and those with the
    widest sets (two 16-column operands side by side, which calls of this size do not choose by themselves).  The
    second case is the launch shape of the 32-sequence rollout workload: 4 prompts of 1024 tokens x 8 samples."""
    shape = ri.SHAPES["layer8b"]
    w, wn = make_both(shape, 34)
    wd = to_device(w)
    B = len(ctxs) * G
    pages = sum((c + 15) // 16 for c in ctxs) + 2 * B + 4
    nkv, d, H = shape["n_kv"], shape["head_dim"], shape["hidden"]
    ks = [ri.normal((c, nkv, d), 1.0, 34, 2000 + 2 * b, dtype=torch.bfloat16) for b, c in enumerate(ctxs)]
    vs = [ri.normal((c, nkv, d), 1.0, 34, 2001 + 2 * b, dtype=torch.bfloat16) for b, c in enumerate(ctxs)]
    x = ri.normal((B, H), 1.0, 34, 1999).to(torch.bfloat16).float()
    outs = []
    for share in (1, 0, 2):
        ro = amd.Rollout(shape, wd, max_seqs=B, max_ctx=5040, max_rows=B, kv_pages=pages)
        ro.rl_debug_shuffle_free_pages(5)
        ro.rl_debug_share_attention(share)
        for b in range(len(ctxs)):
            ro.rl_seq_import_kv(b * G, [ks[b].to(DEV)], [vs[b].to(DEV)])
            ro.rl_seq_fork(b * G, [b * G + j for j in range(1, G)])
        assert ro.rl_kv_stats()[0] == pages - sum((c + 15) // 16 for c in ctxs) - (G - 1) * sum(1 for c in ctxs if c % 16)
        order = ri.permutation(B, 34, 77).tolist()          # members of a prompt need not be adjacent rows
        out = torch.empty(B, H)
        out[order] = ro.rl_decode_hidden(order, x[order].to(DEV)).cpu()
        nxt = ro.rl_decode_hidden(order, x[order].to(DEV)).cpu()     # a second step: own keys differ per member now
        torch.cuda.synchronize()
        outs.append((out, nxt))
        assert all(ro.rl_seq_len(i) == ctxs[i // G] + 2 for i in range(B))
        ro.close()
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert torch.equal(outs[0][0], outs[2][0]) and torch.equal(outs[0][1], outs[2][1])
    out = outs[0][0].numpy()
    for i in range(B):
        b = i // G
        ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[i], ctxs[b])
        err = rel_inf(out[i] - x[i].numpy(), ref - x[i].numpy())
        assert err < 3e-2, (i, err)


def test_append_kv_equals_import_and_extends_forked_sequences(amd):
    """rl_seq_append_kv: a context imported in two pieces (the cut inside a page) gives the bits of the same context
    imported at once; samples forked from one cached prompt and then given private tokens of different lengths match
    the oracle row by row (shared prompt pages + private tails); error paths leave the state untouched."""
    B = amd.binding
    shape = ri.SHAPES["layer8b"]
    w, wn = make_both(shape, 36)
    nkv, d, H = shape["n_kv"], shape["head_dim"], shape["hidden"]
    ro = amd.Rollout(shape, to_device(w), max_seqs=8, max_ctx=1024, max_rows=8, kv_pages=160)
    ro.rl_debug_shuffle_free_pages(21)
    k = ri.normal((700, nkv, d), 1.0, 36, 2000, dtype=torch.bfloat16)
    v = ri.normal((700, nkv, d), 1.0, 36, 2001, dtype=torch.bfloat16)
    ro.rl_seq_import_kv(0, [k.to(DEV)], [v.to(DEV)])
    ro.rl_seq_import_kv(1, [k[:299].to(DEV)], [v[:299].to(DEV)])
    ro.rl_seq_append_kv(1, [k[299:].to(DEV).contiguous()], [v[299:].to(DEV).contiguous()])
    assert ro.rl_seq_len(1) == 700
    # a cached prompt of 100 tokens continued as three samples with 0, 37 and 50 private tokens
    kp = ri.normal((100, nkv, d), 1.0, 36, 2002, dtype=torch.bfloat16)
    vp = ri.normal((100, nkv, d), 1.0, 36, 2003, dtype=torch.bfloat16)
    ro.rl_seq_import_kv(2, [kp.to(DEV)], [vp.to(DEV)])
    ro.rl_seq_fork(2, [3, 4])
    priv = {2: 0, 3: 37, 4: 50}
    tails = {}
    for s_id, n in priv.items():
        if n:
            tk = ri.normal((n, nkv, d), 1.0, 36, 2010 + 2 * s_id, dtype=torch.bfloat16)
            tv = ri.normal((n, nkv, d), 1.0, 36, 2011 + 2 * s_id, dtype=torch.bfloat16)
            ro.rl_seq_append_kv(s_id, [tk.to(DEV)], [tv.to(DEV)])
            tails[s_id] = (tk, tv)
    free_before = ro.rl_kv_stats()[0]
    for args, status in [((5, [k[:4].to(DEV)], [v[:4].to(DEV)]), B.RL_ERR_BAD_SEQ),             # not active
                         ((0, [k[:400].to(DEV)], [v[:400].to(DEV)]), B.RL_ERR_CTX_OVERFLOW)]:   # 700 + 400 > max_ctx - 1
        with pytest.raises(B.RLError) as e:
            ro.rl_seq_append_kv(*args)
        assert e.value.status == status and ro.rl_kv_stats()[0] == free_before and ro.rl_seq_len(0) == 700
    ids = [0, 1, 2, 3, 4]
    x = ri.normal((5, H), 1.0, 36, 1999).to(torch.bfloat16).float()
    x[1] = x[0]
    out = ro.rl_decode_hidden(ids, x.to(DEV)).cpu()
    torch.cuda.synchronize()
    assert torch.equal(out[0], out[1])
    out = out.numpy()
    for r, s_id in enumerate(ids):
        if s_id < 2:
            kk, vv = k, v
        elif priv[s_id]:
            kk, vv = torch.cat([kp, tails[s_id][0]]), torch.cat([vp, tails[s_id][1]])
        else:
            kk, vv = kp, vp
        ref = _oracle_layer_row(shape, wn, kk, vv, x[r], kk.shape[0])
        err = rel_inf(out[r] - x[r].numpy(), ref - x[r].numpy())
        assert err < 3e-2, (s_id, err)
    ro.close()


def test_bf16_layer_batch_and_page_placement_invariance(amd):
    ctxs = [40, 513, 100, 257, 31]
    shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=32)
    full = ro.rl_decode_hidden(list(range(5)), x.to(DEV)).cpu()
    ro.close()
    # same sequences, other pages, decoded alone or in another order
    shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=32, shuffle=1234)
    alone = ro.rl_decode_hidden([3], x[3:4].to(DEV)).cpu()
    rest = ro.rl_decode_hidden([4, 0, 2, 1], x[[4, 0, 2, 1]].to(DEV)).cpu()
    torch.cuda.synchronize()
    assert torch.equal(alone[0], full[3])
    assert torch.equal(rest, full[[4, 0, 2, 1]])
    ro.close()


# --------------------------------------------------------------------------- bf16 small full model, logits
@pytest.mark.parametrize("n_q,n_kv,qk_norm", [(4, 1, 1), (8, 1, 1), (2, 2, 1), (4, 2, 0)])
def test_bf16_small_model_teacher_forced_logits(amd, n_q, n_kv, qk_norm):
    """2-layer bf16 decoder (8B head size, narrow), query groups of 4, 8, 1 and 2 heads per kv head, with and without
    the per-head norm: prefill (three separate prompts and one prompt sampled three times, whose samples share
    pages) + teacher-forced decode; logits within 3e-2, argmax agreement >= 99 %, sampled ids reproduced by the
    oracle sampler from the GPU's logits."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=n_q, n_kv=n_kv, ffn=768, vocab=8192, qk_norm=qk_norm)
    w, wn = make_both(shape, 41, std=0.05)
    ro = amd.Rollout(shape, to_device(w), max_seqs=6, max_ctx=320, max_rows=40, kv_pages=90)
    om = orc.OracleModel(dims_of(shape), wn, max_ctx=320)
    lens = [270, 3, 33, 70, 70, 70]
    prompts = [ri.tokens((n,), shape["vocab"], 41, 920 + i).tolist() for i, n in enumerate(lens[:4])]
    prompts += [prompts[3], prompts[3]]
    seqs = [2, 0, 1, 3, 4, 5]
    seed = 77
    ro.rl_prefill(seqs[:3], prompts[:3], 1.0, seed)
    ro.rl_prefill_groups(seqs[3:], 3, [prompts[3]], 1.0, seed)
    torch.cuda.synchronize()
    for i, s in enumerate(seqs):
        om.prefill(s, prompts[i])
    n = len(seqs)
    steps = 40
    forced_all = ri.tokens((steps, n), shape["vocab"], 41, 930)
    logits = torch.empty(n, shape["vocab"], device=DEV)
    cur = ri.tokens((n,), shape["vocab"], 41, 929).to(DEV)
    count, worst = ArgmaxCount(3e-2), 0.0
    for step in range(steps):
        forced = forced_all[step].clone()
        forced[step % n] = -1                         # leave one row sampled each step
        tok, lp = ro.rl_decode_step(seqs, cur, 1.0, seed, forced_next=forced.to(DEV), debug_logits=logits)
        torch.cuda.synchronize()
        zg = logits.cpu().numpy()
        for i, s in enumerate(seqs):
            z = om.forward_token(s, int(cur[i]))
            worst = max(worst, float(rel_inf(zg[i], z)))
            count.add(zg[i], z)
            t_ref, lp_ref = orc.sample(zg[i], 1.0, seed, s, lens[i] + step + 1, forced=int(forced[i]))
            assert int(tok[i]) == t_ref
            assert abs(float(lp[i]) - lp_ref) < 1e-4
            _, lp_orc = orc.sample(z, 1.0, seed, s, lens[i] + step + 1, forced=t_ref)
            assert abs(float(lp[i]) - lp_orc) < 5e-2
        cur = tok
    assert worst < 3e-2, worst
    count.check(min_rows=100)          # the same rule for every variant
    print(f"[n_q={n_q} n_kv={n_kv} qk_norm={qk_norm}] worst logit error {worst:.2e}; {count.summary()}")
    ro.close()


# ------------------------------------------------------------------------------------------- error handling
def test_rollout_consumes_weights_and_sizes_pool_itself(amd):
    """consume_weights empties the caller's dict while packing (one copy of the model on the card); with
    kv_pages=None the pool takes what is left beside weights and workspace.  Same outputs as a plain instance."""
    shape = ri.SHAPES["tiny"]
    w, _ = make_both(shape, 41)
    prompts = ri.tokens((3, 20), shape["vocab"], 41, 930).tolist()
    ra = amd.Rollout(shape, to_device(w), max_seqs=4, max_ctx=64, max_rows=64, kv_pages=16)
    wd = to_device(w)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()                    # what earlier tests left in the allocator's cache goes back first
    free_before, total = torch.cuda.mem_get_info()
    rb = amd.Rollout(shape, wd, max_seqs=4, max_ctx=64, max_rows=64, kv_pages=None, consume_weights=True,
                     kv_slack_bytes=free_before - (256 << 20))      # leaves about 256 MiB for workspace and pool
    assert set(wd.keys()) == {"layers"} and all(len(l) == 0 for l in wd["layers"])
    n_pages = rb.rl_kv_stats()[1]
    assert n_pages >= 16 and rb.cfg.kv_pool_bytes < (2 << 30)
    ta, la = ra.rl_prefill([0, 1, 2], prompts, 1.0, 3)
    tb, lb = rb.rl_prefill([0, 1, 2], prompts, 1.0, 3)
    for _ in range(3):
        ta, la = ra.rl_decode_step([0, 1, 2], ta, 1.0, 3)
        tb, lb = rb.rl_decode_step([0, 1, 2], tb, 1.0, 3)
    torch.cuda.synchronize()
    assert torch.equal(ta, tb) and torch.equal(la, lb)
    ra.close()
    rb.close()


def test_error_paths_leave_state_untouched(amd):
    B = amd.binding
    shape = ri.SHAPES["tiny"]
    w, _ = make_both(shape, 51)
    ro = amd.Rollout(shape, to_device(w), max_seqs=4, max_ctx=32, max_rows=4, kv_pages=3)
    p = ri.tokens((20,), shape["vocab"], 51, 940).tolist()
    with pytest.raises(B.RLError) as e:
        ro.rl_prefill([0, 1], [p, p], 0.0, 0)         # 2 x 2 pages > 3
    assert e.value.status == B.RL_ERR_KV_FULL and ro.rl_kv_stats() == (3, 3)
    with pytest.raises(B.RLError) as e:
        ro.rl_prefill([4], [p], 0.0, 0)
    assert e.value.status == B.RL_ERR_BAD_SEQ
    with pytest.raises(B.RLError) as e:
        ro.rl_prefill([0], [p + p], 0.0, 0)
    assert e.value.status == B.RL_ERR_CTX_OVERFLOW
    with pytest.raises(B.RLError) as e:
        ro.rl_prefill([0], [[shape["vocab"]]], 0.0, 0)
    assert e.value.status == B.RL_ERR_INVALID_ARG
    with pytest.raises(B.RLError) as e:
        ro.rl_prefill([0], [[]], 0.0, 0)              # an empty prompt
    assert e.value.status == B.RL_ERR_INVALID_ARG
    with pytest.raises(B.RLError) as e:
        ro.rl_decode_step([], torch.empty(0, dtype=torch.int32, device=DEV), 0.0, 0)   # an empty batch
    assert e.value.status == B.RL_ERR_INVALID_ARG
    ro.rl_free_seqs([])                               # freeing nothing is allowed
    assert ro.rl_kv_stats() == (3, 3)
    tok, _ = ro.rl_prefill([0], [p], 0.0, 0)
    assert ro.rl_kv_stats() == (1, 3)
    with pytest.raises(B.RLError) as e:
        ro.rl_prefill([0], [p], 0.0, 0)               # already active
    assert e.value.status == B.RL_ERR_BAD_SEQ
    with pytest.raises(B.RLError) as e:
        ro.rl_decode_step([1], tok, 0.0, 0)           # not active
    assert e.value.status == B.RL_ERR_BAD_SEQ
    with pytest.raises(B.RLError) as e:
        ro.rl_decode_step([0, 0], torch.cat([tok, tok]), 0.0, 0)
    assert e.value.status == B.RL_ERR_INVALID_ARG
    for _ in range(12):                               # 20 -> 32 tokens = max_ctx
        tok, _ = ro.rl_decode_step([0], tok, 0.0, 0)
    assert ro.rl_seq_len(0) == 32
    with pytest.raises(B.RLError) as e:
        ro.rl_decode_step([0], tok, 0.0, 0)
    assert e.value.status == B.RL_ERR_CTX_OVERFLOW and ro.rl_seq_len(0) == 32
    ro.rl_free_seqs([0])
    with pytest.raises(B.RLError) as e:
        ro.rl_free_seqs([0])
    assert e.value.status == B.RL_ERR_BAD_SEQ
    assert ro.rl_kv_stats() == (3, 3)
    torch.cuda.synchronize()
    ro.close()


# ------------------------------------------------------------- full-size workloads, sampled against the oracle
def test_layer8b_full_size_batch64_ctx2048_sampled_rows(amd):
    """The one-layer workload at full size (batch 64, 2048 cached tokens each, shuffled pages): every row against
    the oracle."""
    ctxs = [2048] * 64
    shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=33, shuffle=77)
    out = ro.rl_decode_hidden(list(range(64)), x.to(DEV))
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    assert np.isfinite(out).all()
    for b in range(64):
        ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[b], 2048)
        err = rel_inf(out[b] - x[b].numpy(), ref - x[b].numpy())
        assert err < 3e-2, (b, err)
    ro.close()


def test_layer8b_wave_shape_128_rows_shared_prompt_context_9k_sampled_rows(amd):
    """The launch configuration that the benchmark times, on one layer at full width: 128 rows = 16 prompts x 8 samples,
    a prompt of 2048 tokens whose pages the samples of a group share (imported once, forked), 7168 + j private tokens
    appended per sequence (so that the members of a group stand at different positions within a few steps, as after
    ragged retirements), one decode step.  Rows are sampled (two per group pattern: first and last member of some
    groups) and compared with the oracle, which gets each row's own keys and values as one contiguous history."""
    shape = dict(ri.SHAPES["layer8b"])
    seed, G, n_groups, P, private = 41, 8, 16, 2048, 7168
    w, wn = make_both(shape, seed)
    B = G * n_groups
    nkv, d, H = shape["n_kv"], shape["head_dim"], shape["hidden"]
    extra = [0 if g % 2 == 0 else (j % 3) for g in range(n_groups) for j in range(G)]   # odd groups: members out of step
    max_ctx = (P + private + 3 + 1 + 15) // 16 * 16 + 16
    pages = n_groups * (P // 16) + sum((private + e + 1 + 15) // 16 + 1 for e in extra) + 8
    ro = amd.Rollout(shape, to_device(w), max_seqs=B, max_ctx=max_ctx, max_rows=B, kv_pages=pages)
    sampled = {0, 7, 8 + 1, 8 + 2, 8 + 7, 5 * 8 + 3, 15 * 8, 15 * 8 + 5, 15 * 8 + 7}
    hist = {}
    for g in range(n_groups):
        kp = ri.normal((P, nkv, d), 1.0, seed, 3000 + 2 * g, dtype=torch.bfloat16)
        vp = ri.normal((P, nkv, d), 1.0, seed, 3001 + 2 * g, dtype=torch.bfloat16)
        ro.rl_seq_import_kv(g * G, [kp.to(DEV)], [vp.to(DEV)])
        ro.rl_seq_fork(g * G, list(range(g * G + 1, (g + 1) * G)))
        for j in range(G):
            b = g * G + j
            n = private + extra[b]
            ka = ri.normal((n, nkv, d), 1.0, seed, 4000 + 2 * b, device=DEV, dtype=torch.bfloat16)
            va = ri.normal((n, nkv, d), 1.0, seed, 4001 + 2 * b, device=DEV, dtype=torch.bfloat16)
            ro.rl_seq_append_kv(b, [ka], [va])
            if b in sampled:
                hist[b] = (torch.cat([kp, ka.cpu()]), torch.cat([vp, va.cpu()]))
    assert [ro.rl_seq_len(b) for b in range(B)] == [P + private + e for e in extra]
    x = ri.normal((B, H), 1.0, seed, 1999).to(torch.bfloat16).float()
    out = ro.rl_decode_hidden(list(range(B)), x.to(DEV))
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    assert np.isfinite(out).all()
    worst = 0.0
    for b in sorted(sampled):
        k, v = hist[b]
        ctx = P + private + extra[b]
        ref = _oracle_layer_row(shape, wn, k, v, x[b], ctx)
        err = float(rel_inf(out[b] - x[b].numpy(), ref - x[b].numpy()))
        worst = max(worst, err)
        assert err < 3e-2, (b, err)
    print(f"[wave shape] worst layer error over {len(sampled)} sampled rows at context {P + private}: {worst:.2e}")
    ro.close()


def test_bf16_layer_many_rows_uses_wide_tiles(amd):
    """70 and 130 rows (the 128-column tile, one and two passes) with short histories."""
    for n in (70, 130):
        ctxs = [(7 * i) % 50 for i in range(n)]
        shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=34)
        out = ro.rl_decode_hidden(list(range(n)), x.to(DEV)).cpu().numpy()
        for b in range(n):
            ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[b], ctxs[b])
            err = rel_inf(out[b] - x[b].numpy(), ref - x[b].numpy())
            assert err < 3e-2, (n, b, err)
        ro.close()


@pytest.fixture(scope="module")
def full8b(amd):
    """The 36-layer 8B-shaped model on the card, shared by the tests below (drawing and packing it takes a while).
    Layer weights for the oracle are redrawn from the same seeded streams, one layer at a time."""
    shape = ri.SHAPES["full8b"]
    seed = ri.BASE_SEED + 2
    w = ri.make_weights(shape, seed, device=DEV, dtype=torch.bfloat16)
    m = dict(shape=shape, seed=seed, dims=dims_of(shape),
             final_norm=w["final_norm"].float().cpu().numpy(), lm_head=w["lm_head"].float().cpu().numpy(),
             embed=w["embed"])
    m["ro"] = amd.Rollout(shape, w, max_seqs=16, max_ctx=2064, max_rows=64, kv_pages=8 * 130 + 16, consume_weights=True)
    del w
    torch.cuda.empty_cache()
    yield m
    m["ro"].close()


def _layer_weights_for_oracle(m, l):
    return {k: np.ascontiguousarray(v.float().cpu().numpy())
            for k, v in ri.make_layer(m["shape"], m["seed"], l, device=DEV, dtype=torch.bfloat16).items()}


def test_full8b_prefill_every_layer_and_first_token(full8b):
    """The 36-layer 8B-shaped model, prefill path: two prompts with capture of every layer boundary; each of the 36
    oracle layers is fed the GPU's layer input at every position and must reproduce the GPU's layer output.  The
    first sampled token is pinned through a second route: the same prompt minus its last token is prefilled and that
    token fed as a decode step, which must give the same token and log-probability bit for bit and exposes the logits,
    from which the oracle sampler must draw that very token; the log-probability is compared with the oracle head's."""
    m = full8b
    ro, shape, seed, dims = m["ro"], m["shape"], m["seed"], m["dims"]
    L, V, nkv, d = shape["n_layers"], shape["vocab"], shape["n_kv"], shape["head_dim"]
    cap = ro.rl_set_capture(True)
    lens = [17, 6]
    prompts = [ri.tokens((n,), V, seed, 950 + i).tolist() for i, n in enumerate(lens)]
    tok, lp = ro.rl_prefill([1, 3], prompts, 1.0, seed)
    torch.cuda.synchronize()
    cap_pre = cap[:, :sum(lens)].cpu().numpy()          # [(L+1), rows, H]; rows = seq 1 positions, then seq 3
    row0 = [0, lens[0]]
    logits2 = torch.empty(2, V, device=DEV)
    tok2, lp2 = ro.rl_decode_step([1, 3], tok, 1.0, seed, debug_logits=logits2)
    torch.cuda.synchronize()
    cap_step = cap[L, :2].cpu().numpy()
    zg2 = logits2.cpu().numpy()
    # the first sampled token again, as a decode step at the last prompt position (same ids: same random streams)
    ro.rl_free_seqs([1, 3])
    ro.rl_prefill([1, 3], [p[:-1] for p in prompts], 1.0, seed)
    last = torch.tensor([p[-1] for p in prompts], dtype=torch.int32, device=DEV)
    logits1 = torch.empty(2, V, device=DEV)
    tok_b, lp_b = ro.rl_decode_step([1, 3], last, 1.0, seed, debug_logits=logits1)
    torch.cuda.synchronize()
    ro.rl_free_seqs([1, 3])
    ro.rl_set_capture(False)
    assert torch.equal(tok, tok_b) and torch.equal(lp, lp_b)     # prefill and decode give the same bits
    zg1 = logits1.cpu().numpy()
    for si, s_id in enumerate([1, 3]):
        t_ref, lp_ref = orc.sample(zg1[si], 1.0, seed, s_id, lens[si])
        assert int(tok[si]) == t_ref and abs(float(lp[si]) - lp_ref) < 1e-4
        z = orc.matvec(m["lm_head"], orc.rmsnorm(cap_pre[L, row0[si] + lens[si] - 1], m["final_norm"], shape["rms_eps"]))
        assert rel_inf(zg1[si], z) < 3e-2
        _, lp_orc = orc.sample(z, 1.0, seed, s_id, lens[si], forced=t_ref)
        assert abs(float(lp[si]) - lp_orc) < 5e-2, (si, float(lp[si]), lp_orc)
        z = orc.matvec(m["lm_head"], orc.rmsnorm(cap_step[si], m["final_norm"], shape["rms_eps"]))
        assert rel_inf(zg2[si], z) < 3e-2
        t_ref, lp_ref = orc.sample(zg2[si], 1.0, seed, s_id, lens[si] + 1)
        assert int(tok2[si]) == t_ref and abs(float(lp2[si]) - lp_ref) < 1e-4
    worst = 0.0
    for l in range(L):
        lw = _layer_weights_for_oracle(m, l)
        for si, n in enumerate(lens):
            kc = np.zeros((n, nkv, d), np.float32)
            vc = np.zeros_like(kc)
            for p in range(n):
                x_in = np.ascontiguousarray(cap_pre[l, row0[si] + p].copy())
                xo = x_in.copy()
                orc.layer_forward(dims, lw, xo, p, kc, vc)
                err = float(rel_inf(cap_pre[l + 1, row0[si] + p] - x_in, xo - x_in))
                worst = max(worst, err)
                assert err < 3e-2, (l, si, p, err)
    print(f"[full8b prefill] worst layer error over 36 layers x {sum(lens)} rows: {worst:.2e}")


def test_full8b_decode_at_rollout_contexts_end_to_end(full8b):
    """The 36-layer 8B-shaped model, decode path at the contexts of the 32-sequence rollout workload: eight sequences
    whose KV is imported (N(0,1) on the bf16 grid, identical on both sides) at 1024 and 2034 tokens run 13
    teacher-forced steps (up to context 2047) = 104 rows.  The oracle runs the same rows end to end (its own
    residual stream, its own appended keys and values, all 36 layers and the output projection): logits within 3e-2,
    argmax agreement >= 99 %, log-probabilities within twice the logit bound, ids reproduced from the GPU's logits.  Two sequences
    (one per context) are also checked layer by layer, first and last step, with the oracle layer fed the GPU's
    layer input, and the output projection alone on the GPU's last residual."""
    m = full8b
    ro, shape, seed, dims = m["ro"], m["shape"], m["seed"], m["dims"]
    L, H, V, nkv, d = shape["n_layers"], shape["hidden"], shape["vocab"], shape["n_kv"], shape["head_dim"]
    n_dec, steps = 8, 13
    ctx0 = [1024] * 4 + [2034] * 4
    dec_ids = list(range(4, 4 + n_dec))
    cap = ro.rl_set_capture(True)

    def kv_of(b, l, which):
        return ri.normal((ctx0[b], nkv, d), 1.0, seed, 5000 + (b * L + l) * 2 + which, device=DEV, dtype=torch.bfloat16)

    for b in range(n_dec):
        ro.rl_seq_import_kv(dec_ids[b], [kv_of(b, l, 0) for l in range(L)], [kv_of(b, l, 1) for l in range(L)])
    fed = ri.tokens((steps + 1, n_dec), V, seed, 960)          # row t is fed at step t, row t+1 is forced
    zg = np.empty((steps, n_dec, V), np.float32)
    lp_g = np.empty((steps, n_dec), np.float32)
    tok_g = np.empty((steps, n_dec), np.int64)
    cap_dec = np.empty((steps, L + 1, n_dec, H), np.float32)
    forced_all = fed[1:].clone()
    logits = torch.empty(n_dec, V, device=DEV)
    for t in range(steps):
        forced_all[t, t % n_dec] = -1                          # one row per step is sampled
        tk, lq = ro.rl_decode_step(dec_ids, fed[t].to(DEV), 1.0, seed, forced_next=forced_all[t].to(DEV),
                                   debug_logits=logits)
        torch.cuda.synchronize()
        zg[t], lp_g[t], tok_g[t] = logits.cpu().numpy(), lq.cpu().numpy(), tk.cpu().numpy()
        cap_dec[t] = cap[:, :n_dec].cpu().numpy()
    assert all(ro.rl_seq_len(dec_ids[b]) == ctx0[b] + steps for b in range(n_dec))
    ro.rl_free_seqs(dec_ids)
    ro.rl_set_capture(False)
    x_chain = m["embed"][fed[:steps].to(DEV).long()].float().cpu().numpy()    # [steps, n_dec, H]: the oracle's own stream
    assert np.array_equal(x_chain, cap_dec[:, 0])                             # the gather is exact
    sliced, sliced_steps = (0, 4), (0, steps - 1)                             # one sequence per context class
    worst_layer = 0.0
    for l in range(L):
        lw = _layer_weights_for_oracle(m, l)
        for b in range(n_dec):
            kc = np.zeros((ctx0[b] + steps, nkv, d), np.float32)
            vc = np.zeros_like(kc)
            kc[:ctx0[b]] = kv_of(b, l, 0).float().cpu().numpy()
            vc[:ctx0[b]] = kv_of(b, l, 1).float().cpu().numpy()
            for t in range(steps):
                pos = ctx0[b] + t
                if b in sliced and t in sliced_steps:
                    # The layer alone, fed the GPU's input; the earlier keys and values are the end-to-end oracle's.
                    # It writes slot `pos`, which the end-to-end pass below overwrites with its own.
                    x_in = np.ascontiguousarray(cap_dec[t, l, b].copy())
                    xo = x_in.copy()
                    orc.layer_forward(dims, lw, xo, pos, kc, vc)
                    err = float(rel_inf(cap_dec[t, l + 1, b] - x_in, xo - x_in))
                    worst_layer = max(worst_layer, err)
                    assert err < 3e-2, (l, b, t, err)
                x = np.ascontiguousarray(x_chain[t, b])
                orc.layer_forward(dims, lw, x, pos, kc, vc)
                x_chain[t, b] = x
    count, worst, worst_lp = ArgmaxCount(3e-2), 0.0, 0.0
    for t in range(steps):
        for b in range(n_dec):
            z = orc.matvec(m["lm_head"], orc.rmsnorm(x_chain[t, b], m["final_norm"], shape["rms_eps"]))
            err = float(rel_inf(zg[t, b], z))
            worst = max(worst, err)
            assert err < 3e-2, (t, b, err)
            count.add(zg[t, b], z)
            pos = ctx0[b] + t + 1
            t_ref, lp_ref = orc.sample(zg[t, b], 1.0, seed, dec_ids[b], pos, forced=int(forced_all[t, b]))
            assert int(tok_g[t, b]) == t_ref and abs(float(lp_g[t, b]) - lp_ref) < 1e-4, (t, b)
            # log-probability = z_tok - logsumexp(z): two terms, each within the logit bound 3e-2 max|z|
            _, lp_orc = orc.sample(z, 1.0, seed, dec_ids[b], pos, forced=t_ref)
            worst_lp = max(worst_lp, abs(float(lp_g[t, b]) - lp_orc))
            assert abs(float(lp_g[t, b]) - lp_orc) < 2 * 3e-2 * np.abs(z).max(), (t, b, float(lp_g[t, b]), lp_orc)
            if b in sliced and t in sliced_steps:             # the output projection alone, on the GPU's last residual
                zs = orc.matvec(m["lm_head"], orc.rmsnorm(cap_dec[t, L, b], m["final_norm"], shape["rms_eps"]))
                assert rel_inf(zg[t, b], zs) < 3e-2
    assert count.rows >= 100
    count.check(min_rows=50)
    print(f"[full8b decode] worst layer error {worst_layer:.2e}, worst end-to-end logit error {worst:.2e}, worst "
          f"log-probability error {worst_lp:.2e}; {count.summary()}")


# ------------------------------------------------------ ragged rollout: sequences retire and new ones join
def test_tiny_fp32_ragged_continuous_batch(amd):
    """Eight sequences with pre-drawn prompt and final lengths share a pool that cannot hold them all at once:
    sequences retire individually, their pages are recycled for waiting prompts, and every generated token and
    log-probability still matches the oracle run on each sequence alone (batch- and placement-invariance)."""
    shape = ri.SHAPES["tiny"]
    w, wn = make_both(shape, ri.BASE_SEED + 3)
    n_total, seed = 8, 4242
    p_len = ri.lengths(n_total, 3, 40, seed, 960).tolist()
    f_len = [p + int(e) for p, e in zip(p_len, ri.lengths(n_total, 2, 30, seed, 961).tolist())]
    prompts = [ri.tokens((n,), shape["vocab"], seed, 970 + i).tolist() for i, n in enumerate(p_len)]
    pages_needed = [(f + 15) // 16 for f in f_len]
    ro = amd.Rollout(shape, to_device(w), max_seqs=4, max_ctx=80, max_rows=4, kv_pages=max(pages_needed) * 2 + 1)
    ro.rl_debug_shuffle_free_pages(5)
    B = amd.binding
    waiting = list(range(n_total))
    active = {}                                   # slot id -> dict(idx, tokens, lps)
    results = {}
    logits = torch.empty(4, shape["vocab"], device=DEV)
    steps = 0
    while waiting or active:
        # admit as many waiting prompts as fit (library says KV_FULL when one does not)
        while waiting and len(active) < 4:
            idx = waiting[0]
            slot = next(s for s in range(4) if s not in active)
            free_pages, _ = ro.rl_kv_stats()
            try:
                tok, lp = ro.rl_prefill([slot], [prompts[idx]], 1.0, seed + idx)
            except B.RLError as e:
                assert e.status == B.RL_ERR_KV_FULL and ro.rl_kv_stats()[0] == free_pages
                break
            waiting.pop(0)
            active[slot] = dict(idx=idx, toks=[int(tok[0])], lps=[float(lp[0])], zs=[None])
        assert active, "pool too small for a single sequence"
        slots = sorted(active)
        cur = torch.tensor([active[s]["toks"][-1] for s in slots], dtype=torch.int32, device=DEV)
        # every sequence samples with its own seed in the real loop; here one seed per step call suffices
        # because the RNG stream is keyed by (seed, slot id, position) -- use the first sequence's seed
        try:
            tok, lp = ro.rl_decode_step(slots, cur, 1.0, seed, debug_logits=logits)
        except B.RLError as e:
            assert e.status == B.RL_ERR_KV_FULL
            victim = slots[-1]                    # preempt: give the pages back, requeue the prompt
            waiting.insert(0, active.pop(victim)["idx"])
            ro.rl_free_seqs([victim])
            continue
        torch.cuda.synchronize()
        zg = logits.cpu().numpy()
        done = []
        for i, s in enumerate(slots):
            a = active[s]
            a["toks"].append(int(tok[i]))
            a["lps"].append(float(lp[i]))
            a["zs"].append((zg[i].copy(), s))
            if p_len[a["idx"]] + len(a["toks"]) >= f_len[a["idx"]]:
                done.append(s)
        for s in done:
            a = active.pop(s)
            results[a["idx"]] = a
            ro.rl_free_seqs([s])
        steps += 1
        assert steps < 2000
    assert ro.rl_kv_stats()[0] == ro.rl_kv_stats()[1]
    assert sorted(results) == list(range(n_total))
    for idx, a in results.items():
        om = orc.OracleModel(dims_of(shape), wn, max_ctx=80)
        z = om.prefill(0, prompts[idx])
        pos = p_len[idx]
        for t in range(1, len(a["toks"])):
            z = om.forward_token(0, a["toks"][t - 1])
            pos += 1
            zg, slot = a["zs"][t]
            assert rel_inf(zg, z) < 1e-4, (idx, t)
            t_ref, lp_ref = orc.sample(zg, 1.0, seed, slot, pos)
            assert t_ref == a["toks"][t] and abs(lp_ref - a["lps"][t]) < 1e-5, (idx, t)
    ro.close()


@pytest.mark.parametrize("kind", ["tiny_f32", "small_bf16"])
def test_rollout_with_truncated_sampling_reproduced_from_logits(amd, kind):
    """Prefill + decode with temperature 0.6 / top-p 0.95 (and a top-k step): every drawn id and log-probability is
    what the oracle's truncated sampler gives on the logits the step produced."""
    if kind == "tiny_f32":
        shape = ri.SHAPES["tiny"]
        w, _ = make_both(shape, 81)
    else:
        shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=4, n_kv=1, ffn=768, vocab=8192)
        w, _ = make_both(shape, 81, std=0.05)
    V = shape["vocab"]
    ro = amd.Rollout(shape, to_device(w), max_seqs=8, max_ctx=96, max_rows=8, kv_pages=40)
    lens = [20, 33, 7]
    prompts = [ri.tokens((n,), V, 81, 970 + i).tolist() for i, n in enumerate(lens)]
    ids, seed = [4, 0, 6], 4242
    tok, lp = ro.rl_prefill(ids, prompts, 0.6, seed, top_p=0.95)
    z = torch.empty(3, V, device=DEV)
    pos = list(lens)
    for step in range(12):
        k, p = (0, 0.95) if step % 3 else (30, 0.8)
        tok, lp = ro.rl_decode_step(ids, tok, 0.6, seed, debug_logits=z, top_k=k, top_p=p)
        torch.cuda.synchronize()
        pos = [q + 1 for q in pos]
        zc = z.cpu().numpy()
        for r in range(3):
            t_ref, lp_ref, kept = orc.sample_truncated(zc[r], 0.6, k, p, seed, ids[r], pos[r])
            assert int(tok[r]) == t_ref and 1 <= kept < V, (step, r)
            assert abs(float(lp[r]) - lp_ref) < 1e-5 * max(1.0, abs(lp_ref))
    ro.close()


def test_group_rollout_loop_is_schedule_independent_and_matches_oracle(amd):
    """generate_groups: 5 prompts x 3 samples with pre-drawn ragged lengths in a pool that holds two groups at a
    time.  The tokens and log-probabilities equal those of a run with a pool for everything (the schedule does not
    matter), sequence by sequence the oracle's teacher-forced logits reproduce every draw, and with an end token
    the outputs stop right after it."""
    shape = ri.SHAPES["tiny"]
    w, wn = make_both(shape, ri.BASE_SEED + 4)
    G, seed = 3, 777
    p_len = ri.lengths(5, 5, 40, seed, 962).tolist()
    prompts = [ri.tokens((n,), shape["vocab"], seed, 980 + i).tolist() for i, n in enumerate(p_len)]
    limits = ri.lengths(5 * G, 1, 30, seed, 963).tolist()
    limits[4] = 1                                                  # a sequence that ends with its first token
    needs = [amd.group_page_need(len(p), limits[i * G:(i + 1) * G]) for i, p in enumerate(prompts)]
    wd = to_device(w)
    small = amd.Rollout(shape, wd, max_seqs=15, max_ctx=80, max_rows=4, kv_pages=max(needs) + sorted(needs)[1])
    big = amd.Rollout(shape, wd, max_seqs=15, max_ctx=80, max_rows=15, kv_pages=sum(needs))
    actives = []
    ta, la = amd.generate_groups(small, prompts, G, limits, 1.0, seed, on_step=lambda s, n: actives.append(n))
    tb, lb = amd.generate_groups(big, prompts, G, limits, 1.0, seed)
    assert ta == tb and la == lb
    assert [len(t) for t in ta] == limits
    assert small.rl_kv_stats()[0] == small.rl_kv_stats()[1] and big.rl_kv_stats()[0] == big.rl_kv_stats()[1]
    assert max(actives) <= 2 * G + G and min(actives) >= 0 and len(actives) > max(limits)   # several waves
    for k in (0, 4, 7, 14):                                       # oracle on whole sequences
        i = k // G
        om = orc.OracleModel(dims_of(shape), wn, max_ctx=80)
        z = om.prefill(0, prompts[i])
        pos = p_len[i]
        for t in range(limits[k]):
            t_ref, lp_ref = orc.sample(z, 1.0, seed, k, pos)
            assert t_ref == ta[k][t] and abs(lp_ref - la[k][t]) < 2e-5, (k, t)
            if t + 1 < limits[k]:
                z = om.forward_token(0, ta[k][t])
                pos += 1
    # an end token: every output is cut right after its first occurrence, and is otherwise unchanged
    flat = [t for seq in ta for t in seq[:-1]]
    eos = max(set(flat), key=flat.count)
    tc, lc = amd.generate_groups(small, prompts, G, limits, 1.0, seed, eos_id=eos)
    hit = 0
    for k in range(5 * G):
        cut = ta[k].index(eos) + 1 if eos in ta[k] else len(ta[k])
        assert tc[k] == ta[k][:cut] and lc[k] == la[k][:cut]
        hit += cut < len(ta[k])
    assert hit >= 1
    small.close()
    big.close()


# ------------------------------------------------------------------ grouped sampling with shared prompt pages
@pytest.mark.parametrize("kind", ["tiny_f32", "small_bf16"])
def test_prefill_groups_equals_independent_prefill(amd, kind):
    """G samples per prompt: the prompt runs once, full pages are shared, the partial page is copied.  Tokens,
    log-probs and every later decode step are bit-identical to prefilling the prompt G times; the oracle confirms
    the first tokens; the pool accounting shows the sharing."""
    if kind == "tiny_f32":
        shape = ri.SHAPES["tiny"]
        w, wn = make_both(shape, 61)
    else:
        shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=4, n_kv=1, ffn=768, vocab=8192)
        w, wn = make_both(shape, 61, std=0.05)
    G, seed = 4, 99
    lens = [37, 32, 5]                                 # partial page, exactly two pages, less than a page
    prompts = [ri.tokens((n,), shape["vocab"], 61, 980 + i).tolist() for i, n in enumerate(lens)]
    ids = list(range(len(lens) * G))
    wd = to_device(w)
    ra = amd.Rollout(shape, wd, max_seqs=16, max_ctx=96, max_rows=16, kv_pages=80)
    rb = amd.Rollout(shape, wd, max_seqs=16, max_ctx=96, max_rows=16, kv_pages=80)
    rb.rl_debug_shuffle_free_pages(17)
    ta, la = ra.rl_prefill(ids, [prompts[i // G] for i in ids], 1.0, seed)
    tb, lb = rb.rl_prefill_groups(ids, G, prompts, 1.0, seed)
    torch.cuda.synchronize()
    assert torch.equal(ta, tb) and torch.equal(la, lb)
    # independent: 3+2+1 pages per member; grouped: shared full pages + one private partial page per member
    assert ra.rl_kv_stats()[0] == 80 - G * (3 + 2 + 1)
    assert rb.rl_kv_stats()[0] == 80 - ((2 + G) + 2 + G)
    if kind == "tiny_f32":
        om = orc.OracleModel(dims_of(shape), wn, max_ctx=96)
        for i, p in enumerate(prompts):
            z = om.prefill(i, p)
            for j in range(G):
                t_ref, lp_ref = orc.sample(z, 1.0, seed, i * G + j, lens[i])
                assert int(tb[i * G + j]) == t_ref and abs(float(lb[i * G + j]) - lp_ref) < 2e-5
    assert len(set(tb.tolist())) > 3                   # members draw different first tokens
    za = torch.empty(len(ids), shape["vocab"], device=DEV)
    zb = torch.empty_like(za)
    for step in range(20):                             # crosses page boundaries of every member
        ta, la = ra.rl_decode_step(ids, ta, 1.0, seed, debug_logits=za)
        tb, lb = rb.rl_decode_step(ids, tb, 1.0, seed, debug_logits=zb)
        torch.cuda.synchronize()
        assert torch.equal(za, zb) and torch.equal(ta, tb) and torch.equal(la, lb), step
    # retiring members one by one returns shared pages only with their last holder
    rb.rl_free_seqs(ids[:G - 1] + ids[G:2 * G])
    free_mid = rb.rl_kv_stats()[0]
    rb.rl_free_seqs([ids[G - 1]] + ids[2 * G:])
    assert rb.rl_kv_stats() == (80, 80) and free_mid < 80
    ra.close()
    rb.close()


def test_shared_prompt_attention_is_bit_identical_to_per_row(amd):
    """Samples of one prompt at the same position have the attention over the common prompt pages computed once
    per set of rows.  Logits, tokens and log-probs equal, bit for bit, those with the sharing switched off and
    those of sequences prefilled one by one (which share nothing), for a prompt inside one block's segments, one
    beyond 4096 keys (partials through the workspace) and a short one; with sets of four and of two, a left-over
    row, members that retire, and members that fall out of step.  A fourth instance runs the rotation and the KV
    append as a kernel of their own instead of inside the attention kernel: same bits again, step after step (so
    the keys and values it leaves in the pages are the same too).  A fifth uses the widest sets (all seven samples
    of a prompt in one set, 28 columns in two operands) in the decode steps and in the prefill's window sets."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=8, n_kv=2, ffn=768, vocab=8192)
    w, _ = make_both(shape, 63, std=0.05)
    wd = to_device(w)
    G, seed = 7, 5
    lens = [1100, 4500, 300, 5]                  # the last one: a single 32-key step at first, no full prompt page
    prompts = [ri.tokens((n,), shape["vocab"], 63, 940 + i).tolist() for i, n in enumerate(lens)]
    ids = list(range(len(lens) * G))
    kw = dict(max_seqs=32, max_ctx=4608, max_rows=64, kv_pages=2750)
    ra = amd.Rollout(shape, wd, **kw)       # shared pages, shared attention
    rb = amd.Rollout(shape, wd, **kw)       # shared pages, every row on its own
    rc = amd.Rollout(shape, wd, **kw)       # nothing shared
    rd = amd.Rollout(shape, wd, **kw)       # shared pages and attention, separate rotation + append kernel
    re = amd.Rollout(shape, wd, **kw)       # shared pages and attention, widest sets
    rb.rl_debug_share_attention(False)
    rd.rl_debug_attention_appends(False)
    re.rl_debug_share_attention(2)
    ta, la = ra.rl_prefill_groups(ids, G, prompts, 1.0, seed)
    tb, lb = rb.rl_prefill_groups(ids, G, prompts, 1.0, seed)
    tc, lc = rc.rl_prefill(ids, [prompts[i // G] for i in ids], 1.0, seed)
    td, ld = rd.rl_prefill_groups(ids, G, prompts, 1.0, seed)
    te, le = re.rl_prefill_groups(ids, G, prompts, 1.0, seed)
    torch.cuda.synchronize()
    assert torch.equal(ta, tb) and torch.equal(la, lb) and torch.equal(ta, tc) and torch.equal(la, lc)
    assert torch.equal(ta, td) and torch.equal(la, ld) and torch.equal(ta, te) and torch.equal(la, le)
    V = shape["vocab"]
    every = (ra, rb, rc, rd, re)

    def step(active, tok):
        zs = [torch.empty(len(active), V, device=DEV) for _ in every]
        outs = [r.rl_decode_step(active, tok, 1.0, seed, debug_logits=z) for r, z in zip(every, zs)]
        torch.cuda.synchronize()
        for z, (t_, l_) in zip(zs[1:], outs[1:]):
            assert torch.equal(zs[0], z) and torch.equal(outs[0][0], t_) and torch.equal(outs[0][1], l_)
        return outs[0][0]

    tok = {i: int(ta[k]) for k, i in enumerate(ids)}
    active = list(ids)
    for it in range(36):                         # every slot of a page, both pages of a 32-key step
        if it == 6:                              # one member of each prompt retires: sets of four and two remain
            gone = [0, G + 3, 2 * G + 6]
            for r in every:
                r.rl_free_seqs(gone)
            active = [i for i in active if i not in gone]
        if it == 12:                             # two members of the first prompt fall one step behind
            behind = [1, 2]
            sub = [i for i in active if i not in behind]
            out = step(sub, torch.tensor([tok[i] for i in sub], dtype=torch.int32, device=DEV))
            for k, i in enumerate(sub):
                tok[i] = int(out[k])
        order = active if it % 2 == 0 else active[::-1]          # row order inside the batch is free
        out = step(order, torch.tensor([tok[i] for i in order], dtype=torch.int32, device=DEV))
        for k, i in enumerate(order):
            tok[i] = int(out[k])
    for r in every:
        r.close()


@pytest.mark.parametrize("n_q,n_kv", [(8, 1), (4, 2), (2, 2), (6, 2)])
def test_shared_attention_set_widths_agree_for_other_head_groupings(amd, n_q, n_kv):
    """Query heads per kv head other than the 8B model's four: eight (a set of four rows fills both 16-column
    operands), two (eight rows in one operand), one, and three (a row's heads straddle the two operands).  Logits,
    tokens and log-probs with the wide sets, with the narrow ones and with the sharing switched off are the same
    bits, for a prompt inside one block's segments and one beyond 4096 keys, with a retired member."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=n_q, n_kv=n_kv, ffn=768, vocab=8192)
    w, _ = make_both(shape, 64, std=0.05)
    wd = to_device(w)
    G, seed = 8, 9
    lens = [700, 4400]
    prompts = [ri.tokens((n,), shape["vocab"], 64, 950 + i).tolist() for i, n in enumerate(lens)]
    ids = list(range(len(lens) * G))
    kw = dict(max_seqs=16, max_ctx=4480, max_rows=32, kv_pages=700)
    every = [amd.Rollout(shape, wd, **kw) for _ in range(3)]
    for r, mode in zip(every, (0, 2, 3)):           # off, wide sets, narrow sets
        r.rl_debug_share_attention(mode)
    first = [r.rl_prefill_groups(ids, G, prompts, 1.0, seed) for r in every]
    torch.cuda.synchronize()
    for t_, l_ in first[1:]:
        assert torch.equal(first[0][0], t_) and torch.equal(first[0][1], l_)
    V = shape["vocab"]
    tok = {i: int(first[0][0][k]) for k, i in enumerate(ids)}
    active = list(ids)
    for it in range(6):
        if it == 3:                                  # seven and eight members from here on
            for r in every:
                r.rl_free_seqs([5])
            active.remove(5)
        t_in = torch.tensor([tok[i] for i in active], dtype=torch.int32, device=DEV)
        zs = [torch.empty(len(active), V, device=DEV) for _ in every]
        outs = [r.rl_decode_step(active, t_in, 1.0, seed, debug_logits=z) for r, z in zip(every, zs)]
        torch.cuda.synchronize()
        for z, (t_, l_) in zip(zs[1:], outs[1:]):
            assert torch.equal(zs[0], z) and torch.equal(outs[0][0], t_) and torch.equal(outs[0][1], l_), (it, n_q, n_kv)
        for k, i in enumerate(active):
            tok[i] = int(outs[0][0][k])
    for r in every:
        r.close()


def test_prefill_and_score_bits_do_not_depend_on_the_row_chunk(amd):
    """Prompts pushed through the layers 1024, 320 or 48 rows at a time (max_rows): the first tokens, their
    log-probabilities, the teacher-forced scores and the decode steps that follow are the same bits."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=8, n_kv=2, ffn=768, vocab=8192)
    w, _ = make_both(shape, 66, std=0.05)
    wd = to_device(w)
    lens = [1500, 700, 33]
    prompts = [ri.tokens((n,), shape["vocab"], 66, 960 + i).tolist() for i, n in enumerate(lens)]
    ids = [0, 1, 2]
    res = []
    for rows in (1024, 320, 48):
        ro = amd.Rollout(shape, wd, max_seqs=8, max_ctx=1536, max_rows=rows, kv_pages=300)
        t, lp = ro.rl_prefill(ids, prompts, 1.0, 3)
        sc = ro.rl_score([5, 6], [prompts[0][:1200], prompts[1]], 1.0)
        steps = [ro.rl_decode_step(ids, None, 1.0, 3) for _ in range(3)]
        torch.cuda.synchronize()
        res.append([t.cpu(), lp.cpu(), sc.cpu()] + [x.cpu() for st in steps for x in st])
        ro.close()
    for other in res[1:]:
        for a, b in zip(res[0], other):
            assert torch.equal(a, b)


# ------------------------------------------------------------------------------ teacher-forced scoring call
def test_score_matches_oracle_log_softmax(amd):
    shape = ri.SHAPES["tiny"]
    w, wn = make_both(shape, 71)
    ro = amd.Rollout(shape, to_device(w), max_seqs=8, max_ctx=64, max_rows=16, kv_pages=12)
    lens = [40, 2, 17]
    seqs = [ri.tokens((n,), shape["vocab"], 71, 990 + i).tolist() for i, n in enumerate(lens)]
    for T in (1.0, 0.7):
        out = ro.rl_score([4, 0, 7], seqs, T).cpu().numpy()
        assert ro.rl_kv_stats() == (12, 12)             # scratch sequences are gone
        invT = float(np.float32(1.0) / np.float32(T))
        k = 0
        for i, q in enumerate(seqs):
            om = orc.OracleModel(dims_of(shape), wn, max_ctx=64)
            for t in range(len(q) - 1):
                ls = orc.log_softmax(om.forward_token(0, q[t]), invT)
                assert abs(out[k] - ls[q[t + 1]]) < 2e-5, (T, i, t)
                k += 1
        assert k == out.size
    B = amd.binding
    with pytest.raises(B.RLError) as e:
        ro.rl_score([0], [list(range(70))], 1.0)
    assert e.value.status == B.RL_ERR_CTX_OVERFLOW and ro.rl_kv_stats() == (12, 12)
    ro.close()


def test_score_bf16_matches_oracle_log_softmax(amd):
    """The scoring call on the bf16 path (MFMA projections, windowed attention sets, output projection fused with the
    log-sum-exp) against the oracle's log-softmax of its own teacher-forced logits, at two temperatures; sequences
    longer than a chunk of rows, a two-token one, and one that ends exactly on a page."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=4, n_kv=1, ffn=768, vocab=8192)
    w, wn = make_both(shape, 73, std=0.05)
    ro = amd.Rollout(shape, to_device(w), max_seqs=8, max_ctx=128, max_rows=24, kv_pages=24)
    lens = [70, 2, 32, 45]
    seqs = [ri.tokens((n,), shape["vocab"], 73, 990 + i).tolist() for i, n in enumerate(lens)]
    for T in (1.0, 0.7):
        out = ro.rl_score([4, 0, 7, 2], seqs, T).cpu().numpy()
        assert ro.rl_kv_stats() == (24, 24)
        invT = float(np.float32(1.0) / np.float32(T))
        k, worst = 0, 0.0
        for i, q in enumerate(seqs):
            om = orc.OracleModel(dims_of(shape), wn, max_ctx=128)
            for t in range(len(q) - 1):
                ls = orc.log_softmax(om.forward_token(0, q[t]), invT)
                worst = max(worst, abs(float(out[k]) - float(ls[q[t + 1]])))
                k += 1
        assert k == out.size
        assert worst < 5e-2, (T, worst)
    ro.close()


@pytest.mark.parametrize("kind", ["tiny_f32", "small_bf16"])
def test_rescored_rollout_gives_ratio_one(amd, kind):
    """With theta = theta_old the probability ratio of the objective is exactly one: the log-probs returned while
    sampling equal the log-probs of a teacher-forced pass over the finished sequences."""
    if kind == "tiny_f32":
        shape = ri.SHAPES["tiny"]
        w, _ = make_both(shape, 72)
    else:
        shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=4, n_kv=1, ffn=768, vocab=8192)
        w, _ = make_both(shape, 72, std=0.05)
    ro = amd.Rollout(shape, to_device(w), max_seqs=8, max_ctx=96, max_rows=24, kv_pages=40)
    G, seed, n_new = 3, 5, 30
    prompts = [ri.tokens((n,), shape["vocab"], 72, 995 + i).tolist() for i, n in enumerate([21, 16])]
    ids = list(range(2 * G))
    tok, lp = ro.rl_prefill_groups(ids, G, prompts, 1.0, seed)
    toks, lps = [tok.cpu()], [lp.cpu()]
    for _ in range(n_new - 1):
        tok, lp = ro.rl_decode_step(ids, tok, 1.0, seed)
        toks.append(tok.cpu())
        lps.append(lp.cpu())
    toks, lps = torch.stack(toks, 1), torch.stack(lps, 1)          # [6, n_new]
    ro.rl_free_seqs(ids)
    full = [prompts[i // G] + toks[i].tolist() for i in ids]
    sc = ro.rl_score(ids, full, 1.0).cpu()
    k = 0
    for i in ids:
        P = len(prompts[i // G])
        got = sc[k + P - 1:k + P - 1 + n_new]
        ratio = torch.exp(got - lps[i])
        assert torch.all((ratio - 1).abs() < 1e-5), (i, (ratio - 1).abs().max())
        k += len(full[i]) - 1
    assert len({tuple(t.tolist()) for t in toks[:G]}) == G          # the samples of one prompt differ
    ro.close()


# ----------------------------------------------------------------------------------- decode step as a HIP graph
@pytest.mark.parametrize("kv_fp8,G,wide", [(False, 4, False), (True, 4, False), (False, 8, True)])
def test_decode_graph_steps_equal_eager_steps(amd, kv_fp8, G, wide):
    """rl_decode_graph_step against rl_decode_step on a second instance: same tokens and log-probabilities, bit for
    bit, on every one of 40 steps (compared after each launch, with eager work and synchronisations in between).  The
    batch holds two groups of four samples (shared prompt pages: set blocks in the attention launch) and a single
    sequence whose context crosses 1024 tokens on the way, which changes a launch shape and forces a new capture; page
    grants arrive every 16 steps through the device-counted table update.  An eager step in the middle of the graph
    steps keeps both instances in agreement too.  In the third case the groups have eight samples and the graph
    instance uses the wide sets (two operands) while the eager one keeps sets of four."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=8, n_kv=2, ffn=768, vocab=8192)
    w, _ = make_both(shape, 65, std=0.05)
    wd = to_device(w)
    seed = 9
    lens = [1003, 70, 33]
    prompts = [ri.tokens((n,), shape["vocab"], 65, 940 + i).tolist() for i, n in enumerate(lens)]
    ids = list(range(2 * G + 1))
    kw = dict(max_seqs=24, max_ctx=1088, max_rows=64, kv_pages=280, kv_fp8=kv_fp8)
    ra, rb = amd.Rollout(shape, wd, **kw), amd.Rollout(shape, wd, **kw)
    if wide:
        ra.rl_debug_share_attention(2)
    for r in (ra, rb):
        r.rl_prefill_groups(ids[:2 * G], G, prompts[1:], 1.0, seed)
        r.rl_prefill([2 * G], [prompts[0]], 1.0, seed)
    g = ra.decode_graph(ids, 1.0, seed)
    with pytest.raises(amd.binding.RLError) as e:         # the null stream cannot be captured
        g.step()
    assert e.value.status == amd.binding.RL_ERR_INVALID_ARG
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for step in range(40):
            if step == 20:                                # an eager step between graph steps, on both instances
                ta, la = ra.rl_decode_step(ids, None, 1.0, seed)
            else:
                ta, la = g.step()
            tb, lb = rb.rl_decode_step(ids, None, 1.0, seed)
            torch.cuda.synchronize()
            assert torch.equal(ta, tb) and torch.equal(la, lb), step
    assert [ra.rl_seq_len(i) for i in ids] == [rb.rl_seq_len(i) for i in ids] == [110] * G + [73] * G + [1043]
    assert 2 <= g.captures <= 6, g.captures               # two buffers, one change of shape
    g.close()
    ra.close()
    rb.close()


# ------------------------------------------------------------------------------- fp8 keys and values (opt-in)
def _e4m3_exact(shape_, seed, tid):
    """Random values that every fp8 e4m3 variant represents exactly: multiples of 0.25 in [-2, 2]."""
    return (ri.lengths(int(np.prod(shape_)), -8, 8, seed, tid).float() * 0.25).reshape(shape_).to(torch.bfloat16)


def test_fp8_kv_layer_with_exactly_representable_cache_matches_oracle(amd):
    """fp8 pages pin their layout: imported keys and values that e4m3 represents exactly lose nothing in the cache, so
    the layer must match the oracle to the bf16 bound (only each row's own new key and value are rounded to fp8: one
    key among >= 100).  Contexts on page, step and merge boundaries, a forked group (shared pages, set blocks), and
    bit equality with the shared-prompt treatment switched off."""
    shape = ri.SHAPES["layer8b"]
    w, wn = make_both(shape, 38)
    wd = to_device(w)
    nkv, d, H = shape["n_kv"], shape["head_dim"], shape["hidden"]
    ctxs = [100, 255, 256, 257, 700, 1023, 1024, 4095, 5000]
    G = 4                                                   # the last context is continued as four samples
    ks = [_e4m3_exact((c, nkv, d), 38, 2000 + 2 * b) for b, c in enumerate(ctxs)]
    vs = [_e4m3_exact((c, nkv, d), 38, 2001 + 2 * b) for b, c in enumerate(ctxs)]
    n = len(ctxs) + G - 1
    x = ri.normal((n, H), 1.0, 38, 1999).to(torch.bfloat16).float()
    pages = sum((c + 16) // 16 + 1 for c in ctxs) + 2 * G + 8
    outs = []
    for share in (True, False):
        ro = amd.Rollout(shape, wd, max_seqs=n, max_ctx=5056, max_rows=n, kv_pages=pages, kv_fp8=True)
        assert ro.cfg.kv_pool_bytes == pages * 16 * nkv * d * 2          # one byte per element, K and V
        ro.rl_debug_shuffle_free_pages(13)
        ro.rl_debug_share_attention(share)
        for b in range(len(ctxs)):
            ro.rl_seq_import_kv(b, [ks[b].to(DEV)], [vs[b].to(DEV)])
        last = len(ctxs) - 1
        ro.rl_seq_fork(last, list(range(len(ctxs), n)))
        outs.append(ro.rl_decode_hidden(list(range(n)), x.to(DEV)).cpu())
        ro.close()
    assert torch.equal(outs[0], outs[1])
    out = outs[0].numpy()
    for r in range(n):
        b = min(r, len(ctxs) - 1)
        ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[r], ctxs[b])
        err = rel_inf(out[r] - x[r].numpy(), ref - x[r].numpy())
        assert err < 3e-2, (r, ctxs[b], err)


def test_fp8_kv_layer_random_cache_within_the_fp8_tolerance(amd):
    """N(0,1) keys and values cached as fp8 against the oracle, which never rounds them.  e4m3 keeps 4 significant
    bits: each cached element is within 2^-4 relative (about 2.6e-2 rms), the scores and the value average inherit
    that, and the layer's output moves by a few per cent of its change to the residual stream: bound 1e-1."""
    ctxs = [0, 1, 15, 16, 17, 255, 256, 257, 700, 2048, 4500]
    shape = ri.SHAPES["layer8b"]
    w, wn = make_both(shape, 31)
    nkv, d, H = shape["n_kv"], shape["head_dim"], shape["hidden"]
    n = len(ctxs)
    ro = amd.Rollout(shape, to_device(w), max_seqs=n, max_ctx=4544, max_rows=n,
                     kv_pages=sum((c + 16) // 16 + 1 for c in ctxs) + 4, kv_fp8=True)
    ro.rl_debug_shuffle_free_pages(9)
    ks = [ri.normal((c, nkv, d), 1.0, 31, 2000 + 2 * b, dtype=torch.bfloat16) for b, c in enumerate(ctxs)]
    vs = [ri.normal((c, nkv, d), 1.0, 31, 2001 + 2 * b, dtype=torch.bfloat16) for b, c in enumerate(ctxs)]
    for b in range(n):
        ro.rl_seq_import_kv(b, [ks[b].to(DEV)], [vs[b].to(DEV)])
    x = ri.normal((n, H), 1.0, 31, 1999).to(torch.bfloat16).float()
    out = ro.rl_decode_hidden(list(range(n)), x.to(DEV)).cpu().numpy()
    worst = 0.0
    for b, c in enumerate(ctxs):
        ref = _oracle_layer_row(shape, wn, ks[b], vs[b], x[b], c)
        err = float(rel_inf(out[b] - x[b].numpy(), ref - x[b].numpy()))
        worst = max(worst, err)
        assert err < 1e-1, (b, c, err)
    print(f"[fp8 kv] worst layer error with N(0,1) keys and values: {worst:.2e}")
    ro.close()


def test_fp8_kv_small_model_rollout_fused_and_separate_append_agree(amd):
    """A 2-layer bf16 model with fp8 pages: grouped prefill + 36 sampled steps.  The attention kernel's own rotation
    and append (new key and value patched into its operands, bytes written afterwards) give the bits of the separate
    append kernel, with shared-prompt sets on and off; logits stay within the fp8 bound of the oracle's (one layer's
    bound 1e-1, errors of independent roundings add in squares over the two layers: 1.41e-1), and the sampled ids are
    the oracle sampler's on the GPU's logits."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=2, hidden=512, n_q=8, n_kv=2, ffn=768, vocab=8192)
    w, wn = make_both(shape, 64, std=0.05)
    wd = to_device(w)
    G, seed = 4, 5
    lens = [300, 40, 5]
    prompts = [ri.tokens((n,), shape["vocab"], 64, 940 + i).tolist() for i, n in enumerate(lens)]
    ids = list(range(len(lens) * G))
    kw = dict(max_seqs=16, max_ctx=352, max_rows=64, kv_pages=120, kv_fp8=True)
    ra, rb, rc = (amd.Rollout(shape, wd, **kw) for _ in range(3))
    rb.rl_debug_attention_appends(False)
    rc.rl_debug_share_attention(False)
    every = (ra, rb, rc)
    toks = [r.rl_prefill_groups(ids, G, prompts, 1.0, seed) for r in every]
    torch.cuda.synchronize()
    for t_, l_ in toks[1:]:
        assert torch.equal(toks[0][0], t_) and torch.equal(toks[0][1], l_)
    oms = {}
    for i in ids:
        oms[i] = orc.OracleModel(dims_of(shape), wn, max_ctx=352)
        oms[i].prefill(0, prompts[i // G])
    V = shape["vocab"]
    tok = toks[0][0]
    worst = 0.0
    for step in range(36):
        zs = [torch.empty(len(ids), V, device=DEV) for _ in every]
        outs = [r.rl_decode_step(ids, tok, 1.0, seed, debug_logits=z) for r, z in zip(every, zs)]
        torch.cuda.synchronize()
        for z, (t_, l_) in zip(zs[1:], outs[1:]):
            assert torch.equal(zs[0], z) and torch.equal(outs[0][0], t_) and torch.equal(outs[0][1], l_), step
        zg = zs[0].cpu().numpy()
        for k, i in enumerate(ids):
            z = oms[i].forward_token(0, int(tok[k]))
            worst = max(worst, float(rel_inf(zg[k], z)))
            t_ref, lp_ref = orc.sample(zg[k], 1.0, seed, i, lens[i // G] + step + 1)
            assert int(outs[0][0][k]) == t_ref and abs(float(outs[0][1][k]) - lp_ref) < 1e-4
        tok = outs[0][0]
    assert worst < 1e-1 * 2 ** 0.5, worst
    print(f"[fp8 kv] 2-layer model, worst logit error over 36 steps: {worst:.2e}")
    for r in every:
        r.close()


def test_bf16_sampled_step_bits_do_not_depend_on_batch_size_class(amd):
    """The output projection with the sampling epilogue also changes kernels with the batch.  A 1-layer model wide
    enough for every variant (hidden 1024, vocabulary 24576): three sequences decoded alone, among 40, 100, 150,
    300 and 600 rows (more than one batch tile of 256) give the same logits, tokens and log-probabilities, bit for
    bit, sampled and greedy."""
    shape = dict(ri.SHAPES["layer8b"], n_layers=1, hidden=1024, n_q=8, n_kv=2, ffn=1024, vocab=24576)
    w, _ = make_both(shape, 43, std=0.05)
    wd = to_device(w)
    n_max = 600
    prompts = [ri.tokens((3 + i % 5,), shape["vocab"], 43, 3000 + i).tolist() for i in range(n_max)]
    V = shape["vocab"]
    res = []
    for n in (3, 40, 100, 150, 300, 600):
        ro = amd.Rollout(shape, wd, max_seqs=n_max, max_ctx=32, max_rows=256 if n <= 256 else 1024, kv_pages=2 * n_max)
        ids = list(range(n))
        tok, lp = ro.rl_prefill(ids, prompts[:n], 1.0, 9)
        outs = [(tok[:3].clone(), lp[:3].clone())]
        for T in (1.0, 0.0, 0.7):
            z = torch.empty(n, V, device=DEV)
            tok, lp = ro.rl_decode_step(ids, tok, T, 9, debug_logits=z)
            outs.append((tok[:3].clone(), lp[:3].clone(), z[:3].clone()))
        torch.cuda.synchronize()
        res.append(outs)
        ro.close()
    for other in res[1:]:
        for a, b in zip(res[0], other):
            assert all(torch.equal(x, y) for x, y in zip(a, b))


def test_bf16_layer_bits_do_not_depend_on_batch_size_class(amd):
    """The projection kernels change shape with the batch (32-, 64-, 128-, 256-column variants); a row's result must
    keep its bits in all of them."""
    base = [40, 513, 100, 257, 31]
    outs = []
    for n in (5, 40, 70, 140):
        ctxs = base + [(11 * i) % 60 for i in range(n - 5)]
        shape, wn, ro, ks, vs, x = _layer_case(amd, ctxs, seed=35)
        outs.append(ro.rl_decode_hidden(list(range(n)), x.to(DEV)).cpu()[:5])
        ro.close()
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
