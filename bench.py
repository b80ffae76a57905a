"""Benchmark of the rollout hot path on one MI355X.

Workload "wave" (default): the largest batch one GPU holds at the paper's limits (Appendix D: 32 prompts per batch,
prompts up to 2048 tokens, responses up to 16384, G samples per prompt).  The 36-layer 8B-shaped bf16 policy, 16
prompts x group 8 = 128 resident sequences (what fits beside the weights when every sequence may grow to 16384
tokens: one of the two waves of the 32-prompt batch), prompts of 2048 tokens prefilled once per group (pages shared
by the 8 samples), every sample then placed at --ctx-mid tokens of context (default 9216, the mean of a run from
2048 to 16384) by appending private N(0,1) keys and values, then EXACTLY --steps decode steps are timed; one step =
embed, 36 layers (norm, QKV, rotary+append, paged attention, O, norm, gate/up+SwiGLU, down), final norm, lm_head,
Gumbel-max sampling with log-probs, for all 128 sequences.  Everything is resident in HBM when the timed region
starts.  The same model then runs the 32-sequence workload (4 prompts x 8, prompts 1024) for comparison; its
figures are extra keys of the one JSON line that is printed.

Workload "full": the 32-sequence workload alone (4 prompts x group 8, 1024-token prompts, 1024 generated tokens).

Workload "layer8b_b64_ctx2048" (--workload layer): one decoder layer at the same dimensions, batch 64 over
2048 cached tokens per sequence, one decode step per "step".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic of the dominant kernels from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/hbm_traffic_counters.md),
# stored as measured bytes / algorithmic bytes of the same launches, each counter scaled by what it reads for a plain
# 1 GiB device copy (FETCH_SIZE x 2.0000, WRITE_SIZE x 1.0000).  An entry is used only while the kernel's source
# file still has the hash it had when the counters were taken; otherwise "traffic" is null.
TRAFFIC_RATIO = {
    # one layer at the launch shape of the 128-sequence wave (16 groups x 8 samples, 2048 shared + 7168 private tokens)
    ("wave", "attn_decode"): (1.044, "attn_bf16.hip", "bf9a68219783273c"),
    ("layer", "attn_decode"): (1.044, "attn_bf16.hip", "bf9a68219783273c"),
    ("full", "attn_decode"): (1.040, "attn_bf16.hip", "bf9a68219783273c"),
    ("full", "gemm_gate_up_swiglu"): (1.011, "gemm_bf16.hip", "c85762f8c6f26887"),
}


def measured_traffic(workload, kernel, algorithmic_bytes):
    import hashlib
    ent = TRAFFIC_RATIO.get((workload, kernel))
    if ent is None:
        return None
    ratio, src, sha = ent
    path = os.path.join(ROOT, "paper_2510_17891_amd", "csrc", src)
    try:
        cur = hashlib.sha256(open(path, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    return ratio * algorithmic_bytes if cur == sha else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed decode steps; default: full workload 1015 (with the prefill token and 8 warm-up steps "
                         "that is the 1024 generated tokens per sequence of the workload), others 512")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", choices=["wave", "full", "layer", "copy", "ragged", "max", "tiny", "objective", "score", "prefill", "sched"],
                    default="wave")
    ap.add_argument("--score-len", type=int, default=1024, help="score workload: tokens per sequence (32 x 8 sequences)")
    ap.add_argument("--prefill-len", type=int, default=2048, help="prefill workload: tokens per prompt (32 prompts)")
    ap.add_argument("--chunk-rows", type=int, default=1024,
                    help="prefill and score workloads: rows (tokens) pushed through the layers per launch (max_rows)")
    ap.add_argument("--ctx-mid", type=int, default=9216,
                    help="wave workload: tokens of context per sequence when the timed region starts")
    ap.add_argument("--wave-prompts", type=int, default=16, help="wave workload: resident prompts (x 8 samples each)")
    ap.add_argument("--kv-fp8", action="store_true",
                    help="wave / full workloads: cache keys and values as fp8 (opt-in performance variant, not the headline)")
    ap.add_argument("--attn-split", type=int, default=0,
                    help="wave workload: segments per attention block beyond 4096 keys (0: the library's default)")
    ap.add_argument("--graph", action="store_true",
                    help="wave workload: launch every decode step as a HIP graph (rl_decode_graph_step)")
    ap.add_argument("--no-small-batch", action="store_true",
                    help="wave workload: skip the 32-sequence comparison run")
    ap.add_argument("--length-scale", type=float, default=1.0,
                    help="ragged workload: multiply the drawn prompt and final lengths (1.0: prompts U[256,1024], "
                         "final lengths U[1024,8192]); max workload: multiply prompt 2048 and total context 16384")
    ap.add_argument("--profile-steps", type=int, default=8, help="extra steps run with per-kernel events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--contiguous-pages", action="store_true",
                    help="layer workload: give every sequence consecutive pages instead of a random permutation")
    ap.add_argument("--batch", type=int, default=64, help="layer workload: sequences per step")
    ap.add_argument("--ctx", type=int, default=2048, help="layer workload: cached tokens per sequence at the start")
    ap.add_argument("--prefill", choices=["real", "import"], default="real",
                    help="import: fill the prompt KV with random N(0,1) pages instead of running the prefill "
                         "(for counter runs that should only see decode steps)")
    ap.add_argument("--group", type=int, default=1,
                    help="layer workload: every `group` consecutive sequences continue one cached context (shared pages)")
    ap.add_argument("--grow", type=int, default=0,
                    help="layer workload: untimed decode steps after the import (the members of a group get private "
                         "tokens on top of the shared context)")
    ap.add_argument("--grow-append", action="store_true",
                    help="layer workload: --grow tokens are appended as random keys and values instead of decoded")
    ap.add_argument("--n-prompts", type=int, default=4, help="full workload: prompts (x 8 samples each); 4 is the headline")
    ap.add_argument("--temperature", type=float, default=1.0, help="full workload: sampling temperature")
    ap.add_argument("--top-k", type=int, default=0, help="full workload: top-k cut (0: none)")
    ap.add_argument("--top-p", type=float, default=0.0, help="full workload: top-p cut (0: none)")
    ap.add_argument("--no-share-attention", action="store_true",
                    help="full workload: attention over the prompt pages once per row instead of once per set of samples")
    ap.add_argument("--set-width", type=int, choices=[1, 2, 3], default=1,
                    help="full and layer workloads: rows per set of samples; 1: the library's rule, 2: always the wide "
                         "sets (two operands), 3: never")
    ap.add_argument("--separate-append", action="store_true",
                    help="rotation and KV append as a kernel of their own instead of inside the decode attention kernel")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = {"full": 1015, "wave": 20, "tiny": 320, "objective": 200, "sched": 200}.get(args.workload, 512)
    return args


def kernel_bytes(shape, M, ctx_sum, bf=2, kv_bytes=2):
    """Algorithmic HBM bytes of one launch of each kernel class at batch M.  ctx_sum: cached tokens the step must
    read, summed over the batch, pages that several sequences hold in common counted once."""
    H, d, F, V = shape["hidden"], shape["head_dim"], shape["ffn"], shape["vocab"]
    nq, nkv = shape["n_q"], shape["n_kv"]
    nqkv, nqd = (nq + 2 * nkv) * d, nq * d
    return {
        "gemm_qkv": nqkv * H * bf + M * H * bf + M * nqkv * 4,
        "gemm_o": H * nqd * bf + M * nqd * bf + M * H * 4,
        "gemm_gate_up_swiglu": 2 * F * H * bf + M * H * bf + M * F * bf,
        "gemm_down": H * F * bf + M * F * bf + M * H * 4,
        "gemm_lm_head": V * H * bf + M * H * bf + M * V * 4,
        # K/V pages, the QKV projection's output (summed, rotated and appended inside the kernel), the bf16 output
        "attn_decode": ctx_sum * nkv * 2 * d * kv_bytes + M * nqkv * 4 + M * nqd * bf + M * 2 * nkv * d * kv_bytes,
    }


def cpu_baseline_full(shape, ctx, n_seq=16, head_fraction=8):
    """Time the oracle on a bounded sample of a decode step: n_seq sequences at context `ctx`, each pushed through
    n_layers decoder-layer passes (one layer's weights, used for every pass) and 1/head_fraction of the output
    projection's rows, which is scaled up.  Returns tokens/s of the oracle for one sequence at a time."""
    import numpy as np
    import torch
    import rollout_inputs as ri
    from oracle import oracle as orc
    dims = {k: shape[k] for k in ("hidden", "n_q", "n_kv", "head_dim", "ffn", "qk_norm", "rms_eps", "rope_base")}
    lw = {k: np.ascontiguousarray(v.to(torch.bfloat16).float().numpy())
          for k, v in ri.make_layer(shape, ri.BASE_SEED, 0).items()}
    rows = shape["vocab"] // head_fraction
    lm = np.ascontiguousarray(ri.normal((rows, shape["hidden"]), 0.02, ri.BASE_SEED, 2).to(torch.bfloat16).float().numpy())
    kc = np.ascontiguousarray(ri.normal((ctx + 1, shape["n_kv"], shape["head_dim"]), 1.0, ri.BASE_SEED, 7).numpy())
    vc = kc.copy()
    x = ri.normal((n_seq, shape["hidden"]), 1.0, ri.BASE_SEED, 8).numpy()
    orc.matvec(lm[:64], x[0])  # load the library, spin up threads
    t0 = time.perf_counter()
    for s in range(n_seq):
        for _ in range(shape["n_layers"]):
            xs = np.ascontiguousarray(x[s].copy())  # every pass from a unit-scale input: the arithmetic is the same
            orc.layer_forward(dims, lw, xs, ctx, kc, vc)
    t_layers = (time.perf_counter() - t0) / n_seq
    t0 = time.perf_counter()
    for s in range(n_seq):
        orc.matvec(lm, x[s])
    t_head_measured = time.perf_counter() - t0
    t_head = t_head_measured / n_seq * head_fraction
    t_tok = t_layers + t_head
    return {"value": 1.0 / t_tok, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"oracle timed on {n_seq} sequences x {shape['n_layers']} decoder-layer passes at context {ctx} "
                      f"(one layer's weights for every pass) and 1/{head_fraction} of the lm_head rows (scaled up); "
                      f"{n_seq * t_layers + t_head_measured:.1f} s of CPU work timed, sampler excluded"}


def kernel_table(prof, kb):
    """{kernel class: launches, mean microseconds, share of the summed durations, achieved GB/s} from the library's
    event timings `prof` and the algorithmic bytes per launch `kb`."""
    kernels = {}
    for name, (cnt, ms) in prof.items():
        if cnt == 0:
            continue
        avg_us = ms / cnt * 1e3
        entry = {"launches": cnt, "avg_us": avg_us, "share": None}
        if name in kb:
            entry["achieved_GBs"] = kb[name] / (avg_us * 1e-6) / 1e9
            entry["bytes"] = kb[name]
        kernels[name] = entry
    tot = sum(e["avg_us"] * e["launches"] for e in kernels.values())
    for e in kernels.values():
        e["share"] = e["avg_us"] * e["launches"] / tot
    return kernels


def step_bytes_of(shape, kbm):
    return shape["n_layers"] * (kbm["gemm_qkv"] + kbm["gemm_o"] + kbm["gemm_gate_up_swiglu"] + kbm["gemm_down"]
                                + kbm["attn_decode"]) + kbm["gemm_lm_head"]


def run_wave(args):
    """The default workload: one resident wave of the largest batch at mid-run context, then the 32-sequence batch."""
    import torch
    import rollout_inputs as ri
    from paper_2510_17891_amd import Rollout
    from paper_2510_17891_amd.binding import _i32
    dev = "cuda:0"
    torch.cuda.set_device(0)
    seed = ri.BASE_SEED + 2
    shape = ri.SHAPES["full8b"]
    L, nkv, d = shape["n_layers"], shape["n_kv"], shape["head_dim"]
    n_prompts, G, P = args.wave_prompts, 8, 2048
    B = n_prompts * G
    ctx_mid = max(P, args.ctx_mid)
    private = ctx_mid - P
    n_steps = args.warmup + args.steps + 4 + args.profile_steps
    max_ctx = (max(ctx_mid + n_steps, 1024 + 64 + n_steps) + 1 + 15) // 16 * 16
    pages = n_prompts * (P // 16 + G * ((ctx_mid + n_steps + 15) // 16 - P // 16)) + 64
    t_setup = time.perf_counter()
    w = ri.make_weights(shape, seed, device=dev, dtype=torch.bfloat16)
    ro = Rollout(shape, w, max_seqs=B, max_ctx=max_ctx, max_rows=256, kv_pages=pages, consume_weights=True,
                 kv_fp8=args.kv_fp8)
    del w
    torch.cuda.empty_cache()
    if args.attn_split:
        ro.rl_debug_attention_split(args.attn_split)
    if args.separate_append:
        ro.rl_debug_attention_appends(False)
    prompts = ri.tokens((n_prompts, P), shape["vocab"], seed, 960)
    seq_ids = list(range(B))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if args.prefill == "real":
        tok, lp = ro.rl_prefill_groups(seq_ids, G, [prompts[i].tolist() for i in range(n_prompts)], 1.0, seed)
    else:
        # counter runs that should only see decode steps: the prompt's keys and values are imported (N(0,1)) for the
        # first sample of a group and the others are forked from it, which shares the prompt pages like the prefill does
        for g in range(n_prompts):
            kv = [ri.normal((P, nkv, d), 1.0, seed, 6000 + g * L + l, device=dev, dtype=torch.bfloat16) for l in range(L)]
            ro.rl_seq_import_kv(g * G, kv, kv[::-1])
            ro.rl_seq_fork(g * G, list(range(g * G + 1, (g + 1) * G)))
            del kv
        tok = ri.tokens((B,), shape["vocab"], seed, 961).to(dev)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    if private > 0:
        # every sample gets its own response tokens' keys and values: N(0,1) on the bf16 grid, drawn per (sequence, layer)
        for b in seq_ids:
            kv = [ri.normal((private, nkv, d), 1.0, seed, 7000 + b * L + l, device=dev, dtype=torch.bfloat16)
                  for l in range(L)]
            ro.rl_seq_append_kv(b, kv, kv[::-1])
            del kv
        torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup
    ids = _i32(seq_ids)
    bufs = [(torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.float32, device=dev))
            for _ in range(2)]
    state = {"cur": tok, "i": 0}

    graphs = {}

    def step(id_arr=ids, n=B):
        if args.graph:
            if n not in graphs:
                graphs[n] = ro.decode_graph(list(id_arr), 1.0, seed)
            graphs[n].step()
            return
        ot, ol = bufs[state["i"] & 1]
        ro.rl_decode_step(id_arr, state["cur"], 1.0, seed, out_tokens=ot[:n], out_logprobs=ol[:n])
        state["cur"] = ot[:n]
        state["i"] += 1

    if args.graph:   # a graph cannot be captured on the null stream: everything from here on runs on a stream of its own
        torch.cuda.synchronize()
        torch.cuda.set_stream(torch.cuda.Stream())
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # Per-kernel durations: HIP events bracket every launch of the steps that directly follow the timed region (events
    # on every launch cost about 8 % of a step, so they stay out of `value`; the contexts are args.steps tokens longer,
    # 0.2 % at this length).  A graph launch has no per-kernel events.
    n_prof = 0 if (args.no_profile or args.graph) else max(1, min(args.profile_steps, 4))
    if n_prof:
        ro.rl_profile_enable(True)
        for _ in range(n_prof):
            step()
        torch.cuda.synchronize()
        ro.rl_profile_enable(False)
    ms_per_step = elapsed / args.steps * 1e3
    ctx_first = ctx_mid + args.warmup + 1            # keys the first timed step attends to (its own token included)
    ctx_last = ctx_first + args.steps - 1
    ctx_avg = 0.5 * (ctx_first + ctx_last)
    shared_tok = P // 16 * 16

    def ctx_sum(ctx, once):
        return int((n_prompts if once else B) * shared_tok + B * (ctx - shared_tok))

    kvb = 1 if args.kv_fp8 else 2
    kb_once = kernel_bytes(shape, B, ctx_sum(ctx_avg, True), kv_bytes=kvb)
    kb_each = kernel_bytes(shape, B, ctx_sum(ctx_avg, False), kv_bytes=kvb)
    out = {
        "metric": "generated tokens/s (8B-shaped bf16 decode) + % peak HBM GB/s, 1 MI355X",
        "value": B * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"full8b_36L_bf16_wave_{B}seq_prompt{P}_ctx{ctx_mid}_T1.0" + ("_kvfp8" if args.kv_fp8 else ""),
                   "batch": B, "groups": n_prompts,
                   "group_size": G, "context_first_timed_step": ctx_first, "context_last_timed_step": ctx_last,
                   "kv_block": 16, "temperature": 1.0, "logprob_per_token": True, "shared_prompt_tokens": shared_tok,
                   "prefill": (f"{n_prompts} prompts x {P} tokens run once each, pages shared by the {G} samples of a prompt"
                               if args.prefill == "real" else "prompt keys and values imported, samples forked"),
                   "private_context": f"{private} tokens per sequence of appended N(0,1) keys and values",
                   "kv_pool_GB": pages * rl_page_bytes(shape) * kvb / 2 / 1e9},
        # step-level fractions: per-sequence byte formula (weights once + 4096 B per cached token, layer and sequence),
        # and the smaller figure with the prompt pages that 8 samples hold in common counted once
        "step_algorithmic_GB": step_bytes_of(shape, kb_each) / 1e9,
        "step_hbm_fraction": step_bytes_of(shape, kb_each) / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9),
        "step_GB_shared_pages_once": step_bytes_of(shape, kb_once) / 1e9,
        "step_hbm_fraction_shared_pages_once": step_bytes_of(shape, kb_once) / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9),
        "prefill_s": prefill_s, "prefill_prompt_tokens_per_s": n_prompts * P / prefill_s, "setup_s": setup_s,
    }
    if n_prof:
        prof = ro.rl_profile_read()
        out["config"]["kernel_timing"] = f"HIP events on the {n_prof} steps that follow the timed region"
        ctx_p = ctx_last + 0.5 * (n_prof + 1)
        kb_once = kernel_bytes(shape, B, ctx_sum(ctx_p, True), kv_bytes=kvb)
        kb_each = kernel_bytes(shape, B, ctx_sum(ctx_p, False), kv_bytes=kvb)
        kernels = kernel_table(prof, kb_once)
        out["kernels"] = kernels
        dom = max((n for n in kernels if n in kb_once), key=lambda n: kernels[n]["avg_us"] * kernels[n]["launches"])
        out["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["achieved_GBs"], "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": kernels[dom]["achieved_GBs"] / HBM_PEAK_GBS,
                           "traffic": None if args.kv_fp8 else measured_traffic("wave", dom, kb_once[dom]),
                           "bytes_per_launch": kb_once[dom],
                           "achieved_per_sequence_formula": kb_each[dom] / (kernels[dom]["avg_us"] * 1e-6) / 1e9}

    # ---- the 32-sequence workload on the same model: 4 prompts x 8 samples, prompts of 1024 tokens ---------------
    for gr in graphs.values():
        gr.close()
    graphs.clear()
    if not args.no_small_batch:
        ro.rl_free_seqs(seq_ids)
        n2, P2 = 4, 1024
        B2 = n2 * G
        ids2_list = list(range(B2))
        ids2 = _i32(ids2_list)
        prompts2 = ri.tokens((n2, P2), shape["vocab"], seed, 900)
        t0 = time.perf_counter()
        tok2, _ = ro.rl_prefill_groups(ids2_list, G, [prompts2[i].tolist() for i in range(n2)], 1.0, seed)
        torch.cuda.synchronize()
        prefill2_s = time.perf_counter() - t0
        state["cur"], state["i"] = tok2, 0
        for _ in range(args.warmup):
            step(ids2, B2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(ids2, B2)
        torch.cuda.synchronize()
        el2 = time.perf_counter() - t0
        small = {"workload": f"full8b_36L_bf16_{B2}seq_prompt{P2}_T1.0", "tokens_per_s": B2 * args.steps / el2,
                 "ms_per_step": el2 / args.steps * 1e3, "context_first_timed_step": P2 + args.warmup + 1,
                 "context_last_timed_step": P2 + args.warmup + args.steps, "prefill_s": prefill2_s}
        c2 = P2 + args.warmup + 0.5 * (args.steps + 1)
        sh2 = P2 // 16 * 16
        kb2 = kernel_bytes(shape, B2, int(n2 * sh2 + B2 * (c2 - sh2)), kv_bytes=kvb)
        kb2_each = kernel_bytes(shape, B2, int(B2 * c2), kv_bytes=kvb)
        small["step_hbm_fraction"] = step_bytes_of(shape, kb2_each) / (el2 / args.steps) / (HBM_PEAK_GBS * 1e9)
        small["step_hbm_fraction_shared_pages_once"] = step_bytes_of(shape, kb2) / (el2 / args.steps) / (HBM_PEAK_GBS * 1e9)
        if not args.no_profile and not args.graph:
            ro.rl_profile_enable(True)
            for _ in range(args.profile_steps):
                step(ids2, B2)
            torch.cuda.synchronize()
            ro.rl_profile_enable(False)
            small["kernels"] = kernel_table(ro.rl_profile_read(), kb2)
        out["batch32"] = small
    for gr in graphs.values():
        gr.close()
    if args.graph:
        out["config"]["launch"] = "one HIP graph launch per decode step"
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_full(shape, int(ctx_avg), n_seq=8)  # about 25 s of host work at context 9 k
    ro.close()
    print(json.dumps(out))


def run_tiny(args):
    """The tiny fp32 workload end to end (4 prompts x 64 tokens, 32 greedy tokens each) and the oracle's wall time for
    the same run.  A launch-bound case by nature: 2 layers of 256-wide matrices, about 40 small kernels per step."""
    import numpy as np
    import torch
    import rollout_inputs as ri
    from paper_2510_17891_amd import Rollout
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import dims_of, make_both, to_device
    shape = ri.SHAPES["tiny"]
    w, wn = make_both(shape, ri.BASE_SEED + 1)
    ro = Rollout(shape, to_device(w), max_seqs=8, max_ctx=128, max_rows=64, kv_pages=40)
    prompts = ri.tokens((4, 64), shape["vocab"], ri.BASE_SEED + 1, 900).tolist()
    seqs = [0, 1, 2, 3]

    def run():
        tok, lp = ro.rl_prefill(seqs, prompts, 0.0, 0)
        out = [tok]
        for _ in range(31):
            tok, lp = ro.rl_decode_step(seqs, tok, 0.0, 0)
            out.append(tok)
        torch.cuda.synchronize()
        ro.rl_free_seqs(seqs)
        return torch.stack(out, 1).cpu()

    gpu_tokens = run()                                  # warm-up (and the ids to compare)
    reps = max(1, args.steps // 32)
    t0 = time.perf_counter()
    for _ in range(reps):
        run()
    gpu_s = (time.perf_counter() - t0) / reps
    out = {"metric": "generated tokens/s (tiny fp32 decoder, greedy)", "value": 4 * 32 / gpu_s, "unit": "tokens/s",
           "n_gpus": 1, "steps": 32 * reps, "warmup": 32, "ms_per_step": gpu_s / 32 * 1e3, "higher_is_better": True,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": "tiny_2L_fp32_4x64_prompt_32_greedy", "note": "launch-bound: prefill of 256 rows in "
                      "chunks of 64 plus 31 decode steps of about 40 small kernels each; the rate says nothing about HBM"},
           "whole_run_ms": gpu_s * 1e3}
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        om = orc.OracleModel(dims_of(shape), wn, max_ctx=128)
        t0 = time.perf_counter()
        ref = []
        for s, p in zip(seqs, prompts):
            z = om.prefill(s, p)
            row = []
            for k in range(32):
                t, _ = orc.sample(z, 0.0, 0, s, 64 + k)
                row.append(t)
                if k < 31:
                    z = om.forward_token(s, t)
            ref.append(row)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 4 * 32 / cpu_s, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"the whole run (4 x 64 prompt tokens + 4 x 32 greedy tokens), {cpu_s:.2f} s"}
        out["tokens_equal_oracle"] = bool((gpu_tokens.numpy() == np.array(ref)).all())
    ro.close()
    print(json.dumps(out))


def run_objective(args):
    """rl_hrd_objective on one RL batch at the paper's limits: 32 prompts x 8 outputs, lengths U[64, 16384]."""
    import numpy as np
    import torch
    import rollout_inputs as ri
    from paper_2510_17891_amd import binding as B
    dev = "cuda:0"
    n_prompts, G, seed = 32, 8, 11
    n = n_prompts * G
    lens = ri.lengths(n, 64, 16384, seed, 1).numpy()
    lens[-1] = 16384
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(off[-1])
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    lp_old = -ri.normal((total,), 1.0, seed, 3, device=dev).abs() - 0.1
    lp_new = lp_old + ri.normal((total,), 0.25, seed, 4, device=dev)
    toks = ri.tokens((total,), 1000, seed, 2).to(dev)
    rs = ri.normal((n,), 0.6, seed, 5).abs().clamp(max=2.0).to(dev)
    rc = (ri.normal((n,), 1.0, seed, 6) > 0).float().to(dev)
    offd = d(off)
    res = {}
    for label, kw in (("plan_lengths_given", dict(n_plan=d((lens // 2).astype(np.int32)))),
                      ("delimiter_scan", dict(tokens=toks, delimiter_token=7))):
        for _ in range(3):
            B.rl_hrd_objective(n_prompts, G, offd, lp_new, lp_old, rs, rc, **kw)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            B.rl_hrd_objective(n_prompts, G, offd, lp_new, lp_old, rs, rc, **kw)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / args.steps * 1e6
        nbytes = total * (8 + (4 if "tokens" in kw else 0)) + n * 24
        res[label] = {"us_per_call": us, "algorithmic_bytes": nbytes, "GBs": nbytes / us / 1e3}
    out = {"metric": "HRD objective forward, microseconds per RL batch", "value": res["plan_lengths_given"]["us_per_call"],
           "unit": "us", "n_gpus": 1, "steps": args.steps, "higher_is_better": False, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "hrd_objective_32x8_outputs_U[64,16384]_tokens", "tokens": total,
                      "note": "two kernels (one block per output, then a one-block sum): latency- and launch-bound at "
                              "this size, the 8 bytes per token are far from an HBM limit"},
           "variants": res}
    print(json.dumps(out))


def run_score_or_prefill(args):
    """Prompt processing as a matrix-core workload: `prefill` runs 32 prompts of --prefill-len tokens (4 groups of 8
    prompts at a time, the KV stays), `score` runs rl_score over 32 x 8 sequences of --score-len tokens.  Reports
    tokens/s and the fraction of the dense bf16/f16 matrix-core peak that the model's matrix flops amount to."""
    import torch
    import rollout_inputs as ri
    from paper_2510_17891_amd import Rollout
    dev = "cuda:0"
    torch.cuda.set_device(0)
    seed = ri.BASE_SEED + 2
    shape = ri.SHAPES["full8b"]
    score = args.workload == "score"
    n_seq, T = (256, args.score_len) if score else (32, args.prefill_len)
    max_ctx = (T + 16 + 15) // 16 * 16
    w = ri.make_weights(shape, seed, device=dev, dtype=torch.bfloat16)
    ro = Rollout(shape, w, max_seqs=n_seq, max_ctx=max_ctx, max_rows=args.chunk_rows, kv_pages=n_seq * (max_ctx // 16) + 16,
                 consume_weights=True)
    del w
    torch.cuda.empty_cache()
    toks = ri.tokens((n_seq, T), shape["vocab"], seed, 970)
    seqs = [toks[i].tolist() for i in range(n_seq)]
    ids = list(range(n_seq))
    # matrix flops per token: 2 x (layer matrices + lm_head for the scored positions) + attention 4 n_q d ctx per layer
    H, d, F, V = shape["hidden"], shape["head_dim"], shape["ffn"], shape["vocab"]
    nq, nkv, L = shape["n_q"], shape["n_kv"], shape["n_layers"]
    per_tok = 2 * L * (H * (nq + 2 * nkv) * d + nq * d * H + 3 * F * H)
    attn = 4 * nq * d * L * (T + 1) / 2
    head = 2 * V * H
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if score:
        group = 32
        for b0 in range(0, n_seq, group):
            ro.rl_score(ids[b0:b0 + group], seqs[b0:b0 + group], 1.0)
        flops = n_seq * (T * (per_tok + attn) + (T - 1) * head)
    else:
        for b0 in range(0, n_seq, 8):
            ro.rl_prefill(ids[b0:b0 + 8], seqs[b0:b0 + 8], 1.0, seed)
        flops = n_seq * (T * (per_tok + attn) + head)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    out = {"metric": "teacher-forced scoring tokens/s" if score else "prefill prompt tokens/s", "value": n_seq * T / el,
           "unit": "tokens/s", "n_gpus": 1, "steps": 1, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"full8b_{'score' if score else 'prefill'}_{n_seq}x{T}", "rows_per_chunk": args.chunk_rows},
           "seconds": el, "model_TFLOPs": flops / el / 1e12,
           "roofline": {"bound": "mfma", "achieved": flops / el / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                        "frac": flops / el / 1e12 / 2500.0, "traffic": None}}
    ro.close()
    print(json.dumps(out))


def run_sched(args):
    """Host cost of the step scheduler: a one-layer model at 8B layer dimensions (so that the GPU side is short and the
    host side shows), 16 and 32 groups of 8 samples (128 and 256 rows, prompts shared inside a group), generated by the
    group rollout loop.  Reports, per decode call, the library's admission checks and metadata build + upload, its
    kernel launches, and what the Python loop adds around the call."""
    import torch
    import rollout_inputs as ri
    from paper_2510_17891_amd import Rollout, generate_groups, group_page_need
    dev = "cuda:0"
    torch.cuda.set_device(0)
    seed = ri.BASE_SEED + 5
    shape = dict(ri.SHAPES["layer8b"], vocab=4096)
    w = ri.make_weights(shape, seed, device=dev, dtype=torch.bfloat16)
    res = {}
    for n_prompts in (16, 32):
        G, P, new = 8, 64, args.steps
        prompts = [ri.tokens((P,), shape["vocab"], seed, 980 + i).tolist() for i in range(n_prompts)]
        pages = n_prompts * group_page_need(P, [new] * G) + 8
        ro = Rollout(shape, w, max_seqs=n_prompts * G, max_ctx=(P + new + 16) // 16 * 16, max_rows=256, kv_pages=pages)
        generate_groups(ro, prompts[:2], G, 4, 1.0, seed)          # warm-up
        ro.rl_profile_host_read()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        generate_groups(ro, prompts, G, new, 1.0, seed)
        wall = time.perf_counter() - t0
        h = ro.rl_profile_host_read()
        calls = max(1, h["calls"])
        res[f"{n_prompts * G}_rows"] = {
            "decode_calls": h["calls"], "admit_us_per_call": h["admit_us"] / calls, "meta_us_per_call": h["meta_us"] / calls,
            "launch_us_per_call": h["launch_us"] / calls, "wait_for_device_us_per_call": h["wait_us"] / calls,
            "wall_us_per_step": wall / new * 1e6,
            "python_us_per_step": wall / new * 1e6 - (h["admit_us"] + h["meta_us"] + h["launch_us"] + h["wait_us"]) / new}
        ro.close()
    out = {"metric": "host microseconds per decode call spent in the step scheduler", "unit": "us",
           "value": res["256_rows"]["admit_us_per_call"] + res["256_rows"]["meta_us_per_call"], "higher_is_better": False,
           "n_gpus": 1, "steps": args.steps, "data": "synthetic",
           "config": {"workload": "layer8b_1L_vocab4096_groups_of_8_prompt64", "note": "wall_us_per_step includes the "
                      "prefills of the run (one per group); wait_for_device is the time the host, 62 calls ahead, "
                      "stood still for the GPU; the scheduler's own share is admit + meta"}, "rows": res}
    print(json.dumps(out))


def rl_page_bytes(shape):
    return 16 * shape["n_layers"] * shape["n_kv"] * shape["head_dim"] * 2 * 2


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py runs on one GPU only (a rollout shards by whole sequences, with no communication per step, so "
              "N GPUs are N independent copies of this run); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import rollout_inputs as ri
    from paper_2510_17891_amd import Rollout
    dev = "cuda:0"
    torch.cuda.set_device(0)
    seed = ri.BASE_SEED + 2

    if args.workload == "wave":
        run_wave(args)
        return
    if args.workload == "tiny":
        run_tiny(args)
        return
    if args.workload == "objective":
        run_objective(args)
        return
    if args.workload in ("score", "prefill"):
        run_score_or_prefill(args)
        return
    if args.workload == "sched":
        run_sched(args)
        return

    if args.workload == "copy":
        # Plain device copy of known size: the reference against which HBM byte counters are scaled, and the
        # on-box streaming ceiling (reads 1 GiB and writes 1 GiB per launch).
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        red = torch.empty(n // 4, dtype=torch.float32, device=dev).normal_()
        for _ in range(max(1, args.warmup)):
            dst.copy_(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        t0 = time.perf_counter()
        for _ in range(args.steps):
            red.sum()
        torch.cuda.synchronize()
        dr = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"workload": "copy_1GiB", "bytes_read": n, "bytes_written": n, "us_per_copy": dt * 1e6,
                          "copy_GBs_read_plus_write": 2 * n / dt / 1e9, "read_only_sum_GBs": n / dr / 1e9}))
        return

    if args.workload == "ragged":
        # Whole rollout with ragged lengths and continuous batching: 16 prompts x 8 samples, prompt length per prompt
        # U[256,1024], final length per sequence U[1024,8192] (pre-drawn), sequences retire one by one.
        from paper_2510_17891_amd import generate_groups, group_page_need
        shape = ri.SHAPES["full8b"]
        n_prompts, G = 16, 8
        sc = args.length_scale
        p_len = [max(1, int(v * sc)) for v in ri.lengths(n_prompts, 256, 1024, seed, 910).tolist()]
        f_len = [max(2, int(v * sc)) for v in ri.lengths(n_prompts * G, 1024, 8192, seed, 911).tolist()]
        limits = [max(1, f_len[k] - p_len[k // G]) for k in range(n_prompts * G)]
        prompts = [ri.tokens((n,), shape["vocab"], seed, 920 + i).tolist() for i, n in enumerate(p_len)]
        pages = sum(group_page_need(p_len[i], limits[i * G:(i + 1) * G]) for i in range(n_prompts))
        max_ctx = (max(p_len[k // G] + limits[k] for k in range(n_prompts * G)) + 15) // 16 * 16
        w = ri.make_weights(shape, seed, device=dev, dtype=torch.bfloat16)
        kvb = 1 if args.kv_fp8 else 2
        ro = Rollout(shape, w, max_seqs=n_prompts * G, max_ctx=max_ctx, max_rows=256, kv_pages=pages, kv_fp8=args.kv_fp8)
        del w
        torch.cuda.empty_cache()
        torch.cuda.synchronize()
        trace = []
        t0 = time.perf_counter()
        toks, lps = generate_groups(ro, prompts, G, limits, 1.0, seed, on_step=lambda s, n: trace.append(n))
        elapsed = time.perf_counter() - t0
        n_tok = sum(len(t) for t in toks)
        assert [len(t) for t in toks] == limits
        # algorithmic bytes: weights once per step + every cached token of every stepped sequence (shared prompt pages
        # counted per sequence, as the per-sequence formula does)
        steps = len(trace)
        kv_tokens = sum(sum(range(p_len[k // G] + 1, p_len[k // G] + limits[k])) for k in range(n_prompts * G))
        wbytes = 2 * (shape["n_layers"] * (shape["hidden"] * (shape["n_q"] + 2 * shape["n_kv"]) * shape["head_dim"]
                                          + shape["n_q"] * shape["head_dim"] * shape["hidden"]
                                          + 3 * shape["ffn"] * shape["hidden"]) + shape["vocab"] * shape["hidden"])
        total_bytes = steps * wbytes + kv_tokens * shape["n_layers"] * shape["n_kv"] * 2 * shape["head_dim"] * kvb
        print(json.dumps({
            "metric": "generated tokens/s (8B-shaped bf16 decode) + % peak HBM GB/s, 1 MI355X",
            "value": n_tok / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": 0,
            "ms_per_step": elapsed / max(1, steps) * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"full8b_ragged_{n_prompts}x{G}_scale{sc}" + ("_kvfp8" if args.kv_fp8 else ""), "prompts": "U[256,1024] per prompt",
                       "final_lengths": "U[1024,8192] per sequence", "generated_tokens": n_tok, "kv_pages": pages,
                       "prefill": "inside the timed region, prompts run once per group", "temperature": 1.0},
            "whole_run_s": elapsed, "hbm_fraction_per_sequence_formula": total_bytes / elapsed / (HBM_PEAK_GBS * 1e9),
            "active_sequences_first_mid_last": [trace[0], trace[len(trace) // 2], trace[-1]] if trace else None}))
        ro.close()
        return

    if args.workload == "max":
        # The largest rollout batch (Appendix D limits): 32 prompts x 8 samples, prompt 2048, generated up to 16384 tokens
        # of context, KV pool = what the card holds beside the weights.  The 256 sequences need 618 GB of KV, so groups
        # are admitted as pages allow (generate_groups reserves a group's pages up to its limit) and the rest waits.
        from paper_2510_17891_amd import generate_groups, group_page_need
        shape = ri.SHAPES["full8b"]
        n_prompts, G = 32, 8
        sc = args.length_scale
        P, total = max(16, int(2048 * sc)), max(32, int(16384 * sc))
        limits = [total - P] * (n_prompts * G)
        prompts = [ri.tokens((P,), shape["vocab"], seed, 960 + i).tolist() for i in range(n_prompts)]
        need_group = group_page_need(P, limits[:G])
        w = ri.make_weights(shape, seed, device=dev, dtype=torch.bfloat16)
        kvb = 1 if args.kv_fp8 else 2
        page_bytes = 16 * shape["n_layers"] * shape["n_kv"] * shape["head_dim"] * 2 * kvb
        # kv_pages=None: the pool takes what the card holds once the packed weights and the workspace are placed
        ro = Rollout(shape, w, max_seqs=n_prompts * G, max_ctx=(total + 15) // 16 * 16, max_rows=256, kv_pages=None,
                     consume_weights=True, kv_slack_bytes=4 << 30, kv_fp8=args.kv_fp8)
        del w
        pages = ro.rl_kv_stats()[1]
        torch.cuda.synchronize()
        trace = []
        t0 = time.perf_counter()

        def progress(s_, n_):
            trace.append(n_)
            if s_ % 1000 == 0:
                print(f"step {s_}: {n_} sequences active, {time.perf_counter() - t0:.0f} s", file=sys.stderr, flush=True)

        toks, lps = generate_groups(ro, prompts, G, limits, 1.0, seed, on_step=progress)
        elapsed = time.perf_counter() - t0
        n_tok = sum(len(t) for t in toks)
        assert [len(t) for t in toks] == limits and all(len(l) == len(t) for l, t in zip(lps, toks))
        steps = len(trace)
        kv_tokens = n_prompts * G * sum(range(P + 1, total))
        wbytes = 2 * (shape["n_layers"] * (shape["hidden"] * (shape["n_q"] + 2 * shape["n_kv"]) * shape["head_dim"]
                                          + shape["n_q"] * shape["head_dim"] * shape["hidden"]
                                          + 3 * shape["ffn"] * shape["hidden"]) + shape["vocab"] * shape["hidden"])
        total_bytes = steps * wbytes + kv_tokens * shape["n_layers"] * shape["n_kv"] * 2 * shape["head_dim"] * kvb
        print(json.dumps({
            "metric": "generated tokens/s (8B-shaped bf16 decode) + % peak HBM GB/s, 1 MI355X",
            "value": n_tok / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": 0,
            "ms_per_step": elapsed / max(1, steps) * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"full8b_max_{n_prompts}x{G}_prompt{P}_to{total}" + ("_kvfp8" if args.kv_fp8 else ""),
                       "generated_tokens": n_tok,
                       "kv_pages": pages, "kv_pool_GB": pages * page_bytes / 1e9, "pages_per_group": need_group,
                       "groups_resident_at_once": pages // need_group,
                       "prefill": "inside the timed region, prompts run once per group", "temperature": 1.0,
                       "logprob_per_token": True},
            "whole_run_s": elapsed, "hbm_fraction_per_sequence_formula": total_bytes / elapsed / (HBM_PEAK_GBS * 1e9),
            "active_sequences_first_mid_last": [trace[0], trace[len(trace) // 2], trace[-1]] if trace else None}))
        ro.close()
        return

    if args.workload == "full":
        shape = ri.SHAPES["full8b"]
        n_prompts, G, P = args.n_prompts, 8, 1024
        B = n_prompts * G
        total_steps = args.warmup + args.steps + (0 if args.no_profile else args.profile_steps)
        max_ctx = (P + total_steps + 1 + 15) // 16 * 16
        pages = B * (max_ctx // 16)
        w = ri.make_weights(shape, seed, device=dev, dtype=torch.bfloat16)
        ro = Rollout(shape, w, max_seqs=B, max_ctx=max_ctx, max_rows=max(256, B), kv_pages=pages)
        del w
        torch.cuda.empty_cache()
        if args.no_share_attention:
            ro.rl_debug_share_attention(False)
        elif args.set_width != 1:
            ro.rl_debug_share_attention(args.set_width)
        if args.separate_append:
            ro.rl_debug_attention_appends(False)
        prompts = ri.tokens((n_prompts, P), shape["vocab"], seed, 900)
        prompt_list = [prompts[i // G].tolist() for i in range(B)]
        seq_ids = list(range(B))
        torch.cuda.synchronize()
        if args.prefill == "real":
            t0 = time.perf_counter()
            # the G samples of a prompt share its KV pages: each prompt is run once (Section 2.3: G outputs per q_i)
            tok, lp = ro.rl_prefill_groups(seq_ids, G, [prompts[i].tolist() for i in range(n_prompts)], 1.0, seed)
            torch.cuda.synchronize()
            prefill_s = time.perf_counter() - t0
        else:
            kv = [ri.normal((P, shape["n_kv"], shape["head_dim"]), 1.0, seed, 3000 + l, device=dev, dtype=torch.bfloat16)
                  for l in range(shape["n_layers"])]
            for b in seq_ids:
                ro.rl_seq_import_kv(b, kv, kv)
            tok = prompts[0, :B].to(dev).contiguous()
            torch.cuda.synchronize()
            prefill_s = None
        workload = f"full8b_36L_bf16_{B}seq_prompt{P}_T{args.temperature}" \
            + (f"_topk{args.top_k}" if args.top_k else "") + (f"_topp{args.top_p}" if args.top_p else "")
        ctx0 = P
    else:
        shape = ri.SHAPES["layer8b"]
        B, ctx0 = args.batch, args.ctx
        total_steps = args.grow + args.warmup + args.steps + (0 if args.no_profile else args.profile_steps)
        max_ctx = (ctx0 + total_steps + 1 + 15) // 16 * 16
        pages = B * (max_ctx // 16)
        w = ri.make_weights(shape, seed, device=dev, dtype=torch.bfloat16)
        ro = Rollout(shape, w, max_seqs=B, max_ctx=max_ctx, max_rows=B, kv_pages=pages)
        if args.attn_split:
            ro.rl_debug_attention_split(args.attn_split)
        if not args.contiguous_pages:
            ro.rl_debug_shuffle_free_pages(seed)  # block tables are a random permutation of the pool
        if args.no_share_attention:
            ro.rl_debug_share_attention(False)
        elif args.set_width != 1:
            ro.rl_debug_share_attention(args.set_width)
        if args.separate_append:
            ro.rl_debug_attention_appends(False)
        for b in range(0, B, args.group):
            k = ri.normal((ctx0, shape["n_kv"], shape["head_dim"]), 1.0, seed, 2000 + 2 * b, device=dev, dtype=torch.bfloat16)
            v = ri.normal((ctx0, shape["n_kv"], shape["head_dim"]), 1.0, seed, 2001 + 2 * b, device=dev, dtype=torch.bfloat16)
            ro.rl_seq_import_kv(b, [k], [v])
            if args.group > 1:
                ro.rl_seq_fork(b, list(range(b + 1, min(B, b + args.group))))
        seq_ids = list(range(B))
        x_in = ri.normal((B, shape["hidden"]), 1.0, seed, 1999, device=dev)
        x_out = torch.empty_like(x_in)
        prefill_s = None
        workload = f"layer8b_1L_bf16_b{B}_ctx{ctx0}" + (f"_group{args.group}" if args.group > 1 else "") \
            + (f"_plus{args.grow}" if args.grow else "")
        G, P = args.group, ctx0
        n_prompts = (B + G - 1) // G
        ctx0 += args.grow

    from paper_2510_17891_amd.binding import _i32
    ids = _i32(seq_ids)
    if args.workload == "full":
        bufs = [(torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.float32, device=dev))
                for _ in range(2)]
        state = {"cur": tok, "i": 0}

        def step():
            ot, ol = bufs[state["i"] & 1]
            ro.rl_decode_step(ids, state["cur"], args.temperature, seed, out_tokens=ot, out_logprobs=ol,
                              top_k=args.top_k, top_p=args.top_p)
            state["cur"] = ot
            state["i"] += 1
    else:
        def step():
            ro.rl_decode_hidden(ids, x_in, x_out)

    if args.workload == "layer":
        if args.grow_append and args.grow:
            # the grown part as appended N(0,1) keys and values, one private stretch per sequence, instead of decode steps
            for b in seq_ids:
                k = ri.normal((args.grow, shape["n_kv"], shape["head_dim"]), 1.0, seed, 5000 + b, device=dev,
                              dtype=torch.bfloat16)
                ro.rl_seq_append_kv(b, [k], [k])
        else:
            for _ in range(args.grow):
                step()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    ctx_begin = ctx0 + args.warmup
    ctx_end = ctx_begin + args.steps  # context of the last timed step is ctx_end - 1 (+1 for the fed token)
    ctx_avg = 0.5 * (ctx_begin + ctx_end - 1) + 1
    n_layers = shape["n_layers"]
    # tokens in pages that the G samples of a prompt hold in common are read once per prompt, not once per sample
    shared_tok = (P // 16 * 16) if (G > 1 and args.prefill == "real") else 0

    def ctx_sum(ctx):
        return int(n_prompts * shared_tok + B * (ctx - shared_tok))

    step_bytes = None
    if args.workload == "full":
        kbm = kernel_bytes(shape, B, ctx_sum(ctx_avg))
        step_bytes = n_layers * (kbm["gemm_qkv"] + kbm["gemm_o"] + kbm["gemm_gate_up_swiglu"] + kbm["gemm_down"]
                                 + kbm["attn_decode"]) + kbm["gemm_lm_head"]
    else:
        shp = dict(shape, vocab=4)
        kbm = kernel_bytes(shp, B, ctx_sum(ctx_avg))
        step_bytes = kbm["gemm_qkv"] + kbm["gemm_o"] + kbm["gemm_gate_up_swiglu"] + kbm["gemm_down"] + kbm["attn_decode"]

    out = {
        "metric": "generated tokens/s (8B-shaped bf16 decode) + % peak HBM GB/s, 1 MI355X",
        "value": B * args.steps / elapsed,
        "unit": "tokens/s" if args.workload == "full" else "layer-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload, "batch": B, "context_first_timed_step": ctx_begin + 1,
                   "context_last_timed_step": ctx_end, "kv_block": 16, "temperature": args.temperature},
        "step_hbm_fraction": None, "step_algorithmic_GB": None,
    }
    # The per-sequence byte formula (weights once + 4096 B per cached token per layer per sequence) is the unit of
    # the step-level fraction; where the samples of a prompt hold pages in common the step needs fewer bytes, and the
    # fraction against that smaller figure is given as well (per-kernel rates below always use the smaller figure).
    extra = (n_layers if args.workload == "full" else 1) * (B - n_prompts) * shared_tok * shape["n_kv"] * 2 * shape["head_dim"] * 2
    out["step_algorithmic_GB"] = (step_bytes + extra) / 1e9
    out["step_hbm_fraction"] = (step_bytes + extra) / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9)
    if shared_tok:
        out["config"]["shared_prompt_tokens"] = shared_tok
        out["step_GB_shared_pages_once"] = step_bytes / 1e9
        out["step_hbm_fraction_shared_pages_once"] = step_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9)
    if prefill_s is not None:
        out["prefill_s"] = prefill_s
        out["prefill_prompt_tokens_per_s"] = n_prompts * 1024 / prefill_s
        out["config"]["prefill"] = f"{n_prompts} prompts x 1024 tokens run once each, pages shared by the 8 samples of a prompt"
    elif args.workload == "full":
        out["config"]["prompt_kv"] = "imported N(0,1)"

    # ---- per-kernel durations from HIP events on the launch stream, same steps, same state --------------
    if not args.no_profile:
        if args.workload == "full" and args.prefill == "real":
            # The timed region once more, from the same prompts and seed (the same tokens), with the events switched
            # on for every stride-th step: launch durations over the contexts of the timed region, not after it.
            ro.rl_free_seqs(seq_ids)
            tok, _ = ro.rl_prefill_groups(seq_ids, G, [prompts[i].tolist() for i in range(n_prompts)], 1.0, seed)
            state["cur"], state["i"] = tok, 0
            for _ in range(args.warmup):
                step()
            stride = max(1, args.steps // 128)
            ctx_seen = []
            for k in range(args.steps):
                on = k % stride == 0
                if on:
                    ro.rl_profile_enable(True)
                    ctx_seen.append(ctx_begin + k + 1)
                step()
                if on:
                    ro.rl_profile_enable(False)
            torch.cuda.synchronize()
            prof = ro.rl_profile_read()
            ctx_p = sum(ctx_seen) / len(ctx_seen)
            out["config"]["kernel_timing"] = f"HIP events on every {stride}th step of a second pass over the timed region"
        else:
            ro.rl_profile_enable(True)
            for _ in range(args.profile_steps):
                step()
            torch.cuda.synchronize()
            prof = ro.rl_profile_read()
            ro.rl_profile_enable(False)
            ctx_p = ctx_end + 0.5 * (args.profile_steps - 1) + 1
            out["config"]["kernel_timing"] = f"HIP events on {args.profile_steps} steps after the timed region"
        shp = shape if shape["vocab"] else dict(shape, vocab=4)
        kb = kernel_bytes(shp, B, ctx_sum(ctx_p))
        kernels = {}
        for name, (cnt, ms) in prof.items():
            if cnt == 0:
                continue
            avg_us = ms / cnt * 1e3
            entry = {"launches": cnt, "avg_us": avg_us, "share": None}
            if name in kb:
                entry["achieved_GBs"] = kb[name] / (avg_us * 1e-6) / 1e9
                entry["bytes"] = kb[name]
            kernels[name] = entry
        tot = sum(e["avg_us"] * e["launches"] for e in kernels.values())
        for e in kernels.values():
            e["share"] = e["avg_us"] * e["launches"] / tot
        out["kernels"] = kernels
        dom = max((n for n in kernels if n in kb), key=lambda n: kernels[n]["avg_us"] * kernels[n]["launches"])
        out["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["achieved_GBs"], "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": kernels[dom]["achieved_GBs"] / HBM_PEAK_GBS,
                           "traffic": measured_traffic(args.workload, dom, kb[dom])}
    if not args.no_cpu_baseline:
        if args.workload == "full":
            out["cpu_baseline"] = cpu_baseline_full(shape, int(ctx_avg))
        else:
            cb = cpu_baseline_full(dict(shape, vocab=16 * 64), ctx0, n_seq=64, head_fraction=16)
            cb["unit"] = "layer-tokens/s"
            out["cpu_baseline"] = cb
    ro.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
