"""Seeded synthetic inputs for the rollout path.

This module holds no arithmetic of the method: it only names the workload
shapes and draws random tensors.  Both the CPU oracle's tests and the GPU
library's tests/benchmark take their inputs from here, so the two sides see
the very same numbers without sharing any other code.

Workloads (uniform-random token ids and random-weight policies stand in for
the paper's prompts and trained checkpoint, neither of which is available):
  tiny     2-layer fp32 decoder, hidden 256, 4 q / 2 kv heads, head_dim 64,
           FFN 688, vocab 4096
  layer8b  one decoder layer at 8B dimensions, bf16
  full8b   36-layer 8B-shaped policy, vocab 151936, bf16
Matrices and embeddings are N(0, 0.02); every RMSNorm gain is 1 + N(0, 0.02)
so that a missing gain multiply is visible.
"""
import torch

BASE_SEED = 20251017

SHAPES = {
    "tiny": dict(n_layers=2, hidden=256, n_q=4, n_kv=2, head_dim=64, ffn=688, vocab=4096,
                 rms_eps=1e-6, rope_base=1e6, qk_norm=1, dtype="f32"),
    "layer8b": dict(n_layers=1, hidden=4096, n_q=32, n_kv=8, head_dim=128, ffn=12288, vocab=0,
                    rms_eps=1e-6, rope_base=1e6, qk_norm=1, dtype="bf16"),
    "full8b": dict(n_layers=36, hidden=4096, n_q=32, n_kv=8, head_dim=128, ffn=12288,
                   vocab=151936, rms_eps=1e-6, rope_base=1e6, qk_norm=1, dtype="bf16"),
}


def _gen(seed, tensor_id, device):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(tensor_id) * 7919 + 12345) % (2 ** 63 - 1))
    return g


def normal(shape, std, seed, tensor_id, device="cpu", mean=0.0, dtype=torch.float32):
    """N(mean, std) tensor drawn in fp32 from stream (seed, tensor_id), cast to `dtype`."""
    g = _gen(seed, tensor_id, device)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return t.to(dtype)


def tokens(shape, vocab, seed, tensor_id):
    """Uniform-random token ids in [0, vocab) as int32 (CPU)."""
    g = _gen(seed, tensor_id, "cpu")
    return torch.randint(0, vocab, shape, generator=g, dtype=torch.int64).to(torch.int32)


def lengths(n, lo, hi, seed, tensor_id):
    """n integers uniform in [lo, hi] (CPU int64)."""
    g = _gen(seed, tensor_id, "cpu")
    return torch.randint(lo, hi + 1, (n,), generator=g, dtype=torch.int64)


def permutation(n, seed, tensor_id):
    g = _gen(seed, tensor_id, "cpu")
    return torch.randperm(n, generator=g)


LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "q_norm", "k_norm", "wo", "mlp_norm",
                 "w_gate", "w_up", "w_down")


def layer_shapes(s):
    H, d, F = s["hidden"], s["head_dim"], s["ffn"]
    return dict(attn_norm=(H,), wq=(s["n_q"] * d, H), wk=(s["n_kv"] * d, H), wv=(s["n_kv"] * d, H),
                q_norm=(d,), k_norm=(d,), wo=(H, s["n_q"] * d), mlp_norm=(H,),
                w_gate=(F, H), w_up=(F, H), w_down=(H, F))


def make_layer(s, seed, layer, device="cpu", dtype=torch.float32, std=0.02):
    """Logical tensors of one layer, row-major [out, in]."""
    out = {}
    for j, (name, shp) in enumerate(layer_shapes(s).items()):
        tid = 100 + layer * 16 + j
        if name.endswith("norm"):
            out[name] = normal(shp, std, seed, tid, device, mean=1.0, dtype=dtype)
        else:
            out[name] = normal(shp, std, seed, tid, device, dtype=dtype)
    return out


def make_weights(s, seed, device="cpu", dtype=torch.float32, std=0.02):
    """All logical tensors of a model: embed, lm_head, final_norm, layers[...]."""
    w = {"layers": [make_layer(s, seed, l, device, dtype, std) for l in range(s["n_layers"])]}
    w["final_norm"] = normal((s["hidden"],), std, seed, 3, device, mean=1.0, dtype=dtype)
    if s["vocab"] > 0:
        w["embed"] = normal((s["vocab"], s["hidden"]), std, seed, 1, device, dtype=dtype)
        w["lm_head"] = normal((s["vocab"], s["hidden"]), std, seed, 2, device, dtype=dtype)
    return w
