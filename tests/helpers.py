"""Shared helpers of the GPU parity tests: weights on both sides, error norms."""
import numpy as np
import torch

import rollout_inputs as ri
from oracle import oracle as orc

DIM_KEYS = ("hidden", "n_q", "n_kv", "head_dim", "ffn", "qk_norm", "rms_eps", "rope_base")


def dims_of(shape):
    return {k: shape[k] for k in DIM_KEYS}


def storage_dtype(shape):
    return torch.bfloat16 if shape["dtype"] == "bf16" else torch.float32


def make_both(shape, seed, std=0.02):
    """(weights on the storage grid as CPU torch tensors, the same as fp32 numpy for the oracle)."""
    dt = storage_dtype(shape)
    w = ri.make_weights(shape, seed, device="cpu", dtype=dt, std=std)

    def np32(t):
        return np.ascontiguousarray(t.float().numpy())
    wn = {k: (np32(v) if k != "layers" else [{a: np32(b) for a, b in l.items()} for l in v]) for k, v in w.items()}
    return w, wn


def to_device(w, device="cuda:0"):
    return {k: (v.to(device) if k != "layers" else [{a: b.to(device) for a, b in l.items()} for l in v])
            for k, v in w.items()}


def rel_inf(got, ref):
    """max |got - ref| / max |ref| over the last axis (per row)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.abs(got - ref).max(-1) / np.abs(ref).max(-1)
