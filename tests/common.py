"""Helpers shared by the test modules: turn a synth layer (torch tensors, logical layouts)
into the numpy arrays the oracle takes, and run the oracle's route + layer."""
import numpy as np
import torch

from oracle import oracle as orc  # noqa: F401
from oracle.layer_check import oracle_arrays, oracle_draft, oracle_verify, rel_err  # noqa: F401


def routing_gap(logits, k):
    """Smallest gap between consecutive order statistics among the top k+1 logits of each
    row: if it is far above the accumulation error, ids are well defined."""
    s = -np.sort(-logits, axis=1)[:, :k + 1]
    return float(np.min(s[:, :-1] - s[:, 1:]))


def bf16_exact(a):
    """float64/32 array -> torch bf16, asserting nothing is lost."""
    t = torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16)
    assert np.array_equal(t.float().numpy().astype(np.float64), np.asarray(a, np.float64))
    return t
