"""Shared helpers for the parity tests: tolerances and tensor plumbing.

Tolerances (fp32 accumulation against the fp64 oracle):
  log-probabilities, Retrace targets, TD errors, ratios, priorities:
      |g - o| <= 1e-4 * max(|o|, 1)
  entropies:
      |g - o| <= 1e-4 * max(|o|, 1e-2 * log V)
The floors exist because a relative bound is meaningless next to zero (a peaked row's
entropy, a target that happens to cancel); they are the only slack beyond 1e-4 relative.
Indices are compared bit for bit.
"""
import math

import numpy as np
import torch

RTOL = 1e-4


def assert_close(got, want, floor=1.0, what="", rtol=RTOL):
    g = np.asarray(got, dtype=np.float64)
    o = np.asarray(want, dtype=np.float64)
    assert g.shape == o.shape, f"{what}: shape {g.shape} vs {o.shape}"
    if g.size == 0:
        return 0.0
    assert np.all(np.isfinite(g) == np.isfinite(o)), f"{what}: finiteness differs"
    fin = np.isfinite(o)
    np.testing.assert_array_equal(g[~fin], o[~fin], err_msg=f"{what}: non-finite values differ")
    err = np.abs(g[fin] - o[fin])
    bound = rtol * np.maximum(np.abs(o[fin]), floor)
    worst = float(np.max(err / np.maximum(np.abs(o[fin]), floor))) if err.size else 0.0
    bad = err > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {err.size} outside 1e-4 relative "
                           f"(floor {floor}); worst scaled error {worst:.3e}")
    return worst


def ent_floor(V):
    return 1e-2 * math.log(V)


def bits_of(logits_bf16: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns on the host."""
    return logits_bf16.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def npf(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()
