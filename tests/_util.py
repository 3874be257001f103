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
import functools
import math
import os

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


def host_threads() -> int:
    """Threads the oracle may use over independent rows (the GPU machine exports OMP_NUM_THREADS)."""
    return int(os.environ.get("OMP_NUM_THREADS", "0")) or min(os.cpu_count() or 1, 16)


def oracle_score_streamed(oracle, logits, tokens, A, V=None, chunk_bytes=1 << 30):
    """The oracle's score_logits over EVERY row of a device-resident logit matrix: rows are
    independent, so the matrix is brought to the host in chunks of whole steps of at most
    chunk_bytes and the results are concatenated."""
    R, stride = logits.shape
    rows = max(A, (chunk_bytes // (2 * stride)) // A * A)
    parts = []
    tok = npf(tokens)
    for r0 in range(0, R, rows):
        r1 = min(R, r0 + rows)
        parts.append(oracle.score_logits(bits_of(logits[r0:r1]), tok[r0:r1], A, V=V, nthreads=host_threads()))
        print(f"  oracle rows {r1}/{R}", flush=True)
    return {k: np.concatenate([p[k] for p in parts]) for k in parts[0]}


@functools.lru_cache(maxsize=None)
def scored_config(ci: int):
    """A workload with logits at its full size -- inputs on the device, the library's score_logits
    outputs, and the oracle's over every row -- made once per test session and shared by the tests
    that need it (the large-vocabulary workload is 40 GB of logits and 20 s of oracle time)."""
    import oracle
    from paper_2410_14803_amd import binding as b
    from paper_2410_14803_amd import synth
    dev = "cuda"
    cfg = synth.CONFIGS[ci]
    seed = synth.BASE_SEED + cfg.index
    off_np = synth.trajectory_offsets(cfg, seed)
    N = int(off_np[-1])
    R = N * cfg.A
    print(f"config {ci}: R={R} rows, {R * cfg.V * 2 / 1e9:.2f} GB of logits", flush=True)
    logits = synth.logits_bf16(R, cfg.V, seed + 1, dev, heavy_tail=cfg.heavy_tail)
    tokens = synth.action_tokens(logits, seed + 2)
    ws = b.Workspace(cfg.M)
    got = {k: torch.full((R,), 7.0, device=dev) for k in ("tok_logp", "tok_ent")}
    got.update({k: torch.full((N,), 7.0, device=dev) for k in ("step_logp", "step_ent")})
    b.score_logits(logits, tokens, cfg.A, ws, **got)
    torch.cuda.synchronize()
    st, _ = ws.status()
    want = oracle_score_streamed(oracle, logits, tokens, cfg.A)
    return dict(cfg=cfg, seed=seed, off_np=off_np, N=N, R=R, logits=logits, tokens=tokens, ws=ws, got=got,
                flags=st.flags, want=want)
