"""Shared helpers for the parity tests: tolerances and tensor plumbing.

Tolerances (fp32 accumulation against the fp64 oracle): 1e-4 relative, with a floor of one
hundredth of the scale of the quantity's operands,
      |g - o| <= 1e-4 * max(|o|, 1e-2 * scale)
scale = 1 for log-probabilities, Retrace targets, TD errors, ratios and priorities (values,
rewards and ratios of order one), scale = log V for entropies.  The floor exists because a
relative bound is meaningless next to zero (a peaked row's entropy, a TD error or target whose
terms cancel): there the result is held to 1e-6 of the size of what was added up.
Indices are compared bit for bit.
"""
import functools
import math
import os

import numpy as np
import torch

RTOL = 1e-4


FLOOR_FRACTION = 1e-2


# For results at the end of a chain in which each side consumed its own intermediates: a ratio
# rho = exp(log pi - log mu) inherits the absolute error of log pi (one fp32 ulp at |log pi| ~ 500
# is 3e-5, still inside 1e-4 relative), and a target inherits that relative error times the size
# of the correction it sums, however small the target itself comes out.  There the floor is the
# operand scale itself.
CHAINED = dict(floor_fraction=1.0)


def assert_close(got, want, scale=1.0, what="", rtol=RTOL, floor_fraction=FLOOR_FRACTION):
    """scale: a number, or an array shaped like `want` (the size of what each element added up)."""
    g = np.asarray(got, dtype=np.float64)
    o = np.asarray(want, dtype=np.float64)
    assert g.shape == o.shape, f"{what}: shape {g.shape} vs {o.shape}"
    if g.size == 0:
        return 0.0
    assert np.all(np.isfinite(g) == np.isfinite(o)), f"{what}: finiteness differs"
    fin = np.isfinite(o)
    np.testing.assert_array_equal(g[~fin], o[~fin], err_msg=f"{what}: non-finite values differ")
    floor = np.broadcast_to(floor_fraction * np.asarray(scale, dtype=np.float64), o.shape)[fin]
    err = np.abs(g[fin] - o[fin])
    denom = np.maximum(np.abs(o[fin]), floor)
    worst = float(np.max(err / np.maximum(denom, 1e-300))) if err.size else 0.0
    bad = err > rtol * denom
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {err.size} outside 1e-4 relative "
                           f"(floor {float(np.min(floor)):.3g}..{float(np.max(floor)):.3g}); worst scaled error {worst:.3e}")
    return worst


def ent_floor(V):
    """The scale of an entropy over V outcomes (assert_close puts the floor at a hundredth of it)."""
    return math.log(V)


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


GRAD_ULPS = 16 * 2.0 ** -24     # rounding the gradient kernel itself may add, relative to an element's factors


def grad_bound(logits_bits, tokens, V, coef, beta, scale, o_tok_logp, o_tok_ent, g_tok_logp, g_tok_ent):
    """Per-element bound on |device gradient - oracle gradient| (fp32 output), from the arithmetic of
        g[r, v] = scale * p_v * (C_r + beta * (log p_v + H_r))           (v != token)
        g[r, tok] = scale * (C_r * (p - 1) + beta * p * (log p + H_r)),   C_r = rho_t * A_t.
    The second sweep takes log Z_r = x_tok - tok_logp[r] and H_r = tok_ent[r] from the first one, so an
    absolute error e_r in tok_logp scales every p_v of the row by exp(-e_r) and shifts log p_v by e_r,
    and an error h_r in tok_ent shifts H_r.  Where the factor C + beta*(log p + H) does not cancel that
    is a relative error of the element and sits inside 1e-4*|o|; where it cancels, what is left is
        scale * p_v * (|C_r| + beta * (|log p_v| + H_r + 1)) * (e_r + h_r + a few fp32 roundings).
    e_r and h_r are measured here (device first sweep against the oracle's); the roundings are
    GRAD_ULPS (exp2, the two-float log Z, one fused multiply-add per factor, coef in fp32).  The last
    term is fp32's smallest normal number: below it the device flushes to zero.
    Arguments are per row [R] except logits_bits [R, >=V]; returns [R, V]."""
    x = (np.ascontiguousarray(logits_bits[:, :V]).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    tok = np.asarray(tokens)
    live = (tok >= 0) & (tok < V)
    rows = np.arange(x.shape[0])
    xt = x[rows, np.where(live, tok, 0)]
    log_z = xt - np.asarray(o_tok_logp, np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        logp = x - log_z[:, None]
        p = np.exp(logp)
    p = np.where(np.isfinite(p), p, 0.0)
    abs_logp = np.where(np.isfinite(logp), np.abs(logp), 0.0)        # masked vocabulary entries: p = 0
    inherited = np.abs(np.asarray(g_tok_logp, np.float64) - o_tok_logp) + np.abs(np.asarray(g_tok_ent, np.float64) - o_tok_ent)
    factors = np.abs(coef)[:, None] + beta * (abs_logp + np.asarray(o_tok_ent, np.float64)[:, None] + 1.0)
    extra = scale * p * factors * (inherited[:, None] + GRAD_ULPS) + 2.0 ** -126
    return np.where(live[:, None], extra, 0.0)
