"""Seeded synthetic workloads shaped like the paper's learner batches.

This module only draws random inputs (logits, action tokens, trajectory lengths,
rewards, values, behaviour-policy noise, replay priorities, uniforms).  It contains
none of the scoring arithmetic (no softmax, no Retrace, no priorities, no CDF): both
the HIP library's tests and the CPU oracle's tests are fed from here, and neither the
library nor the oracle imports it.

Shapes follow the paper's setting: finite-horizon episodes of at most 15-20 steps
(Appendix A.5, task horizons), sparse 0/1 terminal reward from the evaluator
(Section 3), a token-level language-model policy whose action is a short token
sequence (Appendix A.5, T5-style decoder), and behaviour policies that lag the
target policy (Section 3, asynchronous collection).

All generators take an explicit seed and a torch device; the same (seed, device type)
always yields the same values.  CPU and GPU generators yield different streams, which
is fine: within one test both sides consume the very same arrays.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np
import torch

BASE_SEED = 20241014


@dataclass(frozen=True)
class Config:
    """One synthetic workload.  len_lo == len_hi means fixed-length trajectories."""
    name: str
    B: int                    # trajectories
    len_lo: int               # min steps per trajectory
    len_hi: int               # max steps per trajectory (inclusive)
    A: int                    # action tokens per step (0: no logits in this workload)
    V: int                    # vocabulary (0: no logits)
    heavy_tail: bool = False  # 5% of logits get a +8 spike
    gamma: float = 0.9
    lam: float = 0.95
    w: Tuple[float, float, float] = (1.0, 0.5, 0.1)
    alpha: float = 0.6
    M: int = 0                # replay entries
    K: int = 0                # samples per draw
    reward: str = "terminal"  # "terminal": last step ~ Bernoulli(0.3); "dense": every step ~ Bernoulli(0.05)
    value_lo: float = 0.0
    value_hi: float = 1.0
    mu_sigma: float = 0.3
    replay: str = "exp"       # "exp": p ~ Exp(1); "lognormal": p ~ LogNormal(0,1)
    index: int = 0
    iters: int = 1


CONFIGS = {
    0: Config("tiny", B=32, len_lo=10, len_hi=10, A=8, V=32128, M=4096, K=256, index=0),
    1: Config("learner_batch", B=256, len_lo=1, len_hi=20, A=32, V=32128, M=65536, K=1024, index=1),
    2: Config("large_vocab", B=128, len_lo=16, len_hi=16, A=64, V=151936, heavy_tail=True,
              M=4096, K=256, index=2),
    3: Config("long_scan", B=4096, len_lo=64, len_hi=256, A=0, V=0, gamma=0.99, lam=1.0,
              reward="dense", value_lo=-1.0, value_hi=1.0, mu_sigma=0.5, index=3),
    4: Config("replay_scale", B=0, len_lo=0, len_hi=0, A=0, V=0, M=1 << 24, K=65536,
              replay="lognormal", w=(1.0, 0.0, 0.0), index=4, iters=100),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp64."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def trajectory_offsets(cfg: Config, seed: int) -> np.ndarray:
    """CSR offsets int32[B+1]; lengths uniform on {len_lo..len_hi}."""
    g = _gen(seed, "cpu")
    if cfg.B == 0:
        return np.zeros(1, dtype=np.int32)
    lens = torch.randint(cfg.len_lo, cfg.len_hi + 1, (cfg.B,), generator=g, dtype=torch.int64)
    off = torch.zeros(cfg.B + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(lens, 0)
    return off.numpy().astype(np.int32)


def logits_bf16(R: int, V: int, seed: int, device, heavy_tail: bool = False,
                rows_per_chunk: Optional[int] = None) -> torch.Tensor:
    """bf16 [R, V]: 2*N(0,1), plus 8*Bernoulli(0.05) when heavy_tail; rounded to bf16."""
    g = _gen(seed, device)
    out = torch.empty((R, V), dtype=torch.bfloat16, device=device)
    if rows_per_chunk is None:
        rows_per_chunk = max(1, (1 << 28) // max(V, 1))
    for r0 in range(0, R, rows_per_chunk):
        r1 = min(R, r0 + rows_per_chunk)
        x = torch.randn((r1 - r0, V), generator=g, device=device, dtype=torch.float32) * 2.0
        if heavy_tail:
            spike = torch.rand((r1 - r0, V), generator=g, device=device) < 0.05
            x = x + 8.0 * spike.to(torch.float32)
        out[r0:r1] = x.to(torch.bfloat16)
    return out


def action_tokens(logits: torch.Tensor, seed: int, noise_sigma: float = 0.5,
                  rows_per_chunk: Optional[int] = None) -> torch.Tensor:
    """int32 [R]: one draw per row from Categorical(softmax(logits + N(0, sigma^2))).

    Drawn with the Gumbel-max trick (argmax of perturbed logits), so that no softmax is
    ever formed here.
    """
    R, V = logits.shape
    device = logits.device
    g = _gen(seed, device)
    out = torch.empty(R, dtype=torch.int32, device=device)
    if rows_per_chunk is None:
        rows_per_chunk = max(1, (1 << 27) // max(V, 1))
    for r0 in range(0, R, rows_per_chunk):
        r1 = min(R, r0 + rows_per_chunk)
        x = logits[r0:r1].to(torch.float32)
        x = x + noise_sigma * torch.randn(x.shape, generator=g, device=device)
        u = torch.rand(x.shape, generator=g, device=device).clamp_(1e-20, 1.0 - 1e-7)
        gumbel = -torch.log(-torch.log(u))
        out[r0:r1] = torch.argmax(x + gumbel, dim=1).to(torch.int32)
    return out


def step_inputs(cfg: Config, offsets: np.ndarray, seed: int, device):
    """Per-step fp32 inputs other than the policy's own log-probabilities.

    Returns dict(reward[N], value[N], q[N], mu_noise[N], boot[B]).  The behaviour
    log-probability is formed by the caller as logp_pi + mu_noise, from whichever
    logp_pi that caller computed; this module never evaluates the policy.
    """
    g = _gen(seed, device)
    N = int(offsets[-1])
    B = len(offsets) - 1
    span = cfg.value_hi - cfg.value_lo
    value = torch.rand(N, generator=g, device=device) * span + cfg.value_lo
    q = torch.rand(N, generator=g, device=device) * span + cfg.value_lo
    mu_noise = torch.randn(N, generator=g, device=device) * cfg.mu_sigma
    if cfg.reward == "terminal":
        reward = torch.zeros(N, device=device)
        if B > 0 and N > 0:
            hit = (torch.rand(B, generator=g, device=device) < 0.3).to(torch.float32)
            off = torch.as_tensor(offsets, device=device, dtype=torch.int64)
            nonempty = off[1:] > off[:-1]
            last = (off[1:] - 1)[nonempty]
            reward[last] = hit[nonempty]
    else:
        reward = (torch.rand(N, generator=g, device=device) < 0.05).to(torch.float32)
    boot = torch.zeros(B, device=device)
    return dict(reward=reward, value=value, q=q, mu_noise=mu_noise, boot=boot)


def policy_logprobs(N: int, seed: int, device) -> torch.Tensor:
    """fp32 [N] stand-in for log pi when a workload has no logits: -3*|N(0,1)|."""
    g = _gen(seed, device)
    return -3.0 * torch.randn(N, generator=g, device=device).abs()


def replay_priorities(M: int, kind: str, seed: int, device) -> torch.Tensor:
    """fp32 [M] raw priorities p: Exp(1) or LogNormal(0,1)."""
    g = _gen(seed, device)
    if kind == "exp":
        u = torch.rand(M, generator=g, device=device, dtype=torch.float64).clamp_(1e-300, 1.0)
        return (-torch.log(u)).to(torch.float32)
    if kind == "lognormal":
        return torch.exp(torch.randn(M, generator=g, device=device, dtype=torch.float32))
    raise ValueError(kind)


def uniforms(K: int, seed: int, device) -> torch.Tensor:
    """fp64 [K] in [0, 1) with 53 random bits."""
    g = _gen(seed, device)
    return torch.rand(K, generator=g, device=device, dtype=torch.float64)


def td_errors(K: int, seed: int, device) -> torch.Tensor:
    """fp32 [K] ~ N(0,1): synthetic TD errors for the replay-at-scale loop."""
    g = _gen(seed, device)
    return torch.randn(K, generator=g, device=device, dtype=torch.float32)


def scaled(cfg: Config, **kw) -> Config:
    """A smaller copy of a config (same distributions) for CPU-sized tests."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return Config(**d)
