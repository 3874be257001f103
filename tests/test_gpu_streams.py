"""Calls on different streams share nothing but what the caller hands them: two chains of the hot
path, each with its own inputs, outputs and workspace, run side by side on two streams (both at
the default priority) and give the bits each gives alone."""
import numpy as np
import pytest
import torch

from paper_2410_14803_amd import binding as b
from paper_2410_14803_amd import synth
from _util import npf

pytestmark = pytest.mark.gpu
DEV = "cuda"


class Chain:
    def __init__(self, seed, B, M, K):
        cfg = synth.scaled(synth.CONFIGS[1], B=B, M=M, K=K)
        self.cfg = cfg
        off_np = synth.trajectory_offsets(cfg, seed)
        self.N = N = int(off_np[-1]); self.R = R = N * cfg.A
        self.off = torch.as_tensor(off_np, device=DEV)
        self.logits = synth.logits_bf16(R, cfg.V, seed + 1, DEV)
        self.tokens = synth.action_tokens(self.logits, seed + 2)
        self.si = synth.step_inputs(cfg, off_np, seed + 3, DEV)
        f = lambda n: torch.zeros(n, device=DEV)
        self.out = dict(tok_logp=f(R), tok_ent=f(R), step_logp=f(N), step_ent=f(N), target=f(N), td=f(N), rho=f(N),
                        step_prio=f(N), traj_prio=f(cfg.B), prob=f(K))
        self.idx = torch.zeros(K, dtype=torch.int64, device=DEV)
        self.logmu = torch.randn(N, generator=torch.Generator(device=DEV).manual_seed(seed + 4), device=DEV) * 0.3 - 9.0
        self.u = synth.uniforms(K, seed + 5, DEV)
        self.w0 = synth.replay_priorities(M, "exp", seed + 6, DEV) ** 0.6
        self.weights = self.w0.clone()
        self.ws = b.Workspace(M)

    def reset(self):
        self.weights.copy_(self.w0)
        for v in self.out.values():
            v.zero_()
        self.idx.zero_()
        b.update_priorities(self.weights, None, None, self.cfg.alpha, self.ws)

    def run(self, rounds):
        c, o = self.cfg, self.out
        for _ in range(rounds):
            b.score_logits(self.logits, self.tokens, c.A, self.ws, tok_logp=o["tok_logp"], tok_ent=o["tok_ent"],
                           step_logp=o["step_logp"], step_ent=o["step_ent"])
            b.retrace_priorities(o["step_logp"], self.logmu, self.si["reward"], self.si["value"], o["step_ent"], self.off,
                                 c.gamma, c.lam, c.w, q=self.si["q"], target=o["target"], td=o["td"], rho=o["rho"],
                                 step_prio=o["step_prio"], traj_prio=o["traj_prio"])
            b.sample_prioritized(self.weights, self.u, self.ws, self.idx, o["prob"])
            b.update_priorities(self.weights, self.idx, o["step_prio"][:c.K] if self.N >= c.K else o["step_prio"],
                                c.alpha, self.ws)

    def snapshot(self):
        d = {k: npf(v).copy() for k, v in self.out.items()}
        d["idx"] = npf(self.idx).copy(); d["weights"] = npf(self.weights).copy()
        st, rc = self.ws.status()
        assert rc == b.OK and st.flags == 0
        return d


def test_two_chains_on_two_streams():
    a, c = Chain(100, 40, 70000, 700), Chain(200, 64, 5000, 300)     # the larger and the one-workgroup replay path
    rounds = 6
    alone = []
    for ch in (a, c):
        ch.reset(); ch.run(rounds)
        torch.cuda.synchronize()
        alone.append(ch.snapshot())
    sa, sc = torch.cuda.Stream(), torch.cuda.Stream()
    for trial in range(3):
        for ch in (a, c):
            ch.reset()
        torch.cuda.synchronize()
        with torch.cuda.stream(sa):
            a.run(rounds)
        with torch.cuda.stream(sc):
            c.run(rounds)
        torch.cuda.synchronize()
        for ch, want in ((a, alone[0]), (c, alone[1])):
            got = ch.snapshot()
            for k in want:
                assert np.array_equal(got[k], want[k], equal_nan=True), f"trial {trial}: {k} differs when run beside another stream"
