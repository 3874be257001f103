"""The five calls of the hot path enqueue kernels only (no allocation, no memset, no
synchronisation), so a caller may capture them into a HIP graph.  The graph is replayed several
times with eager work and synchronisation in between, and every replay is compared with the
eager result on the same inputs."""
import numpy as np
import pytest
import torch

from paper_2410_14803_amd import binding as b
from paper_2410_14803_amd import synth
from _util import npf

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_hot_path_in_a_hip_graph():
    cfg = synth.scaled(synth.CONFIGS[1], B=12, M=20000, K=512)
    off_np = synth.trajectory_offsets(cfg, 5)
    N = int(off_np[-1]); R = N * cfg.A
    off = torch.as_tensor(off_np, device=DEV)
    logits = synth.logits_bf16(R, cfg.V, 6, DEV)
    tokens = synth.action_tokens(logits, 7)
    si = synth.step_inputs(cfg, off_np, 8, DEV)
    f = lambda n: torch.zeros(n, device=DEV)
    out = dict(tok_logp=f(R), tok_ent=f(R), step_logp=f(N), step_ent=f(N), target=f(N), td=f(N), rho=f(N),
               step_prio=f(N), traj_prio=f(cfg.B), prob=f(cfg.K))
    idx = torch.zeros(cfg.K, dtype=torch.int64, device=DEV)
    logmu = f(N)
    u = torch.zeros(cfg.K, dtype=torch.float64, device=DEV)
    w0 = synth.replay_priorities(cfg.M, "exp", 9, DEV) ** 0.6
    weights = w0.clone()
    ws = b.Workspace(cfg.M)
    b.update_priorities(weights, None, None, cfg.alpha, ws)

    def chain():
        b.score_logits(logits, tokens, cfg.A, ws, tok_logp=out["tok_logp"], tok_ent=out["tok_ent"],
                       step_logp=out["step_logp"], step_ent=out["step_ent"])
        b.retrace_targets(out["step_logp"], logmu, si["reward"], si["value"], off, cfg.gamma, cfg.lam, q=si["q"],
                          target=out["target"], td=out["td"], rho=out["rho"])
        b.compute_priorities(out["td"], out["rho"], out["step_ent"], off, cfg.w, step_prio=out["step_prio"],
                             traj_prio=out["traj_prio"])
        b.sample_prioritized(weights, u, ws, idx, out["prob"])
        b.update_priorities(weights, idx, out["step_prio"][:cfg.K] if N >= cfg.K else out["step_prio"], cfg.alpha, ws)

    def snapshot():
        torch.cuda.synchronize()
        d = {k: npf(v).copy() for k, v in out.items()}
        d["idx"] = npf(idx).copy(); d["weights"] = npf(weights).copy()
        return d

    def set_inputs(seed):
        logmu.copy_(torch.randn(N, generator=torch.Generator(device=DEV).manual_seed(seed), device=DEV) * 0.3 - 9.0)
        u.copy_(synth.uniforms(cfg.K, seed + 1, DEV))
        weights.copy_(w0)
        b.update_priorities(weights, None, None, cfg.alpha, ws)

    # warm-up on a side stream, then capture
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        set_inputs(100)
        chain()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    set_inputs(100)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        chain()
    for rep, seed in enumerate((11, 12, 13, 11)):
        set_inputs(seed)
        chain()
        eager = snapshot()
        for v in out.values():
            v.fill_(-5.0)                      # eager work between replays
        idx.fill_(-5)
        set_inputs(seed)
        g.replay()
        replayed = snapshot()
        for k in eager:
            np.testing.assert_array_equal(replayed[k].view(np.uint8), eager[k].view(np.uint8),
                                          err_msg=f"replay {rep}: {k} differs from the eager run")
    st, rc = ws.status()
    assert rc == b.OK and st.flags == 0


def test_large_buffer_rebuild_and_patched_insert_in_a_hip_graph(oracle):
    # Whether a rebuild needs its second sweep, and whether an insert can be patched, is decided
    # on the device: a captured graph must take the right route for every input it is replayed on.
    M = 64 * 65536 + 3 * 256 + 9
    K_up, K_in, K_s, cursor = 5000, 3000, 600, M - 1000
    w0_host = np.zeros(M, np.float32)
    oracle.update_priorities(w0_host, np.arange(M), npf(synth.replay_priorities(M, "lognormal", 3, "cpu")), 0.6)
    w0 = torch.as_tensor(w0_host, device=DEV)
    weights = w0.clone()
    ws = b.Workspace(M)
    idx_up = torch.zeros(K_up, dtype=torch.int64, device=DEV)
    p_up = torch.zeros(K_up, device=DEV)
    p_in = torch.zeros(K_in, device=DEV)
    u = torch.zeros(K_s, dtype=torch.float64, device=DEV)
    drawn = [torch.zeros(K_s, dtype=torch.int64, device=DEV) for _ in range(2)]

    def chain():
        b.update_priorities(weights, idx_up, p_up, 0.6, ws)
        b.sample_prioritized(weights, u, ws, drawn[0], None)
        b.replay_insert(weights, cursor, p_in, 0.6, ws)
        b.sample_prioritized(weights, u, ws, drawn[1], None)

    def set_inputs(seed, up_scale, in_scale):
        rng = np.random.default_rng(seed)
        idx_up.copy_(torch.as_tensor(rng.integers(0, M, K_up), device=DEV))
        p_up.copy_(torch.as_tensor((rng.random(K_up) * up_scale).astype(np.float32), device=DEV))
        p_in.copy_(torch.as_tensor((rng.random(K_in) * in_scale).astype(np.float32), device=DEV))
        u.copy_(synth.uniforms(K_s, seed, DEV))
        weights.copy_(w0)
        b.update_priorities(weights, None, None, 0.6, ws)
        torch.cuda.synchronize()

    def check(tag):
        torch.cuda.synchronize()
        oi, _, _ = oracle.sample_prioritized(npf(weights), npf(u))
        np.testing.assert_array_equal(npf(drawn[1]), oi, err_msg=tag)
        st, rc = ws.status()
        _, total = oracle.quantise_weights(npf(weights))
        assert rc == b.OK and st.total == total, tag
        return npf(weights).copy(), npf(drawn[0]).copy()

    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        set_inputs(1, 1.0, 1.0)
        chain()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    set_inputs(1, 1.0, 1.0)
    with torch.cuda.graph(g):
        chain()
    # (update scale, insert scale): same exponent throughout / the update raises it / the insert
    # raises it / back to the first
    for rep, (up_scale, in_scale) in enumerate([(1.0, 1.0), (1e6, 1.0), (1.0, 1e6), (1.0, 1.0)]):
        set_inputs(20 + rep, up_scale, in_scale)
        chain()
        eager = check(f"eager {rep}")
        for d in drawn:
            d.fill_(-5)
        set_inputs(20 + rep, up_scale, in_scale)
        g.replay()
        replayed = check(f"replay {rep}")
        np.testing.assert_array_equal(eager[0], replayed[0])
        np.testing.assert_array_equal(eager[1], replayed[1])
