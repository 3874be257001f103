#!/usr/bin/env python3
"""Throughput of the A-RIDE scoring pass on one MI355X.

One "step" is one pass of the whole hot path over one learner batch (the "learner_batch"
workload: 256 trajectories of 1..20 steps, 32 action tokens per step, V = 32128 bf16
logits; replay buffer of 65536 entries, 1024 draws):

    score_logits -> retrace_priorities (retrace_targets and compute_priorities in one pass)
                 -> sample_prioritized -> update_priorities (scatter + index rebuild)

All inputs are synthetic, seeded, and resident in HBM before the timed region starts.
Prints ONE JSON line: whole-job trajectory-steps/s, the HBM roofline of the dominant
kernel (the logit sweep) from HIP events recorded inside the timed region, and the CPU
oracle timed on a bounded sample of the same batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak

# HBM bytes per step from hardware counters (profiles/*.md): FETCH_SIZE and WRITE_SIZE in KiB per
# dispatch from two `rocprofv3 --pmc` runs of the very command, each scaled by what the same counter
# reads for a plain 1 GiB copy kernel (x2.000 and x1.000), summed over the kernels the roofline entry
# names.  An entry is valid only for the kernel source it was measured on (first 16 hex digits of
# the file's sha256) and for its workload; anything else reports null.
TRAFFIC = {
    # the logit sweep (k_score_rows_split) on configs 0, 1, 2
    ("scoring", 0): ("score_logits.hip", "44710732453a7cf8", 164830618),
    ("scoring", 1): ("score_logits.hip", "44710732453a7cf8", 5287676621),
    ("scoring", 2): ("score_logits.hip", "44710732453a7cf8", 39844374118),
    # k_actor_grad on config 1
    ("actor_grad", 1): ("actor_grad.hip", "afc03ce463a348c2", 10559418982),
    # k_flat_scan on config 3 at batch scales 1, 16, 64: (scale, one pass?)
    ("retrace", (1, True)): ("retrace.hip", "c321b09416a5e31a", 26570957),
    ("retrace", (16, True)): ("retrace.hip", "c321b09416a5e31a", 439354368),
    ("retrace", (64, True)): ("retrace.hip", "c321b09416a5e31a", 1708336128),
    ("retrace", (1, False)): ("retrace.hip", "c321b09416a5e31a", 31978496),
    ("retrace", (16, False)): ("retrace.hip", "c321b09416a5e31a", 537822106),
    ("retrace", (64, False)): ("retrace.hip", "c321b09416a5e31a", 2059197645),
    # config 4: sample + tag + commit + the one sweep + its check + prefix; and the patched insert
    ("replay", None): ("replay.hip", "ad5cde5702f702cb", 117363000),
    ("insert", None): ("replay.hip", "ad5cde5702f702cb", 797000),
    ("insert", "rebuild"): ("replay.hip", "ad5cde5702f702cb", 79412000),    # the patched insert + a full rebuild
}


def _traffic(path, key):
    import hashlib
    entry = TRAFFIC.get((path, key))
    if entry is None:
        return None
    fname, sha, nbytes = entry
    src = os.path.join(ROOT, "paper_2410_14803_amd", "csrc", fname)
    return nbytes if hashlib.sha256(open(src, "rb").read()).hexdigest()[:16] == sha else None


METRIC = "trajectory-steps/sec scored (logits->Retrace->priority) + % peak HBM GB/s"


def bench_actor_grad(args, b, torch, cfg, logits, tokens, tok_logp, tok_ent, step_logp, step_ent, si, N, R):
    """One step = one aride_actor_loss_grad call (bf16 gradient + scalar loss) on the batch."""
    dev = logits.device
    g = torch.Generator(device=dev); g.manual_seed(99)
    rho = torch.exp(0.3 * torch.randn(N, generator=g, device=dev))
    target = torch.rand(N, generator=g, device=dev)
    grad = torch.empty_like(logits)
    loss = torch.zeros(1, device=dev)

    def step():
        b.actor_loss_grad(logits, tokens, cfg.A, tok_logp, tok_ent, step_logp, step_ent, rho, target, si["value"],
                          0.01, 1.0 / N, grad=grad, loss=loss)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = e0.elapsed_time(e1) / args.steps
    alg_bytes = R * cfg.V * 4 + R * 12 + N * 12     # logits in, bf16 gradient out, per-row and per-step scalars
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        h = lambda t: t.detach().cpu().numpy()
        n_s = min(N, 8)                       # a few whole steps: the oracle's gradient is single-threaded
        r_s = n_s * cfg.A
        bits = logits[:r_s].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        t0 = time.perf_counter()
        oracle.actor_loss_grad(bits, h(tokens[:r_s]), cfg.A, h(rho[:n_s]), h(target[:n_s]), h(si["value"][:n_s]),
                               0.01, 1.0 / N)
        dt = time.perf_counter() - t0
        cpu = {"value": n_s / dt, "unit": "trajectory-steps/s", "cores": 1, "kind": "oracle", "seconds": dt,
               "sample": f"first {n_s} steps ({r_s} logit rows) of the batch, fp64 gradient"}
    print(json.dumps({
        "metric": "trajectory-steps/sec through the actor loss + logit gradient (eq. 1) + % peak HBM GB/s",
        "value": N * args.steps / elapsed, "unit": "trajectory-steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} (config {cfg.index}), actor_grad path", "traj_steps": N,
                   "logit_rows": R, "vocab": cfg.V, "grad_dtype": "bf16"},
        "roofline": {"bound": "hbm", "kernel": "k_actor_grad (+ k_actor_loss)", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": _traffic("actor_grad", args.config) if R == 82144 else None,
                     "algorithmic_bytes_per_launch": alg_bytes, "ms_per_launch": ms},
        "cpu_baseline": cpu}), flush=True)


def _sweep_kernel_name(V):
    """The kernel aride_score_logits dispatches for rows of V logits (the rule of score_logits_launch:
    16-byte vectors per row from which a row is shared by 4, 8, 16 waves)."""
    nvec = V >> 3
    for waves, least in ((16, 12288), (8, 3072), (4, 1024)):
        if nvec >= least:
            return f"k_score_rows_split ({waves} waves per row at this row length)"
    return "k_score_rows (one wave per row at this row length)"


def _timed(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return time.perf_counter() - t0, e0.elapsed_time(e1) / steps


def bench_retrace(args, b, torch, synth, dev):
    """One step = retrace_targets + compute_priorities over the long-scan batch (config 3), as the one call
    aride_retrace_priorities unless --two-calls."""
    cfg = synth.CONFIGS[3]
    if args.batch_scale != 1:                 # the same length mix, more trajectories
        cfg = synth.scaled(cfg, B=cfg.B * args.batch_scale)
    seed = synth.BASE_SEED + cfg.index
    off_np = synth.trajectory_offsets(cfg, seed)
    N = int(off_np[-1])
    off = torch.as_tensor(off_np, device=dev)
    lp = synth.policy_logprobs(N, seed + 3, dev)
    si = synth.step_inputs(cfg, off_np, seed + 4, dev)
    lm = lp + si["mu_noise"]
    ent = torch.rand(N, device=dev)
    f = lambda n: torch.empty(n, device=dev)
    tg, td, rho, sp, tp = f(N), f(N), f(N), f(N), f(cfg.B)

    def step():
        if args.one_pass:
            b.retrace_priorities(lp, lm, si["reward"], si["value"], ent, off, cfg.gamma, cfg.lam, cfg.w, q=si["q"],
                                 target=tg, td=td, rho=rho, step_prio=sp, traj_prio=tp)
            return
        b.retrace_targets(lp, lm, si["reward"], si["value"], off, cfg.gamma, cfg.lam, q=si["q"], target=tg, td=td, rho=rho)
        b.compute_priorities(td, rho, ent, off, cfg.w, step_prio=sp, traj_prio=tp)
    # the two sibling kernels of the same scan, a few untimed calls each so that a profile of this
    # command shows them too: V-trace targets and Monte-Carlo returns
    ret, lab = f(N), f(N)
    for _ in range(10):
        b.retrace_targets(lp, lm, si["reward"], si["value"], off, cfg.gamma, cfg.lam, q=si["q"], target=tg, td=td,
                          rho=rho, vtrace=True, rho_bar=1.0, c_bar=1.0)
        b.mc_returns(si["reward"], off, cfg.gamma, ret=ret, label=lab)
    elapsed, ms = _timed(torch, step, args.steps, args.warmup)
    mix = _mix_probe(torch, N, (6, 4) if args.one_pass else (5, 3), dev) if args.mix_probe else None
    alg_bytes = N * (20 + 12) + N * (12 + 4) + cfg.B * 12     # retrace: 5 in + 3 out; priorities: 3 in + 1 out
    if args.one_pass:
        alg_bytes = N * (24 + 16) + cfg.B * 12                # 6 in + 4 out: td and rho are not read back
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        h = lambda t: t.detach().cpu().numpy()
        a = (h(lp), h(lm), h(si["reward"]), h(si["value"]), off_np, cfg.gamma, cfg.lam)
        qh, eh = h(si["q"]), h(ent)
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 2.0:
            o = oracle.retrace_targets(*a, q=qh)
            oracle.compute_priorities(o["td"], o["rho"], eh, off_np, *cfg.w)
            reps += 1
        dt = time.perf_counter() - t0
        cpu = {"value": N * reps / dt, "unit": "trajectory-steps/s", "cores": 1, "kind": "oracle", "seconds": dt,
               "sample": f"the whole batch ({N} steps), {reps} repetitions"}
    print(json.dumps({
        "metric": "trajectory-steps/sec through Retrace + priorities (no logits) + % peak HBM GB/s",
        "value": N * args.steps / elapsed, "unit": "trajectory-steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} (config {cfg.index})", "trajectories": cfg.B, "traj_steps": N,
                   "gamma": cfg.gamma, "lambda": cfg.lam, "one_pass": bool(args.one_pass)},
        "roofline": {"bound": "hbm", "kernel": "k_flat_scan<Retrace, with priorities> (one launch)"
                     if args.one_pass else "k_flat_scan<Retrace> + k_flat_scan<priorities> (two launches)",
                     "achieved": alg_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": _traffic("retrace", (args.batch_scale, bool(args.one_pass))),
                     "algorithmic_bytes_per_launch": alg_bytes, "ms_per_launch": ms, "stream_mix_probe": mix},
        "cpu_baseline": cpu}), flush=True)


def _mix_probe(torch, N, shape, dev):
    """Bare kernels with the scan's traffic and no scan (shape = arrays read, arrays written; 16 bytes
    per lane and array): the rate the memory system allows that mix of streams on N steps, for a
    workgroup per 4 KB in dispatch order and for the scan's own shape (a contiguous span per wave),
    with plain and with non-temporal loads; and the read-only and write-only halves by themselves."""
    import ctypes
    probe = ctypes.CDLL(os.path.join(ROOT, "paper_2410_14803_amd", "libaride_probe.so"))
    probe.aride_probe_mix.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                                      ctypes.c_int, ctypes.c_void_p]
    n = N // 4 * 4
    ins = [torch.rand(n, device=dev) for _ in range(6)]
    outs = [torch.empty(n, device=dev) for _ in range(4)]
    pin = torch.tensor([t.data_ptr() for t in ins], dtype=torch.int64, device=dev)
    pout = torch.tensor([t.data_ptr() for t in outs], dtype=torch.int64, device=dev)
    st = torch.cuda.current_stream().cuda_stream

    def rate(nin, nout, pattern):
        go = lambda: probe.aride_probe_mix(pin.data_ptr(), pout.data_ptr(), nin, nout, n, pattern, st)
        for _ in range(5):
            assert go() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            go()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 20
        gbps = n * 4 * (nin + nout) / (ms * 1e-3) / 1e9
        return {"ms": ms, "GB/s": gbps, "frac": gbps / HBM_PEAK_GBPS}

    nin, nout = shape
    out = {"arrays_read": nin, "arrays_written": nout, "steps": n}
    out.update(rate(nin, nout, 0))
    out["patterns"] = {
        "block_per_4KB": rate(nin, nout, 0), "block_per_4KB_nt_loads": rate(nin, nout, 1),
        "span_per_wave": rate(nin, nout, 2), "span_per_wave_nt_loads": rate(nin, nout, 3),
        "read_only_6": rate(6, 0, 0), "read_only_6_nt_loads": rate(6, 0, 1), "write_only_4": rate(0, 4, 0),
        "write_only_4_span_per_wave": rate(0, 4, 2)}
    return out


def bench_replay(args, b, torch, synth, dev):
    """One step = sample K indices, recompute their priorities, scatter, rebuild the index (config 4)."""
    cfg = synth.CONFIGS[4]
    seed = synth.BASE_SEED + cfg.index
    M, K = cfg.M, cfg.K
    w = torch.zeros(M, device=dev)
    ws = b.Workspace(M, device=dev)
    p0 = synth.replay_priorities(M, cfg.replay, seed + 5, dev)
    for s0 in range(0, M, 1 << 22):
        b.update_priorities(w, torch.arange(s0, min(M, s0 + (1 << 22)), device=dev), p0[s0:s0 + (1 << 22)], cfg.alpha, ws)
    total = args.steps + args.warmup
    uni = synth.uniforms(K * total, seed + 6, dev).view(total, K)
    prio = synth.td_errors(K * total, seed + 7, dev).abs().view(total, K)
    idx = torch.empty(K, dtype=torch.int64, device=dev)
    it = [0]

    def step():
        i = it[0] % total
        it[0] += 1
        b.sample_prioritized(w, uni[i], ws, idx, None)
        b.update_priorities(w, idx, prio[i], cfg.alpha, ws)
    elapsed, ms = _timed(torch, step, args.steps, args.warmup)
    st, rc = ws.status()
    assert rc == b.OK and st.flags == 0, f"status flags {st.flags:#x} rc {rc}"
    # per step: one sweep of the weights (maxima and integer sums together) and the index written
    # once (a u64 per 16 weights and per 256 weights); per draw the 16 sub-block sums of one block,
    # the 16 weights of one sub-block (the upper index levels it consults stay in cache) and 16 B
    # of I/O; per update 12 B in and one 64-byte sector read-modify-written
    alg_bytes = M * 4 + (M // 16) * 8 + (M // 256) * 8 + K * (128 + 64 + 8 + 8) + K * (8 + 4 + 64)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        h = lambda t: t.detach().cpu().numpy()
        wh = h(w).copy()
        t0 = time.perf_counter()
        reps = 0
        while reps < 3:
            oi, _, _ = oracle.sample_prioritized(wh, h(uni[reps]))
            oracle.update_priorities(wh, oi, h(prio[reps]), cfg.alpha)
            reps += 1
        dt = time.perf_counter() - t0
        cpu = {"value": K * reps / dt, "unit": "draws/s", "cores": 1, "kind": "oracle", "seconds": dt,
               "sample": f"{reps} iterations of sample + update on the full {M}-entry buffer"}
    print(json.dumps({
        "metric": "prioritized draws/sec incl. priority update and index rebuild + % peak HBM GB/s",
        "value": K * args.steps / elapsed, "unit": "draws/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": f"{cfg.name} (config {cfg.index})", "replay_entries": M, "draws": K, "alpha": cfg.alpha},
        "roofline": {"bound": "hbm", "kernel": "k_sample + k_update_tag/commit + k_super_sums + k_prefix_super",
                     "achieved": alg_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": _traffic("replay", None),
                     "algorithmic_bytes_per_launch": alg_bytes, "ms_per_launch": ms},
        "cpu_baseline": cpu}), flush=True)


def bench_insert(args, b, torch, synth, dev):
    """One step = K new entries appended to the circular 2^24-entry buffer (config 4 sizes) with the
    sampling index brought up to date; --rebuild-every-insert forces the full rebuild for comparison."""
    cfg = synth.CONFIGS[4]
    seed = synth.BASE_SEED + cfg.index
    M, K = cfg.M, cfg.K
    w = torch.zeros(M, device=dev)
    ws = b.Workspace(M, device=dev)
    p0 = synth.replay_priorities(M, cfg.replay, seed + 5, dev)
    for s0 in range(0, M, 1 << 22):
        b.update_priorities(w, torch.arange(s0, min(M, s0 + (1 << 22)), device=dev), p0[s0:s0 + (1 << 22)], cfg.alpha, ws)
    total = args.steps + args.warmup
    prio = synth.td_errors(K * total, seed + 8, dev).abs().view(total, K)
    it = [0]
    cursor = [M - 3 * K - 17]          # the run wraps around the end of the buffer

    def step():
        i = it[0] % total
        it[0] += 1
        cursor[0] = b.replay_insert(w, cursor[0], prio[i], cfg.alpha, ws)
        if args.rebuild_every_insert:
            b.update_priorities(w, None, None, cfg.alpha, ws)
    elapsed, ms = _timed(torch, step, args.steps, args.warmup)
    st, rc = ws.status()
    assert rc == b.OK and st.flags == 0, f"status flags {st.flags:#x} rc {rc}"
    # per step: K priorities read, K weights written, the touched blocks read once more for their
    # integer sums, their index entries rewritten (a rebuild instead sweeps all M weights)
    alg_bytes = K * (4 + 4 + 4) + (K // 256 + 2) * (8 + 4)
    if args.rebuild_every_insert:
        alg_bytes += M * 4 + (M // 256) * 8
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        h = lambda t: t.detach().cpu().numpy()
        wh = h(w).copy()
        t0 = time.perf_counter()
        reps, cur = 0, 0
        while reps < min(total, 100):
            cur, _ = oracle.replay_insert(wh, cur, h(prio[reps]), cfg.alpha)
            oracle.quantise_weights(wh)          # the oracle's index is the whole prefix, rebuilt from scratch
            reps += 1
        dt = time.perf_counter() - t0
        cpu = {"value": K * reps / dt, "unit": "entries/s", "cores": 1, "kind": "oracle", "seconds": dt,
               "sample": f"{reps} inserts of {K} entries + quantisation of the full {M}-entry buffer"}
    print(json.dumps({
        "metric": "replay entries inserted/sec incl. keeping the sampling index current + % peak HBM GB/s",
        "value": K * args.steps / elapsed, "unit": "entries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": f"{cfg.name} (config {cfg.index}), circular insert", "replay_entries": M,
                   "entries_per_insert": K, "alpha": cfg.alpha, "rebuild_every_insert": bool(args.rebuild_every_insert)},
        "roofline": {"bound": "hbm", "kernel": "k_insert_patch + k_patch_supers + k_patch_finish (+ two gated no-ops)",
                     "achieved": alg_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": _traffic("insert", "rebuild" if args.rebuild_every_insert else None),
                     "algorithmic_bytes_per_launch": alg_bytes, "ms_per_launch": ms},
        "cpu_baseline": cpu}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps first; the first few dozen launches after start-up run a little slower")
    ap.add_argument("--config", type=int, default=1, help="workload index (1 = learner batch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target oracle time for the CPU sample")
    ap.add_argument("--path", choices=["scoring", "actor_grad", "retrace", "replay", "insert"], default="scoring",
                    help="scoring: the five-call hot path on the learner batch (default). actor_grad: the actor "
                         "loss and its logit gradient (eq. (1)), the second sweep over the same logits. "
                         "retrace: retrace_targets + compute_priorities on the long-scan workload (config 3). "
                         "replay: sample + update + index rebuild on the 2^24-entry buffer (config 4). "
                         "insert: circular insert of 65 536 entries into that buffer, index patched")
    ap.add_argument("--launch-series", type=int, default=0,
                    help="with --path scoring: report the duration of each of the first N pre-warm launches of the "
                         "sweep and the shader clock read by a 10 us probe kernel after each of them")
    ap.add_argument("--two-calls", action="store_true",
                    help="with --path scoring or retrace: aride_retrace_targets and aride_compute_priorities as two "
                         "calls instead of the one call aride_retrace_priorities (one launch, TD errors and "
                         "ratios not read back), which is the default")
    ap.add_argument("--prewarm", type=int, default=60,
                    help="with --path scoring: untimed launches of the logit sweep before the warm-up steps. A "
                         "process's first sustained load makes the chip's power management drop the shader clock "
                         "from 2.4 to about 1.3 GHz within 3 ms and let it back up to its sustained 1.8 GHz over "
                         "the next 20 ms; launches in that window take up to 40 percent longer")
    ap.add_argument("--rebuild-every-insert", action="store_true",
                    help="with --path insert: follow every insert by a full index rebuild (the comparison)")
    ap.add_argument("--rotate", type=int, default=0,
                    help="number of copies of the logits swept in turn (0: as many as make 512 MB, i.e. 1 for "
                         "the learner batch and 4 for the tiny one)")
    ap.add_argument("--batch-scale", type=int, default=1,
                    help="with --path retrace: multiply the number of trajectories (the kernels are "
                         "launch-bound at the configured size)")
    ap.add_argument("--mix-probe", action="store_true",
                    help="with --path retrace: also time a bare kernel that reads and writes as many fp32 arrays as "
                         "the scan does and nothing else (the ceiling for that mix of read and write streams)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch a plain 1 GiB copy kernel a few times (calibrates hardware counters)")
    args = ap.parse_args()
    args.one_pass = not args.two_calls
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2410_14803_amd import binding as b
    from paper_2410_14803_amd import synth

    from paper_2410_14803_amd import build as hip_build
    hip_build.ensure_built()   # compiles only a tree with nothing built
    b.lib()   # fails loudly if the HIP library is still missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.path == "retrace":
        return bench_retrace(args, b, torch, synth, dev)
    if args.path == "replay":
        return bench_replay(args, b, torch, synth, dev)
    if args.path == "insert":
        return bench_insert(args, b, torch, synth, dev)
    cfg = synth.CONFIGS[args.config]
    assert cfg.V > 0 and cfg.M > 0, "bench runs a workload with logits and a replay buffer"
    seed = synth.BASE_SEED + cfg.index
    off_np = synth.trajectory_offsets(cfg, seed)
    N = int(off_np[-1]); R = N * cfg.A; B = cfg.B; K = cfg.K; M = cfg.M
    off = torch.as_tensor(off_np, device=dev)
    logits = synth.logits_bf16(R, cfg.V, seed + 1, dev, heavy_tail=cfg.heavy_tail)
    tokens = synth.action_tokens(logits, seed + 2)
    # A batch that fits the 256 MB last-level cache is swept from several copies in turn (at least
    # 512 MB together), so that what is timed is HBM and not the cache; the learner batch is 5 GB.
    copies = args.rotate if args.rotate > 0 else max(1, -(-(512 << 20) // (R * cfg.V * 2)))
    logits_ring = [logits] + [logits.clone() for _ in range(copies - 1)]
    si = synth.step_inputs(cfg, off_np, seed + 4, dev)
    ws = b.Workspace(M, device=dev)
    f = lambda n: torch.empty(n, device=dev)
    tok_logp, tok_ent, step_logp, step_ent = f(R), f(R), f(N), f(N)
    target, td, rho, step_prio, traj_prio = f(N), f(N), f(N), f(N), f(B)
    idx = torch.empty(K, dtype=torch.int64, device=dev)
    prob = f(K)
    ent_scale = float(cfg.A * np.log(cfg.V))

    # input preparation (untimed): behaviour log-probs lag the policy's by seeded noise, and the
    # replay buffer starts from seeded priorities
    b.score_logits(logits, tokens, cfg.A, ws, tok_logp=tok_logp, tok_ent=tok_ent, step_logp=step_logp, step_ent=step_ent)
    logmu = (step_logp + si["mu_noise"]).contiguous()
    weights = torch.zeros(M, device=dev)
    p0 = synth.replay_priorities(M, cfg.replay, seed + 5, dev)
    b.update_priorities(weights, torch.arange(M, device=dev), p0, cfg.alpha, ws)
    total_iters = args.steps + args.warmup
    uni = synth.uniforms(K * total_iters, seed + 6, dev).view(total_iters, K)
    prio_src = (torch.arange(K, device=dev) % N)   # first K step priorities, wrapping if N < K
    torch.cuda.synchronize()

    if args.path == "actor_grad":
        return bench_actor_grad(args, b, torch, cfg, logits, tokens, tok_logp, tok_ent, step_logp, step_ent, si, N, R)

    def one_step(i, ev=None):
        b.score_logits(logits_ring[i % copies], tokens, cfg.A, ws, tok_logp=tok_logp, tok_ent=tok_ent,
                       step_logp=step_logp, step_ent=step_ent, sweep_events=ev)
        if args.one_pass:
            b.retrace_priorities(step_logp, logmu, si["reward"], si["value"], step_ent, off, cfg.gamma, cfg.lam,
                                 cfg.w, q=si["q"], td_scale=2.0, ent_scale=ent_scale, target=target, td=td, rho=rho,
                                 step_prio=step_prio, traj_prio=traj_prio)
        else:
            b.retrace_targets(step_logp, logmu, si["reward"], si["value"], off, cfg.gamma, cfg.lam, q=si["q"],
                              target=target, td=td, rho=rho)
            b.compute_priorities(td, rho, step_ent, off, cfg.w, td_scale=2.0, ent_scale=ent_scale,
                                 step_prio=step_prio, traj_prio=traj_prio)
        b.sample_prioritized(weights, uni[i], ws, idx, prob)
        b.update_priorities(weights, idx, step_prio[prio_src] if N < K else step_prio[:K], cfg.alpha, ws)

    # Pre-warm: the sweep alone, each launch timed like the timed steps below, so that the line can
    # show what the first window of a process costs beside the steady state (see --prewarm).
    n_pre = max(args.prewarm, args.launch_series)
    pre = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_pre)]
    for a, c in pre:
        a.record(); c.record()
    clock_probe, clocks = None, None
    if args.launch_series > 0:
        import ctypes
        lib_probe = ctypes.CDLL(os.path.join(ROOT, "paper_2410_14803_amd", "libaride_probe.so"))
        lib_probe.aride_probe_clock.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
        clocks = torch.zeros(n_pre, 2, dtype=torch.int64, device=dev)
        clock_probe = lambda i: lib_probe.aride_probe_clock(clocks[i].data_ptr(), 1000, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for i, ev in enumerate(pre):
        b.score_logits(logits_ring[i % copies], tokens, cfg.A, ws, tok_logp=tok_logp, tok_ent=tok_ent,
                       step_logp=step_logp, step_ent=step_ent, sweep_events=ev)
        if clock_probe is not None:
            assert clock_probe(i) == 0
    torch.cuda.synchronize()
    pre_ms = [a.elapsed_time(c) for a, c in pre]
    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()
    # One pair of HIP events per timed step, attached to the dispatch of the logit sweep itself
    # (aride_score_logits_timed): they read the kernel's own start and end, and put no marker
    # packets on the stream.  (Events recorded around the call cost a barrier packet each and
    # read ~30 us more than the kernel takes.)  Recording each once creates the HIP event.
    events = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for i in range(args.steps)}
    for a, c in events.values():
        a.record(); c.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(args.warmup + i, events.get(i))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    st, rc = ws.status()
    assert rc == b.OK and st.flags == 0, f"status flags {st.flags:#x} rc {rc}"

    if args.copy_probe:
        import ctypes
        probe = ctypes.CDLL(os.path.join(ROOT, "paper_2410_14803_amd", "libaride_probe.so"))
        probe.aride_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            rcp = probe.aride_probe_copy(dst.data_ptr(), src.data_ptr(), src.numel(),
                                         torch.cuda.current_stream().cuda_stream)
            assert rcp == 0
        torch.cuda.synchronize()
        assert torch.equal(src, dst)

    ms_per_step = elapsed / args.steps * 1e3
    value = N * args.steps / elapsed
    # dominant kernel: the logit sweep.  Algorithmic bytes per launch: every bf16 logit once,
    # one int32 token per row, two fp32 results per row.
    sweep_ms = sum(a.elapsed_time(c) for a, c in events.values()) / len(events)
    expected_rows = {0: 2560, 1: 82144, 2: 131072}.get(args.config)
    traffic = _traffic("scoring", args.config) if R == expected_rows else None
    alg_bytes = R * cfg.V * 2 + R * 4 + R * 8
    achieved = alg_bytes / (sweep_ms * 1e-3) / 1e9
    out = {
        "metric": METRIC, "value": value, "unit": "trajectory-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name} (config {cfg.index})", "trajectories": B, "traj_steps": N,
                   "action_tokens": cfg.A, "vocab": cfg.V, "logit_rows": R, "logit_bytes": R * cfg.V * 2,
                   "replay_entries": M, "draws": K, "gamma": cfg.gamma, "lambda": cfg.lam, "alpha": cfg.alpha,
                   "logit_copies_in_rotation": copies, "one_pass": bool(args.one_pass)},
        "roofline": {"bound": "hbm", "kernel": _sweep_kernel_name(cfg.V), "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "algorithmic_bytes_per_launch": alg_bytes, "ms_per_launch": sweep_ms,
                     "prewarm_launches": args.prewarm,
                     "ms_per_launch_first_window": (sum(pre_ms[:40]) / len(pre_ms[:40])) if pre_ms else None,
                     "ms_per_launch_slowest_of_first_window": max(pre_ms[:40]) if pre_ms else None},
    }

    if clocks is not None:
        ck = clocks.cpu().numpy()[:args.launch_series]
        out["launch_series"] = {"sweep_us": [round(x * 1e3, 1) for x in pre_ms[:args.launch_series]],
                                "shader_mhz_after_launch": [round(100.0 * c / max(w, 1)) for c, w in ck]}
    if not args.no_cpu_baseline:
        import oracle
        threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or min(os.cpu_count() or 1, 16)
        host = lambda t: t.detach().cpu().numpy()
        rows_probe = min(R, 2 * cfg.A)
        bits = lambda r: logits[:r].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        tp0 = time.perf_counter()
        oracle.score_logits(bits(rows_probe), host(tokens[:rows_probe]), cfg.A, nthreads=threads)
        per_row = (time.perf_counter() - tp0) / rows_probe
        # whole trajectories, as many as fit the time budget
        want_rows = max(cfg.A, int(args.cpu_seconds / max(per_row, 1e-9)))
        nb = int(np.searchsorted(off_np * cfg.A, want_rows, side="right")) - 1
        nb = max(1, min(B, nb))
        n_s = int(off_np[nb]); r_s = n_s * cfg.A
        lb, tk = bits(r_s), host(tokens[:r_s])
        lm, rw, vv, qq = host(logmu[:n_s]), host(si["reward"][:n_s]), host(si["value"][:n_s]), host(si["q"][:n_s])
        w_host, u_host = host(weights).copy(), host(uni[0])
        tc0 = time.perf_counter()
        o = oracle.score_logits(lb, tk, cfg.A, nthreads=threads)
        ort = oracle.retrace_targets(o["step_logp"], lm, rw, vv, off_np[:nb + 1], cfg.gamma, cfg.lam, q=qq)
        opr = oracle.compute_priorities(ort["td"], ort["rho"], o["step_ent"], off_np[:nb + 1], *cfg.w,
                                        td_scale=2.0, ent_scale=ent_scale)
        oi, _, _ = oracle.sample_prioritized(w_host, u_host)
        pk = opr["step_prio"][np.arange(K) % n_s].astype(np.float32)
        oracle.update_priorities(w_host, oi, pk, cfg.alpha)
        tc1 = time.perf_counter()
        out["cpu_baseline"] = {"value": n_s / (tc1 - tc0), "unit": "trajectory-steps/s", "cores": threads,
                               "kind": "oracle", "seconds": tc1 - tc0,
                               "sample": f"first {nb} trajectories of the batch ({n_s} steps, {r_s} logit rows), "
                                         f"whole path incl. one {K}-draw sample and update on the {M}-entry buffer"}
        # the same oracle on one thread, on a share of those rows that takes about as long (the logit
        # reduction is all but the whole cost)
        r1 = max(cfg.A, (r_s // threads) // cfg.A * cfg.A)
        ts0 = time.perf_counter()
        oracle.score_logits(lb[:r1], tk[:r1], cfg.A, nthreads=1)
        ts1 = time.perf_counter()
        out["cpu_baseline"]["single_thread"] = {"value": (r1 // cfg.A) / (ts1 - ts0), "unit": "trajectory-steps/s",
                                                "cores": 1, "seconds": ts1 - ts0,
                                                "sample": f"logit reduction of the first {r1} rows"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
