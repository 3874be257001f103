"""Pins for the oracle's V-trace targets (the alternative the paper contrasts Retrace with,
Section 2 / Appendix A.4.1) and Monte-Carlo returns with labels (Section 5.1)."""
import math

import numpy as np
import pytest


def _traj(rng, T):
    lp = -2 * np.abs(rng.standard_normal(T))
    lm = lp + 0.6 * rng.standard_normal(T)
    r = (rng.random(T) < 0.3).astype(float)
    return lp, lm, r, rng.uniform(-1, 1, T), rng.uniform(-1, 1, T)


def brute_vtrace(lp, lm, r, v, q, boot, gamma, lam, rho_bar, c_bar):
    """The published V-trace sum, term by term, for one trajectory."""
    T = len(r)
    rho = [math.exp(lp[i] - lm[i]) for i in range(T)]
    out = []
    for s in range(T):
        acc = 0.0
        for t in range(s, T):
            prod = 1.0
            for i in range(s, t):
                prod *= lam * min(c_bar, rho[i])
            v_next = v[t + 1] if t + 1 < T else boot
            acc += gamma ** (t - s) * prod * min(rho_bar, rho[t]) * (r[t] + gamma * v_next - q[t])
        out.append(q[s] + acc)
    return out


@pytest.mark.parametrize("rho_bar,c_bar,lam", [(1.0, 1.0, 1.0), (2.0, 0.7, 0.9), (1e9, 1e9, 1.0)])
def test_vtrace_brute_force(oracle, rho_bar, c_bar, lam):
    rng = np.random.default_rng(40)
    lens = [1, 2, 5, 9]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    parts = [_traj(rng, T) for T in lens]
    lp, lm, r, v, q = (np.concatenate([p[i] for p in parts]) for i in range(5))
    boot = rng.uniform(-1, 1, len(lens))
    out = oracle.vtrace_targets(lp, lm, r, v, off, 0.95, lam, rho_bar, c_bar, q=q, boot=boot)
    for b, T in enumerate(lens):
        s = slice(off[b], off[b + 1])
        want = brute_vtrace(lp[s], lm[s], r[s], v[s], q[s], boot[b], 0.95, lam, rho_bar, c_bar)
        np.testing.assert_allclose(out["target"][s], want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["rho"], np.exp(lp - lm), rtol=1e-14)


def test_vtrace_on_policy_is_the_n_step_return(oracle):
    # pi == mu, clips >= 1, lambda = 1: v_s = sum gamma^k r + gamma^n boot (the on-policy n-step target)
    rng = np.random.default_rng(41)
    T = 30
    lp, _, r, v, _ = _traj(rng, T)
    out = oracle.vtrace_targets(lp, lp.copy(), r, v, np.array([0, T], np.int32), 0.97, 1.0, 1.0, 1.0,
                                boot=np.array([0.4]))
    want = [sum(0.97 ** (k - t) * r[k] for k in range(t, T)) + 0.97 ** (T - t) * 0.4 for t in range(T)]
    np.testing.assert_allclose(out["target"], want, rtol=1e-12, atol=1e-12)


def test_vtrace_differs_from_retrace_exactly_by_the_own_step_ratio(oracle):
    # with every ratio < 1 (no clipping): V-trace Delta_t = rho_t*delta_t + gamma*lam*rho_t*Delta_{t+1},
    # Retrace Delta_t = delta_t + gamma*lam*rho_{t+1}*Delta_{t+1}  =>  vtrace_Delta_t = rho_t * retrace_Delta_t
    rng = np.random.default_rng(42)
    T = 12
    lp, _, r, v, q = _traj(rng, T)
    lm = lp + rng.uniform(0.1, 1.0, T)          # rho < 1 everywhere
    off = np.array([0, T], np.int32)
    a = oracle.vtrace_targets(lp, lm, r, v, off, 0.9, 0.95, 1.0, 1.0, q=q)
    b = oracle.retrace_targets(lp, lm, r, v, off, 0.9, 0.95, q=q)
    np.testing.assert_allclose(a["target"] - q, b["rho"] * (b["target"] - q), rtol=1e-12, atol=1e-14)


def test_mc_returns_brute_force_and_labels(oracle):
    rng = np.random.default_rng(43)
    lens = [1, 4, 0, 25]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    r = rng.standard_normal(sum(lens)) * (rng.random(sum(lens)) < 0.4)
    ret, label = oracle.mc_returns(r, off, 0.93)
    for b, T in enumerate(lens):
        for t in range(T):
            want = sum(0.93 ** (k - t) * r[off[b] + k] for k in range(t, T))
            assert ret[off[b] + t] == pytest.approx(want, rel=1e-12, abs=1e-14)
    np.testing.assert_array_equal(label, (ret > 0).astype(float))


def test_mc_return_of_a_single_terminal_reward(oracle):
    T = 20
    r = np.zeros(T); r[-1] = 1.0
    ret, label = oracle.mc_returns(r, np.array([0, T], np.int32), 0.9)
    np.testing.assert_allclose(ret, 0.9 ** (T - 1 - np.arange(T)), rtol=1e-13)
    assert np.all(label == 1.0)
    ret0, label0 = oracle.mc_returns(np.zeros(T), np.array([0, T], np.int32), 0.9)
    assert np.all(ret0 == 0) and np.all(label0 == 0)
