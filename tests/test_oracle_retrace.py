"""Pins for the oracle's Retrace(lambda) targets (Section 5.2) and TD errors (Section 5.3).

The oracle runs a backward recursion; these tests pin it to the paper's double
sum/product written out term by term, and to the textbook special cases it must
reduce to.
"""
import math

import numpy as np
import pytest


def brute_force_delta(logp_pi, logp_mu, r, v, q, boot, gamma, lam):
    """Section 5.2 as printed: Delta_t = sum_{k=t}^{T-1} gamma^(k-t) (prod_{i=t+1}^{k} c_i) delta_k
    with c_i = lam * min(1, pi_i/mu_i), for one trajectory, in pure Python."""
    T = len(r)
    delta = []
    for k in range(T):
        v_next = v[k + 1] if k + 1 < T else boot
        delta.append(r[k] + gamma * v_next - q[k])
    out = []
    for t in range(T):
        acc = 0.0
        for k in range(t, T):
            prod = 1.0
            for i in range(t + 1, k + 1):
                prod *= lam * min(1.0, math.exp(logp_pi[i] - logp_mu[i]))
            acc += gamma ** (k - t) * prod * delta[k]
        out.append(acc)
    return out, delta


def _rand_traj(rng, T):
    lp = -3 * np.abs(rng.standard_normal(T))
    lm = lp + 0.5 * rng.standard_normal(T)
    r = (rng.random(T) < 0.3).astype(float)
    v = rng.uniform(-1, 1, T)
    q = rng.uniform(-1, 1, T)
    return lp, lm, r, v, q


@pytest.mark.parametrize("with_q", [False, True])
def test_brute_force_expansion(oracle, with_q):
    rng = np.random.default_rng(10)
    lens = [1, 2, 3, 5, 8, 8, 1, 7]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    parts = [_rand_traj(rng, T) for T in lens]
    lp, lm, r, v, q = (np.concatenate([p[i] for p in parts]) for i in range(5))
    boot = rng.uniform(-1, 1, len(lens))
    gamma, lam = 0.9, 0.95
    out = oracle.retrace_targets(lp, lm, r, v, off, gamma, lam, q=q if with_q else None, boot=boot)
    for b, T in enumerate(lens):
        s = slice(off[b], off[b + 1])
        qq = q[s] if with_q else v[s]
        Delta, delta = brute_force_delta(lp[s], lm[s], r[s], v[s], qq, boot[b], gamma, lam)
        np.testing.assert_allclose(out["target"][s], qq + np.array(Delta), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(out["td"][s], delta, rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(out["rho"][s], np.exp(lp[s] - lm[s]), rtol=1e-13)


def test_lambda_zero_is_one_step_td(oracle):
    rng = np.random.default_rng(11)
    T = 12
    lp, lm, r, v, _ = _rand_traj(rng, T)
    off = np.array([0, T], np.int32)
    out = oracle.retrace_targets(lp, lm, r, v, off, 0.9, 0.0, boot=np.array([0.25]))
    v_next = np.concatenate([v[1:], [0.25]])
    np.testing.assert_allclose(out["target"], r + 0.9 * v_next, rtol=1e-13, atol=1e-14)


def test_on_policy_is_td_lambda(oracle):
    # pi == mu  =>  c_i = lambda  =>  Delta_t = sum_k (gamma*lambda)^(k-t) delta_k  (the GAE sum)
    rng = np.random.default_rng(12)
    T = 15
    lp, _, r, v, _ = _rand_traj(rng, T)
    off = np.array([0, T], np.int32)
    gamma, lam = 0.97, 0.8
    out = oracle.retrace_targets(lp, lp.copy(), r, v, off, gamma, lam)
    v_next = np.concatenate([v[1:], [0.0]])
    delta = r + gamma * v_next - v
    want = [sum((gamma * lam) ** (k - t) * delta[k] for k in range(t, T)) for t in range(T)]
    np.testing.assert_allclose(out["target"] - v, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["rho"], 1.0, rtol=1e-15)


def test_on_policy_lambda_one_is_monte_carlo_return(oracle):
    # pi == mu and lambda == 1 telescope to G_t = sum_k gamma^(k-t) r_k + gamma^(T-t) boot
    rng = np.random.default_rng(13)
    T = 40
    lp, _, r, v, _ = _rand_traj(rng, T)
    off = np.array([0, T], np.int32)
    gamma, boot = 0.99, 0.7
    out = oracle.retrace_targets(lp, lp.copy(), r, v, off, gamma, 1.0, boot=np.array([boot]))
    want = [sum(gamma ** (k - t) * r[k] for k in range(t, T)) + gamma ** (T - t) * boot for t in range(T)]
    np.testing.assert_allclose(out["target"], want, rtol=1e-12, atol=1e-12)


def test_ratios_above_one_truncate(oracle):
    # every rho >= 1 behaves exactly like pi == mu (c_i = lambda)
    rng = np.random.default_rng(14)
    T = 9
    lp, _, r, v, q = _rand_traj(rng, T)
    off = np.array([0, T], np.int32)
    a = oracle.retrace_targets(lp, lp - rng.uniform(0, 2, T), r, v, off, 0.9, 0.95, q=q)
    b = oracle.retrace_targets(lp, lp.copy(), r, v, off, 0.9, 0.95, q=q)
    np.testing.assert_allclose(a["target"], b["target"], rtol=1e-14)
    assert np.all(a["rho"] >= 1.0)


def test_own_ratio_does_not_enter_own_correction(oracle):
    # the product starts at i = t+1: changing mu at step 0 changes rho_0 and nothing else;
    # changing mu at the last step changes targets of every earlier step but not its own
    rng = np.random.default_rng(15)
    T = 6
    lp, lm, r, v, _ = _rand_traj(rng, T)
    lm = lp + 1.0  # all ratios < 1, so the truncation is inactive
    off = np.array([0, T], np.int32)
    base = oracle.retrace_targets(lp, lm, r, v, off, 0.9, 0.95)
    lm0 = lm.copy(); lm0[0] += 0.7
    a = oracle.retrace_targets(lp, lm0, r, v, off, 0.9, 0.95)
    np.testing.assert_array_equal(a["target"], base["target"])
    assert a["rho"][0] != base["rho"][0]
    lml = lm.copy(); lml[-1] += 0.7
    b = oracle.retrace_targets(lp, lml, r, v, off, 0.9, 0.95)
    assert b["target"][-1] == base["target"][-1]
    assert np.all(b["target"][:-1] != base["target"][:-1])


def test_length_one_and_empty(oracle):
    off = np.array([0, 1, 1, 2], np.int32)   # middle trajectory is empty
    lp = np.array([-1.0, -2.0]); lm = np.array([-1.5, -1.0])
    r = np.array([1.0, 0.0]); v = np.array([0.3, 0.6])
    boot = np.array([0.5, 9.0, -0.25])
    out = oracle.retrace_targets(lp, lm, r, v, off, 0.9, 0.95, boot=boot)
    np.testing.assert_allclose(out["target"], [1.0 + 0.9 * 0.5, 0.0 + 0.9 * -0.25], rtol=1e-15)
    e = oracle.retrace_targets(np.zeros(0), np.zeros(0), np.zeros(0), np.zeros(0),
                               np.array([0], np.int32), 0.9, 0.9)
    assert e["target"].shape == (0,)


def test_segment_isolation(oracle):
    # a trajectory's outputs do not depend on its neighbours or on its position in the batch
    rng = np.random.default_rng(16)
    lens = [4, 9, 1, 6]
    parts = [_rand_traj(rng, T) for T in lens]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cat = [np.concatenate([p[i] for p in parts]) for i in range(5)]
    full = oracle.retrace_targets(cat[0], cat[1], cat[2], cat[3], off, 0.9, 0.95, q=cat[4])
    for b, T in enumerate(lens):
        p = parts[b]
        solo = oracle.retrace_targets(p[0], p[1], p[2], p[3], np.array([0, T], np.int32), 0.9, 0.95, q=p[4])
        for k in ("target", "td", "rho"):
            np.testing.assert_array_equal(full[k][off[b]:off[b + 1]], solo[k])
    order = [2, 0, 3, 1]
    offp = np.concatenate([[0], np.cumsum([lens[i] for i in order])]).astype(np.int32)
    catp = [np.concatenate([parts[i][j] for i in order]) for j in range(5)]
    perm = oracle.retrace_targets(catp[0], catp[1], catp[2], catp[3], offp, 0.9, 0.95, q=catp[4])
    for pos, i in enumerate(order):
        np.testing.assert_array_equal(perm["target"][offp[pos]:offp[pos + 1]], full["target"][off[i]:off[i + 1]])
