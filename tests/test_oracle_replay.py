"""Pins for the oracle's priorities (Section 5.3, Appendix A.4.3) and for the
prioritized replay sampler / update (Appendix A.4.2, P(i) = p_i^alpha / sum p^alpha)."""
import math
from fractions import Fraction

import numpy as np
import pytest


# ---------------------------------------------------------------- priorities

def _prio_inputs(rng, lens):
    N = sum(lens)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return off, rng.standard_normal(N), np.exp(rng.standard_normal(N)), rng.uniform(0, 5, N)


def test_priority_terms_isolated_and_linear(oracle):
    rng = np.random.default_rng(20)
    off, td, rho, ent = _prio_inputs(rng, [3, 1, 7, 4])
    a = oracle.compute_priorities(td, rho, ent, off, 1, 0, 0)
    b = oracle.compute_priorities(td, rho, ent, off, 0, 1, 0)
    c = oracle.compute_priorities(td, rho, ent, off, 0, 0, 1)
    np.testing.assert_allclose(a["step_prio"], np.abs(td), rtol=1e-15)
    np.testing.assert_allclose(b["step_prio"], np.minimum(1.0, rho), rtol=1e-15)
    assert b["step_prio"].min() >= 0 and b["step_prio"].max() <= 1   # ratio term lies in [0,1]
    np.testing.assert_allclose(c["step_prio"], ent, rtol=1e-15)
    w = (2.0, 0.5, 0.7)
    full = oracle.compute_priorities(td, rho, ent, off, *w, td_scale=4.0, ent_scale=2.5, eps=1e-3)
    want = w[0] * a["step_prio"] / 4.0 + w[1] * b["step_prio"] + w[2] * c["step_prio"] / 2.5 + 1e-3
    np.testing.assert_allclose(full["step_prio"], want, rtol=1e-14)
    raw = oracle.compute_priorities(td, rho, ent, off, 0, 1, 0, truncate_rho=False)
    np.testing.assert_allclose(raw["step_prio"], rho, rtol=1e-15)


def test_trajectory_priority_is_weighted_sum_of_means(oracle):
    # p(tau) = w1*mean|delta| + w2*mean rho + w3*mean H, as printed in Section 5.3
    rng = np.random.default_rng(21)
    lens = [5, 2, 11, 1]
    off, td, rho, ent = _prio_inputs(rng, lens)
    w = (1.0, 0.5, 0.1)
    out = oracle.compute_priorities(td, rho, ent, off, *w, truncate_rho=False)
    for b in range(len(lens)):
        s = slice(off[b], off[b + 1])
        want = w[0] * np.mean(np.abs(td[s])) + w[1] * np.mean(rho[s]) + w[2] * np.mean(ent[s])
        assert out["traj_prio"][b] == pytest.approx(want, rel=1e-13)
        assert out["traj_prio"][b] == pytest.approx(np.mean(out["step_prio"][s]), rel=1e-13)


def test_empty_trajectory_priority_is_zero(oracle):
    off = np.array([0, 0, 2], np.int32)
    out = oracle.compute_priorities([1.0, -2.0], [0.5, 3.0], [0.1, 0.2], off, 1, 1, 1)
    assert out["traj_prio"][0] == 0.0


# ---------------------------------------------------------------- update

def test_update_is_sequential_last_writer_wins(oracle):
    w = np.zeros(8, np.float32)
    idx = [3, 5, 3, 3, 7]
    prio = [1.0, 4.0, 9.0, 16.0, -2.0]
    bad = oracle.update_priorities(w, idx, prio, 0.5)
    assert bad == 0
    np.testing.assert_array_equal(w, np.array([0, 0, 0, 4, 0, 2, 0, 0], np.float32))
    assert oracle.update_priorities(w, [8, -1, 0], [1.0, 1.0, 1.0], 0.5) == 2
    assert w[0] == 1.0


def test_update_power_closed_forms(oracle):
    p = np.array([0.0, 1.0, 4.0, 2.25, 1e-6, 123.456], np.float32)
    for alpha in (0.0, 0.5, 0.6, 1.0):
        w = np.full(len(p), 7.0, np.float32)
        oracle.update_priorities(w, np.arange(len(p)), p, alpha)
        if alpha == 0.0:
            want = np.ones(len(p))          # alpha = 0 is uniform sampling (0^0 = 1 in IEEE pow)
        elif alpha == 0.5:
            want = np.sqrt(p.astype(np.float64))
        elif alpha == 1.0:
            want = p.astype(np.float64)
        else:
            want = np.exp(np.float64(np.float32(alpha)) * np.log(np.maximum(p.astype(np.float64), 1e-300)))
            want[p == 0] = 0.0
        np.testing.assert_allclose(w, want.astype(np.float32), rtol=2e-7)
    w = np.zeros(2, np.float32)
    oracle.update_priorities(w, [0, 1], [np.nan, -3.0], 0.6)
    np.testing.assert_array_equal(w, [0.0, 0.0])   # no mass for NaN / negative priorities


def test_update_idempotent_without_duplicates(oracle):
    rng = np.random.default_rng(22)
    w1 = rng.random(64).astype(np.float32)
    w2 = w1.copy()
    idx = rng.permutation(64)[:20]
    prio = rng.random(20).astype(np.float32)
    oracle.update_priorities(w1, idx, prio, 0.6)
    oracle.update_priorities(w2, idx, prio, 0.6)
    oracle.update_priorities(w2, idx[::-1].copy(), prio[::-1].copy(), 0.6)
    np.testing.assert_array_equal(w1, w2)


# ---------------------------------------------------------------- sampler

def _brute_sample(weights, us):
    """The sampler's definition in exact rational arithmetic, by linear scan."""
    w = [Fraction(float(x)) if (np.isfinite(x) and x > 0) else Fraction(0) for x in weights]
    wmax = max(w)
    e = math.frexp(float(wmax))[1]            # wmax = m * 2^e with 0.5 <= m < 1, i.e. ilogb + 1
    q = [int(x * Fraction(2) ** (39 - e)) for x in w]   # floor for non-negative rationals
    total = sum(q)
    out = []
    for u in us:
        t = min(int(Fraction(float(u) * float(total))), total - 1)
        c = 0
        for i, qi in enumerate(q):
            c += qi
            if c > t:
                out.append(i)
                break
    return out, q, total


def test_quantisation_matches_rational_definition(oracle):
    rng = np.random.default_rng(23)
    w = np.exp(rng.standard_normal(50) * 4).astype(np.float32)
    w[[3, 9]] = 0.0
    w[11] = np.float32(1e-30)     # far below wmax * 2^-39: quantises to zero
    q, total = oracle.quantise_weights(w)
    _, qb, tb = _brute_sample(w, [])
    assert [int(x) for x in q] == qb and total == tb
    assert max(qb) < 2 ** 39 and max(qb) >= 2 ** 38
    assert q[11] == 0
    # scaling every weight by a power of two leaves the integers unchanged
    q2, total2 = oracle.quantise_weights(w * np.float32(2.0 ** -20))
    assert total2 == total and np.array_equal(q, q2)


def test_exhaustive_enumeration_dyadic(oracle):
    # weights k/16 with sum 4 and wmax 1: q = w * 2^38, Total = 2^40 exactly; u = j / 2^10 hits entry i exactly
    # q_i * 2^10 / Total times
    w = np.array([1, 3, 0, 8, 4, 16, 0, 2, 6, 8, 16], np.float32) / 16.0   # sum = 64/16 = 4
    m = 10
    us = np.arange(2 ** m) / 2.0 ** m
    idx, prob, rc = oracle.sample_prioritized(w, us)
    assert rc == 0
    q, total = oracle.quantise_weights(w)
    assert total == 2 ** 40
    counts = np.bincount(idx, minlength=len(w))
    np.testing.assert_array_equal(counts, (w * 16 * 2 ** m / 64).astype(np.int64))
    np.testing.assert_allclose(prob, (w / 4.0)[idx], rtol=1e-15)
    assert np.all(np.diff(idx) >= 0)                 # non-decreasing in u
    assert not np.isin(idx, [2, 6]).any()            # zero-weight entries are never drawn


def test_against_brute_force_linear_scan(oracle):
    rng = np.random.default_rng(24)
    for M in (1, 2, 5, 16, 33):
        w = np.exp(rng.standard_normal(M) * 2).astype(np.float32)
        if M > 3:
            w[rng.integers(0, M, 2)] = 0.0
        w[0] = max(w[0], np.float32(0.1))
        us = np.concatenate([rng.random(300), [0.0, np.nextafter(1.0, 0.0), 0.5]])
        idx, prob, rc = oracle.sample_prioritized(w, us)
        want, q, total = _brute_sample(w, us)
        assert rc == 0 and list(idx) == want
        np.testing.assert_allclose(prob, [q[i] / total for i in want], rtol=1e-15)


def test_every_integer_threshold_small_total(oracle):
    # tiny integer weights: walk every u that lands on each integer t in [0, Total) after scaling
    w = np.array([3, 0, 1, 4, 0, 2], np.float32)
    q, total = oracle.quantise_weights(w)
    scale = total // 10                      # q_i = w_i * scale, scale a power of two
    assert [int(x) for x in q] == [int(x) * scale for x in w]
    cum = np.cumsum(w).astype(int)
    for t_small in range(10):
        for frac in (0.0, 0.5):
            u = (t_small + frac) / 10.0
            idx, _, _ = oracle.sample_prioritized(w, [u])
            t = min(int(math.floor(u * total)), total - 1)
            want = int(np.searchsorted(cum * scale, t, side="right"))
            assert idx[0] == want


def test_equal_weights_power_of_two(oracle):
    M = 64
    w = np.full(M, 0.37, np.float32)
    rng = np.random.default_rng(25)
    us = rng.random(500)
    idx, prob, _ = oracle.sample_prioritized(w, us)
    np.testing.assert_array_equal(idx, np.floor(us * M).astype(np.int64))
    np.testing.assert_allclose(prob, 1.0 / M, rtol=1e-15)


def test_alpha_zero_uniform_alpha_one_proportional(oracle):
    # alpha = 0 -> uniform, alpha = 1 -> proportional to p  (Appendix A.4.2)
    p = np.array([1.0, 2.0, 4.0, 8.0, 1.0], np.float32)
    us = (np.arange(1600) + 0.5) / 1600.0
    w = np.zeros(5, np.float32)
    oracle.update_priorities(w, np.arange(5), p, 0.0)
    idx, _, _ = oracle.sample_prioritized(w, us)
    np.testing.assert_array_equal(np.bincount(idx, minlength=5), [320] * 5)
    oracle.update_priorities(w, np.arange(5), p, 1.0)
    idx, _, _ = oracle.sample_prioritized(w, us)
    np.testing.assert_array_equal(np.bincount(idx, minlength=5), [100, 200, 400, 800, 100])


def test_degenerate_inputs(oracle):
    idx, prob, rc = oracle.sample_prioritized(np.zeros(7, np.float32), [0.1, 0.9])
    assert rc == -5 and list(idx) == [-1, -1] and list(prob) == [0.0, 0.0]
    w = np.array([np.nan, -1.0, np.inf, 2.0, 0.0], np.float32)
    idx, prob, rc = oracle.sample_prioritized(w, [0.0, 0.5, 0.999, -0.3, np.nan, 1.0, 7.0])
    assert rc == 0 and list(idx) == [3] * 7       # only the finite positive entry carries mass
    np.testing.assert_allclose(prob, 1.0)


def test_chi_square_sanity(oracle):
    rng = np.random.default_rng(26)
    w = np.exp(rng.standard_normal(40)).astype(np.float32)
    n = 200000
    idx, _, _ = oracle.sample_prioritized(w, rng.random(n))
    q, total = oracle.quantise_weights(w)
    expected = q.astype(np.float64) / total * n
    chi2 = np.sum((np.bincount(idx, minlength=40) - expected) ** 2 / expected)
    assert chi2 < 39 + 6 * math.sqrt(2 * 39)     # mean dof, +6 sigma


# ---------------------------------------------------------------- circular insert (Appendix A.4.2)

def test_circular_insert_wraps_and_overwrites_oldest(oracle):
    M = 5
    w = np.zeros(M, np.float32)
    cur, slots = oracle.replay_insert(w, 0, [1.0, 4.0, 9.0], 0.5)
    assert cur == 3 and list(slots) == [0, 1, 2]
    np.testing.assert_array_equal(w, [1, 2, 3, 0, 0])
    cur, slots = oracle.replay_insert(w, cur, [16.0, 25.0, 36.0, 49.0], 0.5)     # wraps past the end
    assert cur == 2 and list(slots) == [3, 4, 0, 1]
    np.testing.assert_array_equal(w, [6, 7, 3, 4, 5])                            # the two oldest were overwritten


def test_circular_insert_batch_equals_one_by_one(oracle):
    rng = np.random.default_rng(30)
    M = 17
    p = rng.random(60).astype(np.float32) * 4
    wa = np.zeros(M, np.float32); wb = np.zeros(M, np.float32)
    cur_a, slots = oracle.replay_insert(wa, 11, p, 0.6)
    cur_b = 11
    for x in p:                                  # the paper's rule, i <- (i + 1) mod N, one entry at a time
        wb[cur_b] = np.float32(float(x) ** np.float64(np.float32(0.6)))
        cur_b = (cur_b + 1) % M
    assert cur_a == cur_b == (11 + 60) % M
    np.testing.assert_allclose(wa, wb, rtol=1e-7)
    # more entries than capacity: only the last M survive, the earlier ones report slot -1
    assert np.all(slots[:60 - M] == -1) and sorted(slots[60 - M:]) == list(range(M))
    np.testing.assert_array_equal(slots[60 - M:], (11 + np.arange(60 - M, 60)) % M)


def test_circular_insert_empty_batch(oracle):
    w = np.ones(4, np.float32)
    cur, slots = oracle.replay_insert(w, 3, [], 0.6)
    assert cur == 3 and len(slots) == 0 and np.all(w == 1)
