"""GPU parity: aride_replay_insert on large buffers, where the sampling index is patched (only
the blocks the insert touched are summed again) instead of rebuilt, against the CPU oracle.

The oracle knows nothing of patching: after every insert it quantises the whole buffer, sums
it and searches its prefix.  Whatever route the library takes, indices and the integer total
must be identical, so each case below is chosen for the route it forces: same exponent (patch),
a larger or smaller exponent of the maximum, no mass left, an index that was never built
(rebuild after all), batches that wrap around the end of the buffer.
"""
import numpy as np
import pytest
import torch

from paper_2410_14803_amd import binding as b
from paper_2410_14803_amd import synth
from _util import npf

pytestmark = pytest.mark.gpu
DEV = "cuda"
M_BIG = 64 * 65536 + 3 * 256 + 9        # 65 super-blocks, last block of 9 weights


def check(oracle, w, ws, seed, tag, n=1200):
    u = synth.uniforms(n, seed, DEV)
    u[:3] = torch.tensor([0.0, np.nextafter(1.0, 0.0), 0.5], dtype=torch.float64)
    idx = torch.full((n,), -7, dtype=torch.int64, device=DEV)
    prob = torch.full((n,), -7.0, device=DEV)
    b.sample_prioritized(w, u, ws, idx, prob)
    torch.cuda.synchronize()
    wh = npf(w)
    oi, op, rc = oracle.sample_prioritized(wh, npf(u))
    np.testing.assert_array_equal(npf(idx), oi, err_msg=f"{tag}: indices differ")
    np.testing.assert_allclose(npf(prob), op.astype(np.float32), rtol=1e-6, atol=0, err_msg=f"{tag}: prob")
    st, _ = ws.status()
    q, total = oracle.quantise_weights(wh)
    assert st.total == total, f"{tag}: total"
    assert np.float32(st.wmax) == wh[np.isfinite(wh) & (wh >= 0)].max(), f"{tag}: maximum"
    return st


def start(oracle, M, seed, scale=1.0):
    p = npf(synth.replay_priorities(M, "lognormal", seed, "cpu")) * np.float32(scale)
    w_host = np.zeros(M, np.float32)
    oracle.update_priorities(w_host, np.arange(M), p, 0.6)
    w = torch.as_tensor(w_host, device=DEV)
    ws = b.Workspace(M)
    b.update_priorities(w, None, None, 0.6, ws)
    return w, ws


def insert(oracle, w, ws, cursor, prio_host, alpha=0.6, slots=True):
    K = len(prio_host)
    prio = torch.as_tensor(np.asarray(prio_host, np.float32), device=DEV)
    so = torch.full((K,), -7, dtype=torch.int64, device=DEV) if slots else None
    wo = npf(w).copy()
    nc = b.replay_insert(w, cursor, prio, alpha, ws, slots_out=so)
    torch.cuda.synchronize()
    oc, o_slots = oracle.replay_insert(wo, cursor, npf(prio), alpha)
    assert nc == oc
    if slots:
        np.testing.assert_array_equal(npf(so), o_slots)
    np.testing.assert_allclose(npf(w), wo, rtol=1e-6)
    return nc


@pytest.mark.parametrize("K,cursor", [
    (1, 0), (1, M_BIG - 1), (255, 1), (256, 256 * 7), (257, 65536 * 3 - 100), (5000, M_BIG - 2500),
    (70000, 65536 * 64 - 10), (M_BIG // 8, 12345), (M_BIG // 8, M_BIG - 1000),
])
def test_patch_same_exponent(oracle, K, cursor):
    print(f"case K={K} cursor={cursor}", flush=True)
    w, ws = start(oracle, M_BIG, 11)
    rng = np.random.default_rng(K + cursor)
    wmax = float(npf(w).max())
    # priorities whose weights stay below half the current maximum: the exponent cannot move
    prio = (rng.random(K) * (0.5 * wmax) ** (1 / 0.6) * 0.9).astype(np.float32)
    prio[rng.random(K) < 0.2] = 0.0
    insert(oracle, w, ws, cursor, prio)
    check(oracle, w, ws, 1000 + K, f"K={K} cursor={cursor}")


def test_patch_leaves_untouched_blocks_alone(oracle):
    # White box: a weight changed behind the library's back in a block the insert does not touch
    # must NOT show up in the total -- that is what tells a patch from a rebuild.
    w, ws = start(oracle, M_BIG, 12)
    before = npf(w).copy()
    j = 65536 * 40 + 77
    w[j] = w[j] * 0.5 + 0.01
    prio = np.full(3000, 0.01, np.float32)
    b.replay_insert(w, 5, torch.as_tensor(prio, device=DEV), 0.6, ws)
    torch.cuda.synchronize()
    st, _ = ws.status()
    seen = npf(w).copy()
    seen[j] = before[j]
    _, total_stale = oracle.quantise_weights(seen)
    _, total_true = oracle.quantise_weights(npf(w))
    assert total_stale != total_true and st.total == total_stale
    b.update_priorities(w, None, None, 0.6, ws)          # a rebuild brings it in
    check(oracle, w, ws, 77, "after rebuild")


def test_a_sequence_of_inserts_with_moving_maximum(oracle):
    M = M_BIG
    w, ws = start(oracle, M, 13)
    rng = np.random.default_rng(5)
    cursor = M - 3000
    wmax = float(npf(w).max())
    steps = [
        ("small", 4000, 0.01),                       # patch
        ("new maximum, same exponent", 300, None),   # patch, wmax_bits moves
        ("exponent up", 700, 1e4),                   # rebuild after all
        ("small again", 66000, 0.02),                # patch under the new exponent
        ("exponent up again", 1, 1e7),
        ("nothing special", 2000, 0.5),
    ]
    for it, (name, K, level) in enumerate(steps):
        print(f"step {it}: {name}", flush=True)
        if level is None:
            e = np.floor(np.log2(wmax)) + 1
            target = 2.0 ** e * (1 - 2.0 ** -10)                   # just below the next power of two
            assert target > wmax
            prio = np.full(K, 1e-3, np.float32)
            prio[K // 2] = np.float32(target ** (1 / 0.6) * (1 - 1e-5))
        else:
            prio = (rng.random(K) * level).astype(np.float32)
            prio[0] = level
        e_before = ws.status()[0].exponent
        cursor = insert(oracle, w, ws, cursor, prio)
        st = check(oracle, w, ws, 200 + it, name)
        assert (st.exponent > e_before) == name.startswith("exponent up"), name
        wmax = float(npf(w).max())


def test_exponent_goes_down_when_the_maximum_is_overwritten(oracle):
    w, ws = start(oracle, M_BIG, 14, scale=1e-3)
    # one dominant entry, then a short insert right over it
    cursor = 65536 * 10 + 250
    insert(oracle, w, ws, cursor + 3, [1e6])
    check(oracle, w, ws, 31, "dominant entry in")
    assert int(np.argmax(npf(w))) == cursor + 3
    insert(oracle, w, ws, cursor, np.full(8, 1e-4, np.float32))
    st = check(oracle, w, ws, 32, "dominant entry overwritten")
    assert st.exponent < 10


def test_first_insert_on_a_workspace_without_an_index(oracle):
    M = M_BIG
    w_host = np.zeros(M, np.float32)
    w = torch.as_tensor(w_host, device=DEV)
    ws = b.Workspace(M)                                   # initialised, never built
    rng = np.random.default_rng(9)
    cursor = insert(oracle, w, ws, M - 10, rng.random(500).astype(np.float32))
    check(oracle, w, ws, 41, "first insert")
    cursor = insert(oracle, w, ws, cursor, (rng.random(9000) * 0.3).astype(np.float32))
    check(oracle, w, ws, 42, "second insert")
    assert cursor == (M - 10 + 9500) % M


def test_mass_removed_and_restored(oracle):
    M = M_BIG
    w = torch.zeros(M, device=DEV)
    ws = b.Workspace(M)
    insert(oracle, w, ws, 100, np.linspace(0.1, 2.0, 3000, dtype=np.float32))
    check(oracle, w, ws, 51, "some mass")
    insert(oracle, w, ws, 0, np.zeros(4000, np.float32))          # wipes it all
    st, rc = ws.status()
    assert rc == b.E_ZERO_MASS and st.total == 0 and (st.flags & b.ST_ZERO_MASS)
    idx = torch.full((50,), -7, dtype=torch.int64, device=DEV)
    b.sample_prioritized(w, synth.uniforms(50, 52, DEV), ws, idx, None)
    torch.cuda.synchronize()
    assert (npf(idx) == -1).all()
    insert(oracle, w, ws, M - 5, np.full(12, 0.7, np.float32))    # wraps, brings mass back
    st, rc = ws.status()
    assert rc == b.OK
    check(oracle, w, ws, 53, "mass back")


def test_patch_interleaved_with_updates_and_an_infinite_priority(oracle):
    w, ws = start(oracle, M_BIG, 15)
    rng = np.random.default_rng(21)
    cursor = 999_000
    for it in range(4):
        cursor = insert(oracle, w, ws, cursor, (rng.random(30_000) * 0.2).astype(np.float32), slots=False)
        check(oracle, w, ws, 60 + it, f"insert {it}", n=400)
        idx = torch.as_tensor(rng.integers(0, M_BIG, 5000), device=DEV)
        prio = torch.as_tensor(rng.random(5000).astype(np.float32), device=DEV)
        wo = npf(w).copy()
        b.update_priorities(w, idx, prio, 0.6, ws)
        torch.cuda.synchronize()
        oracle.update_priorities(wo, npf(idx), npf(prio), 0.6)
        np.testing.assert_allclose(npf(w), wo, rtol=1e-6)
        check(oracle, w, ws, 70 + it, f"update {it}", n=400)
    st, _ = ws.status()
    assert not (st.flags & b.ST_BAD_WEIGHT)
    prio = np.full(600, 0.05, np.float32)
    prio[17] = np.inf                                              # weight +inf: no mass, flagged
    b.replay_insert(w, cursor, torch.as_tensor(prio, device=DEV), 0.6, ws)
    torch.cuda.synchronize()
    st, _ = ws.status()
    assert st.flags & b.ST_BAD_WEIGHT
    u = synth.uniforms(300, 80, DEV)
    idx = torch.empty(300, dtype=torch.int64, device=DEV)
    b.sample_prioritized(w, u, ws, idx, None)
    torch.cuda.synchronize()
    oi, _, _ = oracle.sample_prioritized(npf(w), npf(u))
    np.testing.assert_array_equal(npf(idx), oi)


def test_patch_at_maximum_capacity(oracle):
    # M = ARIDE_MAX_REPLAY: 256 super-blocks, 4096 chunks, every fixed-size array of the workspace full
    M = b.MAX_REPLAY
    w, ws = start(oracle, M, 16)
    rng = np.random.default_rng(3)
    cursor = M - 40_000
    for it, K in enumerate((65_536, 1, M // 8)):
        prio = (rng.random(K) * 0.5).astype(np.float32)
        cursor = insert(oracle, w, ws, cursor, prio, slots=(K < 100_000))
        check(oracle, w, ws, 90 + it, f"max capacity K={K}", n=800)
    assert cursor == (M - 40_000 + 65_536 + 1 + M // 8) % M


@pytest.mark.parametrize("top", [3.0e38, 1.0, 2.0 ** -126, 1.0e-41, 1.4e-45])
def test_large_buffer_extreme_magnitudes(oracle, top):
    # weights written directly (then a rebuild with K = 0): the largest finite values, the smallest
    # normal, subnormals down to the last one -- the exponent of the maximum runs over its whole range
    M = M_BIG
    rng = np.random.default_rng(int(-np.log2(top)) + 200)
    w_host = (rng.random(M) * top).astype(np.float32)
    w_host[rng.random(M) < 0.5] = 0.0
    w_host[12345] = np.float32(top)
    w = torch.as_tensor(w_host, device=DEV)
    ws = b.Workspace(M)
    b.update_priorities(w, None, None, 1.0, ws)
    b.update_priorities(w, None, None, 1.0, ws)     # again: now the standing exponent is the right guess
    st = check(oracle, w, ws, 300, f"top={top}")
    assert st.exponent == int(np.floor(np.log2(float(np.float32(top))))) + 1
    # a patched insert of entries of the same magnitude (alpha = 1 stores the priorities as they are)
    prio = (rng.random(5000) * top * 0.5).astype(np.float32)
    insert(oracle, w, ws, M - 2000, prio, alpha=1.0)
    check(oracle, w, ws, 301, f"top={top} after insert")


def test_largest_insert_batch():
    # K = 2^31 - 256 entries, the most one call accepts, into a buffer of 2^20: what inserting them one
    # by one would leave are the last M of them; every earlier entry reports slot -1
    M = 1 << 20
    K = (1 << 31) - 256
    torch.cuda.empty_cache()
    if torch.cuda.mem_get_info()[0] < (40 << 30):
        pytest.skip("needs 26 GB of free device memory")
    print(f"case insert K={K} M={M}", flush=True)
    w = torch.zeros(M, device=DEV)
    ws = b.Workspace(M)
    prio = (torch.arange(K, device=DEV, dtype=torch.int32) % 7 + 1).float()      # 1 .. 7, period 7
    slots = torch.full((K,), -7, dtype=torch.int64, device=DEV)
    cursor = b.replay_insert(w, 12345, prio, 1.0, ws, slots_out=slots)           # alpha = 1 stores the priorities as they are
    torch.cuda.synchronize()
    assert cursor == (12345 + K) % M
    assert bool((slots[: K - M] == -1).all())
    k_last = torch.arange(K - M, K, device=DEV, dtype=torch.int64)
    assert bool((slots[K - M:] == (12345 + k_last) % M).all())
    want = torch.empty(M, device=DEV)
    want[(12345 + k_last) % M] = prio[K - M:]
    assert torch.equal(w, want)
    st, rc = ws.status()
    assert rc == b.OK and st.flags == 0
