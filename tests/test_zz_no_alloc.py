"""GPU check of aride_sample_prioritized_static, the draw for callers that cannot allocate: its
indices and probabilities against aride_update_priorities (K = 0) + aride_sample_prioritized with
a caller-owned workspace (bit for bit), and against the CPU oracle, on two calls in a row that
share the library's static array -- the second on a smaller buffer that takes another route."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2410_14803_amd import binding as b
from paper_2410_14803_amd import synth
from _util import npf

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _status(buf):
    return b.Status.from_buffer_copy(bytes(npf(buf)[:ctypes.sizeof(b.Status)]))


def _one_call(oracle, M, K, seed, bad=False):
    print(f"static draw M={M} K={K}", flush=True)
    p = npf(synth.replay_priorities(M, "lognormal", seed, "cpu"))
    w_host = np.zeros(M, np.float32)
    oracle.update_priorities(w_host, np.arange(M), p, 0.6)
    w = torch.as_tensor(w_host, device=DEV)
    w[torch.arange(0, M, 11, device=DEV)] = 0.0
    if bad:
        w[1] = float("nan")
    u = synth.uniforms(K, seed + 1, DEV)
    u[0] = 0.0
    u[K - 1] = float(np.nextafter(1.0, 0.0))
    idx = torch.full((K,), -7, dtype=torch.int64, device=DEV)
    prob = torch.full((K,), -7.0, device=DEV)
    stat = torch.zeros(24, dtype=torch.uint8, device=DEV)
    before = torch.cuda.memory_allocated()
    b.sample_prioritized_static(w, u, idx, prob, stat)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    # the existing entry points with a workspace of the caller's
    ws = b.Workspace(M)
    b.update_priorities(w, None, None, 0.6, ws)
    idx2 = torch.full((K,), -7, dtype=torch.int64, device=DEV)
    prob2 = torch.full((K,), -7.0, device=DEV)
    b.sample_prioritized(w, u, ws, idx2, prob2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(npf(idx), npf(idx2))
    np.testing.assert_array_equal(npf(prob).view(np.uint32), npf(prob2).view(np.uint32))
    st, st2 = _status(stat), ws.status()[0]
    assert (st.flags, st.total, st.wmax, st.exponent) == (st2.flags, st2.total, st2.wmax, st2.exponent)
    assert bool(st.flags & b.ST_BAD_WEIGHT) == bad
    # and the oracle, from the same weight bits
    oi, op, _ = oracle.sample_prioritized(npf(w), npf(u))
    np.testing.assert_array_equal(npf(idx), oi)
    np.testing.assert_allclose(npf(prob), op.astype(np.float32), rtol=1e-6)


def test_static_draw_two_calls_in_a_row(oracle):
    _one_call(oracle, 1000003, 5000, 31, bad=True)     # several super-blocks, ragged tail; leaves a flag behind
    _one_call(oracle, 5000, 301, 33)                   # the single-workgroup route, flags start from zero
    _one_call(oracle, b.STATIC_MAX_REPLAY, 64, 35)     # the largest capacity


def test_static_draw_rejects_what_it_cannot_serve():
    w = torch.ones(16, device=DEV)
    u = torch.zeros(4, dtype=torch.float64, device=DEV)
    idx = torch.empty(4, dtype=torch.int64, device=DEV)
    L = b.lib()
    call = lambda wp, M, up, K, ip: L.aride_sample_prioritized_static(wp, M, up, K, ip, None, None, None)
    assert call(b._p(w), b.STATIC_MAX_REPLAY + 1, b._p(u), 4, b._p(idx)) == b.E_RANGE
    assert call(b._p(w), 0, b._p(u), 4, b._p(idx)) == b.E_SHAPE
    assert call(None, 16, b._p(u), 4, b._p(idx)) == b.E_NULL
    assert call(b._p(w), 16, None, 4, b._p(idx)) == b.E_NULL
    assert call(b._p(w) + 4, 12, b._p(u), 4, b._p(idx)) == b.E_ALIGN
    assert call(b._p(w), 16, b._p(u), 0, None) == b.OK
    # no mass: every index is -1
    z = torch.zeros(16, device=DEV)
    stat = torch.zeros(24, dtype=torch.uint8, device=DEV)
    b.sample_prioritized_static(z, u, idx, None, stat)
    torch.cuda.synchronize()
    assert np.all(npf(idx) == -1) and _status(stat).flags & b.ST_ZERO_MASS
