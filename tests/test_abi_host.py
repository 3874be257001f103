"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, sizes its workspace as documented and rejects bad
arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2410_14803_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = ctypes.c_void_p


@pytest.fixture(scope="module")
def L():
    return b.lib()


def test_every_declared_symbol_is_exported(L):
    text = open(os.path.join(ROOT, "include", "aride.h")).read()
    declared = sorted(set(re.findall(r"^int\s+(aride_\w+)\s*\(", text, flags=re.M)))
    assert declared == sorted(b.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_error_codes_match_header():
    text = open(os.path.join(ROOT, "include", "aride.h")).read()
    codes = dict(re.findall(r"#define\s+(ARIDE_E_\w+)\s+(-?\d+)", text))
    assert int(codes["ARIDE_E_NULL"]) == b.E_NULL and int(codes["ARIDE_E_SHAPE"]) == b.E_SHAPE
    assert int(codes["ARIDE_E_ALIGN"]) == b.E_ALIGN and int(codes["ARIDE_E_RANGE"]) == b.E_RANGE
    assert int(codes["ARIDE_E_ZERO_MASS"]) == b.E_ZERO_MASS and int(codes["ARIDE_E_WORKSPACE"]) == b.E_WORKSPACE
    assert int(codes["ARIDE_E_HIP"]) == b.E_HIP
    assert ctypes.sizeof(b.Status) == 24 and ctypes.sizeof(b.PrioCfg) == 28 and ctypes.sizeof(b.RetraceCfg) == 20


def test_workspace_bytes(L):
    assert b.workspace_bytes(0) == 256                       # status block only
    # status, super-block prefixes, partial maxima, new super-block totals, chunk and quarter-chunk
    # maxima, block sums of a patched insert, every 16th block prefix again
    fixed = 256 + 2048 + 4096 + 2048 + 16384 + 65536 + 67584 + 32768
    # per block of 256 weights: one u64 prefix and 16 u64 sub-block sums, each array rounded to 256 bytes
    assert b.workspace_bytes(1) == fixed + 256 + 256
    assert b.workspace_bytes(256 * 32) == fixed + 256 + 32 * 128
    assert b.workspace_bytes(256 * 32 + 1) == fixed + 512 + 4352
    assert b.workspace_bytes(1 << 24) == fixed + 8 * 65536 + 128 * 65536
    out = ctypes.c_size_t(0)
    assert L.aride_workspace_bytes(-1, ctypes.byref(out)) == b.E_SHAPE
    assert L.aride_workspace_bytes((1 << 24) + 1, ctypes.byref(out)) == b.E_RANGE
    assert L.aride_workspace_bytes(10, None) == b.E_NULL


def test_score_logits_rejects_bad_arguments(L):
    ws, x, t = P(4096), P(4096), P(8192)   # never dereferenced: every call fails validation first
    f = L.aride_score_logits
    assert f(x, 4, 10, 10, t, 3, None, None, None, None, ws, 256, None) == b.E_SHAPE    # R % A
    assert f(x, -1, 10, 10, t, 1, None, None, None, None, ws, 256, None) == b.E_SHAPE
    assert f(x, 4, 0, 10, t, 1, None, None, None, None, ws, 256, None) == b.E_SHAPE
    assert f(x, 4, 10, 9, t, 1, None, None, None, None, ws, 256, None) == b.E_SHAPE     # stride < V
    assert f(x, 4, 10, 10, t, 0, None, None, None, None, ws, 256, None) == b.E_SHAPE
    assert f(x, 4, 1 << 31, 1 << 31, t, 1, None, None, None, None, ws, 256, None) == b.E_RANGE
    assert f(x, (1 << 33) - 60, 10, 10, t, 4, None, None, None, None, ws, 256, None) == b.E_RANGE     # ARIDE_MAX_ROWS + 4
    assert f(None, 4, 10, 10, t, 1, None, None, None, None, ws, 256, None) == b.E_NULL
    assert f(x, 4, 10, 10, None, 1, None, None, None, None, ws, 256, None) == b.E_NULL
    assert f(P(4098), 4, 10, 10, t, 1, None, None, None, None, ws, 256, None) == b.E_ALIGN
    assert f(x, 4, 10, 10, t, 1, None, None, None, None, None, 256, None) == b.E_WORKSPACE
    assert f(x, 4, 10, 10, t, 1, None, None, None, None, P(4100), 256, None) == b.E_WORKSPACE
    assert f(x, 4, 10, 10, t, 1, None, None, None, None, ws, 100, None) == b.E_WORKSPACE
    assert f(x, 4, 10, 10, t, 1, None, None, P(64), None, ws, 256, None) == b.E_NULL    # step sums need tok arrays
    assert f(x, 4, 10, 10, t, 1, P(64), None, None, P(64), ws, 256, None) == b.E_NULL
    assert f(x, 0, 10, 10, t, 1, None, None, None, None, ws, 256, None) == b.OK         # empty: no-op
    # the timed variant: both events are required, then the same validation
    g = L.aride_score_logits_timed
    ev = P(4096)
    assert g(x, 4, 10, 10, t, 1, None, None, None, None, ws, 256, None, None, ev) == b.E_NULL
    assert g(x, 4, 10, 10, t, 1, None, None, None, None, ws, 256, None, ev, None) == b.E_NULL
    assert g(x, 4, 10, 10, t, 3, None, None, None, None, ws, 256, None, ev, ev) == b.E_SHAPE
    assert g(x, 0, 10, 10, t, 1, None, None, None, None, ws, 256, None, ev, ev) == b.OK


def test_retrace_and_priorities_reject_bad_arguments(L):
    a = P(4096)
    cfg = b.RetraceCfg(0.9, 0.95, 0, 1.0, 1.0)
    f = L.aride_retrace_targets
    assert f(a, a, a, a, None, None, a, -1, 4, cfg, a, a, a, None) == b.E_SHAPE
    assert f(a, a, a, a, None, None, a, 2, -4, cfg, a, a, a, None) == b.E_SHAPE
    assert f(a, a, a, a, None, None, a, 2, 1 << 31, cfg, a, a, a, None) == b.E_RANGE
    assert f(a, a, a, a, None, None, a, 2, (1 << 31) - 8192, cfg, a, a, a, None) == b.E_RANGE   # ARIDE_MAX_STEPS + 1
    assert f(a, a, a, a, None, None, a, 1 << 25, 4, cfg, a, a, a, None) == b.E_RANGE             # ARIDE_MAX_TRAJECTORIES + 1
    assert f(a, a, a, a, None, None, None, 2, 4, cfg, a, a, a, None) == b.E_NULL
    assert f(None, a, a, a, None, None, a, 2, 4, cfg, a, a, a, None) == b.E_NULL
    assert f(a, a, a, a, None, None, a, 0, 0, cfg, a, a, a, None) == b.OK
    assert f(a, a, a, a, None, None, a, 2, 4, b.RetraceCfg(0.9, 0.95, 7, 1.0, 1.0), a, a, a, None) == b.E_RANGE
    m = L.aride_mc_returns
    assert m(a, a, -1, 4, 0.9, a, a, None) == b.E_SHAPE
    assert m(a, None, 2, 4, 0.9, a, a, None) == b.E_NULL
    assert m(None, a, 2, 4, 0.9, a, a, None) == b.E_NULL
    assert m(a, a, 2, 1 << 31, 0.9, a, a, None) == b.E_RANGE
    assert m(a, a, 0, 0, 0.9, a, a, None) == b.OK
    g = L.aride_compute_priorities
    pc = b.PrioCfg(1, 0.5, 0.1, 1, 1, 0, 1)
    assert g(a, a, a, a, -1, 4, pc, a, a, None) == b.E_SHAPE
    assert g(a, a, a, None, 2, 4, pc, a, a, None) == b.E_NULL
    assert g(a, None, a, a, 2, 4, pc, a, a, None) == b.E_NULL
    assert g(a, a, a, a, 2, 4, b.PrioCfg(1, 1, 1, 0, 1, 0, 1), a, a, None) == b.E_RANGE
    assert g(a, a, a, a, 2, 4, b.PrioCfg(1, 1, 1, 1, 0, 0, 1), a, a, None) == b.E_RANGE
    assert g(a, a, a, a, 0, 0, pc, a, a, None) == b.OK
    # the two in one pass: the union of their checks
    h = L.aride_retrace_priorities
    assert h(a, a, a, a, None, None, a, a, -1, 4, cfg, pc, a, a, a, a, a, None) == b.E_SHAPE
    assert h(a, a, a, a, None, None, a, a, 2, 1 << 31, cfg, pc, a, a, a, a, a, None) == b.E_RANGE
    assert h(a, a, a, a, None, None, a, None, 2, 4, cfg, pc, a, a, a, a, a, None) == b.E_NULL     # offsets
    assert h(a, a, a, a, None, None, None, a, 2, 4, cfg, pc, a, a, a, a, a, None) == b.E_NULL     # entropy
    assert h(a, a, None, a, None, None, a, a, 2, 4, cfg, pc, a, a, a, a, a, None) == b.E_NULL     # reward
    assert h(a, a, a, a, None, None, a, a, 2, 4, b.RetraceCfg(0.9, 0.95, 7, 1.0, 1.0), pc, a, a, a, a, a,
             None) == b.E_RANGE
    assert h(a, a, a, a, None, None, a, a, 2, 4, cfg, b.PrioCfg(1, 1, 1, 0, 1, 0, 1), a, a, a, a, a,
             None) == b.E_RANGE
    assert h(a, a, a, a, None, None, a, a, 0, 0, cfg, pc, a, a, a, a, a, None) == b.OK


def test_replay_rejects_bad_arguments(L):
    w, ws, a = P(4096), P(8192), P(16384)
    need = b.workspace_bytes(1000)
    u = L.aride_update_priorities
    assert u(w, 0, a, a, 4, 0.6, ws, need, None) == b.E_SHAPE
    assert u(w, 1000, a, a, -1, 0.6, ws, need, None) == b.E_SHAPE
    assert u(w, (1 << 24) + 1, a, a, 4, 0.6, ws, 1 << 30, None) == b.E_RANGE
    assert u(None, 1000, a, a, 4, 0.6, ws, need, None) == b.E_NULL
    assert u(P(4100), 1000, a, a, 4, 0.6, ws, need, None) == b.E_ALIGN
    assert u(w, 1000, a, a, 4, 0.6, ws, need - 1, None) == b.E_WORKSPACE
    assert u(w, 1000, a, a, 4, 0.6, None, need, None) == b.E_WORKSPACE
    assert u(w, 1000, a, a, 4, -0.5, ws, need, None) == b.E_RANGE
    assert u(w, 1000, a, a, 4, float("nan"), ws, need, None) == b.E_RANGE
    assert u(w, 1000, a, a, 1 << 23, 0.6, ws, need, None) == b.E_RANGE
    assert u(w, 1000, None, a, 4, 0.6, ws, need, None) == b.E_NULL
    assert u(w, 1000, a, None, 4, 0.6, ws, need, None) == b.E_NULL
    s = L.aride_sample_prioritized
    assert s(w, 1000, ws, need, a, -1, a, None, None) == b.E_SHAPE
    assert s(w, 0, ws, need, a, 4, a, None, None) == b.E_SHAPE
    assert s(w, 1000, ws, need - 8, a, 4, a, None, None) == b.E_WORKSPACE
    assert s(w, 1000, ws, need, None, 4, a, None, None) == b.E_NULL
    assert s(w, 1000, ws, need, a, 4, None, None, None) == b.E_NULL
    assert s(w, 1000, ws, need, P(16388), 4, a, None, None) == b.E_ALIGN
    assert s(w, 1000, ws, need, a, 0, a, None, None) == b.OK
    ins = L.aride_replay_insert
    assert ins(w, 1000, 0, a, -1, 0.6, None, ws, need, None, None) == b.E_SHAPE
    assert ins(w, 1000, 1000, a, 4, 0.6, None, ws, need, None, None) == b.E_RANGE     # cursor outside the buffer
    assert ins(w, 1000, -1, a, 4, 0.6, None, ws, need, None, None) == b.E_RANGE
    assert ins(w, 1000, 0, a, (1 << 31) - 255, 0.6, None, ws, need, None, None) == b.E_RANGE   # more entries than one launch's threads
    assert ins(w, 1000, 0, None, 4, 0.6, None, ws, need, None, None) == b.E_NULL
    assert ins(w, 1000, 0, a, 4, 0.6, None, ws, need - 1, None, None) == b.E_WORKSPACE
    assert ins(w, 1000, 0, a, 4, 0.6, P(16388), ws, need, None, None) == b.E_ALIGN
    assert L.aride_workspace_init(None, 256, None) == b.E_WORKSPACE
    assert L.aride_workspace_init(ws, 100, None) == b.E_WORKSPACE
    assert L.aride_status_read(None, None, None) == b.E_NULL


def test_static_draw_rejects_bad_arguments(L):
    # everything below is turned away before the library's static array is even looked up
    w, a = P(4096), P(16384)
    s = L.aride_sample_prioritized_static
    assert s(w, 0, a, 4, a, None, None, None) == b.E_SHAPE
    assert s(w, 1000, a, -1, a, None, None, None) == b.E_SHAPE
    assert s(w, b.STATIC_MAX_REPLAY + 1, a, 4, a, None, None, None) == b.E_RANGE      # beyond the array's size
    assert s(None, 1000, a, 4, a, None, None, None) == b.E_NULL
    assert s(P(4100), 1000, a, 4, a, None, None, None) == b.E_ALIGN
    assert s(w, 1000, None, 4, a, None, None, None) == b.E_NULL
    assert s(w, 1000, a, 4, None, None, None, None) == b.E_NULL
    assert s(w, 1000, P(16388), 4, a, None, None, None) == b.E_ALIGN
    assert s(w, 1000, a, 4, a, None, P(16388), None) == b.E_ALIGN
    assert s(w, 1000, a, 0, a, None, None, None) == b.OK
    text = open(os.path.join(ROOT, "include", "aride.h")).read()
    assert int(re.search(r"#define\s+ARIDE_STATIC_MAX_REPLAY\s+\(1 << (\d+)\)", text).group(1)) == 20
