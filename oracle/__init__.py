"""ctypes front end of the CPU oracle (oracle/aride_oracle.c).

TEST INFRASTRUCTURE ONLY.  Callers allowed: tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The product package never imports this module, and this
module imports nothing from the product package.

All floating-point inputs are widened to fp64 here and all results come back as fp64
numpy arrays (indices as int64).  bf16 logits are passed as their raw uint16 bit
patterns.  The passages each routine follows are cited in aride_oracle.c.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaride_oracle.so")
_lib = None

_c_dp = ctypes.POINTER(ctypes.c_double)
_c_fp = ctypes.POINTER(ctypes.c_float)
_c_i32p = ctypes.POINTER(ctypes.c_int32)
_c_i64p = ctypes.POINTER(ctypes.c_int64)
_c_u16p = ctypes.POINTER(ctypes.c_uint16)
_c_u64p = ctypes.POINTER(ctypes.c_uint64)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _b
        _b.build()
    lib = ctypes.CDLL(_LIB_PATH)
    lib.oracle_score_logits.restype = ctypes.c_int
    lib.oracle_score_logits.argtypes = [_c_u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                        _c_i32p, ctypes.c_int32, _c_dp, _c_dp, _c_dp, _c_dp,
                                        ctypes.c_int]
    lib.oracle_retrace_targets.restype = ctypes.c_int
    lib.oracle_retrace_targets.argtypes = [_c_dp, _c_dp, _c_dp, _c_dp, _c_dp, _c_dp, _c_i32p,
                                           ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
                                           ctypes.c_double, _c_dp, _c_dp, _c_dp]
    lib.oracle_compute_priorities.restype = ctypes.c_int
    lib.oracle_compute_priorities.argtypes = [_c_dp, _c_dp, _c_dp, _c_i32p, ctypes.c_int64,
                                              ctypes.c_int64] + [ctypes.c_double] * 6 + \
                                             [ctypes.c_int, _c_dp, _c_dp]
    lib.oracle_update_priorities.restype = ctypes.c_int64
    lib.oracle_update_priorities.argtypes = [_c_fp, ctypes.c_int64, _c_i64p, _c_fp,
                                             ctypes.c_int64, ctypes.c_float]
    lib.oracle_quantise_weights.restype = ctypes.c_uint64
    lib.oracle_quantise_weights.argtypes = [_c_fp, ctypes.c_int64, _c_u64p]
    lib.oracle_sample_prioritized.restype = ctypes.c_int
    lib.oracle_sample_prioritized.argtypes = [_c_fp, ctypes.c_int64, _c_dp, ctypes.c_int64,
                                              _c_i64p, _c_dp]
    lib.oracle_vtrace_targets.restype = ctypes.c_int
    lib.oracle_vtrace_targets.argtypes = [_c_dp, _c_dp, _c_dp, _c_dp, _c_dp, _c_dp, _c_i32p, ctypes.c_int64,
                                          ctypes.c_int64] + [ctypes.c_double] * 4 + [_c_dp, _c_dp, _c_dp]
    lib.oracle_mc_returns.restype = ctypes.c_int
    lib.oracle_mc_returns.argtypes = [_c_dp, _c_i32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_double, _c_dp, _c_dp]
    lib.oracle_replay_insert.restype = ctypes.c_int64
    lib.oracle_replay_insert.argtypes = [_c_fp, ctypes.c_int64, ctypes.c_int64, _c_fp, ctypes.c_int64,
                                         ctypes.c_float, _c_i64p]
    lib.oracle_actor_loss_grad.restype = ctypes.c_int
    lib.oracle_actor_loss_grad.argtypes = [_c_u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, _c_i32p,
                                           ctypes.c_int32, _c_dp, _c_dp, _c_dp, _c_dp, ctypes.c_double,
                                           ctypes.c_double, ctypes.c_double, _c_dp, _c_dp]
    _lib = lib
    return lib


def _f64(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a, ctype):
    return None if a is None else a.ctypes.data_as(ctype)


def score_logits(logits_bits, tokens, A, V=None, nthreads=1):
    """logits_bits: uint16 [R, row_stride] bf16 bit patterns (the first V columns of each
    row are the vocabulary; V defaults to row_stride); tokens: int32 [R].

    Returns dict(tok_logp[R], tok_ent[R], step_logp[N], step_ent[N]) in fp64.
    """
    lib = _load()
    lb = np.ascontiguousarray(np.asarray(logits_bits, dtype=np.uint16))
    assert lb.ndim == 2
    R, stride = lb.shape
    V = stride if V is None else int(V)
    tok = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
    assert tok.shape == (R,)
    N = R // A if A > 0 else 0
    out = dict(tok_logp=np.zeros(R), tok_ent=np.zeros(R), step_logp=np.zeros(N), step_ent=np.zeros(N))
    rc = lib.oracle_score_logits(_ptr(lb, _c_u16p), R, V, stride, _ptr(tok, _c_i32p), A,
                                 _ptr(out["tok_logp"], _c_dp), _ptr(out["tok_ent"], _c_dp),
                                 _ptr(out["step_logp"], _c_dp), _ptr(out["step_ent"], _c_dp),
                                 int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_score_logits rc={rc}")
    return out


def retrace_targets(logp_pi, logp_mu, reward, value, traj_offsets, gamma, lam, q=None, boot=None):
    """Returns dict(target[N], td[N], rho[N]) in fp64."""
    lib = _load()
    lp, lm, r, v = _f64(logp_pi), _f64(logp_mu), _f64(reward), _f64(value)
    qq, bb = _f64(q), _f64(boot)
    off = np.ascontiguousarray(np.asarray(traj_offsets, dtype=np.int32))
    B, N = off.shape[0] - 1, lp.shape[0]
    out = dict(target=np.zeros(N), td=np.zeros(N), rho=np.zeros(N))
    rc = lib.oracle_retrace_targets(_ptr(lp, _c_dp), _ptr(lm, _c_dp), _ptr(r, _c_dp), _ptr(v, _c_dp),
                                    _ptr(qq, _c_dp), _ptr(bb, _c_dp), _ptr(off, _c_i32p), B, N,
                                    float(gamma), float(lam), _ptr(out["target"], _c_dp),
                                    _ptr(out["td"], _c_dp), _ptr(out["rho"], _c_dp))
    if rc != 0:
        raise ValueError(f"oracle_retrace_targets rc={rc}")
    return out


def compute_priorities(td, rho, ent, traj_offsets, w_td, w_rho, w_ent, td_scale=1.0,
                       ent_scale=1.0, eps=0.0, truncate_rho=True):
    """Returns dict(step_prio[N], traj_prio[B]) in fp64."""
    lib = _load()
    a, b, c = _f64(td), _f64(rho), _f64(ent)
    off = np.ascontiguousarray(np.asarray(traj_offsets, dtype=np.int32))
    B, N = off.shape[0] - 1, a.shape[0]
    out = dict(step_prio=np.zeros(N), traj_prio=np.zeros(B))
    rc = lib.oracle_compute_priorities(_ptr(a, _c_dp), _ptr(b, _c_dp), _ptr(c, _c_dp),
                                       _ptr(off, _c_i32p), B, N, float(w_td), float(w_rho),
                                       float(w_ent), float(td_scale), float(ent_scale), float(eps),
                                       int(bool(truncate_rho)), _ptr(out["step_prio"], _c_dp),
                                       _ptr(out["traj_prio"], _c_dp))
    if rc != 0:
        raise ValueError(f"oracle_compute_priorities rc={rc}")
    return out


def update_priorities(weights, idx, prio, alpha):
    """In-place on a float32 numpy array `weights`; returns the count of bad indices."""
    lib = _load()
    assert weights.dtype == np.float32 and weights.flags["C_CONTIGUOUS"]
    ii = np.ascontiguousarray(np.asarray(idx, dtype=np.int64))
    pp = np.ascontiguousarray(np.asarray(prio, dtype=np.float32))
    return int(lib.oracle_update_priorities(_ptr(weights, _c_fp), weights.shape[0], _ptr(ii, _c_i64p),
                                            _ptr(pp, _c_fp), ii.shape[0], np.float32(alpha)))


def quantise_weights(weights):
    """Returns (q[M] uint64, Total)."""
    lib = _load()
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.float32))
    q = np.zeros(w.shape[0], dtype=np.uint64)
    total = lib.oracle_quantise_weights(_ptr(w, _c_fp), w.shape[0], _ptr(q, _c_u64p))
    return q, int(total)


def sample_prioritized(weights, uniforms):
    """Returns (idx[K] int64, prob[K] fp64, rc); rc = -5 when the buffer has no mass."""
    lib = _load()
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.float32))
    u = _f64(uniforms)
    K = u.shape[0]
    idx = np.zeros(K, dtype=np.int64)
    prob = np.zeros(K, dtype=np.float64)
    rc = lib.oracle_sample_prioritized(_ptr(w, _c_fp), w.shape[0], _ptr(u, _c_dp), K,
                                       _ptr(idx, _c_i64p), _ptr(prob, _c_dp))
    if rc not in (0, -5):
        raise ValueError(f"oracle_sample_prioritized rc={rc}")
    return idx, prob, rc


def actor_loss_grad(logits_bits, tokens, A, rho, target, baseline, beta, scale, penalty=None,
                    lambda_pen=0.0, V=None, want_grad=True):
    """Returns (loss, grad[R, V] fp64 or None)."""
    lib = _load()
    lb = np.ascontiguousarray(np.asarray(logits_bits, dtype=np.uint16))
    R, stride = lb.shape
    V = stride if V is None else int(V)
    tok = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
    r_, t_, b_, p_ = _f64(rho), _f64(target), _f64(baseline), _f64(penalty)
    grad = np.zeros((R, V)) if want_grad else None
    loss = np.zeros(1)
    rc = lib.oracle_actor_loss_grad(_ptr(lb, _c_u16p), R, V, stride, _ptr(tok, _c_i32p), A, _ptr(r_, _c_dp),
                                    _ptr(t_, _c_dp), _ptr(b_, _c_dp), _ptr(p_, _c_dp), float(beta),
                                    float(lambda_pen), float(scale), _ptr(grad, _c_dp), _ptr(loss, _c_dp))
    if rc != 0:
        raise ValueError(f"oracle_actor_loss_grad rc={rc}")
    return float(loss[0]), grad


def vtrace_targets(logp_pi, logp_mu, reward, value, traj_offsets, gamma, lam, rho_bar, c_bar, q=None, boot=None):
    """Returns dict(target[N], td[N], rho[N]) in fp64."""
    lib = _load()
    lp, lm, r, v = _f64(logp_pi), _f64(logp_mu), _f64(reward), _f64(value)
    qq, bb = _f64(q), _f64(boot)
    off = np.ascontiguousarray(np.asarray(traj_offsets, dtype=np.int32))
    B, N = off.shape[0] - 1, lp.shape[0]
    out = dict(target=np.zeros(N), td=np.zeros(N), rho=np.zeros(N))
    rc = lib.oracle_vtrace_targets(_ptr(lp, _c_dp), _ptr(lm, _c_dp), _ptr(r, _c_dp), _ptr(v, _c_dp),
                                   _ptr(qq, _c_dp), _ptr(bb, _c_dp), _ptr(off, _c_i32p), B, N, float(gamma),
                                   float(lam), float(rho_bar), float(c_bar), _ptr(out["target"], _c_dp),
                                   _ptr(out["td"], _c_dp), _ptr(out["rho"], _c_dp))
    if rc != 0:
        raise ValueError(f"oracle_vtrace_targets rc={rc}")
    return out


def mc_returns(reward, traj_offsets, gamma):
    """Returns (ret[N], label[N]) in fp64."""
    lib = _load()
    r = _f64(reward)
    off = np.ascontiguousarray(np.asarray(traj_offsets, dtype=np.int32))
    N = r.shape[0]
    ret, label = np.zeros(N), np.zeros(N)
    rc = lib.oracle_mc_returns(_ptr(r, _c_dp), _ptr(off, _c_i32p), off.shape[0] - 1, N, float(gamma),
                               _ptr(ret, _c_dp), _ptr(label, _c_dp))
    if rc != 0:
        raise ValueError(f"oracle_mc_returns rc={rc}")
    return ret, label


def replay_insert(weights, cursor, prio, alpha):
    """In place on a float32 numpy array; returns (new_cursor, slots[K] int64)."""
    lib = _load()
    assert weights.dtype == np.float32 and weights.flags["C_CONTIGUOUS"]
    pp = np.ascontiguousarray(np.asarray(prio, dtype=np.float32))
    slots = np.zeros(pp.shape[0], dtype=np.int64)
    cur = lib.oracle_replay_insert(_ptr(weights, _c_fp), weights.shape[0], int(cursor), _ptr(pp, _c_fp),
                                   pp.shape[0], np.float32(alpha), _ptr(slots, _c_i64p))
    return int(cur), slots
