"""ctypes binding of libaride.so (the C ABI declared in include/aride.h).

Argument marshalling only: every function takes torch CUDA tensors (or None for
nullable arguments), checks dtype/contiguity, and passes raw device pointers plus the
current torch stream to the library.  Nothing is computed here and there is no
fallback: if the shared library has not been built, lib() raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaride.so")
_lib = None

OK = 0
E_NULL, E_SHAPE, E_ALIGN, E_RANGE, E_ZERO_MASS, E_WORKSPACE, E_HIP = -1, -2, -3, -4, -5, -6, -7
ST_BAD_TOKEN, ST_BAD_WEIGHT, ST_ZERO_MASS, ST_BAD_INDEX, ST_BAD_UNIFORM = 1, 2, 4, 8, 16
MAX_REPLAY = 1 << 24
STATIC_MAX_REPLAY = 1 << 20

EXPORTS = ["aride_workspace_bytes", "aride_workspace_init", "aride_status_read",
           "aride_score_logits", "aride_score_logits_timed", "aride_retrace_targets", "aride_compute_priorities",
           "aride_retrace_priorities",
           "aride_update_priorities", "aride_sample_prioritized", "aride_actor_loss_grad", "aride_mc_returns", "aride_replay_insert",
           "aride_sample_prioritized_static"]


class RetraceCfg(ctypes.Structure):
    _fields_ = [("gamma", ctypes.c_float), ("lam", ctypes.c_float), ("mode", ctypes.c_int32),
                ("rho_bar", ctypes.c_float), ("c_bar", ctypes.c_float)]


TRACE_RETRACE, TRACE_VTRACE = 0, 1


class PrioCfg(ctypes.Structure):
    _fields_ = [("w_td", ctypes.c_float), ("w_rho", ctypes.c_float), ("w_ent", ctypes.c_float),
                ("td_scale", ctypes.c_float), ("ent_scale", ctypes.c_float), ("eps", ctypes.c_float),
                ("truncate_rho", ctypes.c_int32)]


class ActorCfg(ctypes.Structure):
    _fields_ = [("beta", ctypes.c_float), ("lambda_pen", ctypes.c_float), ("scale", ctypes.c_float),
                ("grad_f32", ctypes.c_int32)]


class Status(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32), ("total", ctypes.c_uint64),
                ("wmax", ctypes.c_float), ("exponent", ctypes.c_int32)]


class ArideError(RuntimeError):
    def __init__(self, fn, rc):
        super().__init__(f"{fn} failed with code {rc}")
        self.rc = rc


def lib():
    """Loads libaride.so (raises FileNotFoundError / OSError if it is not built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2410_14803_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    L.aride_workspace_bytes.restype = ctypes.c_int
    L.aride_workspace_bytes.argtypes = [i64, ctypes.POINTER(sz)]
    L.aride_workspace_init.restype = ctypes.c_int
    L.aride_workspace_init.argtypes = [vp, sz, vp]
    L.aride_status_read.restype = ctypes.c_int
    L.aride_status_read.argtypes = [vp, ctypes.POINTER(Status), vp]
    L.aride_score_logits.restype = ctypes.c_int
    L.aride_score_logits.argtypes = [vp, i64, i64, i64, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    L.aride_score_logits_timed.restype = ctypes.c_int
    L.aride_score_logits_timed.argtypes = [vp, i64, i64, i64, vp, i32, vp, vp, vp, vp, vp, sz, vp, vp, vp]
    L.aride_retrace_targets.restype = ctypes.c_int
    L.aride_retrace_targets.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, RetraceCfg, vp, vp, vp, vp]
    L.aride_retrace_priorities.restype = ctypes.c_int
    L.aride_retrace_priorities.argtypes = [vp] * 8 + [i64, i64, RetraceCfg, PrioCfg] + [vp] * 6
    L.aride_compute_priorities.restype = ctypes.c_int
    L.aride_compute_priorities.argtypes = [vp, vp, vp, vp, i64, i64, PrioCfg, vp, vp, vp]
    L.aride_update_priorities.restype = ctypes.c_int
    L.aride_update_priorities.argtypes = [vp, i64, vp, vp, i64, f32, vp, sz, vp]
    L.aride_sample_prioritized.restype = ctypes.c_int
    L.aride_sample_prioritized.argtypes = [vp, i64, vp, sz, vp, i64, vp, vp, vp]
    L.aride_sample_prioritized_static.restype = ctypes.c_int
    L.aride_sample_prioritized_static.argtypes = [vp, i64, vp, i64, vp, vp, vp, vp]
    L.aride_replay_insert.restype = ctypes.c_int
    L.aride_replay_insert.argtypes = [vp, i64, i64, vp, i64, f32, vp, vp, sz, ctypes.POINTER(ctypes.c_int64), vp]
    L.aride_mc_returns.restype = ctypes.c_int
    L.aride_mc_returns.argtypes = [vp, vp, i64, i64, f32, vp, vp, vp]
    L.aride_actor_loss_grad.restype = ctypes.c_int
    L.aride_actor_loss_grad.argtypes = [vp, i64, i64, i64, vp, i32] + [vp] * 8 + [ActorCfg, vp, vp, vp]
    _lib = L
    return L


def _p(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return t.data_ptr()


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream():
    """Handle of torch's current stream on the current device (what every call is enqueued on)."""
    if _raw_stream is not None:        # the short way to the same handle: a third of the cost of the call below
        return _raw_stream(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


def _check(fn, rc):
    if rc != OK:
        raise ArideError(fn, rc)


def workspace_bytes(M: int) -> int:
    out = ctypes.c_size_t(0)
    _check("aride_workspace_bytes", lib().aride_workspace_bytes(int(M), ctypes.byref(out)))
    return out.value


class Workspace:
    """Device workspace (status block + replay index for capacity M), caller-owned memory."""

    def __init__(self, M: int = 0, device="cuda"):
        self.M = int(M)
        self.nbytes = workspace_bytes(M)
        self.buf = torch.empty(self.nbytes, dtype=torch.uint8, device=device)
        assert self.buf.data_ptr() % 256 == 0
        _check("aride_workspace_init", lib().aride_workspace_init(_p(self.buf), self.nbytes, _stream()))

    @property
    def ptr(self):
        return ctypes.c_void_p(self.buf.data_ptr())

    def status(self):
        """Synchronising read of the status block; returns (Status, rc)."""
        st = Status()
        rc = lib().aride_status_read(self.ptr, ctypes.byref(st), _stream())
        return st, rc


def score_logits(logits, tokens, A, ws, tok_logp=None, tok_ent=None, step_logp=None, step_ent=None, V=None,
                 sweep_events=None):
    """logits: bf16 [R, row_stride]; tokens int32 [R]; outputs are written in place.
    sweep_events: a pair of torch.cuda.Event(enable_timing=True), each recorded once before (which is
    what creates the HIP event); they are attached to the row-sweep kernel's own dispatch."""
    assert logits.dtype == torch.bfloat16 and logits.dim() == 2
    R, stride = logits.shape
    V = stride if V is None else int(V)
    args = (_p(logits), R, V, stride, _p(tokens, torch.int32), int(A),
            _p(tok_logp, torch.float32), _p(tok_ent, torch.float32),
            _p(step_logp, torch.float32), _p(step_ent, torch.float32), ws.ptr, ws.nbytes, _stream())
    if sweep_events is None:
        _check("aride_score_logits", lib().aride_score_logits(*args))
    else:
        e0, e1 = (ctypes.c_void_p(e.cuda_event) for e in sweep_events)
        assert e0.value and e1.value, "record each event once before passing it"
        _check("aride_score_logits_timed", lib().aride_score_logits_timed(*args, e0, e1))


def retrace_targets(logp_pi, logp_mu, reward, value, traj_offsets, gamma, lam, q=None, boot=None,
                    target=None, td=None, rho=None, vtrace=False, rho_bar=1.0, c_bar=1.0):
    B = traj_offsets.numel() - 1
    N = logp_pi.numel()
    f = torch.float32
    rc = lib().aride_retrace_targets(_p(logp_pi, f), _p(logp_mu, f), _p(reward, f), _p(value, f), _p(q, f),
                                     _p(boot, f), _p(traj_offsets, torch.int32), B, N,
                                     RetraceCfg(float(gamma), float(lam), TRACE_VTRACE if vtrace else TRACE_RETRACE,
                                                float(rho_bar), float(c_bar)), _p(target, f), _p(td, f),
                                     _p(rho, f), _stream())
    _check("aride_retrace_targets", rc)


def compute_priorities(td, rho, ent, traj_offsets, w, td_scale=1.0, ent_scale=1.0, eps=0.0,
                       truncate_rho=True, step_prio=None, traj_prio=None):
    B = traj_offsets.numel() - 1
    N = td.numel()
    f = torch.float32
    cfg = PrioCfg(float(w[0]), float(w[1]), float(w[2]), float(td_scale), float(ent_scale), float(eps),
                  int(bool(truncate_rho)))
    rc = lib().aride_compute_priorities(_p(td, f), _p(rho, f), _p(ent, f), _p(traj_offsets, torch.int32),
                                        B, N, cfg, _p(step_prio, f), _p(traj_prio, f), _stream())
    _check("aride_compute_priorities", rc)


def retrace_priorities(logp_pi, logp_mu, reward, value, ent, traj_offsets, gamma, lam, w, q=None, boot=None,
                       td_scale=1.0, ent_scale=1.0, eps=0.0, truncate_rho=True, target=None, td=None, rho=None,
                       step_prio=None, traj_prio=None, vtrace=False, rho_bar=1.0, c_bar=1.0):
    """retrace_targets and compute_priorities in one pass (one launch)."""
    B = traj_offsets.numel() - 1
    N = logp_pi.numel()
    f = torch.float32
    rcfg = RetraceCfg(float(gamma), float(lam), TRACE_VTRACE if vtrace else TRACE_RETRACE, float(rho_bar),
                      float(c_bar))
    pcfg = PrioCfg(float(w[0]), float(w[1]), float(w[2]), float(td_scale), float(ent_scale), float(eps),
                   int(bool(truncate_rho)))
    rc = lib().aride_retrace_priorities(_p(logp_pi, f), _p(logp_mu, f), _p(reward, f), _p(value, f), _p(q, f),
                                        _p(boot, f), _p(ent, f), _p(traj_offsets, torch.int32), B, N, rcfg, pcfg,
                                        _p(target, f), _p(td, f), _p(rho, f), _p(step_prio, f), _p(traj_prio, f),
                                        _stream())
    _check("aride_retrace_priorities", rc)


def update_priorities(weights, idx, prio, alpha, ws):
    """weights fp32 [M] updated in place; idx int64 [K] / prio fp32 [K] may be None (rebuild only)."""
    K = 0 if idx is None else idx.numel()
    rc = lib().aride_update_priorities(_p(weights, torch.float32), weights.numel(), _p(idx, torch.int64),
                                       _p(prio, torch.float32), K, float(alpha), ws.ptr, ws.nbytes, _stream())
    _check("aride_update_priorities", rc)


def sample_prioritized(weights, uniforms, ws, idx_out, prob_out=None):
    rc = lib().aride_sample_prioritized(_p(weights, torch.float32), weights.numel(), ws.ptr, ws.nbytes,
                                        _p(uniforms, torch.float64), uniforms.numel(),
                                        _p(idx_out, torch.int64), _p(prob_out, torch.float32), _stream())
    _check("aride_sample_prioritized", rc)


def sample_prioritized_static(weights, uniforms, idx_out, prob_out=None, status_out=None):
    """The draw without a workspace: the index lives in the library's own static device array.
    status_out: uint8 [24] device tensor (or None) that receives this call's status block."""
    if status_out is not None:
        assert status_out.dtype == torch.uint8 and status_out.numel() >= ctypes.sizeof(Status)
    rc = lib().aride_sample_prioritized_static(_p(weights, torch.float32), weights.numel(),
                                               _p(uniforms, torch.float64), uniforms.numel(),
                                               _p(idx_out, torch.int64), _p(prob_out, torch.float32),
                                               _p(status_out), _stream())
    _check("aride_sample_prioritized_static", rc)


def actor_loss_grad(logits, tokens, A, tok_logp, tok_ent, step_logp, step_ent, rho, target, baseline,
                    beta, scale, penalty=None, lambda_pen=0.0, grad=None, loss=None, V=None):
    """grad: bf16 or fp32 tensor shaped like logits (or None); loss: fp32 tensor [1] (or None)."""
    assert logits.dtype == torch.bfloat16 and logits.dim() == 2
    R, stride = logits.shape
    V = stride if V is None else int(V)
    f = torch.float32
    grad_f32 = 0
    if grad is not None:
        assert grad.shape == logits.shape and grad.dtype in (torch.bfloat16, torch.float32)
        grad_f32 = int(grad.dtype == torch.float32)
    cfg = ActorCfg(float(beta), float(lambda_pen), float(scale), grad_f32)
    rc = lib().aride_actor_loss_grad(_p(logits), R, V, stride, _p(tokens, torch.int32), int(A), _p(tok_logp, f),
                                     _p(tok_ent, f), _p(step_logp, f), _p(step_ent, f), _p(rho, f),
                                     _p(target, f), _p(baseline, f), _p(penalty, f), cfg, _p(grad),
                                     _p(loss, f), _stream())
    _check("aride_actor_loss_grad", rc)


def mc_returns(reward, traj_offsets, gamma, ret=None, label=None):
    B = traj_offsets.numel() - 1
    f = torch.float32
    rc = lib().aride_mc_returns(_p(reward, f), _p(traj_offsets, torch.int32), B, reward.numel(), float(gamma),
                                _p(ret, f), _p(label, f), _stream())
    _check("aride_mc_returns", rc)


def replay_insert(weights, cursor, prio, alpha, ws, slots_out=None):
    """Appends prio.numel() entries at the circular cursor; returns the advanced cursor."""
    new_cursor = ctypes.c_int64(-1)
    rc = lib().aride_replay_insert(_p(weights, torch.float32), weights.numel(), int(cursor),
                                   _p(prio, torch.float32), prio.numel(), float(alpha),
                                   _p(slots_out, torch.int64), ws.ptr, ws.nbytes, ctypes.byref(new_cursor),
                                   _stream())
    _check("aride_replay_insert", rc)
    return new_cursor.value
