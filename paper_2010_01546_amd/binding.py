"""ctypes binding of the C ABI in include/fw.h -- argument marshalling only.

Every function has the name and argument order of its C entry point.  Tensors are torch tensors on the GPU
(PyTorch supplies device memory and streams, nothing else); each call passes ``tensor.data_ptr()`` through and
raises :class:`FwError` on a non-OK status.  There is no fallback: if ``libfw.so`` is missing, importing this
module fails.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfw.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not found: build it first (python -m paper_2010_01546_amd.build); there is no fallback path")
lib = C.CDLL(LIB_PATH)

FW_OK, FW_ERR_INVALID_ARG, FW_ERR_UNSUPPORTED, FW_ERR_ALIGNMENT, FW_ERR_WORKSPACE, FW_ERR_HIP, FW_ERR_NOT_CONVERGED = range(7)
FW_F32, FW_BF16 = 0, 1
FW_LAYOUT_ROWS, FW_LAYOUT_NCHW, FW_LAYOUT_NHWC, FW_LAYOUT_NHWC_KKC = 0, 1, 2, 3
(FW_OP_COV_ACCUMULATE, FW_OP_GRAD_TRANSFORM, FW_OP_COND_REDUCE_STEP, FW_OP_WHITEN_EVD, FW_OP_COND_STATE_REFRESH,
 FW_OP_GRAD_TRANSFORM_TAPS, FW_OP_SGD_UPDATE, FW_OP_DIAGNOSTICS, FW_OP_COND_PROBE) = range(9)

EXPORTS = ["fw_cov_accumulate", "fw_cov_finalize", "fw_grad_transform", "fw_cond_state_init", "fw_cond_reduce_step",
           "fw_whiten_evd", "fw_cond_state_refresh", "fw_grad_transform_taps", "fw_sgd_update", "fw_bias_compensate",
           "fw_diagnostics", "fw_cov_plan_query", "fw_cond_reduce_step_static", "fw_cond_probe", "fw_cond_refresh_plan_query",
           "fw_grad_plan_query", "fw_mfma_rate_probe", "fw_workspace_bytes", "fw_status_string", "fw_version"]
N_STATUS_EXPORTS = 17   # the leading entries of EXPORTS return fw_status


class fw_conv_desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("B", "Cin", "H", "W", "kh", "kw", "stride", "pad", "form")]


class fw_cond_params(C.Structure):
    _fields_ = [("gamma", C.c_float), ("delta", C.c_float), ("eps", C.c_float), ("c_rel", C.c_float), ("c_abs", C.c_float),
                ("beta", C.c_float), ("n_power_iters", C.c_int), ("guard", C.c_int)]


class fw_cond_state(C.Structure):
    _fields_ = [("M", C.c_int), ("Phi_x", C.c_void_p), ("lambda_bar", C.c_void_p), ("T", C.c_void_p), ("Q", C.c_void_p),
                ("Qs", C.c_void_p), ("Phi_y", C.c_void_p), ("Psi", C.c_void_p), ("xi2", C.c_void_p)]


class fw_cond_info(C.Structure):
    _fields_ = [("lambda_e", C.c_float), ("g_e", C.c_float), ("a_e", C.c_float), ("v_norm", C.c_float),
                ("m_prime", C.c_int), ("set_size", C.c_int), ("applied", C.c_int), ("flags", C.c_int)]


class fw_sgd_params(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float)]


class fw_cov_plan(C.Structure):
    _fields_ = [("shift", C.c_int), ("regions", C.c_int), ("differences", C.c_int), ("workgroups", C.c_int), ("ranges", C.c_int),
                ("covered_pixels", C.c_longlong), ("mfma_flops_issued", C.c_double), ("split_bf16", C.c_int)]


class fw_refresh_plan(C.Structure):
    _fields_ = [("split", C.c_int), ("mfma_flops_issued", C.c_double)]


class fw_grad_plan(C.Structure):
    _fields_ = [("split", C.c_int), ("mfma_flops_issued", C.c_double)]


class fw_evd_params(C.Structure):
    _fields_ = [("eps", C.c_float), ("g_max", C.c_float), ("beta", C.c_float), ("tol", C.c_float),
                ("gain_mode", C.c_int), ("max_sweeps", C.c_int)]


_P = C.c_void_p
lib.fw_cov_accumulate.argtypes = [_P, C.c_int, C.c_int, C.POINTER(fw_conv_desc), _P, _P, _P, C.c_size_t, _P]
lib.fw_cov_finalize.argtypes = [_P, _P, C.c_longlong, C.c_int, C.c_float, C.c_int, _P, _P, _P, _P, _P]
lib.fw_grad_transform.argtypes = [_P, C.c_int, C.c_int, C.c_int, _P, _P, _P, _P, C.c_size_t, _P]
lib.fw_cond_state_init.argtypes = [C.POINTER(fw_cond_state), _P]
lib.fw_cond_state_refresh.argtypes = [C.POINTER(fw_cond_state), _P, C.c_size_t, _P]
lib.fw_cond_reduce_step.argtypes = [C.POINTER(fw_cond_state), C.POINTER(fw_cond_params), _P, _P, C.c_size_t, _P]
lib.fw_cond_reduce_step_static.argtypes = [C.POINTER(fw_cond_state), C.POINTER(fw_cond_params), _P, _P]
lib.fw_whiten_evd.argtypes = [_P, C.c_int, C.POINTER(fw_evd_params), _P, _P, _P, _P, _P, C.c_size_t, _P]
lib.fw_grad_transform_taps.argtypes = [_P, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, _P, C.c_size_t, _P]
lib.fw_sgd_update.argtypes = [_P, C.c_int, C.c_int, C.c_int, C.c_int, _P, C.POINTER(fw_sgd_params), _P, _P, _P, C.c_size_t, _P]
lib.fw_bias_compensate.argtypes = [_P, _P, C.c_int, C.c_int, C.c_int, _P, _P, C.c_float, _P]
lib.fw_diagnostics.argtypes = [_P, _P, C.c_int, _P, _P, C.c_size_t, _P]
lib.fw_cond_probe.argtypes = [_P, C.c_int, _P, C.c_int, _P, _P, C.c_size_t, _P]
lib.fw_cond_refresh_plan_query.argtypes = [C.c_int, C.c_size_t, C.POINTER(fw_refresh_plan)]
lib.fw_cov_plan_query.argtypes = [C.c_int, C.c_int, C.POINTER(fw_conv_desc), C.POINTER(fw_cov_plan)]
lib.fw_grad_plan_query.argtypes = [C.c_int, C.c_int, C.c_int, C.c_size_t, C.POINTER(fw_grad_plan)]
lib.fw_mfma_rate_probe.argtypes = [C.c_int, C.c_int, _P, C.POINTER(C.c_double), _P]
lib.fw_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(fw_conv_desc), C.c_int]
lib.fw_workspace_bytes.restype = C.c_size_t
lib.fw_status_string.argtypes = [C.c_int]
lib.fw_status_string.restype = C.c_char_p
lib.fw_version.restype = C.c_int
for _n in EXPORTS[:N_STATUS_EXPORTS]:
    getattr(lib, _n).restype = C.c_int


class FwError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib.fw_status_string(status).decode()} (status {status})")


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _check(status, where, allow=()):
    if status != FW_OK and status not in allow:
        raise FwError(status, where)
    return status


def conv_desc(B, Cin, H=1, W=1, kh=1, kw=1, stride=1, pad=0, form=0) -> fw_conv_desc:
    return fw_conv_desc(B, Cin, H, W, kh, kw, stride, pad, form)


def fw_workspace_bytes(op, M, S=0, d=None, dt=FW_F32) -> int:
    return int(lib.fw_workspace_bytes(op, M, S, C.byref(d) if d is not None else None, dt))


def fw_status_string(status) -> str:
    return lib.fw_status_string(status).decode()


def fw_version() -> int:
    return int(lib.fw_version())


def fw_cov_accumulate(X, dt, lay, d, A, s, ws, stream=None):
    p, n = _ws(ws)
    return _check(lib.fw_cov_accumulate(_ptr(X), dt, lay, C.byref(d), _ptr(A), _ptr(s), p, n, _stream(stream)), "fw_cov_accumulate")


def fw_cov_finalize(A, s, n, M, alpha, first_block, mu, Phi_x, phi_x, lambda_bar, stream=None):
    return _check(lib.fw_cov_finalize(_ptr(A), _ptr(s), int(n), M, float(alpha), int(first_block), _ptr(mu), _ptr(Phi_x),
                                      _ptr(phi_x), _ptr(lambda_bar), _stream(stream)), "fw_cov_finalize")


def fw_grad_transform(G, dt, S, M, T, Q, G_out, ws=None, stream=None):
    p, n = _ws(ws)
    return _check(lib.fw_grad_transform(_ptr(G), dt, S, M, _ptr(T), _ptr(Q), _ptr(G_out), p, n, _stream(stream)), "fw_grad_transform")


def fw_grad_transform_taps(G, dt, S, M, taps, Q, G_out, ws, stream=None):
    p, n = _ws(ws)
    return _check(lib.fw_grad_transform_taps(_ptr(G), dt, S, M, taps, _ptr(Q), _ptr(G_out), p, n, _stream(stream)),
                  "fw_grad_transform_taps")


def sgd_params(lr, momentum=0.0, weight_decay=0.0) -> fw_sgd_params:
    return fw_sgd_params(lr, momentum, weight_decay)


def fw_sgd_update(G, dt, S, M, taps, Q, p, W, V=None, ws=None, stream=None):
    wp, n = _ws(ws)
    return _check(lib.fw_sgd_update(_ptr(G), dt, S, M, taps, _ptr(Q), C.byref(p), _ptr(W), _ptr(V), wp, n, _stream(stream)),
                  "fw_sgd_update")


def fw_bias_compensate(b, W, S, M, taps, mu_old, mu_new, scale=1.0, stream=None):
    return _check(lib.fw_bias_compensate(_ptr(b), _ptr(W), S, M, taps, _ptr(mu_old), _ptr(mu_new), float(scale), _stream(stream)),
                  "fw_bias_compensate")


def fw_diagnostics(Phi_y, lam, M, out, ws=None, stream=None):
    wp, n = _ws(ws)
    return _check(lib.fw_diagnostics(_ptr(Phi_y), _ptr(lam), M, _ptr(out), wp, n, _stream(stream)), "fw_diagnostics")


FW_COND_PROBE_MAX_K = 32


def fw_cond_probe(Phi_y, M, b0, k, out, ws, stream=None):
    wp, n = _ws(ws)
    return _check(lib.fw_cond_probe(_ptr(Phi_y), M, _ptr(b0), k, _ptr(out), wp, n, _stream(stream)), "fw_cond_probe")


def fw_cond_refresh_plan_query(M, ws_bytes) -> fw_refresh_plan:
    """Host arithmetic only: works without a GPU."""
    plan = fw_refresh_plan()
    _check(lib.fw_cond_refresh_plan_query(M, ws_bytes, C.byref(plan)), "fw_cond_refresh_plan_query")
    return plan


def fw_grad_plan_query(dt, S, M, ws_bytes) -> fw_grad_plan:
    """Host arithmetic only: works without a GPU."""
    plan = fw_grad_plan()
    _check(lib.fw_grad_plan_query(dt, S, M, ws_bytes, C.byref(plan)), "fw_grad_plan_query")
    return plan


def fw_mfma_rate_probe(zero_operands, iters, sink, stream=None) -> float:
    """Launches the measurement kernel; returns the flops it executes (time it with events)."""
    flops = C.c_double(0.0)
    _check(lib.fw_mfma_rate_probe(int(bool(zero_operands)), int(iters), _ptr(sink), C.byref(flops), _stream(stream)), "fw_mfma_rate_probe")
    return flops.value


def fw_cov_plan_query(dt, lay, d) -> fw_cov_plan:
    """Host arithmetic only: works without a GPU."""
    plan = fw_cov_plan()
    _check(lib.fw_cov_plan_query(dt, lay, C.byref(d), C.byref(plan)), "fw_cov_plan_query")
    return plan


FW_COV_FORM_AUTO, FW_COV_FORM_SHIFT, FW_COV_FORM_DIRECT, FW_COV_FORM_SPLIT = 0, 1, 2, 3


def cond_state(M, Phi_x, lambda_bar, T, Q, Qs, Phi_y, Psi, xi2) -> fw_cond_state:
    """The struct holds raw device addresses; the tensors behind them are attached to it (``tensors``) so that the
    memory lives as long as the struct does: a caller that keeps only the struct would otherwise hand the library
    addresses that the allocator has already given to somebody else."""
    st = fw_cond_state(M, _ptr(Phi_x), _ptr(lambda_bar), _ptr(T), _ptr(Q), _ptr(Qs), _ptr(Phi_y), _ptr(Psi), _ptr(xi2))
    st.tensors = (Phi_x, lambda_bar, T, Q, Qs, Phi_y, Psi, xi2)
    return st


def cond_params(gamma=0.99, delta=0.25, eps=1e-5, c_rel=0.025, c_abs=1e-6, beta=0.1, n_power_iters=0, guard=1) -> fw_cond_params:
    """Defaults are the hyper-parameters of the recursive variant in Sec. 6."""
    return fw_cond_params(gamma, delta, eps, c_rel, c_abs, beta, n_power_iters, guard)


def evd_params(eps=1e-5, g_max=10.0, beta=0.95, tol=0.0, gain_mode=0, max_sweeps=0) -> fw_evd_params:
    """Defaults are the hyper-parameters of the EVD variant in Sec. 6."""
    return fw_evd_params(eps, g_max, beta, tol, gain_mode, max_sweeps)


def fw_cond_state_init(st, stream=None):
    return _check(lib.fw_cond_state_init(C.byref(st), _stream(stream)), "fw_cond_state_init")


def fw_cond_state_refresh(st, ws=None, stream=None):
    wp, n = _ws(ws)
    return _check(lib.fw_cond_state_refresh(C.byref(st), wp, n, _stream(stream)), "fw_cond_state_refresh")


def fw_cond_reduce_step(st, p, info_dev, ws, stream=None):
    wp, n = _ws(ws)
    return _check(lib.fw_cond_reduce_step(C.byref(st), C.byref(p), _ptr(info_dev), wp, n, _stream(stream)), "fw_cond_reduce_step")


FW_COND_STATIC_MAX_M = 4608
FW_REFRESH_SPLIT_MIN_M = 1536
FW_GRAD_SPLIT_MIN_SM, FW_GRAD_SPLIT_MIN_SM_WIDE = 1500000, 1100000


def fw_cond_reduce_step_static(st, p, info_dev, stream=None):
    return _check(lib.fw_cond_reduce_step_static(C.byref(st), C.byref(p), _ptr(info_dev), _stream(stream)), "fw_cond_reduce_step_static")


def fw_whiten_evd(Phi_x, M, p, T, Q, Qs, lam, ws, stream=None, allow_not_converged=False):
    wp, n = _ws(ws)
    allow = (FW_ERR_NOT_CONVERGED,) if allow_not_converged else ()
    return _check(lib.fw_whiten_evd(_ptr(Phi_x), M, C.byref(p), _ptr(T), _ptr(Q), _ptr(Qs), _ptr(lam), wp, n, _stream(stream)),
                  "fw_whiten_evd", allow)


def read_cond_info(info_dev) -> fw_cond_info:
    """Copy a device-side fw_cond_info (8 x 4 bytes, held in an int32 tensor) to a host struct."""
    raw = info_dev.cpu().numpy().tobytes()
    return fw_cond_info.from_buffer_copy(raw[:C.sizeof(fw_cond_info)])
