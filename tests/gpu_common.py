"""Shared helpers of the GPU parity tests: upload seeded inputs, call the C ABI through the binding, fetch results."""
import numpy as np
import torch

import workloads as wl
from oracle import fw_oracle as ora
from paper_2010_01546_amd import binding as b

DEV = "cuda:0"


def relF(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / (den if den > 0 else 1.0))


def dev(x, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(x)).to(DEV).to(dtype).contiguous()


def upload_act(layer: wl.Layer, layout: int):
    """Activation of a layer on the GPU in the given layout and the layer's element type."""
    tdt = torch.bfloat16 if layer.dtype == "bf16" else torch.float32
    if layer.is_rows:
        return dev(layer.act, tdt), b.FW_LAYOUT_ROWS
    return dev(wl.to_layout(layer.act, layout), tdt), layout


def desc_of(layer: wl.Layer):
    return b.conv_desc(*layer.desc.astuple())


def dt_of(layer: wl.Layer):
    return b.FW_BF16 if layer.dtype == "bf16" else b.FW_F32


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=DEV)


def run_cov(layer: wl.Layer, layout: int, A=None, s=None):
    """fw_cov_accumulate on one batch; returns device tensors A [M,M] (lower triangle valid) and s [M]."""
    M = layer.desc.M
    X, lay = upload_act(layer, layout)
    d = desc_of(layer)
    if A is None:
        A = torch.zeros(M, M, device=DEV)
        s = torch.zeros(M, device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, M, 0, d, dt_of(layer)))
    b.fw_cov_accumulate(X, dt_of(layer), lay, d, A, s, ws)
    torch.cuda.synchronize()
    return A, s


def run_finalize(A, s, n, M, alpha, first, mu=None, Phi=None, phi=None):
    if mu is None:
        mu = torch.zeros(M, device=DEV)
        Phi = torch.zeros(M, M, device=DEV)
        phi = torch.zeros(M, device=DEV)
    lbar = torch.zeros(4, device=DEV)
    b.fw_cov_finalize(A, s, n, M, alpha, first, mu, Phi, phi, lbar)
    torch.cuda.synchronize()
    return mu, Phi, phi, lbar


def oracle_rows(layer: wl.Layer, layout: int = 0):
    """Patch rows of the layer in the feature order the given layout implies."""
    if layer.is_rows:
        return np.asarray(layer.act, dtype=np.float64)
    return ora.patch_rows(layer.act, *layer.desc.astuple(), order="kkc" if layout == b.FW_LAYOUT_NHWC_KKC else "ckk")


def lower(Am):
    return np.tril(np.asarray(Am, dtype=np.float64))


class CondRunner:
    """Device state of the recursive method for one layer."""

    def __init__(self, Phi_x_np, lambda_bar, gamma_lt_one=True):
        M = Phi_x_np.shape[0]
        self.M = M
        self.Phi_x = dev(Phi_x_np)
        self.lbar = torch.full((4,), float(lambda_bar), device=DEV)
        z = lambda: torch.empty(M, M, device=DEV)
        self.T, self.Q, self.Qs, self.Phi_y = z(), z(), z(), z()
        self.Psi = z() if gamma_lt_one else None
        self.xi2 = torch.empty(M, device=DEV)
        self.info = torch.zeros(8, dtype=torch.int32, device=DEV)
        self.ws = workspace(b.fw_workspace_bytes(b.FW_OP_COND_REDUCE_STEP, M))
        self.st = b.cond_state(M, self.Phi_x, self.lbar, self.T, self.Q, self.Qs, self.Phi_y, self.Psi, self.xi2)
        b.fw_cond_state_init(self.st)
        torch.cuda.synchronize()

    def step(self, params):
        b.fw_cond_reduce_step(self.st, params, self.info, self.ws)
        torch.cuda.synchronize()
        return b.read_cond_info(self.info)

    def host(self, name):
        return getattr(self, name).cpu().numpy().astype(np.float64)
