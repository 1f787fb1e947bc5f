"""GPU parity of the EVD / ZCA whitening matrix (Sec. 2, Sec. 3.2) against the CPU oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import b, dev, ora, relF, workspace, DEV

pytestmark = pytest.mark.gpu


def run_evd(Phi32, Qs=None, **kw):
    M = Phi32.shape[0]
    T = torch.empty(M, M, device=DEV); Q = torch.empty(M, M, device=DEV); lam = torch.empty(M, device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_WHITEN_EVD, M))
    b.fw_whiten_evd(dev(Phi32), M, b.evd_params(**kw), T, Q, Qs, lam, ws)
    torch.cuda.synchronize()
    return T.cpu().numpy(), Q.cpu().numpy(), lam.cpu().numpy()


@pytest.mark.parametrize("M,lo", [(2, -1), (7, -2), (64, -4), (65, -3), (130, -5), (256, -3), (1100, -4)])
def test_plain_gains(M, lo):
    Phi32 = wl.spd_matrix(M, M, np.logspace(0, lo, M)).astype(np.float32)
    T, Q, lam = run_evd(Phi32, eps=1e-5)
    To, Qo, lo_ = ora.whiten_evd(Phi32, eps=1e-5)
    assert relF(T, To) < 1e-4 and relF(Q, Qo) < 1e-4
    assert np.max(np.abs(lam - lo_)) <= 1e-6 * lo_[0] and np.all(np.diff(lam) <= 0)
    # whitening identity on the part of the spectrum that is not clamped (eq. (whitening))
    P = Phi32.astype(np.float64)
    if lo_[-1] > 1e-5:
        assert np.linalg.norm(T @ P @ T.T - np.eye(M)) / np.sqrt(M) < 1e-3
    assert np.array_equal(T, T.T) and np.array_equal(Q, Q.T)


def test_gain_variant_and_smoothing():
    M = 48
    Phi32 = wl.spd_matrix(8, M, np.logspace(1, -3, M)).astype(np.float32)
    Qs0 = np.eye(M, dtype=np.float32)
    Qs = dev(Qs0)
    T, Q, lam = run_evd(Phi32, Qs=Qs, gain_mode=1, g_max=10.0, beta=0.95)
    To, Qo, lo_ = ora.whiten_evd(Phi32, gain_mode=1, g_max=10.0)
    assert relF(T, To) < 1e-4 and relF(Q, Qo) < 1e-4
    assert relF(Qs.cpu().numpy(), ora.smooth_Q(Qs0, Qo, 0.95)) < 1e-5


def test_clamped_and_degenerate_spectrum():
    M = 40
    lam = np.r_[np.full(10, 2.0), np.full(10, 0.5), np.logspace(-4, -9, 20)]
    Phi32 = wl.spd_matrix(9, M, lam).astype(np.float32)
    T, Q, l = run_evd(Phi32, eps=1e-5)
    To, Qo, lo_ = ora.whiten_evd(Phi32, eps=1e-5)
    assert relF(T, To) < 1e-4 and relF(Q, Qo) < 1e-4


def test_config1_full_whitening():
    L = wl.config1()
    mu, Phi, phi, lbar = ora.block_moments(L.act, 0.0, True)
    Phi32 = Phi.astype(np.float32)
    T, Q, lam = run_evd(Phi32)
    To, Qo, lo_ = ora.whiten_evd(Phi32)
    assert relF(T, To) < 1e-4 and relF(Q, Qo) < 1e-4
    assert np.linalg.norm(T @ Phi32.astype(np.float64) @ T.T - np.eye(64)) / 8 < 1e-3
