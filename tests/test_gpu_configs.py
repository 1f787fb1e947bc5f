"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration bench.py times.

Configs 1-4 are small enough for the float64 oracle to compute whole (seconds to tens of seconds); the ResNet-18
sweep of config 5 is checked on sampled covariance entries that the oracle computes one by one from the activation."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import (CondRunner, b, dev, ora, oracle_rows, relF, run_cov, run_finalize, workspace, DEV)

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def full_config_check(layer, layouts, n_forced, n_free, evd, prm_kw=None):
    M, S = layer.desc.M, layer.S
    Phi_dev = None
    for layout in layouts:
        X = oracle_rows(layer, layout)
        mu_o, Phi_o, phi_o, lbar_o = ora.block_moments(X, 0.0, True)
        n = X.shape[0]
        del X
        A, s = run_cov(layer, layout)
        mu, Phi, phi, lbar = run_finalize(A, s, n, M, 0.0, 1)
        e = relF(Phi.cpu().numpy(), Phi_o)
        print(f"{layer.name} layout {layout}: rel-F(Phi_x) = {e:.3e}")
        assert e < TOL[layer.dtype]
        assert relF(mu.cpu().numpy(), mu_o) < 1e-5 and abs(float(lbar[0]) - lbar_o) < 1e-5 * lbar_o
        Phi_dev = Phi
    Phi32 = Phi_dev.cpu().numpy()
    P64 = Phi32.astype(np.float64)
    lbar32 = float(np.float32(lbar_o))

    # recursive steps: teacher-forced first, then free running with the invariants checked at the end
    run = CondRunner(Phi32, lbar32)
    gp = b.cond_params(**(prm_kw or {}))
    op = ora.CondParams(gamma=gp.gamma, delta=gp.delta, eps=gp.eps, c_rel=gp.c_rel, c_abs=gp.c_abs, beta=gp.beta)
    for k in range(n_forced):
        st = ora.CondState(P64, run.host("T"), run.host("Q"), run.host("Qs"))
        info = run.step(gp)
        new, oi = ora.cond_reduce_step(st, lbar32, op)
        if info.m_prime != oi.m_prime or info.set_size != oi.set_size:
            assert oi.xi[info.m_prime] >= oi.xi[oi.m_prime] * (1 - 2e-5)
            assert abs(info.set_size - oi.set_size) <= max(2, oi.set_size // 100)
            continue
        errs = [relF(run.host("T"), new.T), relF(run.host("Q"), new.Q), relF(run.host("Qs"), new.Qs)]
        print(f"{layer.name} step {k}: m'={info.m_prime} |set|={info.set_size} lambda_e={info.lambda_e:.4g} errs={errs}")
        assert max(errs) < 1e-4
        assert abs(info.lambda_e - oi.lambda_e) <= 2e-4 * abs(oi.lambda_e)
    for k in range(n_free):
        run.step(gp)
    T = run.host("T")
    assert relF(run.host("Q"), T.T @ T) < 1e-4
    assert relF(run.host("Phi_y"), T @ P64 @ T.T) < 1e-4
    assert relF(run.host("Psi"), T @ P64) < 1e-4

    # gradient transform with the smoothed Q of the recursion
    Qs = run.Qs
    Gd = dev(layer.G)
    out = torch.empty_like(Gd)
    b.fw_grad_transform(Gd, b.FW_F32, S, M, None, Qs, out)
    torch.cuda.synchronize()
    assert relF(out.cpu().numpy(), ora.grad_transform(layer.G, Qs.cpu().numpy())) < 1e-5
    if layer.dtype == "bf16":
        Gb = wl.round_to_bf16(layer.G)
        outb = torch.empty(S, M, device=DEV, dtype=torch.bfloat16)
        b.fw_grad_transform(dev(Gb, torch.bfloat16), b.FW_BF16, S, M, None, Qs, outb)
        torch.cuda.synchronize()
        assert relF(outb.float().cpu().numpy(), ora.grad_transform(Gb, Qs.cpu().numpy())) < 2e-2
        wsb = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S, None, b.FW_BF16))
        b.fw_grad_transform(dev(Gb, torch.bfloat16), b.FW_BF16, S, M, None, Qs, outb, wsb)
        torch.cuda.synchronize()
        assert relF(outb.float().cpu().numpy(), ora.grad_transform(Gb, Qs.cpu().numpy())) < 3e-3

    if evd:
        Tt = torch.empty(M, M, device=DEV); Qt = torch.empty(M, M, device=DEV); lam = torch.empty(M, device=DEV)
        ws = workspace(b.fw_workspace_bytes(b.FW_OP_WHITEN_EVD, M))
        b.fw_whiten_evd(Phi_dev, M, b.evd_params(), Tt, Qt, None, lam, ws)
        torch.cuda.synchronize()
        To, Qo, lo = ora.whiten_evd(P64)
        eT, eQ = relF(Tt.cpu().numpy(), To), relF(Qt.cpu().numpy(), Qo)
        print(f"{layer.name} EVD: rel-F(T) = {eT:.3e}, rel-F(Q) = {eQ:.3e}")
        assert eT < 1e-4 and eQ < 1e-4
        assert np.max(np.abs(lam.cpu().numpy() - lo)) <= 1e-6 * lo[0]
        # gradient through the EVD path: T given, Q built inside
        ws2 = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S))
        b.fw_grad_transform(Gd, b.FW_F32, S, M, Tt, None, out, ws2)
        torch.cuda.synchronize()
        assert relF(out.cpu().numpy(), ora.grad_transform(layer.G, ora.Q_from_T(Tt.cpu().numpy()))) < 1e-5


def test_config1_pipeline():
    full_config_check(wl.config1(), [b.FW_LAYOUT_ROWS], n_forced=16, n_free=0, evd=True)


def test_config2_cifar_layer():
    full_config_check(wl.config2(), [b.FW_LAYOUT_NCHW, b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC], n_forced=6, n_free=26, evd=False)


def test_config3_resnet50_14x14():
    full_config_check(wl.config3(), [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC], n_forced=3, n_free=61, evd=True)


def test_config4_resnet50_7x7():
    full_config_check(wl.config4(), [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC], n_forced=2, n_free=62, evd=True)


@pytest.mark.parametrize("index", list(range(len(wl.RESNET18_LAYERS))))
def test_config5_resnet18_layer_sampled(index):
    """Full-size layer of the ResNet-18 sweep: sampled covariance entries against the oracle, one entry at a time."""
    layer = wl.config5_layer(index)
    d = layer.desc
    M = d.M
    A, s = run_cov(layer, b.FW_LAYOUT_NHWC)
    mu, Phi, phi, lbar = run_finalize(A, s, d.n_rows, M, 0.0, 1)
    Ph = Phi.cpu().numpy()
    rng = np.random.default_rng(index)
    feats = sorted(set([0, M - 1, M // 2] + list(rng.integers(0, M, 5))))
    if layer.is_rows:
        cols = {m: np.asarray(layer.act[:, m], dtype=np.float64) for m in feats}
    else:
        cols = {m: ora.patch_feature_column(layer.act, *d.astuple(), m) for m in feats}
    mus = {m: cols[m].mean() for m in feats}
    want = np.array([[ora.cov_entry_centered(cols[i], cols[j], mus[i], mus[j]) for j in feats] for i in feats])
    got = Ph[np.ix_(feats, feats)]
    assert relF(got, want) < 2e-2
    assert relF(mu.cpu().numpy()[feats], np.array([mus[m] for m in feats])) < 1e-4
    # properties that hold at any size
    assert np.array_equal(Ph, Ph.T) and np.all(np.diag(Ph) >= 0)
    assert abs(float(lbar[0]) - float(phi.mean())) < 1e-5 * float(lbar[0])
