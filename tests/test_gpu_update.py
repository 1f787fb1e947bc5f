"""GPU parity of the companions of the gradient transform: per-tap transform, fused weight update, bias compensation
(Sec. 3.1, eqs. (vtWrn_SGD), (mod_weight_grad), (vtb_corr)) and the monitoring figures of Sec. 6 (eq. (rho), kappa)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import CondRunner, b, dev, ora, relF, workspace, DEV

pytestmark = pytest.mark.gpu


def sym_q(M, seed):
    rng = np.random.default_rng(seed)
    T = np.eye(M) + 0.2 * rng.standard_normal((M, M)) / np.sqrt(M)
    return (T.T @ T).astype(np.float32)


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("S,M,taps,dtype", [(5, 8, 9, "f32"), (33, 64, 9, "f32"), (64, 130, 9, "bf16"), (17, 67, 4, "f32"),
                                            (40, 256, 9, "bf16"), (3, 5, 1, "f32"), (128, 512, 9, "f32"), (12, 96, 49, "bf16"),
                                            (44, 3072, 9, "f32"), (41, 3076, 9, "bf16")])   # large products: split form
def test_per_tap_transform(S, M, taps, dtype):
    rng = np.random.default_rng(S * 1000 + M)
    G = (0.03 * rng.standard_normal((S, M, taps))).astype(np.float32)
    if dtype == "bf16":
        G = wl.round_to_bf16(G)
    Q = sym_q(M, M)
    tdt, dt = (torch.bfloat16, b.FW_BF16) if dtype == "bf16" else (torch.float32, b.FW_F32)
    Gd = dev(G, tdt)
    out = torch.full_like(Gd, float("nan"))
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM_TAPS, M, S * taps, None, dt))
    b.fw_grad_transform_taps(Gd, dt, S, M, taps, dev(Q), out, ws)
    torch.cuda.synchronize()
    k = int(round(np.sqrt(taps)))
    if k * k == taps:
        want = ora.grad_transform_taps(G.reshape(S, M, k, k), Q).reshape(S, M, taps)
    else:
        want = np.stack([ora.grad_transform(G[:, :, t], Q) for t in range(taps)], axis=2)
    assert relF(host(out), want) < (1e-4 if dtype == "f32" else 2e-2)
    if dtype == "bf16":   # float32 products, one rounding at the end: each element within half a bfloat16 ulp
        assert np.all(np.abs(host(out) - want) <= np.abs(want) * 2.0 ** -8 + 1e-6)   # + float32 error of the sum


@pytest.mark.parametrize("S,M,taps,dtype,mom,wd", [(32, 64, 1, "f32", 0.0, 0.0), (64, 576, 1, "f32", 0.9, 5e-4), (19, 67, 1, "f32", 0.9, 1e-4),
                                                   (48, 128, 9, "f32", 0.9, 5e-4), (40, 256, 1, "bf16", 0.9, 5e-4),
                                                   (33, 96, 9, "bf16", 0.5, 0.0), (512, 2304, 1, "f32", 0.9, 1e-4),
                                                   # large products with the workspace: the product takes the split form
                                                   (400, 3072, 1, "f32", 0.9, 5e-4), (370, 3076, 1, "bf16", 0.9, 5e-4),
                                                   (48, 3072, 9, "f32", 0.5, 1e-4), (1100, 1536, 1, "f32", 0.9, 5e-4)])
def test_fused_weight_update(S, M, taps, dtype, mom, wd):
    rng = np.random.default_rng(S + 7 * M + taps)
    shape = (S, M) if taps == 1 else (S, M, taps)
    W0 = rng.standard_normal(shape).astype(np.float32)
    Q = sym_q(M, M + 1)
    tdt, dt = (torch.bfloat16, b.FW_BF16) if dtype == "bf16" else (torch.float32, b.FW_F32)
    Wd = dev(W0)
    Vd = torch.zeros_like(Wd) if mom > 0 else None
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_SGD_UPDATE, M, S * taps, None, dt))
    prm = b.sgd_params(0.1, mom, wd)
    W_o, V_o = W0.astype(np.float64), None
    for step in range(3):
        G = (0.05 * rng.standard_normal(shape)).astype(np.float32)
        if dtype == "bf16":
            G = wl.round_to_bf16(G)
        b.fw_sgd_update(dev(G, tdt), dt, S, M, taps, dev(Q), prm, Wd, Vd, ws if (dtype == "bf16" or taps > 1 or M >= 1536) else None)
        torch.cuda.synchronize()
        # teacher-forced: the oracle starts every update from the GPU's previous float32 state
        W_prev = W_o
        if taps == 1:
            W_o, V_o = ora.sgd_update(W_prev, V_o, G, Q, 0.1, mom, wd)
        else:
            cols = [ora.sgd_update(W_prev[:, :, t], None if V_o is None else V_o[:, :, t], G[:, :, t], Q, 0.1, mom, wd) for t in range(taps)]
            W_o, V_o = np.stack([c[0] for c in cols], axis=2), np.stack([c[1] for c in cols], axis=2)
        assert relF(host(Wd) - W_prev, W_o - W_prev) < 1e-4, f"step {step}"     # the change itself, not W (it is tiny against W)
        if Vd is not None:
            assert relF(host(Vd), V_o) < 1e-4
            V_o = host(Vd)
        else:
            V_o = None
        W_o = host(Wd)


def test_update_rejects_bad_arguments():
    S, M = 8, 16
    G, W, Q = torch.zeros(S, M, device=DEV), torch.zeros(S, M, device=DEV), torch.eye(M, device=DEV)
    with pytest.raises(RuntimeError):
        b.fw_sgd_update(G, b.FW_F32, S, M, 1, Q, b.sgd_params(0.1, 0.9), W, None)          # momentum without a buffer
    with pytest.raises(RuntimeError):
        b.fw_sgd_update(G, b.FW_F32, S, M, 9, Q, b.sgd_params(0.1), W, None)                # per-tap without workspace
    with pytest.raises(RuntimeError):
        b.fw_sgd_update(W, b.FW_F32, S, M, 1, Q, b.sgd_params(0.1), W, None)                # gradient aliases the weights
    with pytest.raises(RuntimeError):
        b.fw_grad_transform_taps(G, b.FW_F32, S, M, 1, Q, G, workspace(1 << 16))           # in place
    torch.cuda.synchronize()
    assert float(W.abs().sum()) == 0.0


@pytest.mark.parametrize("S,M,taps", [(3, 5, 1), (64, 576, 1), (33, 64, 9), (1000, 512, 1)])
def test_bias_compensation(S, M, taps):
    rng = np.random.default_rng(S + M)
    shape = (S, M) if taps == 1 else (S, M, taps)
    W = rng.standard_normal(shape).astype(np.float32)
    b0 = rng.standard_normal(S).astype(np.float32)
    mu0, mu1 = rng.standard_normal(M).astype(np.float32), rng.standard_normal(M).astype(np.float32)
    bd = dev(b0)
    b.fw_bias_compensate(bd, dev(W), S, M, taps, dev(mu0), dev(mu1))
    torch.cuda.synchronize()
    Wsum = W.astype(np.float64) if taps == 1 else W.astype(np.float64).sum(axis=2)
    want = ora.bias_compensation(b0, Wsum, 1, mu0, mu1)
    assert np.allclose(host(bd), want, rtol=1e-5, atol=1e-5)
    # the property the rule exists for: the layer output does not move with the mean
    x = rng.standard_normal(M)
    assert np.allclose(Wsum @ (x - mu0) + b0, Wsum @ (x - mu1) + host(bd), atol=1e-3)


@pytest.mark.parametrize("M", [5, 64, 577, 2304])
def test_diagnostics(M):
    rng = np.random.default_rng(M)
    lam = np.sort(rng.uniform(0.0, 1.0, M) ** 4)[::-1].astype(np.float32)
    lam[-1] = -1e-7                                     # a rounding-negative eigenvalue counts as zero
    A = rng.standard_normal((M, M)) / np.sqrt(M)
    P = (A @ A.T + np.diag(rng.uniform(0.5, 1.5, M))).astype(np.float32)
    P = ((P + P.T) / 2).astype(np.float32)
    out = torch.full((4,), float("nan"), device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_DIAGNOSTICS, M))
    b.fw_diagnostics(dev(P), dev(lam), M, out, ws)
    torch.cuda.synchronize()
    rho, kappa, ms = (float(v) for v in out[:3])
    assert rho == pytest.approx(ora.whiteness(P.astype(np.float64)), rel=1e-5)
    assert kappa == pytest.approx(ora.normalized_rank(lam.astype(np.float64)), rel=1e-5)
    assert ms == pytest.approx(ora.aic_signal_rank(lam.astype(np.float64)), rel=1e-5)
    # the stated extremes: a diagonal matrix is perfectly white, equal eigenvalues have full rank
    out.fill_(float("nan"))
    b.fw_diagnostics(dev(np.diag(rng.uniform(0.5, 2.0, M))), None, M, out, ws)
    b.fw_diagnostics(None, dev(np.full(M, 0.3)), M, out)
    torch.cuda.synchronize()
    assert float(out[0]) == pytest.approx(1.0, rel=1e-6) and float(out[1]) == pytest.approx(1.0, rel=1e-5)
    u = rng.uniform(0.5, 2.0, M)
    b.fw_diagnostics(dev(np.outer(u, u)), None, M, out, ws)
    torch.cuda.synchronize()
    assert float(out[0]) == pytest.approx(1.0 / M, rel=1e-4)


@pytest.mark.parametrize("M,k", [(8, 8), (33, 6), (200, 16), (577, 16), (2304, 12), (64, 32), (2500, 10), (4608, 16)])
def test_condition_probe_against_the_oracle(M, k):
    """Extreme Ritz values of a symmetric positive definite matrix on a k-dimensional Krylov space: the GPU's Lanczos
    recurrence against the oracle's projection form, same start vector.  Both work in float64 on the float32 matrix, so
    what is left is the rounding of the float32 outputs and of a differently ordered orthogonalisation."""
    rng = np.random.default_rng(1000 + M)
    P = wl.spd_matrix(M, M, np.logspace(1.0, -2.0, M)).astype(np.float32)
    P = ((P + P.T) / 2).astype(np.float32)
    b0 = rng.standard_normal(M).astype(np.float32)
    out = torch.full((4,), float("nan"), device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_COND_PROBE, M, k))
    b.fw_cond_probe(dev(P), M, dev(b0), k, out, ws)
    torch.cuda.synchronize()
    hi, lo, cond, steps = ora.condition_probe(P.astype(np.float64), b0.astype(np.float64), k)
    g_hi, g_lo, g_cond, g_steps = (float(v) for v in out)
    assert int(g_steps) == steps == min(k, M)
    assert g_hi == pytest.approx(hi, rel=2e-6) and g_lo == pytest.approx(lo, rel=2e-6) and g_cond == pytest.approx(cond, rel=4e-6)
    # never an overestimate of the true condition number
    w = np.linalg.eigvalsh(P.astype(np.float64))
    assert g_cond <= w[-1] / w[0] * (1 + 1e-5)


def test_condition_probe_special_cases():
    # invariant subspace: the start vector lives in the span of two eigenvectors -> stops at dimension 2, exact there
    P = np.diag([7.0, 3.0, 2.0, 1.0, 0.5]).astype(np.float32)
    b0 = np.array([1.0, 0.0, 1.0, 0.0, 0.0], dtype=np.float32)
    out = torch.full((4,), float("nan"), device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_COND_PROBE, 5, 5))
    b.fw_cond_probe(dev(P), 5, dev(b0), 5, out, ws)
    torch.cuda.synchronize()
    assert [float(v) for v in out] == pytest.approx([7.0, 2.0, 3.5, 2.0], rel=1e-6)
    assert ora.condition_probe(P.astype(np.float64), b0.astype(np.float64), 5)[3] == 2
    # default start vector (all ones); a white matrix has condition number 1 after a single step
    b.fw_cond_probe(dev(np.eye(5) * 0.3), 5, None, 4, out, ws)
    torch.cuda.synchronize()
    assert [float(v) for v in out] == pytest.approx([0.3, 0.3, 1.0, 1.0], rel=1e-6)
    want = ora.condition_probe(P.astype(np.float64), np.ones(5), 3)
    b.fw_cond_probe(dev(P), 5, None, 3, out, ws)
    torch.cuda.synchronize()
    assert [float(v) for v in out] == pytest.approx(list(want), rel=2e-6)


def test_condition_probe_follows_the_recursion():
    """The figure the recursion is built to reduce: probe Phi_y before and after a run of steps; the estimate drops with
    the true condition number and stays below it."""
    M = 96
    Phi = wl.spd_matrix(5, M, np.logspace(2.0, -2.0, M)).astype(np.float32)
    run = CondRunner(Phi, float(np.trace(Phi) / M))
    out = torch.zeros(4, device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_COND_PROBE, M, 24))
    b.fw_cond_probe(run.Phi_y, M, None, 24, out, ws)
    torch.cuda.synchronize()
    before = float(out[2])
    gp = b.cond_params()
    for _ in range(40):
        run.step(gp)
    b.fw_cond_probe(run.Phi_y, M, None, 24, out, ws)
    torch.cuda.synchronize()
    after = float(out[2])
    w = np.linalg.eigvalsh(run.host("Phi_y"))
    assert after < before / 3 and after <= w[-1] / w[0] * (1 + 1e-5)
    assert float(out[0]) == pytest.approx(w[-1], rel=1e-3)


def test_condition_probe_breakdown_with_many_features():
    """The form for many features (the step spread over several workgroups): an invariant subspace of dimension 3 stops the
    recurrence there, on the device, and the later launches of the call do nothing."""
    M = 3000
    d = np.full(M, 0.25, dtype=np.float32)
    d[7], d[1234], d[2999] = 9.0, 4.0, 1.0
    b0 = np.zeros(M, dtype=np.float32)
    b0[7] = b0[1234] = b0[2999] = 1.0
    out = torch.full((4,), float("nan"), device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_COND_PROBE, M, 12))
    b.fw_cond_probe(torch.diag(dev(d)).contiguous(), M, dev(b0), 12, out, ws)
    torch.cuda.synchronize()
    assert [float(v) for v in out] == pytest.approx([9.0, 1.0, 9.0, 3.0], rel=1e-6)
    assert ora.condition_probe(np.diag(d.astype(np.float64)), b0.astype(np.float64), 12)[3] == 3


def test_matrix_core_rate_probe():
    """The measurement kernel behind the bench's ceiling: runs, reports its flops, and multiplying zeros is not slower than
    multiplying pseudo-random values (the chip is power-limited under dense matrix instructions)."""
    sink = torch.zeros(4, device=DEV)
    rates = {}
    for zero in (0, 1):
        b.fw_mfma_rate_probe(zero, 200, sink); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = sum(b.fw_mfma_rate_probe(zero, 200, sink) for _ in range(5))
        e1.record(); torch.cuda.synchronize()
        assert flops == 5 * 4096 * 200 * 16 * 2 * 32 * 32 * 16
        rates[zero] = flops / (e0.elapsed_time(e1) * 1e-3)
    assert float(sink.abs().sum()) == 0.0                      # the sink is never written
    assert 0.3e15 < rates[0] < 2.6e15 and rates[1] > 0.9 * rates[0]

