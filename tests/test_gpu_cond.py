"""GPU parity of the recursive condition-number reduction (Sec. 4) against the CPU oracle.

The step is iterated and data dependent, so parity is judged teacher-forced: before every GPU step the oracle is
given the GPU's own state (T, Q, Qs up-cast to float64) and both take one step; T, Q, Qs, Phi_y, lambda_e, g_e are
compared after it.  The integer decisions (arg-max m', membership in the coherence set) must agree unless the deciding
margin is within rounding distance, in which case the oracle is re-run with the GPU's decision."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import BAND, CondRunner, b, dev, forced_step, ora, relF, workspace

pytestmark = pytest.mark.gpu


def teacher_forced(Phi_x, lbar, prm_kw, steps, tol=1e-4):
    M = Phi_x.shape[0]
    Phi32 = Phi_x.astype(np.float32)
    run = CondRunner(Phi32, lbar, gamma_lt_one=prm_kw.get("gamma", 0.99) < 1.0)
    gp = b.cond_params(**prm_kw)
    op = ora.CondParams(gamma=gp.gamma, delta=gp.delta, eps=gp.eps, c_rel=gp.c_rel, c_abs=gp.c_abs, beta=gp.beta,
                        n_power_iters=gp.n_power_iters, guard=bool(gp.guard))
    # initial state
    assert np.array_equal(run.host("T"), np.eye(M)) and np.array_equal(run.host("Phi_y"), Phi32.astype(np.float64))
    assert relF(run.host("xi2"), np.sum(Phi32.astype(np.float64) ** 2, axis=0)) < 1e-6
    applied = 0
    worst = 0.0
    lbar32 = float(np.float32(lbar))
    P64 = Phi32.astype(np.float64)
    compared = 0
    for k in range(steps):
        ok, info, oi, new = forced_step(run, P64, lbar32, gp, op, tol, label=f"step {k}")
        if not ok:
            continue
        compared += 1
        applied += int(oi.applied)
    assert compared >= max(1, steps // 2), "too few steps were compared element by element"
    return run, applied, worst


def spd(M, seed, hi=2.0, lo=-2.0):
    return wl.spd_matrix(seed, M, np.logspace(hi, lo, M))


@pytest.mark.parametrize("M", [8, 33, 64, 100, 200])
@pytest.mark.parametrize("kw", [dict(gamma=1.0, beta=0.0), dict(), dict(gamma=0.9, beta=0.5, n_power_iters=2)])
def test_teacher_forced_steps(M, kw):
    Phi = spd(M, M)
    run, applied, worst = teacher_forced(Phi, np.trace(Phi) / M, kw, steps=8)
    assert applied >= 2


def test_invariants_free_running():
    """After many free-running steps Q = T^T T and Phi_y = T Phi_x T^T still hold, and the condition number has dropped."""
    M = 96
    Phi = spd(M, 5).astype(np.float32).astype(np.float64)
    lbar = np.trace(Phi) / M
    run = CondRunner(Phi, lbar)
    gp = b.cond_params()
    for _ in range(40):
        run.step(gp)
    T = run.host("T")
    assert relF(run.host("Q"), T.T @ T) < 1e-4
    assert relF(run.host("Phi_y"), T @ Phi @ T.T) < 1e-4
    assert relF(run.host("Psi"), T @ Phi) < 1e-4
    assert np.linalg.cond(T @ Phi @ T.T) < np.linalg.cond(Phi) / 5


def test_guard_and_empty_set_flags():
    M = 16
    Phi = np.diag(np.linspace(1.0, 0.5, M))
    run = CondRunner(Phi, 1.0)
    info = run.step(b.cond_params(delta=4.0))           # target above every eigenvalue
    assert info.applied == 0 and info.flags & 2 and info.a_e == 0.0
    assert relF(run.host("T"), 0.99 * np.eye(M) + 0.01 * np.eye(M)) < 1e-6
    run2 = CondRunner(1e-6 * Phi, 1.0)
    info2 = run2.step(b.cond_params())
    assert info2.set_size == 0 and info2.flags & 1 and info2.applied == 0
    assert np.allclose(run2.host("T"), np.eye(M))


def test_config1_sixteen_steps():
    """Config 1: covariance of the ill-conditioned fully connected layer, 16 steps with the paper's hyper-parameters."""
    L = wl.config1()
    mu, Phi, phi, lbar = ora.block_moments(L.act, 0.0, True)
    run, applied, worst = teacher_forced(Phi, lbar, dict(), steps=16)
    assert applied >= 8


@pytest.mark.parametrize("split", [False, True])
@pytest.mark.parametrize("M,leak", [(96, True), (130, True), (64, False), (70, False), (147, True), (1152, True), (1536, True), (1600, False), (2304, True)])
def test_refresh_for_a_new_block(M, leak, split):
    """A new block changes Phi_x while T carries over: Psi, Phi_y and the column norms are rebuilt for the T at hand, and
    the next steps agree with the oracle, which forms T Phi_x T^T explicitly from the new Phi_x.  Both forms of the two
    products: plain float32 (no workspace beyond a stand-in for Psi) and bfloat16 hi + lo splits (full workspace), whose
    operands carry 16 significant bits: relative residual 2^-17 per operand, about 2^-16 = 1.5e-5 per product term at
    worst and a few 1e-6 in Frobenius norm, hence the tolerance 2e-5 there."""
    Phi1 = spd(M, 11).astype(np.float32).astype(np.float64)
    Phi2 = spd(M, 12, hi=1.5, lo=-1.0).astype(np.float32).astype(np.float64)
    kw = dict() if leak else dict(gamma=1.0, beta=0.0)
    gp = b.cond_params(**kw)
    op = ora.CondParams(gamma=gp.gamma, delta=gp.delta, eps=gp.eps, c_rel=gp.c_rel, c_abs=gp.c_abs, beta=gp.beta)
    run = CondRunner(Phi1, np.trace(Phi1) / M, gamma_lt_one=leak)
    for _ in range(6):
        run.step(gp)
    T = run.host("T")
    assert not np.allclose(T, np.eye(M))
    run.Phi_x.copy_(dev(Phi2))
    lbar2 = float(np.float32(np.trace(Phi2) / M))
    run.lbar.fill_(lbar2)
    full = b.fw_workspace_bytes(b.FW_OP_COND_STATE_REFRESH, M)
    assert full >= 4 * 4 * M * M
    if split:
        ws = workspace(full)
    else:
        ws = None if leak else workspace((4 * M * M + 255) // 256 * 256)   # room for Psi only: the float32 form
    b.fw_cond_state_refresh(run.st, ws)
    torch.cuda.synchronize()
    tol = 2e-5 if split else 1e-5
    want = ora.transformed_covariance(T, Phi2)
    Py = run.host("Phi_y")
    e_py = relF(Py, want)
    print(f"M={M} split={split}: rel-F(Phi_y) = {e_py:.2e}")
    assert e_py < tol and np.array_equal(Py, Py.T)
    if split and M >= b.FW_REFRESH_SPLIT_MIN_M:
        assert e_py > 1e-6, "the split form was due but the error is that of plain float32"
    else:
        assert e_py < 1e-6, "plain float32 was due"
    if leak:
        assert relF(run.host("Psi"), T @ Phi2) < tol
    assert relF(run.host("xi2"), np.sum(want ** 2, axis=0)) < 2 * tol
    assert np.array_equal(run.host("T"), T)
    for _ in range(3):   # teacher-forced steps on the new block
        st = ora.CondState(Phi2, run.host("T"), run.host("Q"), run.host("Qs"))
        info = run.step(gp)
        new, oi = ora.cond_reduce_step(st, lbar2, op)
        if info.m_prime != oi.m_prime or info.set_size != oi.set_size:
            continue
        assert max(relF(run.host("T"), new.T), relF(run.host("Q"), new.Q), relF(run.host("Qs"), new.Qs)) < 1e-4
    Tn = run.host("T")
    assert relF(run.host("Phi_y"), Tn @ Phi2 @ Tn.T) < 1e-4


@pytest.mark.timeout(600)
def test_refresh_at_the_largest_config_size():
    """M = 4608, as the benchmark calls it (whole workspace: both products in the split form on 192 x 256 tiles, the second
    on the lower triangle only): Psi, Phi_y and the column norms against explicit float64 products."""
    M = 4608
    Phi1 = spd(M, 21).astype(np.float32).astype(np.float64)
    Phi2 = spd(M, 22, hi=1.5, lo=-1.0).astype(np.float32).astype(np.float64)
    gp = b.cond_params()
    run = CondRunner(Phi1, np.trace(Phi1) / M, gamma_lt_one=True)
    for _ in range(8):
        run.step(gp)
    T = run.host("T")
    assert not np.allclose(T, np.eye(M))
    run.Phi_x.copy_(dev(Phi2))
    run.lbar.fill_(float(np.float32(np.trace(Phi2) / M)))
    full = b.fw_workspace_bytes(b.FW_OP_COND_STATE_REFRESH, M)
    assert b.fw_cond_refresh_plan_query(M, full).split == 1
    b.fw_cond_state_refresh(run.st, workspace(full))
    torch.cuda.synchronize()
    Psi_o = T @ Phi2
    want = Psi_o @ T.T
    Py = run.host("Phi_y")
    e_psi, e_py = relF(run.host("Psi"), Psi_o), relF(Py, want)
    print(f"M={M}: rel-F(Psi) = {e_psi:.2e}, rel-F(Phi_y) = {e_py:.2e}")
    assert e_psi < 2e-5 and e_py < 2e-5 and np.array_equal(Py, Py.T)
    assert relF(run.host("xi2"), np.sum(want ** 2, axis=0)) < 4e-5
