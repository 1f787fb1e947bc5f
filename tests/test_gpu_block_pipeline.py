"""Block pipeline through the C-ABI (Sec. 2: moments re-estimated block by block with forgetting; Sec. 4: the recursion
continues on the transformed covariance of the new block; Sec. 3.1: gradients multiplied by the smoothed Q).

Several blocks of L batches each with drifting statistics.  Per block: L covariance calls into one (A, s), one finalize
with the recursive average, the state refresh for the T carried over, K recursive steps, one gradient transform.  The
oracle side stacks the patch rows of the block and applies its own block moments; the recursive steps are compared
teacher-forced (oracle step applied to the GPU's previous state in float64), as in the single-block tests."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import b, dev, desc_of, dt_of, ora, oracle_rows, relF, upload_act, workspace, DEV

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def drifting_batches(dtype, n_blocks, L, seed0):
    """L x n_blocks small conv batches; the channel amplitudes change from block to block, so Phi_x really moves."""
    out = []
    for i in range(n_blocks):
        amp = 1.0 + 0.5 * np.cos(0.9 * i + np.arange(8))
        blk = []
        for l in range(L):
            lay = wl.small_conv(seed0 + 10 * i + l, B=6, Cin=8, H=10, W=9, k=3, stride=1, pad=1, S=20, dtype="f32")
            act = lay.act * amp[None, None, None, :]
            if dtype == "bf16":
                act = wl.round_to_bf16(act)
            blk.append(wl.Layer(lay.name, lay.desc, lay.S, dtype, act.astype(np.float32), lay.G))
        out.append(blk)
    return out


@pytest.mark.parametrize("dtype,layout", [("f32", 2), ("f32", 1), ("bf16", 2), ("bf16", 3)])
def test_blocks_with_forgetting(dtype, layout):
    n_blocks, L, K, alpha = 3, 2, 4, 0.6
    blocks = drifting_batches(dtype, n_blocks, L, 500)
    d0 = blocks[0][0].desc
    M, S = d0.M, blocks[0][0].S
    A = torch.zeros(M, M, device=DEV); s = torch.zeros(M, device=DEV)
    mu = torch.zeros(M, device=DEV); Phi = torch.zeros(M, M, device=DEV); phi = torch.zeros(M, device=DEV)
    lbar = torch.zeros(4, device=DEV)
    T, Q, Qs, Py, Psi = (torch.empty(M, M, device=DEV) for _ in range(5))
    xi2 = torch.empty(M, device=DEV)
    info = torch.zeros(8, dtype=torch.int32, device=DEV)
    st = b.cond_state(M, Phi, lbar, T, Q, Qs, Py, Psi, xi2)
    ws_cov = workspace(b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, M, 0, desc_of(blocks[0][0]), dt_of(blocks[0][0])))
    ws_cond = workspace(b.fw_workspace_bytes(b.FW_OP_COND_REDUCE_STEP, M))
    gp = b.cond_params()
    op = ora.CondParams(gamma=gp.gamma, delta=gp.delta, eps=gp.eps, c_rel=gp.c_rel, c_abs=gp.c_abs, beta=gp.beta)
    host = lambda t: t.cpu().numpy().astype(np.float64)
    mu_o = Phi_o = phi_o = None
    applied = 0
    for i, blk in enumerate(blocks):
        A.zero_(); s.zero_()
        rows = []
        for layer in blk:
            X, lay = upload_act(layer, layout)
            b.fw_cov_accumulate(X, dt_of(layer), lay, desc_of(layer), A, s, ws_cov)
            rows.append(oracle_rows(layer, layout))
        rows = np.concatenate(rows, axis=0)
        b.fw_cov_finalize(A, s, rows.shape[0], M, alpha, 1 if i == 0 else 0, mu, Phi, phi, lbar)
        mu_o, Phi_o, phi_o, lbar_o = ora.block_moments(rows, alpha, i == 0, mu_o, Phi_o, phi_o)
        torch.cuda.synchronize()
        assert relF(host(Phi), Phi_o) < TOL[dtype], f"block {i}"
        assert relF(host(mu), mu_o) < 1e-5 and relF(host(phi), phi_o) < 1e-5
        assert abs(float(lbar[0]) - lbar_o) < 1e-5 * lbar_o
        if i == 0:
            b.fw_cond_state_init(st)
        else:
            b.fw_cond_state_refresh(st)
        torch.cuda.synchronize()
        P64, lb32 = host(Phi), float(lbar[0])
        assert np.array_equal(P64, P64.T)
        assert relF(host(Py), ora.transformed_covariance(host(T), P64)) < 1e-5, f"block {i}"
        for k in range(K):
            prev = ora.CondState(P64, host(T), host(Q), host(Qs))
            b.fw_cond_reduce_step(st, gp, info, ws_cond)
            torch.cuda.synchronize()
            gi = b.read_cond_info(info)
            new, oi = ora.cond_reduce_step(prev, lb32, op)
            if gi.m_prime != oi.m_prime or gi.set_size != oi.set_size:
                assert oi.xi[gi.m_prime] >= oi.xi[oi.m_prime] * (1 - 2e-5)
                continue
            applied += int(oi.applied)
            errs = [relF(host(T), new.T), relF(host(Q), new.Q), relF(host(Qs), new.Qs),
                    relF(host(Py), ora.transformed_covariance(new.T, P64)), relF(host(Psi), new.T @ P64)]
            assert max(errs) < 1e-4, f"block {i} step {k}: {errs}"
        G = blk[-1].G
        Gout = torch.empty(S, M, device=DEV)
        b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, Qs, Gout)
        torch.cuda.synchronize()
        assert relF(host(Gout), ora.grad_transform(G.astype(np.float64), host(Qs))) < 1e-4
    assert applied >= n_blocks      # the recursion really shrank something in every block
    Tn = host(T)
    assert not np.allclose(Tn, np.eye(M), atol=1e-3)
    assert relF(host(Q), Tn.T @ Tn) < 1e-4


@pytest.mark.parametrize("dtype,layout", [("f32", 2), ("bf16", 3)])
def test_blocks_on_the_evd_leg_with_rank_limited_gains(dtype, layout):
    """The EVD variant over several blocks (Sec. 2, Sec. 3.2): block moments with forgetting, eigen-decomposition of every
    block's covariance, gains limited to the estimated signal rank with g_max (eqs. (hMs), (g_mod)), Q smoothed across
    blocks (eq. (vQs), beta = 0.95 as in Sec. 6), gradient multiplied by the smoothed Q.  The oracle does the same block by
    block from its own moments of the GPU's covariance (T, Q are spectral functions of Phi_x: compared, never V)."""
    n_blocks, L, alpha, beta, g_max, eps = 4, 2, 0.9, 0.95, 10.0, 1e-5
    blocks = drifting_batches(dtype, n_blocks, L, 900)
    d0 = blocks[0][0].desc
    M, S = d0.M, blocks[0][0].S
    A = torch.zeros(M, M, device=DEV); s = torch.zeros(M, device=DEV)
    mu = torch.zeros(M, device=DEV); Phi = torch.zeros(M, M, device=DEV); phi = torch.zeros(M, device=DEV)
    lbar = torch.zeros(4, device=DEV)
    T, Q = torch.empty(M, M, device=DEV), torch.empty(M, M, device=DEV)
    Qs = torch.eye(M, device=DEV)                      # Qs(-1) = I
    lam = torch.empty(M, device=DEV)
    diag = torch.zeros(4, device=DEV)
    ws_cov = workspace(b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, M, 0, desc_of(blocks[0][0]), dt_of(blocks[0][0])))
    ws_evd = workspace(b.fw_workspace_bytes(b.FW_OP_WHITEN_EVD, M))
    ep = b.evd_params(eps=eps, g_max=g_max, beta=beta, gain_mode=1)
    host = lambda t: t.cpu().numpy().astype(np.float64)
    mu_o = Phi_o = phi_o = None
    Qs_o = np.eye(M)
    ranks = []
    for i, blk in enumerate(blocks):
        A.zero_(); s.zero_()
        rows = []
        for layer in blk:
            X, lay = upload_act(layer, layout)
            b.fw_cov_accumulate(X, dt_of(layer), lay, desc_of(layer), A, s, ws_cov)
            rows.append(oracle_rows(layer, layout))
        rows = np.concatenate(rows, axis=0)
        b.fw_cov_finalize(A, s, rows.shape[0], M, alpha, 1 if i == 0 else 0, mu, Phi, phi, lbar)
        mu_o, Phi_o, phi_o, lbar_o = ora.block_moments(rows, alpha, i == 0, mu_o, Phi_o, phi_o)
        b.fw_whiten_evd(Phi, M, ep, T, Q, Qs, lam, ws_evd)
        b.fw_diagnostics(None, lam, M, diag)
        torch.cuda.synchronize()
        assert relF(host(Phi), Phi_o) < TOL[dtype], f"block {i}"
        # the oracle continues from the GPU's covariance of this block
        P64 = host(Phi)
        T_o, Q_o, lam_o = ora.whiten_evd(P64, eps=eps, gain_mode=1, g_max=g_max)
        Qs_o = ora.smooth_Q(Qs_o, Q_o, beta)
        assert np.max(np.abs(host(lam) - lam_o)) <= 1e-6 * lam_o[0]
        assert relF(host(T), T_o) < 1e-4 and relF(host(Q), Q_o) < 1e-4, f"block {i}"
        assert relF(host(Qs), Qs_o) < 1e-4, f"block {i}"
        ms = ora.aic_signal_rank(lam_o)
        ranks.append(ora.round_rank(ms, M))
        assert float(diag[2]) == pytest.approx(ms, rel=1e-4)
        # gains really are the rank-limited ones: beyond the signal rank the transform leaves the eigen-directions alone
        g = ora.evd_gains(lam_o, eps, 1, g_max)
        assert np.all(g[ranks[-1]:] == 1.0) and np.all(g[:ranks[-1]] <= g_max)
        Qs_o = host(Qs)                                # carry the GPU's smoothed Q forward: every block is compared on its own
        G = blk[-1].G
        Gout = torch.empty(S, M, device=DEV)
        b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, Qs, Gout)
        torch.cuda.synchronize()
        assert relF(host(Gout), ora.grad_transform(G.astype(np.float64), host(Qs))) < 1e-4
    assert 1 <= min(ranks) and max(ranks) < M          # the rank limit was active
    assert relF(host(Qs), np.eye(M)) > 1e-3            # and the smoothing has moved Qs away from its start


@pytest.mark.parametrize("dtype,Cin,H", [("f32", 64, 20), ("bf16", 128, 14)])
def test_next_batch_accumulated_on_a_second_stream(dtype, Cin, H):
    """The sums of batch k+1 are accumulated on a second stream while batch k's refresh, recursion and gradient product
    run, ordered by two events (the sums are free once finalize has read them; finalize waits for the sums).  The calls
    share nothing but their arguments, so every matrix must come out bit for bit as on one stream."""
    B, S, steps = 16, 48, 5
    lays = [wl.small_conv(900 + i, B=B, Cin=Cin, H=H, W=H, k=3, stride=1, pad=1, S=S, dtype=dtype) for i in range(2)]
    d = desc_of(lays[0])
    dt = dt_of(lays[0])
    M, n_rows = lays[0].desc.M, lays[0].desc.n_rows
    up = [upload_act(l, 2) for l in lays]
    lay = up[0][1]
    Xs = [u[0] for u in up]
    G = torch.as_tensor(lays[0].G).to(DEV)
    gp = b.cond_params()

    def run(two_streams):
        A = torch.zeros(M, M, device=DEV); s = torch.zeros(M, device=DEV)
        mu = torch.zeros(M, device=DEV); Phi = torch.zeros(M, M, device=DEV); phi = torch.zeros(M, device=DEV)
        lbar = torch.zeros(4, device=DEV)
        T, Q, Qs, Py, Psi = (torch.empty(M, M, device=DEV) for _ in range(5))
        xi2 = torch.empty(M, device=DEV)
        info = torch.zeros(8, dtype=torch.int32, device=DEV)
        Gout = torch.empty_like(G)
        st = b.cond_state(M, Phi, lbar, T, Q, Qs, Py, Psi, xi2)
        ws_cov = workspace(b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, M, 0, d, dt))
        ws_cond = workspace(b.fw_workspace_bytes(b.FW_OP_COND_REDUCE_STEP, M))
        ws_ref = workspace(b.fw_workspace_bytes(b.FW_OP_COND_STATE_REFRESH, M))
        ws_grad = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S))
        b.fw_cov_accumulate(Xs[0], dt, lay, d, A, s, ws_cov)
        b.fw_cov_finalize(A, s, n_rows, M, 0.3, 1, mu, Phi, phi, lbar)
        b.fw_cond_state_init(st)
        torch.cuda.synchronize()
        main = torch.cuda.current_stream()
        side = torch.cuda.Stream() if two_streams else main
        sums_read, sums_ready = torch.cuda.Event(), torch.cuda.Event()

        def accumulate(k):
            with torch.cuda.stream(side):
                side.wait_event(sums_read)
                A.zero_(); s.zero_()
                b.fw_cov_accumulate(Xs[k & 1], dt, lay, d, A, s, ws_cov)
                sums_ready.record(side)

        sums_read.record(main)
        accumulate(1)
        for k in range(1, steps + 1):
            main.wait_event(sums_ready)
            b.fw_cov_finalize(A, s, n_rows, M, 0.3, 0, mu, Phi, phi, lbar)
            sums_read.record(main)
            if k < steps:
                accumulate(k + 1)
            b.fw_cond_state_refresh(st, ws_ref)
            b.fw_cond_reduce_step(st, gp, info, ws_cond)
            b.fw_grad_transform(G, b.FW_F32, S, M, None, Qs, Gout, ws_grad)
        main.wait_stream(side)
        torch.cuda.synchronize()
        return [t.clone() for t in (Phi, mu, T, Q, Qs, Py, Psi, xi2, Gout)]

    one = run(False)
    two = run(True)
    for x, y in zip(one, two):
        assert torch.isfinite(x).all()
        assert torch.equal(x, y)
