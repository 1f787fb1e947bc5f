"""Pins for the CPU oracle: each test ties an oracle function to something other than itself --
a hand-worked fixture, a closed form, an identity the paper states, a library routine on a
special case, or brute force on a tiny input.  CPU only."""
import numpy as np
import pytest

import workloads as wl
from conftest import golden
from oracle import fw_oracle as ora

rng0 = np.random.default_rng(1234)


# ----------------------------------------------------------------------------- unfolding
def test_unfold_matches_hand_enumeration():
    want = np.array(golden("unfold_3x3_single_channel.txt"), dtype=float)
    img = np.arange(1, 10, dtype=float).reshape(1, 3, 3, 1)
    got = ora.patch_rows(img, 1, 1, 3, 3, 3, 3, 1, 1)
    assert got.shape == (9, 9)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("B,Cin,H,W,k,stride,pad", [(2, 3, 5, 4, 3, 1, 1), (2, 2, 7, 6, 3, 2, 1), (1, 3, 9, 9, 7, 2, 3),
                                                  (2, 4, 6, 6, 1, 2, 0), (3, 5, 1, 1, 1, 1, 0)])
def test_unfold_matches_six_nested_loops(B, Cin, H, W, k, stride, pad):
    act = rng0.standard_normal((B, H, W, Cin))
    Ho = (H + 2 * pad - k) // stride + 1
    Wo = (W + 2 * pad - k) // stride + 1
    want = np.zeros((B * Ho * Wo, Cin * k * k))
    for b in range(B):
        for oy in range(Ho):
            for ox in range(Wo):
                for c in range(Cin):
                    for ky in range(k):
                        for kx in range(k):
                            iy, ix = oy * stride + ky - pad, ox * stride + kx - pad
                            if 0 <= iy < H and 0 <= ix < W:
                                want[(b * Ho + oy) * Wo + ox, (c * k + ky) * k + kx] = act[b, iy, ix, c]
    got = ora.patch_rows(act, B, Cin, H, W, k, k, stride, pad)
    assert np.array_equal(got, want)
    for m in (0, Cin * k * k - 1, (Cin * k * k) // 2):
        col = ora.patch_feature_column(act, B, Cin, H, W, k, k, stride, pad, m)
        assert np.array_equal(col, want[:, m])


def test_unfold_channels_last_feature_order():
    """order="kkc": feature (ky*kw+kx)*Cin + c, i.e. X @ weight.permute(0,2,3,1).reshape(S,-1).T is the convolution."""
    B, Cin, H, W, k, S = 2, 3, 5, 4, 3, 2
    act = rng0.standard_normal((B, H, W, Cin))
    Xc = ora.patch_rows(act, B, Cin, H, W, k, k, 1, 1)
    Xk = ora.patch_rows(act, B, Cin, H, W, k, k, 1, 1, order="kkc")
    for c in range(Cin):
        for t in range(k * k):
            assert np.array_equal(Xk[:, t * Cin + c], Xc[:, c * k * k + t])
    wgt = rng0.standard_normal((S, Cin, k, k))
    assert np.allclose(Xk @ wgt.transpose(0, 2, 3, 1).reshape(S, -1).T, Xc @ wgt.reshape(S, -1).T, atol=1e-12)
    m = 7
    assert np.array_equal(ora.patch_feature_column(act, B, Cin, H, W, k, k, 1, 1, m, order="kkc"), Xk[:, m])


def test_unfold_feature_order_is_torch_weight_view_order():
    """With patch rows in this feature order, X @ weight.view(S,-1).T is the convolution output."""
    torch = pytest.importorskip("torch")
    B, Cin, H, W, k, S = 2, 3, 6, 5, 3, 4
    act = rng0.standard_normal((B, H, W, Cin))
    wgt = rng0.standard_normal((S, Cin, k, k))
    X = ora.patch_rows(act, B, Cin, H, W, k, k, 1, 1)
    z = X @ wgt.reshape(S, -1).T
    ref = torch.nn.functional.conv2d(torch.from_numpy(act).permute(0, 3, 1, 2), torch.from_numpy(wgt), padding=1)
    ref = ref.permute(0, 2, 3, 1).reshape(-1, S).numpy()
    assert np.allclose(z, ref, atol=1e-12)


# ----------------------------------------------------------------------------- moments
def test_two_block_moments_match_hand_worked_values():
    g = {r[0]: np.array(r[1:], dtype=float) for r in golden("two_block_moments.txt")}
    X0 = np.array([[1.0, 2.0], [3.0, 6.0]])
    X1 = np.array([[0.0, 0.0], [2.0, 2.0]])
    mu0, Phi0, phi0, lb0 = ora.block_moments(X0, 0.5, True)
    assert np.allclose(mu0, g["mu0"]) and np.allclose(Phi0.ravel(), g["Phi0"]) and np.allclose(phi0, g["phi0"])
    assert lb0 == pytest.approx(g["lbar0"][0])
    mu1, Phi1, phi1, lb1 = ora.block_moments(X1, 0.5, False, mu0, Phi0, phi0)
    assert np.allclose(mu1, g["mu1"]) and np.allclose(Phi1.ravel(), g["Phi1"]) and np.allclose(phi1, g["phi1"])
    assert lb1 == pytest.approx(g["lbar1"][0])


def test_first_block_is_numpy_biased_covariance():
    X = rng0.standard_normal((200, 7)) @ rng0.standard_normal((7, 7)) + 3.0
    mu, Phi, phi, lbar = ora.block_moments(X, 0.3, True)
    assert np.allclose(mu, X.mean(0), atol=1e-13)
    assert np.allclose(Phi, np.cov(X.T, bias=True), atol=1e-12)
    assert np.allclose(phi, np.mean(X ** 2, axis=0)) and lbar == pytest.approx(np.mean(X ** 2))
    # raw power relates to the centred moments: mean(phi) = tr(Phi)/M + |mu|^2/M
    assert lbar == pytest.approx(np.trace(Phi) / 7 + mu @ mu / 7)


def test_raw_sums_and_centred_form_agree():
    """The centred covariance of eq. (vPhixi) expands into raw sums: C = A/n - mhat mu^T - mu mhat^T + mu mu^T."""
    X = rng0.standard_normal((50, 5)) + 1.5
    mu_prev, Phi_prev, phi_prev, _ = ora.block_moments(rng0.standard_normal((40, 5)), 0.0, True)
    A, s, n = ora.raw_sums(X)
    assert np.allclose(A, sum(np.outer(x, x) for x in X)) and np.allclose(s, sum(X)) and n == 50
    alpha = 0.7
    mu, Phi, phi, _ = ora.block_moments(X, alpha, False, mu_prev, Phi_prev, phi_prev)
    mhat = s / n
    C = A / n - np.outer(mhat, mu) - np.outer(mu, mhat) + np.outer(mu, mu)
    assert np.allclose(Phi, alpha * Phi_prev + (1 - alpha) * C, atol=1e-12)
    assert np.allclose(phi, alpha * phi_prev + (1 - alpha) * np.diag(A) / n)
    i, j = 1, 3
    assert ora.cov_entry_centered(X[:, i], X[:, j], mu[i], mu[j]) == pytest.approx(
        ((X[:, i] - mu[i]) * (X[:, j] - mu[j])).mean())


# ----------------------------------------------------------------------------- EVD / ZCA
def test_zca_2x2_closed_form():
    g = {r[0]: np.array(r[1:], dtype=float) for r in golden("zca_2x2.txt")}
    for solver in ("lapack", "jacobi"):
        T, Q, lam = ora.whiten_evd(np.array([[2.0, 1.0], [1.0, 2.0]]), eps=1e-5, solver=solver)
        assert np.allclose(T.ravel(), g["T"], atol=1e-14)
        assert np.allclose(Q.ravel(), g["Q"], atol=1e-14)
        assert np.allclose(lam, g["lam"], atol=1e-14)


@pytest.mark.parametrize("solver", ["lapack", "jacobi"])
def test_full_whitening_gives_identity(solver):
    """Eq. (whitening): T Phi T^T = I when every eigenvalue exceeds eps."""
    M = 24
    Phi = wl.spd_matrix(5, M, np.logspace(0, -3, M))
    T, Q, lam = ora.whiten_evd(Phi, eps=1e-9, solver=solver)
    assert np.allclose(T @ Phi @ T.T, np.eye(M), atol=1e-10)
    assert np.allclose(T, T.T, atol=1e-12)                      # ZCA is symmetric
    assert np.allclose(Q, T.T @ T, atol=1e-10)
    assert np.all(np.diff(lam) <= 0) and np.allclose(lam, np.logspace(0, -3, M), rtol=1e-10)


def test_diagonal_covariance_gives_diagonal_gains_and_clamp():
    phi = np.array([4.0, 1.0, 0.25, 1e-8])
    T, Q, lam = ora.whiten_evd(np.diag(phi), eps=1e-4)
    assert np.allclose(T, np.diag([0.5, 1.0, 2.0, 100.0]), atol=1e-12)     # last gain clamped to 1/sqrt(eps)
    assert np.allclose(Q, np.diag([0.25, 1.0, 4.0, 1e4]), atol=1e-9)


def test_jacobi_brute_force_agrees_with_lapack():
    M = 20
    Phi = wl.spd_matrix(9, M, np.linspace(3.0, 0.1, M))
    lam_j, V = ora.jacobi_eigh(Phi)
    assert np.allclose(lam_j, np.linalg.eigvalsh(Phi)[::-1], atol=1e-12)
    assert np.allclose(V @ np.diag(lam_j) @ V.T, Phi, atol=1e-12) and np.allclose(V.T @ V, np.eye(M), atol=1e-12)
    Tj, Qj, _ = ora.whiten_evd(Phi, solver="jacobi")
    Tl, Ql, _ = ora.whiten_evd(Phi, solver="lapack")
    assert np.allclose(Tj, Tl, atol=1e-11) and np.allclose(Qj, Ql, atol=1e-11)


def test_degenerate_cluster_T_is_unique():
    M = 6
    lam = np.array([2.0, 2.0, 2.0, 0.5, 0.5, 0.1])
    Phi = wl.spd_matrix(3, M, lam)
    Tj, _, _ = ora.whiten_evd(Phi, solver="jacobi")
    Tl, _, _ = ora.whiten_evd(Phi, solver="lapack")
    assert np.allclose(Tj, Tl, atol=1e-11)


def test_rank_and_whiteness_stated_extremes():
    for kind, case, M, want in golden("stated_extremes.txt"):
        M, want = int(M), float(want)
        if kind == "rank":
            lam = np.ones(M) if case == "equal" else np.r_[1.0, np.full(M - 1, 1e-300)]
            assert ora.aic_signal_rank(lam) == pytest.approx(want, rel=1e-9)
        else:
            P = np.diag(rng0.uniform(0.5, 2.0, M)) if case == "diagonal" else np.outer(u := rng0.uniform(0.5, 2, M), u)
            assert ora.whiteness(P) == pytest.approx(want, rel=1e-12)
    assert ora.normalized_rank(np.ones(8)) == pytest.approx(1.0)
    assert ora.round_rank(2.5, 8) == 3 and ora.round_rank(0.2, 8) == 1 and ora.round_rank(9.7, 8) == 8


def test_gain_variant_keeps_average_variance_and_caps():
    """Eq. (g_mod): with every eigenvalue in the signal subspace and no cap hit, T Phi T^T = mean(lam) I."""
    M = 8
    lam = np.linspace(1.2, 0.8, M)                          # near-flat: entropy rank rounds to M
    Phi = wl.spd_matrix(4, M, lam)
    T, Q, lam_o = ora.whiten_evd(Phi, gain_mode=1, g_max=10.0)
    assert ora.round_rank(ora.aic_signal_rank(lam_o), M) == M
    assert np.allclose(T @ Phi @ T.T, lam.mean() * np.eye(M), atol=1e-10)
    # spread spectrum: rank < M, tail gains are 1, capped gains equal g_max
    lam2 = np.array([10.0, 5.0, 1.0, 1e-3, 1e-4, 1e-5])
    g = ora.evd_gains(lam2, eps=1e-5, gain_mode=1, g_max=3.0)
    r = ora.round_rank(ora.aic_signal_rank(lam2), 6)
    assert 1 <= r < 6 and np.all(g[r:] == 1.0)
    want = np.minimum(lam2.sum() / (6 * lam2[:r]), 3.0)
    assert np.allclose(g[:r], want)
    assert np.allclose(ora.evd_gains(lam2, 1e-2, 0), 1 / np.maximum(lam2, 1e-2))


def test_smoothed_Q():
    Q = np.diag([2.0, 4.0])
    assert np.allclose(ora.smooth_Q(np.eye(2), Q, 0.25), 0.25 * np.eye(2) + 0.75 * Q)


# ----------------------------------------------------------------------------- gradient transformation
def test_gradient_update_equals_direct_whitening_update():
    """Sec. 3.1: one SGD step on W~ with G Q equals the direct method's step on W, mapped through W~ = W T.
    T is non-symmetric here, so T^T T and T T^T differ and a transposed Q fails."""
    n, M, S, eta = 40, 6, 3, 0.05
    X = rng0.standard_normal((n, M)) @ rng0.standard_normal((M, M)) + 1.0
    mu = X.mean(0)
    T = np.eye(M) + 0.3 * rng0.standard_normal((M, M))
    W = rng0.standard_normal((S, M))
    b = rng0.standard_normal(S)
    tgt = rng0.standard_normal((n, S))
    # direct method: y = T(x - mu), z = W y + b, quadratic loss
    Y = ora.direct_whiten_forward(X, mu, T)
    assert np.allclose(Y[3], T @ (X[3] - mu))
    Z = Y @ W.T + b
    D = Z - tgt                                   # dL/dz
    W_direct = W - eta * (D.T @ Y)                # eqs. (dWrn), (vWrn_SGD)
    # gradient-based method: same network with W~ = W T
    Wt = W @ T
    Zt = (X - mu) @ Wt.T + b
    assert np.allclose(Z, Zt)
    G = (Zt - tgt).T @ (X - mu)                   # ordinary back-prop gradient w.r.t. W~
    Wt_new = Wt - eta * ora.grad_transform(G, ora.Q_from_T(T))
    assert np.allclose(Wt_new, W_direct @ T, atol=1e-12)
    wrong = Wt - eta * ora.grad_transform(G, T @ T.T)
    assert not np.allclose(wrong, W_direct @ T, atol=1e-6)
    # explicit triple loop for G Q on a corner
    Q = ora.Q_from_T(T)
    assert ora.grad_transform(G, Q)[1, 2] == pytest.approx(sum(G[1, k] * Q[k, 2] for k in range(M)))
    assert Q[0, 1] == pytest.approx(sum(T[k, 0] * T[k, 1] for k in range(M)))


def test_bias_compensation_keeps_the_layer_output():
    """Eq. (vtb_corr) for a fully connected layer (R = N = 1): output unchanged when mu moves."""
    M, S = 5, 3
    W = rng0.standard_normal((S, M)); b = rng0.standard_normal(S)
    mu0, mu1, x = rng0.standard_normal(M), rng0.standard_normal(M), rng0.standard_normal(M)
    b1 = ora.bias_compensation(b, W, 1, mu0, mu1)
    assert np.allclose(W @ (x - mu0) + b, W @ (x - mu1) + b1)


def test_sgd_update_reduces_to_the_plain_rule_and_to_geometric_sums():
    """Momentum and decay arithmetic against closed forms: constant gradient -> W_k = W_0 - lr GQ sum_j (1-m^j)/(1-m);
    zero gradient with decay only -> W_k = (1 - lr wd)^k W_0."""
    S, M, lr, m = 3, 5, 0.1, 0.9
    W0, G = rng0.standard_normal((S, M)), rng0.standard_normal((S, M))
    T = np.eye(M) + 0.2 * rng0.standard_normal((M, M))
    Q = T.T @ T
    W1, V1 = ora.sgd_update(W0, None, G, Q, lr)
    assert np.allclose(W1, W0 - lr * G @ T.T @ T, atol=1e-14) and np.allclose(V1, G @ Q)
    W, V = W0, None
    for k in range(1, 8):
        W, V = ora.sgd_update(W, V, G, Q, lr, momentum=m)
        geo = sum((1 - m ** j) / (1 - m) for j in range(1, k + 1))
        assert np.allclose(W, W0 - lr * geo * (G @ Q), atol=1e-12)
    W, V = W0, None
    for k in range(1, 6):
        W, V = ora.sgd_update(W, V, np.zeros((S, M)), Q, lr, weight_decay=0.05)
        assert np.allclose(W, (1 - lr * 0.05) ** k * W0, atol=1e-14)
    # decay acts on the stored parameter, not through Q
    W2, _ = ora.sgd_update(W0, None, G, Q, lr, weight_decay=0.5)
    assert np.allclose(W2, W0 - lr * (G @ Q) - lr * 0.5 * W0, atol=1e-14)


def test_per_tap_transform_equals_direct_whitening_of_a_convolution():
    """Per-channel form (eq. (vzrp3) with one weight matrix per kernel tap): a 3x3 valid convolution on channel-whitened
    input y = T(x - mu), updated by plain SGD, equals the convolution with W~[:, :, ky, kx] = W[:, :, ky, kx] T on the
    centred input updated with every tap's gradient times Q = T^T T.  Convolutions by explicit loops."""
    B, C, H, Wd, S, k, eta = 2, 3, 5, 4, 2, 3, 0.07
    x = rng0.standard_normal((B, C, H, Wd)) + 0.5
    mu = x.mean(axis=(0, 2, 3))
    T = np.eye(C) + 0.3 * rng0.standard_normal((C, C))
    Wc = rng0.standard_normal((S, C, k, k))
    Ho, Wo = H - k + 1, Wd - k + 1
    tgt = rng0.standard_normal((B, S, Ho, Wo))

    def conv(inp, Wt):
        out = np.zeros((B, S, Ho, Wo))
        for b_ in range(B):
            for s_ in range(S):
                for oy in range(Ho):
                    for ox in range(Wo):
                        out[b_, s_, oy, ox] = sum(Wt[s_, c, ky, kx] * inp[b_, c, oy + ky, ox + kx]
                                                   for c in range(C) for ky in range(k) for kx in range(k))
        return out

    def wgrad(inp, D):
        g = np.zeros((S, C, k, k))
        for s_ in range(S):
            for c in range(C):
                for ky in range(k):
                    for kx in range(k):
                        g[s_, c, ky, kx] = sum(D[b_, s_, oy, ox] * inp[b_, c, oy + ky, ox + kx]
                                               for b_ in range(B) for oy in range(Ho) for ox in range(Wo))
        return g

    xc = x - mu[None, :, None, None]
    y = np.einsum("dc,bchw->bdhw", T, xc)
    Z = conv(y, Wc)
    W_direct = Wc - eta * wgrad(y, Z - tgt)
    Wt = np.einsum("sdkl,dc->sckl", Wc, T)            # W~ = W T, tap by tap
    Zt = conv(xc, Wt)
    assert np.allclose(Z, Zt)
    G4 = wgrad(xc, Zt - tgt)
    Wt_new = Wt - eta * ora.grad_transform_taps(G4, ora.Q_from_T(T))
    assert np.allclose(Wt_new, np.einsum("sdkl,dc->sckl", W_direct, T), atol=1e-12)
    wrong = Wt - eta * ora.grad_transform_taps(G4, T @ T.T)
    assert not np.allclose(wrong, np.einsum("sdkl,dc->sckl", W_direct, T), atol=1e-6)


# ----------------------------------------------------------------------------- recursive whitening
def _rank1_plus_noise(M, snr, seed):
    r = np.random.default_rng(seed)
    u = r.standard_normal(M); u /= np.linalg.norm(u)
    N = r.standard_normal((M, M)); N = N @ N.T / M
    return snr * np.outer(u, u) + N, u


def test_estimator_converges_to_principal_eigenvector_at_high_snr():
    """Sec. 4.2 premise: in the high signal-to-noise case the estimate is the principal eigenvector."""
    angles = []
    for snr in (1e3, 1e5, 1e7):
        P, _ = _rank1_plus_noise(12, snr, 7)
        v, m_prime, members, xi, c = ora.high_power_subspace(P, 0.025, 1e-6)
        lam, V = ora.jacobi_eigh(P)
        angles.append(np.arccos(min(1.0, abs(v @ V[:, 0]))))
        assert np.linalg.norm(v) == pytest.approx(1.0)
        assert m_prime == int(np.argmax(np.linalg.norm(P, axis=0)))
    assert angles[0] > angles[1] > angles[2] and angles[2] < 1e-4


def test_estimator_pieces_by_brute_force():
    M = 7
    B = rng0.standard_normal((M, M)); P = B @ B.T
    v, mp, members, xi, c = ora.high_power_subspace(P, 0.3, 1e-6)
    for m in range(M):
        assert xi[m] == pytest.approx(np.sqrt(sum(P[k, m] ** 2 for k in range(M))))
        assert c[m] == pytest.approx(sum(P[k, mp] * P[k, m] for k in range(M)))
        assert members[m] == (abs(c[m]) >= max(0.3 * xi[mp] * xi[m], 1e-6))
    assert members[mp]
    vt = sum(P[:, m] / c[m] for m in range(M) if members[m]) / members.sum()
    assert np.allclose(v, vt / np.linalg.norm(vt))


def test_coherence_set_excludes_uncorrelated_and_weak_columns():
    u = np.array([3.0, 2.0, 1.0])
    P = np.zeros((6, 6)); P[:3, :3] = np.outer(u, u); P[3, 3] = 0.5; P[4, 4] = 1e-4; P[5, 5] = 0.2
    v, mp, members, xi, c = ora.high_power_subspace(P, 0.025, 1e-6)
    assert mp == 0 and list(members) == [True, True, True, False, False, False]
    assert np.allclose(np.abs(v[:3]), u / np.linalg.norm(u)) and np.allclose(v[3:], 0)
    # the absolute threshold alone can empty the set
    v2, _, members2, _, _ = ora.high_power_subspace(1e-5 * P, 0.025, 1e-6)
    assert v2 is None and members2.sum() == 0
    # power refinement moves a rough estimate to the principal eigenvector
    Pn, _ = _rank1_plus_noise(10, 5.0, 3)
    vr, *_ = ora.high_power_subspace(Pn, 0.025, 1e-6, n_power_iters=500)
    lam, V = ora.jacobi_eigh(Pn)
    assert abs(vr @ V[:, 0]) == pytest.approx(1.0, abs=1e-10)


def test_recursion_Q_equals_TtT_and_T_equals_product_form():
    """Eq. (vQ_rec) reproduces T^T T and eq. (vT_rec) reproduces gamma*T~*T + (1-gamma) I, step after step."""
    M = 10
    Phi = wl.spd_matrix(11, M, np.logspace(1, -2, M))
    lbar = np.trace(Phi) / M
    p = ora.CondParams(gamma=0.9, beta=0.3, delta=0.25)
    st = ora.CondState.initial(Phi)
    Qs_ref = np.eye(M)
    for step in range(12):
        T_old = st.T
        st, info = ora.cond_reduce_step(st, lbar, p)
        assert np.allclose(st.Q, st.T.T @ st.T, atol=1e-12)
        Ttil = np.eye(M) + info.a_e * np.outer(info.v, info.v)                       # eq. (tvT)
        assert np.allclose(st.T, p.gamma * Ttil @ T_old + (1 - p.gamma) * np.eye(M), atol=1e-12)
        Qs_ref = 0.3 * Qs_ref + 0.7 * st.Q
        assert np.allclose(st.Qs, Qs_ref, atol=1e-12)
        if info.applied:
            assert info.g_e == pytest.approx(0.25 * lbar / max(info.lambda_e, p.eps))
            assert info.a_e == pytest.approx(np.sqrt(info.g_e) - 1)
            assert info.lambda_e == pytest.approx(info.v @ info.Phi_y @ info.v)
    assert not np.allclose(st.T, st.T.T, atol=1e-6)        # T really is non-symmetric here


def test_shrink_sets_power_to_target_and_leaves_orthogonal_subspaces():
    """Sec. 4.1 after eq. (xi): the power along v becomes delta*lambda_bar, all orthogonal subspaces keep theirs."""
    M = 8
    lam = np.array([50.0, 3.0, 2.0, 1.5, 1.0, 0.7, 0.4, 0.2])
    Phi = wl.spd_matrix(21, M, lam)
    lbar = 6.0
    p = ora.CondParams(gamma=1.0, beta=0.0, delta=0.25, n_power_iters=3000)
    st, info = ora.cond_reduce_step(ora.CondState.initial(Phi), lbar, p)
    Py = ora.transformed_covariance(st.T, Phi)
    assert info.applied and info.lambda_e == pytest.approx(50.0, rel=1e-9)
    assert info.v @ Py @ info.v == pytest.approx(0.25 * lbar, rel=1e-9)
    got = np.sort(np.linalg.eigvalsh(Py))
    want = np.sort(np.r_[0.25 * lbar, lam[1:]])
    assert np.allclose(got, want, rtol=1e-8)
    # first step from T = I with gamma = 1 is exactly eq. (tvT)
    assert np.allclose(st.T, np.eye(M) + info.a_e * np.outer(info.v, info.v), atol=1e-12)
    assert np.allclose(st.Qs, st.Q)


def test_condition_number_is_non_increasing():
    """With gamma = 1, an exact principal direction, the guard on and delta*lambda_bar >= lambda_min, cond(Phi_y)
    never grows from step to step."""
    M = 12
    lam = np.logspace(2, -1, M)
    Phi = wl.spd_matrix(31, M, lam)
    lbar = np.trace(Phi) / M
    p = ora.CondParams(gamma=1.0, beta=0.0, delta=0.25, n_power_iters=4000, guard=True)
    assert p.delta * lbar >= lam.min()
    st = ora.CondState.initial(Phi)
    conds = [np.linalg.cond(Phi)]
    for _ in range(M + 3):
        st, info = ora.cond_reduce_step(st, lbar, p)
        conds.append(np.linalg.cond(ora.transformed_covariance(st.T, Phi)))
    assert all(b <= a * (1 + 1e-9) for a, b in zip(conds, conds[1:]))
    assert conds[-1] < conds[0] / 10
    assert conds[-1] == pytest.approx(p.delta * lbar / lam.min(), rel=1e-6)   # all high directions now sit at the target
    assert not info.applied                                    # nothing above the target is left


def test_guard_and_empty_set_apply_only_the_leak():
    M = 5
    Phi = np.diag([1.0, 0.9, 0.8, 0.7, 0.6])
    p = ora.CondParams(gamma=0.9, beta=0.5, delta=4.0)          # target above every eigenvalue: g_e >= 1
    st0 = ora.CondState.initial(Phi)
    st0.T = np.eye(M) * 1.1; st0.Q = st0.T.T @ st0.T
    st, info = ora.cond_reduce_step(st0, 1.0, p)
    assert not info.applied and info.a_e == 0.0 and info.g_e >= 1.0
    assert np.allclose(st.T, 0.9 * st0.T + 0.1 * np.eye(M))
    assert np.allclose(st.Q, st.T.T @ st.T)
    p2 = ora.CondParams(gamma=0.9, beta=0.5, delta=4.0, guard=False)
    st2, info2 = ora.cond_reduce_step(st0, 1.0, p2)
    assert info2.applied and info2.a_e > 0
    st3, info3 = ora.cond_reduce_step(ora.CondState.initial(1e-6 * Phi), 1.0, ora.CondParams(gamma=0.5))
    assert info3.set_size == 0 and not info3.applied and np.allclose(st3.T, np.eye(M))


def test_forced_decisions_are_honoured():
    P, _ = _rank1_plus_noise(6, 10.0, 2)
    v, mp, members, xi, c = ora.high_power_subspace(P, 0.025, 1e-6)
    alt = (mp + 1) % 6
    v2, mp2, mem2, _, c2 = ora.high_power_subspace(P, 0.025, 1e-6, forced_m_prime=alt, forced_members=np.ones(6, bool))
    assert mp2 == alt and mem2.all() and np.allclose(c2, P.T @ P[:, alt])


# ----------------------------------------------------------------------------- workloads are pure data
def test_workload_recipes_shapes_and_bf16():
    L1 = wl.config1()
    assert L1.act.shape == (128, 64) and L1.G.shape == (32, 64) and L1.is_rows
    s = np.linalg.svd(L1.act.astype(float), compute_uv=False)
    assert s[0] / s[-1] > 50
    L = wl.small_conv(3, 2, 4, 5, 6, 3, 1, 1, 8, dtype="bf16")
    assert np.array_equal(wl.round_to_bf16(L.act), L.act) and wl.bf16_bits(L.act).dtype == np.uint16
    x = np.array([1.0, 1.00390625, 1.01171875, 3.14159], dtype=np.float32)
    r = wl.round_to_bf16(x)                        # 1+2^-8 ties to even (1.0); 1+3*2^-8 ties to even (1+2^-6)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625) and abs(r[3] - 3.140625) < 1e-6
    assert len(wl.RESNET18_LAYERS) == 21
    L5 = wl.config5_layer(6, B=2, scale=0.25)
    assert L5.desc.kh == 1 and L5.desc.stride == 2 and L5.desc.M == 64


# ----------------------------------------------------------------------------- condition-number probe (Sec. 4, purpose of the recursion)
def _three_term_lanczos(A, b0, k):
    """Textbook Lanczos recurrence, written independently of the oracle's projection form: alpha_j = q_j^T A q_j,
    r = A q_j - alpha_j q_j - beta_(j-1) q_(j-1), beta_j = |r|; Ritz values = eigenvalues of tridiag(alpha, beta)."""
    q_prev = np.zeros_like(b0)
    q = b0 / np.linalg.norm(b0)
    alpha, beta = [], []
    b_prev = 0.0
    for j in range(k):
        w = A @ q
        a = float(q @ w)
        alpha.append(a)
        r = w - a * q - b_prev * q_prev
        b_prev = float(np.linalg.norm(r))
        if j + 1 < k:
            beta.append(b_prev)
            q_prev, q = q, r / b_prev
    Tk = np.diag(alpha) + np.diag(beta, 1) + np.diag(beta, -1)
    return np.linalg.eigvalsh(Tk)[::-1]


def test_probe_single_step_is_the_rayleigh_quotient():
    A = np.array([[4.0, 1.0], [1.0, 3.0]])
    b0 = np.array([1.0, 2.0])
    ritz, steps = ora.krylov_ritz_values(A, b0, 1)
    assert steps == 1 and abs(ritz[0] - (b0 @ A @ b0) / (b0 @ b0)) < 1e-14      # (4 + 4 + 12) / 5 = 4
    assert abs(ritz[0] - 4.0) < 1e-14


def test_probe_full_dimension_gives_the_spectrum():
    M = 12
    lam = np.linspace(5.0, 0.5, M)
    A = wl.spd_matrix(3, M, lam)
    b0 = np.random.default_rng(0).standard_normal(M)
    ritz, steps = ora.krylov_ritz_values(A, b0, M)
    assert steps == M and np.allclose(ritz, lam, rtol=0, atol=1e-9)
    hi, lo, cond, _ = ora.condition_probe(A, b0, M)
    assert abs(cond - 10.0) < 1e-7


def test_probe_stops_on_an_invariant_subspace_and_is_exact_there():
    A = np.diag([7.0, 3.0, 2.0, 1.0])
    b0 = np.array([1.0, 0.0, 1.0, 0.0])        # lives in the span of two eigenvectors
    ritz, steps = ora.krylov_ritz_values(A, b0, 4)
    assert steps == 2 and np.allclose(ritz, [7.0, 2.0], atol=1e-12)


def test_probe_ritz_values_stay_inside_the_spectrum_and_improve_with_k():
    M = 60
    A = wl.spd_matrix(8, M, np.logspace(1.0, -2.0, M))
    w = np.linalg.eigvalsh(A)
    b0 = np.random.default_rng(1).standard_normal(M)
    last_hi, last_lo = -np.inf, np.inf
    for k in (1, 2, 4, 8, 16, 32):
        hi, lo, cond, steps = ora.condition_probe(A, b0, k)
        assert w[0] - 1e-12 <= lo <= hi <= w[-1] + 1e-12
        assert hi >= last_hi - 1e-12 and lo <= last_lo + 1e-12          # nested Krylov spaces: the extremes can only widen
        assert cond <= w[-1] / w[0] * (1 + 1e-9)                        # never an overestimate
        last_hi, last_lo = hi, lo
    assert abs(last_hi / w[-1] - 1) < 1e-6                              # the top converges fast


def test_probe_matches_the_three_term_recurrence():
    M = 40
    A = wl.spd_matrix(9, M, np.logspace(0.5, -1.5, M))
    b0 = np.random.default_rng(2).standard_normal(M)
    for k in (2, 5, 9):
        ritz, steps = ora.krylov_ritz_values(A, b0, k)
        assert steps == k
        assert np.allclose(ritz, _three_term_lanczos(A, b0, k), rtol=1e-9, atol=1e-12)
