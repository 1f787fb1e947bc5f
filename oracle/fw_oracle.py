"""CPU oracle for feature whitening by gradient transformation (arXiv 2010.01546).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, float64 numpy restatement of what
the paper's per-layer hot path computes.  It shares no code with the GPU library and
must never be imported by it; only tests, the smoke check and the benchmark's
CPU-baseline leg call it.

Every function cites the passage of the paper it follows.  Where the paper is
garbled, silent or inconsistent the reading taken is stated in the docstring.

Notation (paper, Sec. 2): a layer input has M features; a conv layer is taken in its
unfolded form, so a "sample row" x is one k*k*Cin patch and the rows of X are the
B*P patches of a batch (Sec. 2 allows any spatial dimension to be vectorised, and
convolution is named as a special case of the generic linear layer, eq. (vzrp)).
Feature order is m = (c*kh + ky)*kw + kx, the order of ``weight.view(S, Cin*kh*kw)``.

Parity pins: see tests/test_oracle_pins.py.  Functions with no pin from the paper
or from mathematics are marked "parity unpinned" in their docstring.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

F64 = np.float64


# =============================================================================
# Patch rows (explicit unfolding) -- Sec. 2, eq. (vXp): the matrix whose columns are
# the spatial elements x_n; here stored row-wise.
# =============================================================================
def patch_rows(act_nhwc: np.ndarray, B, Cin, H, W, kh, kw, stride, pad, order: str = "ckk") -> np.ndarray:
    """Explicit unfolding of an activation tensor [B,H,W,Cin] into patch rows [B*Ho*Wo, Cin*kh*kw].

    X[(b*Ho+oy)*Wo+ox, (c*kh+ky)*kw+kx] = act[b, oy*stride+ky-pad, ox*stride+kx-pad, c], zero outside the image.
    Padding zeros are data of the patch vectors like any other value.
    order "kkc" puts the same values in the feature order m = (ky*kw+kx)*Cin + c (channels-last weights).
    """
    a = np.asarray(act_nhwc, dtype=F64).reshape(B, H, W, Cin)
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    ap = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), dtype=F64)
    ap[:, pad:pad + H, pad:pad + W, :] = a
    X = np.empty((B, Ho, Wo, Cin, kh, kw), dtype=F64)
    for ky in range(kh):
        for kx in range(kw):
            X[:, :, :, :, ky, kx] = ap[:, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride, :]
    if order == "kkc":
        X = np.ascontiguousarray(np.transpose(X, (0, 1, 2, 4, 5, 3)))
    elif order != "ckk":
        raise ValueError(order)
    return X.reshape(B * Ho * Wo, Cin * kh * kw)


def patch_feature_column(act_nhwc: np.ndarray, B, Cin, H, W, kh, kw, stride, pad, m: int, order: str = "ckk") -> np.ndarray:
    """One column of the patch-row matrix (feature m over all B*P rows), without forming the matrix."""
    a = np.asarray(act_nhwc).reshape(B, H, W, Cin)
    if order == "ckk":
        c, r = divmod(m, kh * kw)
    else:
        r, c = divmod(m, Cin)
    ky, kx = divmod(r, kw)
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    col = np.zeros((B, Ho, Wo), dtype=F64)
    for oy in range(Ho):
        iy = oy * stride + ky - pad
        if iy < 0 or iy >= H:
            continue
        for ox in range(Wo):
            ix = ox * stride + kx - pad
            if 0 <= ix < W:
                col[:, oy, ox] = a[:, iy, ix, c]
    return col.reshape(-1)


# =============================================================================
# Raw block sums: what one call of the accumulation step adds up.
# =============================================================================
def raw_sums(X: np.ndarray):
    """A = sum_rows x x^T, s = sum_rows x, n = number of rows (the sums inside eqs. (vmuxi), (vPhixi), (phixmi))."""
    X = np.asarray(X, dtype=F64)
    return X.T @ X, X.sum(axis=0), X.shape[0]


# =============================================================================
# Block moments -- eqs. (vmuxi), (vPhixi), (vmuxnz), (vPhixnz), (phixmi), (blambday)
# =============================================================================
def block_moments(X: np.ndarray, alpha: float, first_block: bool,
                  mu_prev=None, Phi_prev=None, phi_prev=None):
    """Moments of block i from all rows X of the block (the L*B*N spatial elements).

    mu(i)  = alpha*mu(i-1) + (1-alpha)*mean_rows(x)                         eq. (vmuxi)
    Phi(i) = alpha*Phi(i-1) + (1-alpha)*mean_rows((x-mu(i))(x-mu(i))^T)      eq. (vPhixi)
    first block (i = 0): the same without the recursive average               eqs. (vmuxnz), (vPhixnz)
    phi_m(i) = alpha*phi_m(i-1) + (1-alpha)*mean_rows(x_m^2)                 eq. (phixmi)
    lambda_bar = mean_m phi_m(i)                                              eq. (blambday)

    Readings: the covariance is centred on the *updated* mean mu(i), as printed.  phi uses raw
    (uncentred) squares, as printed.  The paper gives no first-block form for phi; the first
    block is taken without the recursive average, like the other two moments (parity unpinned).
    The centred form is evaluated as written: subtract, then multiply.
    """
    X = np.asarray(X, dtype=F64)
    n = X.shape[0]
    mhat = X.sum(axis=0) / n
    raw_pow = (X * X).sum(axis=0) / n
    if first_block:
        mu = mhat
    else:
        mu = alpha * np.asarray(mu_prev, F64) + (1.0 - alpha) * mhat
    Xc = X - mu[None, :]
    C = (Xc.T @ Xc) / n
    if first_block:
        Phi = C
        phi = raw_pow
    else:
        Phi = alpha * np.asarray(Phi_prev, F64) + (1.0 - alpha) * C
        phi = alpha * np.asarray(phi_prev, F64) + (1.0 - alpha) * raw_pow
    return mu, Phi, phi, float(phi.mean())


def cov_entry_centered(col_i: np.ndarray, col_j: np.ndarray, mu_i: float, mu_j: float) -> float:
    """One entry of the centred block covariance of eq. (vPhixnz) from two feature columns."""
    n = col_i.shape[0]
    return float(np.dot(col_i - mu_i, col_j - mu_j) / n)


# =============================================================================
# EVD / ZCA whitening -- eqs. (whitening), (vPhix_evd), (vT_EVD), (vg); Sec. 3.2 for the gain variant
# =============================================================================
def jacobi_eigh(Phi: np.ndarray, max_sweeps: int = 60, tol: float = 1e-15):
    """Cyclic two-sided Jacobi eigen-decomposition of a symmetric matrix (brute-force reference solver).

    Returns (eigenvalues sorted decreasing, V with eigenvectors in the columns): Phi = V diag(lam) V^T, eq. (vPhix_evd).
    """
    A = np.array(Phi, dtype=F64, copy=True)
    M = A.shape[0]
    V = np.eye(M, dtype=F64)
    for _ in range(max_sweeps):
        off = np.sqrt(max(np.sum(A * A) - np.sum(np.diag(A) ** 2), 0.0))
        if off <= tol * np.sqrt(np.sum(A * A)):
            break
        for p in range(M - 1):
            for q in range(p + 1, M):
                apq = A[p, q]
                if abs(apq) <= 1e-300:
                    continue
                with np.errstate(over="ignore"):
                    theta = (A[q, q] - A[p, p]) / (2.0 * apq)
                if not np.isfinite(theta):
                    continue
                t = np.sign(theta) / (abs(theta) + np.hypot(theta, 1.0)) if theta != 0.0 else 1.0
                c = 1.0 / np.sqrt(t * t + 1.0)
                s = t * c
                # A <- J^T A J with J the plane rotation in (p, q)
                Ap = A[:, p].copy()
                Aq = A[:, q].copy()
                A[:, p] = c * Ap - s * Aq
                A[:, q] = s * Ap + c * Aq
                Ap = A[p, :].copy()
                Aq = A[q, :].copy()
                A[p, :] = c * Ap - s * Aq
                A[q, :] = s * Ap + c * Aq
                Vp = V[:, p].copy()
                Vq = V[:, q].copy()
                V[:, p] = c * Vp - s * Vq
                V[:, q] = s * Vp + c * Vq
    lam = np.diag(A).copy()
    order = np.argsort(-lam, kind="stable")
    return lam[order], V[:, order]


def aic_signal_rank(lam: np.ndarray) -> float:
    """Signal-subspace rank estimate of Sec. 3.2, eq. (hMs).

    Reading: the printed sum of exponentials contradicts both extremes the text states (M for equal
    eigenvalues, 1 for a single non-zero eigenvalue); the exponential of the entropy of the normalised
    eigenvalues, exp(-sum_m lb_m log lb_m) with 0 log 0 = 0, satisfies both and is what is computed.
    Non-positive eigenvalues (rounding) count as zero.
    """
    lam = np.maximum(np.asarray(lam, dtype=F64), 0.0)
    tot = lam.sum()
    if tot <= 0.0:
        return 1.0
    lb = lam / tot
    nz = lb > 0.0
    return float(np.exp(-np.sum(lb[nz] * np.log(lb[nz]))))


def round_rank(ms_hat: float, M: int) -> int:
    """Integer rank used as the index bound of eq. (g_mod): round half up, clamped to [1, M] (parity unpinned)."""
    return int(min(max(np.floor(ms_hat + 0.5), 1), M))


def evd_gains(lam: np.ndarray, eps: float, gain_mode: int = 0, g_max: float = 10.0) -> np.ndarray:
    """Gains per eigenvalue (eigenvalues sorted decreasing).

    gain_mode 0: g_m = 1 / max(lam_m, eps)                                              eq. (vg)
    gain_mode 1: g_m = min(1/(M*lb_m), g_max) for m < round(Ms_hat), 1 otherwise         eq. (g_mod)
                 with lb_m = lam_m / sum(lam); lam_m <= 0 takes the limit g_max.
    """
    lam = np.asarray(lam, dtype=F64)
    M = lam.shape[0]
    if gain_mode == 0:
        return 1.0 / np.maximum(lam, eps)
    tot = np.maximum(lam, 0.0).sum()
    g = np.ones(M, dtype=F64)
    r = round_rank(aic_signal_rank(lam), M)
    for m in range(r):
        if lam[m] <= 0.0 or tot <= 0.0:
            g[m] = g_max
        else:
            g[m] = min(tot / (M * lam[m]), g_max)
    return g


def whiten_evd(Phi_x: np.ndarray, eps: float = 1e-5, gain_mode: int = 0, g_max: float = 10.0, solver: str = "lapack"):
    """ZCA whitening matrix from the eigen-decomposition of Phi_x.

    Phi_x = V Lam V^T with eigenvalues sorted decreasing       eq. (vPhix_evd)
    T = V diag(sqrt(g)) V^T                                     eq. (vT_EVD)
    Q = T^T T = V diag(g) V^T                                   eq. (vQ)
    Returns (T, Q, lam).  T and Q are spectral functions of Phi_x and so do not depend on the
    choice of eigenvectors inside a degenerate cluster.
    """
    P = np.asarray(Phi_x, dtype=F64)
    P = 0.5 * (P + P.T)
    if solver == "lapack":
        lam, V = np.linalg.eigh(P)
        lam, V = lam[::-1].copy(), V[:, ::-1].copy()
    elif solver == "jacobi":
        lam, V = jacobi_eigh(P)
    else:
        raise ValueError(solver)
    g = evd_gains(lam, eps, gain_mode, g_max)
    T = (V * np.sqrt(g)[None, :]) @ V.T
    Q = (V * g[None, :]) @ V.T
    return T, Q, lam


def smooth_Q(Qs_prev: np.ndarray, Q: np.ndarray, beta: float) -> np.ndarray:
    """Qs(i) = beta*Qs(i-1) + (1-beta)*Q(i), Qs(-1) = I                  eq. (vQs)"""
    return beta * np.asarray(Qs_prev, F64) + (1.0 - beta) * np.asarray(Q, F64)


# =============================================================================
# Gradient transformation -- eqs. (mod_weight_grad), (vQ)
# =============================================================================
def Q_from_T(T: np.ndarray) -> np.ndarray:
    """Q = T^T T, eq. (vQ).  (Not T T^T: they differ for the non-symmetric T of the recursive method.)"""
    T = np.asarray(T, dtype=F64)
    return T.T @ T


def grad_transform(G: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """dL/dWbar = (dL/dWtilde) Q, eq. (mod_weight_grad); G is [S, M], Q is [M, M]."""
    return np.asarray(G, dtype=F64) @ np.asarray(Q, dtype=F64)


def grad_transform_taps(G4: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """Per-channel form of eq. (mod_weight_grad): a layer of eq. (vzrp3) has one S x M weight matrix W~_rn per spatial
    offset n (for a convolution: per kernel tap, M = Cin), and every one of them is multiplied by the same M x M Q.
    G4 is [S, Cin, kh, kw] (the layout of a convolution weight); Q is [Cin, Cin]."""
    G4 = np.asarray(G4, dtype=F64)
    Q = np.asarray(Q, dtype=F64)
    out = np.empty_like(G4)
    for ky in range(G4.shape[2]):
        for kx in range(G4.shape[3]):
            out[:, :, ky, kx] = G4[:, :, ky, kx] @ Q
    return out


def sgd_update(W: np.ndarray, V, G: np.ndarray, Q: np.ndarray, lr: float, momentum: float = 0.0, weight_decay: float = 0.0):
    """One update of the stored weights W~ [S, M] from the raw gradient G [S, M]:

        d  = G Q + weight_decay * W~          eq. (mod_weight_grad), plus the decay term of Sec. 6
        V' = momentum * V + d                 (V' = d when there is no momentum buffer yet: V is None)
        W~' = W~ - lr * V'                    eq. (vtWrn_SGD)

    With momentum = weight_decay = 0 this is exactly eqs. (vtWrn_SGD), (mod_weight_grad).  Sec. 6 only names "momentum
    0.9" and "weight decay" without formulas; the reading is the common heavy-ball form with the decay term added to
    the already transformed gradient (it acts on the stored parameter W~).  That convention is parity unpinned by the
    paper; its arithmetic is pinned by closed forms (geometric sums) in the tests.
    Returns (W~', V')."""
    W = np.asarray(W, dtype=F64)
    d = grad_transform(G, Q) + weight_decay * W
    Vn = d if V is None else momentum * np.asarray(V, dtype=F64) + d
    return W - lr * Vn, Vn


# --- the direct method of Sec. 2, used only to pin the equivalence claimed in Sec. 3.1 ---------
def direct_whiten_forward(X: np.ndarray, mu: np.ndarray, T: np.ndarray) -> np.ndarray:
    """y = T (x - mu) for every row, eq. (vyn)."""
    return (np.asarray(X, F64) - np.asarray(mu, F64)[None, :]) @ np.asarray(T, F64).T


def bias_compensation(b: np.ndarray, W_sum_over_rn: np.ndarray, R: int, mu_old: np.ndarray, mu_new: np.ndarray):
    """Bias compensation when the tracked mean moves from mu(i-1) to mu(i), eq. (vtb_corr); W_sum_over_rn = sum_{r,n} Wtilde_rn.

    Reading: b|i = b|i- + (1/R) sum_{r,n} Wtilde_rn (mu(i) - mu(i-1)).  The printed equation has the difference the
    other way round, which contradicts the relation it is derived from in the sentence before it (the layer output
    must be the same before and after the update); the sign that keeps that relation is used.
    """
    return np.asarray(b, F64) + (np.asarray(W_sum_over_rn, F64) @ (np.asarray(mu_new, F64) - np.asarray(mu_old, F64))) / R


# =============================================================================
# Recursive whitening -- Sec. 4
# =============================================================================
@dataclass
class CondParams:
    """Hyper-parameters of the recursive method; defaults are the values of Sec. 6."""
    gamma: float = 0.99
    delta: float = 0.25
    eps: float = 1e-5
    c_rel: float = 0.025
    c_abs: float = 1e-6      # printed as a second "c_rel" in Sec. 6; its role in the set rule makes it c_abs
    beta: float = 0.1
    n_power_iters: int = 0   # optional refinements v <- Phi_y v / |Phi_y v| (not in the paper; off by default)
    guard: bool = True       # skip the shrink when it would amplify (g_e >= 1); the paper assumes it never does


@dataclass
class CondState:
    Phi_x: np.ndarray
    T: np.ndarray
    Q: np.ndarray
    Qs: np.ndarray

    @staticmethod
    def initial(Phi_x: np.ndarray) -> "CondState":
        """T(-1) = I (eq. (vT_init)), hence Q = I; Qs(-1) = I (Sec. 3.2)."""
        M = Phi_x.shape[0]
        return CondState(np.array(Phi_x, dtype=F64), np.eye(M), np.eye(M), np.eye(M))


@dataclass
class CondInfo:
    m_prime: int = -1
    set_size: int = 0
    lambda_e: float = 0.0
    g_e: float = 1.0
    a_e: float = 0.0
    applied: bool = False
    members: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=bool))
    xi: np.ndarray = field(default_factory=lambda: np.zeros(0))
    c: np.ndarray = field(default_factory=lambda: np.zeros(0))
    v: np.ndarray = field(default_factory=lambda: np.zeros(0))
    Phi_y: np.ndarray = field(default_factory=lambda: np.zeros((0, 0)))


def transformed_covariance(T: np.ndarray, Phi_x: np.ndarray) -> np.ndarray:
    """Phi_y = T Phi_x T^T: covariance of y = T(x - mu) (Sec. 4, first paragraph; eq. (whitening) is its target)."""
    T = np.asarray(T, F64)
    return T @ np.asarray(Phi_x, F64) @ T.T


def high_power_subspace(Phi_y: np.ndarray, c_rel: float, c_abs: float, n_power_iters: int = 0,
                        forced_m_prime=None, forced_members=None):
    """Principal-direction estimate of Sec. 4.2.

    xi_m = |Phi_y e_m|                                       eq. (xim)
    m'   = argmax_m xi_m  (lowest index on ties)             eq. (mt)
    c^T  = e_m'^T Phi_y^T Phi_y                              eq. (vc)
    set  = { m : |c_m| >= max(c_rel*xi_m'*xi_m, c_abs) }     (set rule after eq. (vc))
    v~   = (1/|set|) sum_{m in set} (1/c_m) Phi_y e_m        eq. (tve)
    v    = v~ / |v~|
    e_m is the 0-based selection vector.  An empty set returns v = None (the paper does not cover it).
    ``forced_*`` let a test substitute a decision that differs from this one only by rounding.
    """
    P = np.asarray(Phi_y, F64)
    M = P.shape[0]
    xi = np.sqrt(np.sum(P * P, axis=0))
    m_prime = int(np.argmax(xi)) if forced_m_prime is None else int(forced_m_prime)
    c = P.T @ P[:, m_prime]
    if forced_members is None:
        members = np.abs(c) >= np.maximum(c_rel * xi[m_prime] * xi, c_abs)
    else:
        members = np.asarray(forced_members, dtype=bool)
    k = int(members.sum())
    if k == 0:
        return None, m_prime, members, xi, c
    vt = np.zeros(M, dtype=F64)
    for m in np.nonzero(members)[0]:
        vt += P[:, m] / c[m]
    vt /= k
    v = vt / np.linalg.norm(vt)
    for _ in range(n_power_iters):
        w = P @ v
        v = w / np.linalg.norm(w)
    return v, m_prime, members, xi, c


def cond_reduce_step(st: CondState, lambda_bar: float, p: CondParams,
                     forced_m_prime=None, forced_members=None):
    """One step of the recursive condition-number reduction (Sec. 4.1), returning the new state and diagnostics.

    lambda_e = v^T Phi_y v                                                 eq. (lambda)
    g_e = delta*lambda_bar / max(lambda_e, eps);  a_e = sqrt(g_e) - 1      eqs. (ge), (xi)
    T(i) = gamma*(T + a_e v t^T) + (1-gamma) I                             eq. (vT_rec)
    Q(i) by the O(M^2) recursion                                          eq. (vQ_rec)
    Qs(i) = beta*Qs(i-1) + (1-beta)*Q(i)                                   eq. (vQs)

    Readings: t = T(i-1)^T v.  Eq. (vtve) prints T v, but only the transposed form makes the two sides of
    eq. (vT_rec) equal and makes eq. (vQ_rec) equal T^T T for the non-symmetric T the recursion produces.
    Phi_y is formed explicitly as T Phi_x T^T with Phi_x fixed.  If the estimate holds no more power than the
    target (g_e >= 1) and ``guard`` is set, or the coherence set is empty, the shrink is skipped (a_e = 0) and
    only the leak is applied (parity unpinned: the paper assumes a high-power direction is always found).
    """
    T, Q, Qs, Phi_x = st.T, st.Q, st.Qs, st.Phi_x
    M = T.shape[0]
    I = np.eye(M)
    Phi_y = transformed_covariance(T, Phi_x)
    v, m_prime, members, xi, c = high_power_subspace(Phi_y, p.c_rel, p.c_abs, p.n_power_iters,
                                                     forced_m_prime, forced_members)
    info = CondInfo(m_prime=m_prime, set_size=int(members.sum()), members=members, xi=xi, c=c, Phi_y=Phi_y)
    a_e = 0.0
    if v is None:
        v = np.zeros(M)
    else:
        lam_e = float(v @ Phi_y @ v)
        g_e = p.delta * lambda_bar / max(lam_e, p.eps)
        info.lambda_e, info.g_e = lam_e, g_e
        if not (p.guard and g_e >= 1.0):
            a_e = np.sqrt(g_e) - 1.0
            info.applied = True
    info.a_e, info.v = a_e, v
    t = T.T @ v
    g = p.gamma
    T_new = g * (T + a_e * np.outer(v, t)) + (1.0 - g) * I
    Q_new = (g * g * (Q + a_e * (a_e + 2.0) * np.outer(t, t)) + (1.0 - g) ** 2 * I
             + g * (1.0 - g) * (a_e * (np.outer(v, t) + np.outer(t, v)) + T + T.T))
    Qs_new = smooth_Q(Qs, Q_new, p.beta)
    return CondState(Phi_x, T_new, Q_new, Qs_new), info


# =============================================================================
# Diagnostics of Sec. 6
# =============================================================================
def normalized_rank(lam: np.ndarray) -> float:
    """kappa = Ms_hat / M (Sec. 6)."""
    lam = np.asarray(lam, F64)
    return aic_signal_rank(lam) / lam.shape[0]


def whiteness(Phi_y: np.ndarray) -> float:
    """rho = M / sum_{m,m'} Phi[m',m]^2 / (Phi[m,m] Phi[m',m'])        eq. (rho)

    Reading: the sum runs over all pairs including m = m'.  The printed m != m' gives infinity for a diagonal
    matrix, against the stated extreme rho = 1; with the diagonal included both stated extremes (1 and 1/M) hold.
    """
    P = np.asarray(Phi_y, F64)
    d = np.diag(P)
    return float(P.shape[0] / np.sum(P * P / np.outer(d, d)))


# =============================================================================
# Condition-number probe -- Sec. 4, opening paragraphs: the quantity the recursion is built to reduce is the condition
# number of Phi_y (convergence time is proportional to it; 1 means white).  A monitoring companion to kappa and rho of
# Sec. 6.  The paper gives no procedure for it; the estimate taken here is the classical one: the extreme Ritz values
# of Phi_y on a Krylov subspace of small dimension k.
# =============================================================================
def krylov_ritz_values(A: np.ndarray, b0: np.ndarray, k: int, breakdown: float = 1e-7):
    """Ritz values of the symmetric matrix A on span{b0, A b0, ..., A^(k-1) b0}, by the definition: an orthonormal basis
    Q of that space (Gram-Schmidt on the successive images, each orthogonalised twice against all earlier vectors),
    H = Q^T A Q, eigenvalues of H in decreasing order.

    The basis stops early when the next image lies in the span already built (its remainder is below ``breakdown``
    times its own length): the space is then invariant and its Ritz values are eigenvalues of A.  Returns (ritz, steps).
    Every Ritz value lies between the extreme eigenvalues of A, so max/min of them never overestimates the condition
    number.
    """
    A = np.asarray(A, F64)
    q = np.asarray(b0, F64).copy()
    q /= np.linalg.norm(q)
    Q = [q]
    for _ in range(1, k):
        w = A @ Q[-1]
        n0 = np.linalg.norm(w)
        for _rep in range(2):
            for qi in Q:
                w = w - (qi @ w) * qi
        nw = np.linalg.norm(w)
        if not nw > breakdown * n0:
            break
        Q.append(w / nw)
    Qm = np.stack(Q, axis=1)
    H = Qm.T @ A @ Qm
    H = 0.5 * (H + H.T)
    return np.linalg.eigvalsh(H)[::-1], Qm.shape[1]


def condition_probe(Phi_y: np.ndarray, b0: np.ndarray, k: int):
    """(lambda_max estimate, lambda_min estimate, their ratio, Krylov dimension reached) of Phi_y from ``k`` Krylov steps
    started at b0.  A non-positive lower estimate gives an infinite ratio (parity unpinned: the paper defines no probe;
    the arithmetic is pinned against LAPACK, the Rayleigh quotient, the textbook three-term recurrence and exactness on an
    invariant subspace)."""
    ritz, steps = krylov_ritz_values(Phi_y, b0, k)
    hi, lo = float(ritz[0]), float(ritz[-1])
    return hi, lo, (hi / lo if lo > 0.0 else float("inf")), steps
