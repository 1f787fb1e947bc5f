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
    """The layer's geometry; ``layer.meta["form"]`` (a fw_cov_form) asks for one of the two covariance forms."""
    return b.conv_desc(*layer.desc.astuple(), form=layer.meta.get("form", 0))


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


BAND = 2e-5   # relative guard band of a decision taken in float32 on the GPU and in float64 by the oracle


def membership_band(M, c_rel):
    """Guard band (relative to the threshold) of the coherence-set decision |c_m| >= c_rel xi_m' xi_m taken in float32:
    c_m is an M-term float32 dot product, rounding error about 2^-24 sqrt(M) xi_m' xi_m (random-sign model, four standard
    deviations allowed), which is that amount divided by c_rel when measured against the threshold."""
    return max(BAND, 4.0 * 2.0 ** -24 * np.sqrt(M) / max(c_rel, 1e-3))


def marginal_decision_ok(info, oi, op, band_argmax=BAND, band_set=None):
    """The GPU's integer decisions differ from the oracle's: true when the difference is explained by rounding (the
    GPU's arg-max is within the band of the oracle's maximum, and the GPU's set size lies between the number of members
    that are in beyond doubt and that number plus the members inside the band).  Prints what it found otherwise."""
    M = oi.xi.shape[0]
    band_set = membership_band(M, op.c_rel) if band_set is None else band_set
    if not oi.xi[info.m_prime] >= oi.xi[oi.m_prime] * (1 - band_argmax):
        print(f"arg-max: gpu {info.m_prime} (xi {oi.xi[info.m_prime]:.9g}) oracle {oi.m_prime} (xi {oi.xi[oi.m_prime]:.9g}), band {band_argmax:g}")
        return False
    xi, c = oi.xi, ora.high_power_subspace(oi.Phi_y, op.c_rel, op.c_abs, 0, forced_m_prime=info.m_prime)[4]
    thr = np.maximum(op.c_rel * xi[info.m_prime] * xi, op.c_abs)
    sure_in = np.abs(c) >= thr * (1 + band_set)
    sure_out = np.abs(c) < thr * (1 - band_set)
    n_marg = int((~sure_in & ~sure_out).sum())
    ok = bool(sure_in.sum() <= info.set_size <= sure_in.sum() + n_marg)
    if not ok:
        ratio = np.sort(np.abs(np.abs(c) / thr - 1.0))[:6]
        print(f"coherence set: gpu size {info.set_size}, oracle {oi.set_size} (m' gpu {info.m_prime}, oracle {oi.m_prime}); sure members "
              f"{int(sure_in.sum())}, inside the band {n_marg} (band {band_set:g}); smallest relative margins {ratio}")
    return ok


def oracle_params(gp):
    return ora.CondParams(gamma=gp.gamma, delta=gp.delta, eps=gp.eps, c_rel=gp.c_rel, c_abs=gp.c_abs, beta=gp.beta,
                          n_power_iters=gp.n_power_iters, guard=bool(gp.guard))


def forced_step(run: CondRunner, P64, lbar32, gp, op, tol=1e-4, label=""):
    """One teacher-forced step: the oracle starts from the GPU's own state (up-cast), both take one step.

    Returns (compared, info, oracle_info, new_oracle_state).  The integer decisions (arg-max m', membership in the
    coherence set) must agree unless the deciding margin lies inside the guard band: then `compared` is False (marginal
    members cannot be told apart from outside) and the caller resynchronises from the GPU state at the next step.
    Otherwise T, Q, Qs, Phi_y (and Psi) are compared element by element and lambda_e, g_e as scalars."""
    st = ora.CondState(P64, run.host("T"), run.host("Q"), run.host("Qs"))
    info = run.step(gp)
    new, oi = ora.cond_reduce_step(st, lbar32, op)
    if info.m_prime != oi.m_prime or info.set_size != oi.set_size:
        assert marginal_decision_ok(info, oi, op), f"{label}: arg-max or coherence set differs beyond rounding"
        return False, info, oi, new
    assert bool(info.applied) == oi.applied, label
    if oi.applied:
        assert abs(info.lambda_e - oi.lambda_e) <= 2e-4 * abs(oi.lambda_e), label
        assert abs(info.g_e - oi.g_e) <= 2e-4 * abs(oi.g_e), label
    errs = [relF(run.host("T"), new.T), relF(run.host("Q"), new.Q), relF(run.host("Qs"), new.Qs),
            relF(run.host("Phi_y"), ora.transformed_covariance(new.T, P64))]
    if run.Psi is not None:
        errs.append(relF(run.host("Psi"), new.T @ P64))
    assert max(errs) < tol, f"{label}: {errs}"
    # carried column norms belong to the new Phi_y
    assert relF(run.host("xi2"), np.sum(run.host("Phi_y") ** 2, axis=0)) < 1e-5, label
    return True, info, oi, new


def oracle_first_block_moments_chunked(layer: wl.Layer, layout: int, images_per_chunk: int):
    """First-block moments of a layer too large to unfold at once: mean over image chunks, then the centred products
    sum (x - mu)(x - mu)^T over the same chunks (the centred form of eqs. (vmuxnz), (vPhixnz), raw squares for eq.
    (phixmi)), all through the oracle's own unfolding and sums."""
    d = layer.desc
    order = "kkc" if layout == b.FW_LAYOUT_NHWC_KKC else "ckk"
    if layer.is_rows:
        return ora.block_moments(np.asarray(layer.act, dtype=np.float64), 0.0, True)
    M = d.M
    geo = (d.Cin, d.H, d.W, d.kh, d.kw, d.stride, d.pad)
    s = np.zeros(M); sq = np.zeros(M); n = 0
    for lo in range(0, d.B, images_per_chunk):
        hi = min(d.B, lo + images_per_chunk)
        X = ora.patch_rows(layer.act[lo:hi], hi - lo, *geo, order=order)
        s += X.sum(axis=0); sq += (X * X).sum(axis=0); n += X.shape[0]
    mu = s / n
    C = np.zeros((M, M))
    for lo in range(0, d.B, images_per_chunk):
        hi = min(d.B, lo + images_per_chunk)
        X = ora.patch_rows(layer.act[lo:hi], hi - lo, *geo, order=order)
        X -= mu[None, :]
        C += ora.raw_sums(X)[0]
    phi = sq / n
    return mu, C / n, phi, float(phi.mean())
