"""GPU parity of the gradient transformation G Q, Q = T^T T (Sec. 3.1) against the CPU oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import b, dev, ora, relF, workspace, DEV

pytestmark = pytest.mark.gpu
rng = np.random.default_rng(77)


def sym_Q(M, seed):
    r = np.random.default_rng(seed)
    T = np.eye(M) + 0.2 * r.standard_normal((M, M)) / np.sqrt(M)
    return T.astype(np.float32), (T.astype(np.float32).astype(np.float64).T @ T.astype(np.float32).astype(np.float64))


@pytest.mark.parametrize("S,M", [(32, 64), (5, 7), (64, 576), (70, 200), (1, 129), (130, 147), (256, 300), (40, 260), (200, 1156),
                                 (256, 2304), (96, 1024), (17, 4608)])
def test_f32_with_Q(S, M):
    T32, Q64 = sym_Q(M, M)
    Q32 = Q64.astype(np.float32)
    G = (rng.standard_normal((S, M)) * 0.1).astype(np.float32)
    out = torch.full((S, M), float("nan"), device=DEV)
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, dev(Q32), out)
    torch.cuda.synchronize()
    want = ora.grad_transform(G, Q32)
    assert relF(out.cpu().numpy(), want) < 1e-5


@pytest.mark.parametrize("S,M", [(32, 64), (64, 576), (70, 200), (256, 2304), (96, 1024), (17, 4608), (1, 2052), (33, 1156), (512, 1152)])
def test_f32_with_Q_and_the_workspace(S, M):
    """With the whole workspace a product with few output tiles cuts its contraction index into runs (ragged last run
    included) and adds them in a fixed order: same result to float32 rounding, and the same bits on a second call."""
    T32, Q64 = sym_Q(M, M + 5)
    Q32 = Q64.astype(np.float32)
    G = (rng.standard_normal((S, M)) * 0.1).astype(np.float32)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S))
    out = torch.full((S, M), float("nan"), device=DEV)
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, dev(Q32), out, ws)
    torch.cuda.synchronize()
    assert relF(out.cpu().numpy(), ora.grad_transform(G, Q32)) < 1e-5
    out2 = torch.full((S, M), float("nan"), device=DEV)
    ws.fill_(0xFF)                     # nothing in the workspace may matter between calls
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, dev(Q32), out2, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    # bfloat16 gradient through the same path (widened, product in float32, rounded on the way out)
    Gb = wl.round_to_bf16(G)
    wsb = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S, None, b.FW_BF16))
    outb = torch.zeros(S, M, device=DEV, dtype=torch.bfloat16)
    b.fw_grad_transform(dev(Gb, torch.bfloat16), b.FW_BF16, S, M, None, dev(Q32), outb, wsb)
    torch.cuda.synchronize()
    assert relF(outb.float().cpu().numpy(), ora.grad_transform(Gb, Q32)) < 3e-3


@pytest.mark.parametrize("S,M", [(512, 4608), (400, 3076), (384, 3072), (1000, 3200), (1100, 1536), (2100, 1028)])
def test_f32_split_form_for_many_features(S, M):
    """float32 gradients past the size rule of the split form, with the whole workspace: G and Q as bfloat16 hi + lo planes on the
    bfloat16 matrix cores (three products per term, float32 accumulation), the contraction index cut into runs when S
    gives few tiles.  Operands carry 16 significant bits: tolerance 2e-5 (float32 form: 1e-5); reproducible bit for bit."""
    T32, Q64 = sym_Q(M, M + 9)
    Q32 = Q64.astype(np.float32)
    G = (rng.standard_normal((S, M)) * 0.1).astype(np.float32)
    want = ora.grad_transform(G, Q32)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S))
    out = torch.full((S, M), float("nan"), device=DEV)
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, dev(Q32), out, ws)
    torch.cuda.synchronize()
    e = relF(out.cpu().numpy(), want)
    print(f"S={S} M={M}: rel-F = {e:.2e}")
    assert 1e-6 < e < 2e-5            # the split form ran (float32 would be below 1e-6) and is inside its tolerance
    ws.fill_(0xFF)
    out2 = torch.full((S, M), float("nan"), device=DEV)
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, dev(Q32), out2, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    # without the workspace: plain float32
    out3 = torch.full((S, M), float("nan"), device=DEV)
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, dev(Q32), out3)
    torch.cuda.synchronize()
    assert relF(out3.cpu().numpy(), want) < 1e-6
    # bfloat16 gradients of the same size: widened, split form, one rounding at the end
    if M % 4 == 0:
        Gb = wl.round_to_bf16(G)
        wsb = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S, None, b.FW_BF16))
        outb = torch.zeros(S, M, device=DEV, dtype=torch.bfloat16)
        b.fw_grad_transform(dev(Gb, torch.bfloat16), b.FW_BF16, S, M, None, dev(Q32), outb, wsb)
        torch.cuda.synchronize()
        wantb = ora.grad_transform(Gb, Q32)
        assert relF(outb.float().cpu().numpy(), wantb) < 3e-3
        assert np.all(np.abs(outb.float().cpu().numpy() - wantb) <= np.abs(wantb) * 2.0 ** -8 + 1e-5 * np.abs(wantb).max())


@pytest.mark.parametrize("S,M", [(32, 64), (5, 7), (64, 576), (70, 200), (130, 147), (33, 260)])
def test_bf16_with_Q(S, M):
    T32, Q64 = sym_Q(M, M + 1)
    Q32 = Q64.astype(np.float32)
    G = wl.round_to_bf16((rng.standard_normal((S, M)) * 0.1).astype(np.float32))
    out = torch.zeros(S, M, device=DEV, dtype=torch.bfloat16)
    b.fw_grad_transform(dev(G, torch.bfloat16), b.FW_BF16, S, M, None, dev(Q32), out)
    torch.cuda.synchronize()
    want = ora.grad_transform(G, Q32)
    assert relF(out.float().cpu().numpy(), want) < 2e-2
    # against the same computation with Q rounded to bf16 the only error left is accumulation order and output rounding
    want_r = ora.grad_transform(G, wl.round_to_bf16(Q32))
    assert relF(out.float().cpu().numpy(), want_r) < 4e-3
    # with the workspace G is widened and Q is used as it is: only the rounding of the output is left
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S, None, b.FW_BF16))
    out2 = torch.zeros(S, M, device=DEV, dtype=torch.bfloat16)
    b.fw_grad_transform(dev(G, torch.bfloat16), b.FW_BF16, S, M, None, dev(Q32), out2, ws)
    torch.cuda.synchronize()
    assert relF(out2.float().cpu().numpy(), want) < 3e-3
    assert np.array_equal(out2.float().cpu().numpy(), wl.round_to_bf16(ora.grad_transform(G, Q32).astype(np.float32))) or \
        relF(out2.float().cpu().numpy(), wl.round_to_bf16(ora.grad_transform(G, Q32).astype(np.float32))) < 1e-3


@pytest.mark.parametrize("S,M", [(8, 64), (33, 150), (64, 576)])
def test_f32_from_nonsymmetric_T(S, M):
    """Q is built as T^T T (eq. (vQ)); a transposed product would fail for this non-symmetric T."""
    T32, Q64 = sym_Q(M, 3 * M)
    assert not np.allclose(T32, T32.T)
    G = (rng.standard_normal((S, M)) * 0.1).astype(np.float32)
    out = torch.zeros(S, M, device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S))
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, dev(T32), None, out, ws)
    torch.cuda.synchronize()
    want = ora.grad_transform(G, ora.Q_from_T(T32))
    assert relF(out.cpu().numpy(), want) < 1e-5
    wrong = ora.grad_transform(G, T32.astype(np.float64) @ T32.astype(np.float64).T)
    assert relF(out.cpu().numpy(), wrong) > 1e-3


@pytest.mark.parametrize("S,M", [(40, 1536), (24, 1670), (160, 3072)])
def test_f32_from_nonsymmetric_T_split_build(S, M):
    """From FW_REFRESH_SPLIT_MIN_M features on Q = T^T T (eq. (vQ)) is built on the bfloat16 matrix cores from the hi + lo
    planes of T's columns (the product G Q stays in float32 at these sizes): float32-grade results,
    and still T^T T, not T T^T."""
    T32, Q64 = sym_Q(M, 5 * M)
    G = (rng.standard_normal((S, M)) * 0.1).astype(np.float32)
    out = torch.zeros(S, M, device=DEV)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S))
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, dev(T32), None, out, ws)
    torch.cuda.synchronize()
    want = ora.grad_transform(G, ora.Q_from_T(T32))
    err = relF(out.cpu().numpy(), want)
    print(f"raw T, split build: S={S} M={M} rel-F {err:.2e}")
    assert err < 2e-5
    wrong = ora.grad_transform(G, T32.astype(np.float64) @ T32.astype(np.float64).T)
    assert relF(out.cpu().numpy(), wrong) > 1e-3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_large_feature_count(dtype):
    """M = 9216: Q = I + u u^T keeps the float64 reference cheap."""
    S, M = 24, 9216
    r = np.random.default_rng(9)
    u = (r.standard_normal(M) / np.sqrt(M)).astype(np.float32)
    Q32 = (np.eye(M, dtype=np.float32) + np.outer(u, u)).astype(np.float32)
    Q32 = np.maximum(Q32, Q32.T)   # exactly symmetric
    G = (r.standard_normal((S, M)) * 0.1).astype(np.float32)
    want = ora.grad_transform(wl.round_to_bf16(G) if dtype == "bf16" else G, Q32)
    if dtype == "f32":
        out = torch.zeros(S, M, device=DEV)
        b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, dev(Q32), out)
        torch.cuda.synchronize()
        assert relF(out.cpu().numpy(), want) < 1e-5
    else:
        ws = workspace(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S, None, b.FW_BF16))
        out = torch.zeros(S, M, device=DEV, dtype=torch.bfloat16)
        b.fw_grad_transform(dev(wl.round_to_bf16(G), torch.bfloat16), b.FW_BF16, S, M, None, dev(Q32), out, ws)
        torch.cuda.synchronize()
        assert relF(out.float().cpu().numpy(), want) < 3e-3


def test_config1_gradient_with_identity_is_copy():
    L = wl.config1()
    S, M = L.G.shape
    out = torch.zeros(S, M, device=DEV)
    b.fw_grad_transform(dev(L.G), b.FW_F32, S, M, None, torch.eye(M, device=DEV), out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), L.G)


def test_largest_feature_count():
    """M = 16384, the library's limit (Q is 1 GiB): Q = I + u u^T + v v^T keeps the float64 reference a few dot products."""
    S, M = 40, 16384
    r = np.random.default_rng(12)
    u = (r.standard_normal(M) / np.sqrt(M)).astype(np.float32)
    v = (r.standard_normal(M) / np.sqrt(M)).astype(np.float32)
    Q = torch.eye(M, device=DEV)
    ud, vd = dev(u), dev(v)
    Q += torch.outer(ud, ud) + torch.outer(vd, vd)
    Q = torch.maximum(Q, Q.T).contiguous()                       # exactly symmetric
    G = (r.standard_normal((S, M)) * 0.1).astype(np.float32)
    out = torch.full((S, M), float("nan"), device=DEV)
    b.fw_grad_transform(dev(G), b.FW_F32, S, M, None, Q, out)
    torch.cuda.synchronize()
    # the reference from the same float32 Q, block of columns by block of columns
    G64 = G.astype(np.float64)
    num = den = 0.0
    for c0 in range(0, M, 2048):
        want = G64 @ Q[:, c0:c0 + 2048].cpu().numpy().astype(np.float64)
        got = out[:, c0:c0 + 2048].cpu().numpy().astype(np.float64)
        num += float(((got - want) ** 2).sum()); den += float((want ** 2).sum())
    assert (num / den) ** 0.5 < 1e-5
    with pytest.raises(b.FwError):
        b.fw_grad_transform(dev(G[:, :64]), b.FW_F32, S, M + 4, None, Q, out)
