"""GPU parity of the moment accumulation and block-moment epilogue against the CPU oracle (Sec. 2, Sec. 4.1)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import (b, lower, oracle_rows, ora, relF, run_cov, run_finalize, workspace, DEV)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}     # relative Frobenius error on the centred covariance
RAW_TOL = {"f32": 1e-5, "bf16": 1e-5}  # raw sums: products of bf16 values are exact in float32, only summation rounds


def check_layer(layer, layout):
    X = oracle_rows(layer, layout)
    A_o, s_o, n = ora.raw_sums(X)
    A, s = run_cov(layer, layout)
    A_h, s_h = A.cpu().numpy(), s.cpu().numpy()
    assert np.array_equal(np.triu(A_h, 1), np.zeros_like(A_h)), "entries above the diagonal must stay untouched"
    assert relF(lower(A_h), lower(A_o)) < RAW_TOL[layer.dtype]
    assert relF(s_h, s_o) < RAW_TOL[layer.dtype]
    M = layer.desc.M
    mu, Phi, phi, lbar = run_finalize(A, s, n, M, 0.0, 1)
    mu_o, Phi_o, phi_o, lbar_o = ora.block_moments(X, 0.0, True)
    assert relF(Phi.cpu().numpy(), Phi_o) < TOL[layer.dtype]
    # the split form keeps 16 significant bits of every value (residual <= 2^-17 |x|): the column sums of a few hundred rows
    # with means near zero then agree to 1e-5 rather than to float32's 1e-6
    mu_tol = 1e-5 if layer.meta.get("form") == b.FW_COV_FORM_SPLIT else 1e-6
    assert relF(mu.cpu().numpy(), mu_o) < mu_tol and relF(phi.cpu().numpy(), phi_o) < 1e-5
    assert abs(float(lbar[0]) - lbar_o) <= 1e-5 * abs(lbar_o)
    Ph = Phi.cpu().numpy()
    assert np.array_equal(Ph, Ph.T)


ROWS_CASES = [  # (n_rows, M, dtype): ragged tails in both dimensions, single block, odd/even block counts
    (128, 64, "f32"), (37, 5, "f32"), (1000, 147, "f32"), (513, 200, "f32"), (300, 321, "f32"), (64, 1, "f32"),
    (129, 64, "bf16"), (1000, 147, "bf16"), (777, 330, "bf16"),
]


@pytest.mark.parametrize("n_rows,M,dtype", ROWS_CASES)
def test_rows_layout(n_rows, M, dtype):
    check_layer(wl.small_rows(10 + M, n_rows, M, 4, dtype=dtype), b.FW_LAYOUT_ROWS)


CONV_CASES = [  # (B, Cin, H, W, k, stride, pad, dtype)
    (3, 8, 9, 7, 3, 1, 1, "f32"), (2, 16, 8, 8, 3, 2, 1, "f32"), (2, 3, 20, 20, 7, 2, 3, "f32"), (4, 24, 6, 6, 1, 2, 0, "f32"),
    (2, 70, 5, 5, 3, 1, 1, "f32"), (1, 4, 3, 3, 3, 1, 0, "f32"),
    (3, 8, 9, 7, 3, 1, 1, "bf16"), (2, 32, 7, 7, 3, 1, 1, "bf16"), (2, 3, 20, 20, 7, 2, 3, "bf16"), (2, 40, 8, 8, 1, 2, 0, "bf16"),
]


@pytest.mark.parametrize("layout", [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NCHW, b.FW_LAYOUT_NHWC_KKC])
@pytest.mark.parametrize("B,Cin,H,W,k,stride,pad,dtype", CONV_CASES)
def test_conv_layouts(B, Cin, H, W, k, stride, pad, dtype, layout):
    check_layer(wl.small_conv(B * 100 + Cin, B, Cin, H, W, k, stride, pad, 8, dtype=dtype), layout)


SHIFT_CASES = [  # stride-1 windows (B, Cin, H, W, kh, kw, pad): every border shape of the shift-correlation path
    (3, 64, 9, 7, 3, 3, 1), (2, 64, 8, 8, 3, 3, 0), (2, 64, 5, 6, 3, 3, 2), (2, 32, 9, 9, 5, 5, 2), (5, 128, 2, 2, 3, 3, 1),
    (2, 64, 6, 5, 3, 1, 0), (2, 64, 5, 7, 1, 3, 0), (3, 96, 7, 7, 2, 2, 1), (1, 64, 3, 8, 4, 4, 3), (2, 200, 6, 6, 3, 3, 1),
    (40, 64, 12, 11, 3, 3, 1), (1, 256, 1, 1, 3, 3, 1), (2, 64, 3, 3, 3, 3, 0),
    (1, 8, 10, 10, 3, 3, 1), (2, 12, 7, 9, 3, 3, 1), (1, 64, 12, 12, 7, 7, 3), (3, 64, 6, 6, 5, 3, 2), (300, 4, 5, 5, 3, 3, 1), (9, 320, 4, 5, 3, 3, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NCHW, b.FW_LAYOUT_NHWC_KKC])
@pytest.mark.parametrize("B,Cin,H,W,kh,kw,pad", SHIFT_CASES)
def test_stride_one_windows(B, Cin, H, W, kh, kw, pad, layout, dtype):
    rng = np.random.default_rng(B + 10 * Cin + H)
    act = np.abs(rng.standard_normal((B, H, W, Cin)) @ (np.eye(Cin) + 0.3 * rng.standard_normal((Cin, Cin)) / np.sqrt(Cin)))
    act = act.astype(np.float32)
    if dtype == "bf16":
        act = wl.round_to_bf16(act)
    d = wl.ConvDesc(B=B, Cin=Cin, H=H, W=W, kh=kh, kw=kw, stride=1, pad=pad)
    G = np.zeros((4, d.M), dtype=np.float32)
    check_layer(wl.Layer("shift", d, 4, dtype, act, G), layout)


@pytest.fixture
def forced_form(request):
    """The covariance form a test asks for; it travels in the layer's descriptor (``layer.meta["form"]``)."""
    return request.param


# the same border shapes, plus pair-unit specials (odd widths, width 4, even and 1-wide windows, few channels), at sizes
# where the run-time estimate would keep the other form: both forms must give the sums of Sec. 2
FORCED_CASES = SHIFT_CASES + [(9, 64, 4, 4, 3, 3, 1), (3, 16, 13, 4, 3, 2, 0), (5, 60, 9, 5, 3, 3, 1), (2, 36, 15, 15, 3, 3, 1),
                              (17, 48, 7, 7, 2, 2, 1), (2, 128, 6, 7, 3, 3, 1), (3, 100, 5, 8, 3, 3, 1), (3, 64, 5, 9, 3, 4, 2), (2, 64, 7, 5, 2, 5, 0), (8, 24, 6, 10, 5, 5, 4)]


@pytest.mark.parametrize("forced_form", [b.FW_COV_FORM_SHIFT, b.FW_COV_FORM_DIRECT], indirect=True)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NCHW, b.FW_LAYOUT_NHWC_KKC])
@pytest.mark.parametrize("B,Cin,H,W,kh,kw,pad", FORCED_CASES)
def test_stride_one_windows_in_either_form(B, Cin, H, W, kh, kw, pad, layout, dtype, forced_form):
    d = wl.ConvDesc(B=B, Cin=Cin, H=H, W=W, kh=kh, kw=kw, stride=1, pad=pad)
    cd = b.conv_desc(B, Cin, H, W, kh, kw, 1, pad, form=forced_form)
    plan = b.fw_cov_plan_query(b.FW_BF16 if dtype == "bf16" else b.FW_F32, layout, cd)
    if forced_form == b.FW_COV_FORM_DIRECT:
        assert plan.shift == 0
    elif Cin % 4 == 0 and 1 < kh * kw <= 25 and (dtype == "bf16" or layout != b.FW_LAYOUT_NCHW):   # 7 x 7: too many regions
        assert plan.shift == 1, "the shift form applies to this layer and was asked for"
    rng = np.random.default_rng(7 * B + 10 * Cin + H + W)
    act = np.abs(rng.standard_normal((B, H, W, Cin)) @ (np.eye(Cin) + 0.3 * rng.standard_normal((Cin, Cin)) / np.sqrt(Cin)))
    act = act.astype(np.float32)
    if dtype == "bf16":
        act = wl.round_to_bf16(act)
    G = np.zeros((4, d.M), dtype=np.float32)
    check_layer(wl.Layer("forced", d, 4, dtype, act, G, meta={"form": forced_form}), layout)


SKINNY_ROWS = [(5000, 64, "f32"), (4096, 100, "bf16"), (3001, 17, "f32"), (2500, 128, "bf16"), (3000, 5, "f32"), (2049, 33, "bf16"),
               (70000, 96, "f32")]


@pytest.mark.parametrize("n_rows,M,dtype", SKINNY_ROWS)
def test_few_features_many_rows(n_rows, M, dtype):
    """Plain rows with M <= 128 and thousands of rows take the streaming kernel (no staging, one partial result per workgroup)."""
    layer = wl.small_rows(20 + M, n_rows, M, 4, dtype=dtype)
    assert b.fw_cov_plan_query(b.FW_BF16 if dtype == "bf16" else b.FW_F32, b.FW_LAYOUT_ROWS, b.conv_desc(*layer.desc.astuple())).shift == 0
    check_layer(layer, b.FW_LAYOUT_ROWS)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NCHW, b.FW_LAYOUT_NHWC_KKC])
@pytest.mark.parametrize("B,Cin,H,W,stride", [(16, 64, 31, 30, 2), (8, 96, 20, 20, 1), (40, 16, 9, 9, 1), (6, 128, 33, 17, 3)])
def test_pointwise_windows(B, Cin, H, W, stride, layout, dtype):
    """1x1 windows (the per-channel variant, shortcut convolutions): strided pixel subsets of a channels-last tensor."""
    check_layer(wl.small_conv(B + Cin, B, Cin, H, W, 1, stride, 0, 8, dtype=dtype), layout)


def test_accumulates_over_batches_and_two_block_recursion():
    """Two batches added into one block equal the block of their union; the second block follows eqs. (vmuxi), (vPhixi)."""
    L0 = wl.small_conv(1, 3, 8, 6, 6, 3, 1, 1, 8)
    L1 = wl.small_conv(2, 3, 8, 6, 6, 3, 1, 1, 8)
    L2 = wl.small_conv(3, 3, 8, 6, 6, 3, 1, 1, 8, relu=True)
    X0, X1, X2 = (oracle_rows(L) for L in (L0, L1, L2))
    M = L0.desc.M
    A, s = run_cov(L0, b.FW_LAYOUT_NHWC)
    A, s = run_cov(L1, b.FW_LAYOUT_NHWC, A, s)
    X01 = np.vstack([X0, X1])
    mu, Phi, phi, lbar = run_finalize(A, s, X01.shape[0], M, 0.3, 1)
    mu_o, Phi_o, phi_o, lb_o = ora.block_moments(X01, 0.3, True)
    assert relF(Phi.cpu().numpy(), Phi_o) < 1e-4
    A2, s2 = run_cov(L2, b.FW_LAYOUT_NHWC)
    mu, Phi, phi, lbar = run_finalize(A2, s2, X2.shape[0], M, 0.3, 0, mu, Phi, phi)
    mu_o2, Phi_o2, phi_o2, lb_o2 = ora.block_moments(X2, 0.3, False, mu_o, Phi_o, phi_o)
    assert relF(Phi.cpu().numpy(), Phi_o2) < 1e-4 and relF(mu.cpu().numpy(), mu_o2) < 1e-6
    assert relF(phi.cpu().numpy(), phi_o2) < 1e-5 and abs(float(lbar[0]) - lb_o2) < 1e-5 * lb_o2


@pytest.mark.parametrize("layout", [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC])
@pytest.mark.parametrize("B,Cin,HW,dtype", [(16, 96, 6, "bf16"), (9, 160, 5, "bf16"), (16, 64, 8, "f32")])
def test_several_tiles_and_single_range(B, Cin, HW, dtype, layout):
    """M = 9*Cin spans several 256-feature tiles with a ragged last one; few rows, so a tile gets a single row range."""
    check_layer(wl.small_conv(B + Cin, B, Cin, HW, HW, 3, 1, 1, 8, dtype=dtype), layout)


@pytest.mark.parametrize("layout", [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC])
@pytest.mark.parametrize("B,Cin,HW,dtype", [(8, 1024, 4, "bf16"), (4, 1024, 3, "f32")])
def test_large_feature_count(B, Cin, HW, dtype, layout):
    """M = 9216 features (more than half of the limit of 16384): dozens of tile rows, few patch rows."""
    check_layer(wl.small_conv(41, B, Cin, HW, HW, 3, 1, 1, 8, dtype=dtype), layout)


def test_config1_covariance():
    check_layer(wl.config1(), b.FW_LAYOUT_ROWS)


def test_empty_and_bad_arguments_on_device():
    M = 8
    A = torch.zeros(M, M, device=DEV); s = torch.zeros(M, device=DEV)
    X = torch.zeros(4, M, device=DEV)
    ws = workspace(1 << 20)
    d = b.conv_desc(0, M)
    with pytest.raises(b.FwError) as e:
        b.fw_cov_accumulate(X, b.FW_F32, b.FW_LAYOUT_ROWS, d, A, s, ws)
    assert e.value.status == b.FW_ERR_INVALID_ARG
    with pytest.raises(b.FwError) as e:
        b.fw_cov_accumulate(X, b.FW_F32, b.FW_LAYOUT_ROWS, b.conv_desc(4, M), A, s, workspace(256))
    assert e.value.status == b.FW_ERR_WORKSPACE
    assert float(A.abs().sum()) == 0.0


def test_run_to_run_determinism():
    L = wl.small_conv(5, 4, 32, 10, 10, 3, 1, 1, 8)
    A1, s1 = run_cov(L, b.FW_LAYOUT_NHWC)
    A2, s2 = run_cov(L, b.FW_LAYOUT_NHWC)
    assert torch.equal(A1, A2) and torch.equal(s1, s2)


@pytest.mark.parametrize("forced_form", [b.FW_COV_FORM_AUTO, b.FW_COV_FORM_SHIFT], indirect=True)
def test_seeded_sweep_of_window_shapes(forced_form):
    """Eighty seeded random layers (windows 1..5 squared or not, strides 1..3, every layout, both precisions, odd sizes):
    raw sums against the oracle's, once with the estimate's own choice of form and once with the shift form wherever it
    applies."""
    rng = np.random.default_rng(1546 + forced_form)
    done = 0
    while done < 80:
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride = int(rng.choice([1, 1, 1, 2, 3]))
        pad = int(rng.integers(0, min(kh, kw)))
        H, W = int(rng.integers(1, 14)), int(rng.integers(1, 14))
        Cin = int(rng.choice([1, 3, 4, 8, 12, 16, 20, 32, 64, 68, 96, 128, 132, 200, 256]))
        if Cin * kh * kw > 2400:
            Cin = max(4, 2400 // (kh * kw) // 4 * 4)
        B = int(rng.choice([1, 2, 3, 5, 8, 9, 17, 40, 130]))
        dtype = str(rng.choice(["f32", "bf16"]))
        layout = int(rng.choice([b.FW_LAYOUT_NCHW, b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC]))
        if H + 2 * pad < kh or W + 2 * pad < kw:
            continue
        d = wl.ConvDesc(B=B, Cin=Cin, H=H, W=W, kh=kh, kw=kw, stride=stride, pad=pad)
        if d.n_rows * d.M * d.M > 1.5e9 or d.n_rows * d.M > 3e7:
            continue
        act = np.abs(rng.standard_normal((B, H, W, Cin))).astype(np.float32)
        if dtype == "bf16":
            act = wl.round_to_bf16(act)
        layer = wl.Layer("sweep", d, 4, dtype, act, np.zeros((4, d.M), np.float32), meta={"form": forced_form})
        case = (B, Cin, H, W, kh, kw, stride, pad, dtype, layout)
        A_o, s_o, n = ora.raw_sums(oracle_rows(layer, layout))
        A, s = run_cov(layer, layout)
        A_h = A.cpu().numpy()
        assert relF(lower(A_h), lower(A_o)) < RAW_TOL[dtype], case
        assert relF(s.cpu().numpy(), s_o) < RAW_TOL[dtype], case
        assert np.array_equal(np.triu(A_h, 1), np.zeros_like(A_h)), case
        done += 1


SPLIT_CASES = [  # B, Cin, H, W, kh, kw, stride, pad
    (9, 64, 8, 8, 3, 3, 1, 1), (5, 24, 9, 7, 3, 3, 1, 1), (4, 16, 11, 10, 5, 5, 2, 2), (6, 6, 7, 9, 3, 3, 1, 0), (3, 32, 6, 6, 1, 1, 1, 0),
    (17, 12, 5, 6, 2, 3, 1, 1), (2, 132, 6, 5, 3, 3, 1, 1)]


@pytest.mark.parametrize("layout", [b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NCHW, b.FW_LAYOUT_NHWC_KKC])
@pytest.mark.parametrize("B,Cin,H,W,kh,kw,stride,pad", SPLIT_CASES)
def test_float32_input_in_the_split_form(B, Cin, H, W, kh, kw, stride, pad, layout):
    """float32 activations taken as hi + lo bfloat16 pairs on the bfloat16 kernels (asked for through the descriptor): the
    same sums to the accuracy of a 16-bit split, every layout and feature order, windows with and without stride."""
    d = wl.ConvDesc(B=B, Cin=Cin, H=H, W=W, kh=kh, kw=kw, stride=stride, pad=pad)
    cd = b.conv_desc(B, Cin, H, W, kh, kw, stride, pad, form=b.FW_COV_FORM_SPLIT)
    plan = b.fw_cov_plan_query(b.FW_F32, layout, cd)
    if layout == b.FW_LAYOUT_NCHW and Cin % 4 != 0:
        assert plan.split_bf16 == 0        # raw NCHW with odd channel counts stays on the float32 kernels
    else:
        assert plan.split_bf16 == 1
    rng = np.random.default_rng(B * 131 + Cin)
    act = np.abs(rng.standard_normal((B, H, W, Cin)) @ (np.eye(Cin) + 0.3 * rng.standard_normal((Cin, Cin)) / np.sqrt(Cin))).astype(np.float32)
    check_layer(wl.Layer("split", d, 4, "f32", act, np.zeros((4, d.M), np.float32), meta={"form": b.FW_COV_FORM_SPLIT}), layout)


def test_split_form_on_plain_rows_and_by_estimate():
    # plain rows, asked for
    layer = wl.small_rows(31, 700, 200, 4, dtype="f32")
    layer.meta["form"] = b.FW_COV_FORM_SPLIT
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_ROWS, b.conv_desc(*layer.desc.astuple(), form=b.FW_COV_FORM_SPLIT)).split_bf16 == 1
    check_layer(layer, b.FW_LAYOUT_ROWS)
    # the estimate takes it for large layers only, and never for bfloat16 input or when a float32 form is asked for
    big = dict(B=128, Cin=64, H=32, W=32, kh=3, kw=3, stride=1, pad=1)
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC_KKC, b.conv_desc(**big)).split_bf16 == 1
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC_KKC, b.conv_desc(**big, form=b.FW_COV_FORM_SHIFT)).split_bf16 == 0
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC_KKC, b.conv_desc(**big, form=b.FW_COV_FORM_DIRECT)).split_bf16 == 0
    assert b.fw_cov_plan_query(b.FW_BF16, b.FW_LAYOUT_NHWC_KKC, b.conv_desc(**big, form=b.FW_COV_FORM_SPLIT)).split_bf16 == 0
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC, b.conv_desc(4, 64, 8, 8, 3, 3, 1, 1)).split_bf16 == 0


@pytest.mark.parametrize("n_rows,M", [(1100, 2304), (300, 4100), (9000, 1028)])
def test_many_features_go_to_the_split_form_by_estimate(n_rows, M):
    """float32 rows with many features: past the measured break-even the estimate itself hands the layer to the split form
    (the float32 kernel's 64 x 64 blocks re-read their panels per block); same parity bar."""
    layer = wl.small_rows(n_rows + M, n_rows, M, 4, dtype="f32")
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_ROWS, b.conv_desc(*layer.desc.astuple())).split_bf16 == 1
    layer.meta["form"] = b.FW_COV_FORM_SPLIT      # the mean's bound of the split form (the plan is the same)
    check_layer(layer, b.FW_LAYOUT_ROWS)
    # just below the break-even the float32 kernel stays
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_ROWS, b.conv_desc(1000, 2304, 1, 1, 1, 1, 1, 0)).split_bf16 == 0
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_ROWS, b.conv_desc(100000, 500, 1, 1, 1, 1, 1, 0)).split_bf16 == 0



@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_largest_feature_count(dtype):
    """M = 16384, the library's limit (A is 1 GiB): a handful of rows keeps the float64 reference cheap; compared row
    block by row block on the device-side copy; one more feature is refused."""
    n_rows, M = 6, 16384
    rng = np.random.default_rng(5)
    X = (rng.standard_normal((n_rows, M)) + 0.25).astype(np.float32)
    if dtype == "bf16":
        X = wl.round_to_bf16(X)
    layer = wl.Layer("max-M", wl.ConvDesc(B=n_rows, Cin=M, H=1, W=1), 4, dtype, X, np.zeros((4, M), np.float32), is_rows=True)
    A, s = run_cov(layer, b.FW_LAYOUT_ROWS)
    X64 = X.astype(np.float64)
    assert relF(s.cpu().numpy(), X64.sum(axis=0)) < 1e-5
    num = den = 0.0
    for r0 in range(0, M, 2048):
        want = X64[:, r0:r0 + 2048].T @ X64                       # rows r0 .. of X^T X
        got = A[r0:r0 + 2048].cpu().numpy().astype(np.float64)
        mask = np.arange(M)[None, :] <= (r0 + np.arange(want.shape[0]))[:, None]
        assert not got[~mask].any(), "entries above the diagonal must stay untouched"
        num += float(((got - want)[mask] ** 2).sum())
        den += float((want[mask] ** 2).sum())
    assert (num / den) ** 0.5 < 1e-5
    del A
    d = b.conv_desc(n_rows, M + 1, 1, 1, 1, 1, 1, 0)
    assert b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, M + 1, 0, d, b.FW_F32) == 0
