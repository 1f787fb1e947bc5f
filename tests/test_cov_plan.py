"""Host logic of the covariance planning (no GPU): which form a layer takes, and invariants of the shift-correlation
decomposition (Sec. 2 sums over unfolded rows, re-grouped by tap difference): the regions partition the pixels, the
number of kept differences is one of each +/- pair, the grid of the float32 kernel fits one round of the compute units."""
import pytest

from paper_2010_01546_amd import binding as b

SHAPES = [  # B, Cin, H, W, kh, kw, stride, pad
    (128, 64, 32, 32, 3, 3, 1, 1), (256, 256, 14, 14, 3, 3, 1, 1), (256, 512, 7, 7, 3, 3, 1, 1), (2, 64, 8, 8, 3, 3, 1, 0),
    (2, 64, 5, 6, 3, 3, 1, 2), (2, 32, 9, 9, 5, 5, 1, 2), (5, 128, 2, 2, 3, 3, 1, 1), (2, 64, 6, 5, 3, 1, 1, 0), (3, 96, 7, 7, 2, 2, 1, 1),
    (1, 64, 3, 8, 4, 4, 1, 3), (1, 256, 1, 1, 3, 3, 1, 1), (256, 64, 56, 56, 3, 3, 1, 1), (256, 128, 28, 28, 3, 3, 1, 1),
]


@pytest.mark.parametrize("dt", [b.FW_F32, b.FW_BF16])
@pytest.mark.parametrize("shape", SHAPES)
def test_stride_one_windows_take_the_shift_form(shape, dt):
    B, Cin, H, W, kh, kw, stride, pad = shape
    # float32: the shift form in the input's own precision is asked for (left to itself the estimate would hand the large
    # layers to the split form, whose plan is that of a bfloat16 layer with twice the channels)
    d = b.conv_desc(*shape, form=b.FW_COV_FORM_SHIFT if dt == b.FW_F32 else b.FW_COV_FORM_AUTO)
    for lay in (b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC, b.FW_LAYOUT_NCHW):
        p = b.fw_cov_plan_query(dt, lay, d)
        assert p.split_bf16 == 0
        if dt == b.FW_BF16 and B < 128 and p.shift == 0:
            continue   # tiny bfloat16 layers: the cost estimate may keep the direct form
        assert p.shift == 1, (shape, lay)
        pairs = dt == b.FW_BF16 and Cin <= 128 and W >= 4   # bfloat16 with few channels: units are pairs of pixels
        kwu = kw // 2 + 1 if pairs else kw
        assert p.differences == ((2 * kh - 1) * (2 * kwu - 1) + 1) // 2
        # every pixel of a stride-1 window with pad < k lies under some window; the regions are disjoint
        assert p.covered_pixels == B * H * W
        assert 1 <= p.regions <= 32 and p.ranges >= p.regions
        Ho, Wo = H + 2 * pad - kh + 1, W + 2 * pad - kw + 1
        M = Cin * kh * kw
        algorithmic = float(B * Ho * Wo) * M * (M + 1)
        assert p.mfma_flops_issued > 0
        if Cin % 64 == 0 and H * W >= 49 and 2 * pad == kh - 1 and dt == b.FW_F32:
            assert p.mfma_flops_issued < 0.5 * algorithmic      # the point of the form: far fewer multiplications
        if dt == b.FW_F32:
            assert p.workgroups <= 256 or p.ranges == p.regions  # one round of the 256 compute units


@pytest.mark.parametrize("dt", [b.FW_F32, b.FW_BF16])
@pytest.mark.parametrize("shape,lay", [((256, 3, 224, 224, 7, 7, 2, 3), b.FW_LAYOUT_NHWC), ((256, 64, 56, 56, 3, 3, 2, 1), b.FW_LAYOUT_NHWC),
                                       ((256, 64, 56, 56, 1, 1, 2, 0), b.FW_LAYOUT_NHWC), ((256, 512, 1, 1, 1, 1, 1, 0), b.FW_LAYOUT_ROWS),
                                       ((4, 6, 8, 8, 3, 3, 1, 1), b.FW_LAYOUT_NHWC)])
def test_other_shapes_keep_the_direct_form(shape, lay, dt):
    p = b.fw_cov_plan_query(dt, lay, b.conv_desc(*shape))
    assert p.shift == 0 and p.regions == 0 and p.covered_pixels == 0
    assert p.workgroups >= 1 and p.mfma_flops_issued > 0


def test_headline_workload_numbers():
    """Config 2: 9 regions, 13 differences, 64 x 832 x 131072 products."""
    p = b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC_KKC, b.conv_desc(128, 64, 32, 32, 3, 3, 1, 1, form=b.FW_COV_FORM_SHIFT))
    assert (p.shift, p.regions, p.differences) == (1, 9, 13)
    assert p.mfma_flops_issued == 2.0 * 64 * 832 * 131072
    assert p.workgroups <= 256
    # left to the estimate, the same layer goes to the bfloat16 matrix cores as 128 channels of hi + lo planes (pairs of
    # pixels as units: 8 differences), and issues bfloat16 flops
    q = b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC_KKC, b.conv_desc(128, 64, 32, 32, 3, 3, 1, 1))
    bf = b.fw_cov_plan_query(b.FW_BF16, b.FW_LAYOUT_NHWC_KKC, b.conv_desc(128, 128, 32, 32, 3, 3, 1, 1))
    assert q.split_bf16 == 1 and (q.shift, q.regions, q.differences, q.mfma_flops_issued) == (bf.shift, bf.regions, bf.differences, bf.mfma_flops_issued)


def test_bad_arguments():
    with pytest.raises(b.FwError):
        b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC, b.conv_desc(0, 64, 8, 8, 3, 3, 1, 1))
    with pytest.raises(b.FwError):
        b.fw_cov_plan_query(7, b.FW_LAYOUT_NHWC, b.conv_desc(2, 64, 8, 8, 3, 3, 1, 1))


def test_form_preference():
    """The form asked for in the descriptor overrides the estimate where both forms apply, and nothing else; workspace
    size and plan follow the same descriptor, and there is no setting outside it."""
    small = dict(B=2, Cin=64, H=9, W=7, kh=3, kw=3, stride=1, pad=1)
    strided = dict(small, stride=2)
    big = dict(B=128, Cin=64, H=32, W=32, kh=3, kw=3, stride=1, pad=1)
    assert b.fw_cov_plan_query(b.FW_BF16, b.FW_LAYOUT_NHWC, b.conv_desc(**small)).shift == 0
    p = b.fw_cov_plan_query(b.FW_BF16, b.FW_LAYOUT_NHWC, b.conv_desc(**small, form=b.FW_COV_FORM_SHIFT))
    assert p.shift == 1 and p.covered_pixels == 2 * 9 * 7
    assert b.fw_cov_plan_query(b.FW_BF16, b.FW_LAYOUT_NHWC, b.conv_desc(**small)).shift == 0      # the request left no trace
    assert b.fw_cov_plan_query(b.FW_BF16, b.FW_LAYOUT_NHWC, b.conv_desc(**strided, form=b.FW_COV_FORM_SHIFT)).shift == 0
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC, b.conv_desc(**big, form=b.FW_COV_FORM_DIRECT)).shift == 0
    assert b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC, b.conv_desc(**big)).shift == 1
    with pytest.raises(b.FwError):
        b.fw_cov_plan_query(b.FW_F32, b.FW_LAYOUT_NHWC, b.conv_desc(**big, form=4))
    assert b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, 576, 0, b.conv_desc(**big, form=4), b.FW_F32) == 0
    # the two forms need different scratch: sized from the same descriptor the call will get
    w_shift = b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, 576, 0, b.conv_desc(**big, form=b.FW_COV_FORM_SHIFT), b.FW_BF16)
    w_direct = b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, 576, 0, b.conv_desc(**big, form=b.FW_COV_FORM_DIRECT), b.FW_BF16)
    assert w_shift > 0 and w_direct > 0 and w_shift != w_direct
    assert not hasattr(b.lib, "fw_cov_set_form")


def test_plan_invariants_on_random_layers():
    """Seeded sweep of stride-1 layers in both precisions, the shift form asked for: wherever it is taken the regions
    partition the pixels that lie under some window, one of each +/- pair of differences is kept (of pixel pairs for
    bfloat16 up to 128 channels), the matrix cores are not asked for more than the direct form's work on a chip-filling
    layer, and the query is repeatable (cached geometry == fresh geometry)."""
    import random
    rnd = random.Random(20101546)
    if True:
        taken = 0
        for _ in range(300):
            kh, kw = rnd.choice([(3, 3), (3, 3), (5, 5), (2, 2), (1, 3), (3, 1), (4, 2), (7, 7), (2, 5)])
            Cin = 4 * rnd.randint(1, 80)
            H, W = rnd.randint(1, 40), rnd.randint(1, 40)
            pad = rnd.randint(0, min(kh, kw) - 1)   # a window may not lie wholly in the padding
            B = rnd.choice([1, 3, 8, 64, 256])
            if H + 2 * pad < kh or W + 2 * pad < kw:
                continue
            d = b.conv_desc(B, Cin, H, W, kh, kw, 1, pad, form=b.FW_COV_FORM_SHIFT)
            Ho, Wo = H + 2 * pad - kh + 1, W + 2 * pad - kw + 1
            # pixels under some window: rows y with an output row oy = y - ty + pad in [0, Ho) for some tap row ty
            rows = sum(1 for y in range(H) if any(0 <= y - t + pad < Ho for t in range(kh)))
            cols = sum(1 for x in range(W) if any(0 <= x - t + pad < Wo for t in range(kw)))
            for dt in (b.FW_F32, b.FW_BF16):
                lay = rnd.choice([b.FW_LAYOUT_NHWC, b.FW_LAYOUT_NHWC_KKC])
                p = b.fw_cov_plan_query(dt, lay, d)
                again = b.fw_cov_plan_query(dt, lay, d)
                assert (p.shift, p.regions, p.differences, p.workgroups, p.ranges, p.covered_pixels, p.mfma_flops_issued) == \
                       (again.shift, again.regions, again.differences, again.workgroups, again.ranges, again.covered_pixels,
                        again.mfma_flops_issued)
                if not p.shift:
                    continue
                taken += 1
                assert p.covered_pixels == B * rows * cols, (B, Cin, H, W, kh, kw, pad, dt)
                kwu = kw // 2 + 1 if (dt == b.FW_BF16 and Cin <= 128 and W >= 4) else kw
                assert p.differences == ((2 * kh - 1) * (2 * kwu - 1) + 1) // 2
                assert 1 <= p.regions <= 32 and p.ranges >= p.regions and p.workgroups >= 1
                assert p.mfma_flops_issued > 0
        assert taken > 200


def test_refresh_plan():
    """The refresh takes the split form only with the full workspace and from FW_REFRESH_SPLIT_MIN_M features on; its
    issued flops are three bfloat16 terms per product on whole tiles, the second product on the lower triangle only."""
    full = b.fw_workspace_bytes(b.FW_OP_COND_STATE_REFRESH, 4608)
    p = b.fw_cond_refresh_plan_query(4608, full)
    assert p.split == 1
    dense = 2.0 * 4608 ** 3
    assert 3 * dense * 1.5 <= p.mfma_flops_issued <= 3 * dense * 1.7        # one full product + a good half
    assert b.fw_cond_refresh_plan_query(4608, full - 256).split == 0
    assert b.fw_cond_refresh_plan_query(4608, 0).mfma_flops_issued == 2 * dense
    small = b.fw_cond_refresh_plan_query(b.FW_REFRESH_SPLIT_MIN_M - 64, 1 << 40)
    assert small.split == 0
    assert b.fw_cond_refresh_plan_query(b.FW_REFRESH_SPLIT_MIN_M, 1 << 40).split == 1
    with pytest.raises(b.FwError):
        b.fw_cond_refresh_plan_query(0, 0)


def test_grad_plan():
    """The gradient product takes the split form for float32 gradients of large products (size rule of the header) when the
    call has its whole workspace; its issued flops are then three bfloat16 terms on whole tiles."""
    S, M = 512, 4608
    full = b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S)
    p = b.fw_grad_plan_query(b.FW_F32, S, M, full)
    dense = 2.0 * S * M * M
    assert p.split == 1 and 3 * dense <= p.mfma_flops_issued <= 3 * dense * 1.2
    q = b.fw_grad_plan_query(b.FW_F32, S, M, full - 256)
    assert q.split == 0 and q.mfma_flops_issued == dense
    assert b.fw_grad_plan_query(b.FW_F32, 256, 2304, 1 << 40).split == 0      # product too small (config 3)
    assert b.fw_grad_plan_query(b.FW_F32, 512, 2304, 1 << 40).split == 1
    assert b.fw_grad_plan_query(b.FW_F32, 1024, 1152, 1 << 40).split == 0
    assert b.fw_grad_plan_query(b.FW_F32, 2048, 1152, 1 << 40).split == 1
    assert b.fw_grad_plan_query(b.FW_F32, 4096, 1000, 1 << 40).split == 0     # too few features
    assert b.fw_grad_plan_query(b.FW_F32, 64, 4608, 1 << 40).split == 0       # too few rows
    assert b.fw_grad_plan_query(b.FW_BF16, S, M, 1 << 40).split == 0          # bfloat16 gradients take the widened form
    with pytest.raises(b.FwError):
        b.fw_grad_plan_query(b.FW_F32, 0, M, 0)

