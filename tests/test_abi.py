"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares, reports sizes and
rejects bad arguments before touching a device.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2010_01546_amd", "libfw.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2010_01546_amd.build import build
        build(verbose=False)
    return C.CDLL(LIB)


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fw.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fw_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"fw_cov_accumulate", "fw_grad_transform", "fw_cond_reduce_step", "fw_whiten_evd"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_names_match_header():
    from paper_2010_01546_amd import binding
    for n in declared_symbols():
        assert hasattr(binding, n), n
    assert binding.fw_version() == 103
    assert binding.fw_status_string(0) == "ok" and "workspace" in binding.fw_status_string(4)
    assert C.sizeof(binding.fw_cond_info) == 32 and C.sizeof(binding.fw_conv_desc) == 36


def test_workspace_sizes():
    from paper_2010_01546_amd import binding as b
    d = b.conv_desc(128, 64, 32, 32, 3, 3, 1, 1)
    n = b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, 576, 0, d, b.FW_F32)
    assert n > 0 and n % 256 == 0 and n < (1 << 30)
    assert b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, 576, 0, None, b.FW_F32) == 0
    assert b.fw_workspace_bytes(b.FW_OP_COND_REDUCE_STEP, 4608) > 7 * 4608 * 4
    assert b.fw_workspace_bytes(b.FW_OP_WHITEN_EVD, 64) >= 2 * 64 * 64 * 8
    assert b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, 64, 32) >= 64 * 64 * 4
    assert (b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, 64, 32, None, b.FW_BF16)
            >= b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, 64, 32) + 32 * 64 * 4)
    assert b.fw_workspace_bytes(b.FW_OP_COND_REDUCE_STEP, 0) == 0
    assert b.fw_workspace_bytes(b.FW_OP_WHITEN_EVD, 1 << 20) == 0


def test_argument_validation_without_a_device():
    from paper_2010_01546_amd import binding as b
    L = b.lib
    d = b.conv_desc(4, 8, 5, 5, 3, 3, 1, 1)
    fake = 0x1000  # aligned, never dereferenced: validation fails first
    # NULL pointers
    assert L.fw_cov_accumulate(None, 0, 2, C.byref(d), fake, fake, fake, 1 << 30, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_cov_accumulate(fake, 0, 2, None, fake, fake, fake, 1 << 30, None) == b.FW_ERR_INVALID_ARG
    # bad enum, bad geometry
    assert L.fw_cov_accumulate(fake, 7, 2, C.byref(d), fake, fake, fake, 1 << 30, None) == b.FW_ERR_INVALID_ARG
    bad = b.conv_desc(4, 8, 5, 5, 3, 3, 0, 1)
    assert L.fw_cov_accumulate(fake, 0, 2, C.byref(bad), fake, fake, fake, 1 << 30, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_cov_accumulate(fake, 0, 0, C.byref(d), fake, fake, fake, 1 << 30, None) == b.FW_ERR_INVALID_ARG  # ROWS with a window
    # alignment, workspace
    assert L.fw_cov_accumulate(fake + 4, 0, 2, C.byref(d), fake, fake, fake, 1 << 30, None) == b.FW_ERR_ALIGNMENT
    assert L.fw_cov_accumulate(fake, 0, 2, C.byref(d), fake, fake, None, 0, None) == b.FW_ERR_WORKSPACE
    assert L.fw_cov_accumulate(fake, 0, 2, C.byref(d), fake, fake, fake, 16, None) == b.FW_ERR_WORKSPACE
    # measurement helper
    assert L.fw_mfma_rate_probe(0, 100, None, None, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_mfma_rate_probe(0, 0, fake, None, None) == b.FW_ERR_INVALID_ARG
    # finalize
    assert L.fw_cov_finalize(fake, fake, 0, 8, 0.5, 0, fake, fake, fake, fake, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_cov_finalize(fake, fake, 10, 8, 1.5, 0, fake, fake, fake, fake, None) == b.FW_ERR_INVALID_ARG
    # gradient transform
    assert L.fw_grad_transform(fake, 0, 4, 8, None, None, fake + 64, None, 0, None) == b.FW_ERR_INVALID_ARG   # neither T nor Q
    assert L.fw_grad_transform(fake, 0, 4, 8, None, fake, fake, None, 0, None) == b.FW_ERR_INVALID_ARG        # in place
    assert L.fw_grad_transform(fake, 0, 4, 8, fake, None, fake + 64, None, 0, None) == b.FW_ERR_WORKSPACE     # T needs scratch
    assert L.fw_grad_transform(fake, 0, 0, 8, None, fake, fake + 64, None, 0, None) == b.FW_ERR_INVALID_ARG
    # recursive step
    st = b.fw_cond_state(8, fake, fake, fake, fake, fake, fake, None, fake)
    p = b.cond_params()
    assert L.fw_cond_reduce_step(C.byref(st), C.byref(p), None, fake, 1 << 20, None) == b.FW_ERR_INVALID_ARG  # gamma<1 needs Psi
    p1 = b.cond_params(gamma=1.0)
    assert L.fw_cond_reduce_step(C.byref(st), C.byref(p1), None, None, 0, None) == b.FW_ERR_WORKSPACE
    for kw in (dict(gamma=0.0), dict(gamma=1.5), dict(delta=0.0), dict(eps=0.0), dict(beta=1.0), dict(c_rel=-1.0), dict(n_power_iters=-1)):
        pb = b.cond_params(**kw)
        assert L.fw_cond_reduce_step(C.byref(st), C.byref(pb), None, fake, 1 << 20, None) == b.FW_ERR_INVALID_ARG, kw
    assert L.fw_cond_state_init(None, None) == b.FW_ERR_INVALID_ARG
    # the allocation-free form: same checks, and its own size limit, all before any device call
    assert L.fw_cond_reduce_step_static(C.byref(st), C.byref(p), None, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_cond_reduce_step_static(None, C.byref(p1), None, None) == b.FW_ERR_INVALID_ARG
    big = b.fw_cond_state(b.FW_COND_STATIC_MAX_M + 1, fake, fake, fake, fake, fake, fake, fake, fake)
    assert L.fw_cond_reduce_step_static(C.byref(big), C.byref(p), None, None) == b.FW_ERR_UNSUPPORTED
    # condition-number probe
    assert L.fw_cond_probe(None, 8, None, 4, fake, fake, 1 << 20, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_cond_probe(fake, 8, None, 0, fake, fake, 1 << 20, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_cond_probe(fake, 8, None, b.FW_COND_PROBE_MAX_K + 1, fake, fake, 1 << 20, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_cond_probe(fake, 8, None, 4, fake, fake, 16, None) == b.FW_ERR_WORKSPACE
    assert b.fw_workspace_bytes(b.FW_OP_COND_PROBE, 4608, 16) >= 17 * 4608 * 8
    # EVD
    e = b.evd_params()
    assert L.fw_whiten_evd(None, 8, C.byref(e), fake, fake, None, fake, fake, 1 << 20, None) == b.FW_ERR_INVALID_ARG
    assert L.fw_whiten_evd(fake, 8, C.byref(e), fake, fake, None, fake, fake, 16, None) == b.FW_ERR_WORKSPACE
    e2 = b.evd_params(gain_mode=3)
    assert L.fw_whiten_evd(fake, 8, C.byref(e2), fake, fake, None, fake, fake, 1 << 20, None) == b.FW_ERR_INVALID_ARG
    with pytest.raises(b.FwError):
        b._check(b.FW_ERR_WORKSPACE, "x")
