"""fw_cond_reduce_step_static -- the recursive step for callers that cannot allocate (its scratch is a static device
array inside the library) -- against fw_cond_reduce_step on identical copies of the state: bit for bit, two calls in a
row, the second on a smaller layer so that it runs over what the first left in the shared array."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import DEV, dev, workspace
from paper_2010_01546_amd import binding as b

pytestmark = pytest.mark.gpu

NAMES = ("T", "Q", "Qs", "Phi_y", "Psi", "xi2")


def make_state(Phi_np, lbar):
    M = Phi_np.shape[0]
    t = {"Phi_x": dev(Phi_np), "lbar": torch.full((4,), float(lbar), device=DEV)}
    for n in NAMES[:5]:
        t[n] = torch.empty(M, M, device=DEV)
    t["xi2"] = torch.empty(M, device=DEV)
    t["info"] = torch.zeros(8, dtype=torch.int32, device=DEV)
    t["st"] = b.cond_state(M, t["Phi_x"], t["lbar"], t["T"], t["Q"], t["Qs"], t["Phi_y"], t["Psi"], t["xi2"])
    b.fw_cond_state_init(t["st"])
    return t


def run_pair(M, seed, steps, params):
    spectrum = np.logspace(0.0, 3.0, M)[::-1]
    Phi = wl.spd_matrix(seed, M, spectrum).astype(np.float32)
    lbar = float(np.mean(np.diag(Phi)))
    ref, sta = make_state(Phi, lbar), make_state(Phi, lbar)
    ws = workspace(b.fw_workspace_bytes(b.FW_OP_COND_REDUCE_STEP, M))
    for k in range(steps):
        b.fw_cond_reduce_step(ref["st"], params, ref["info"], ws)
        b.fw_cond_reduce_step_static(sta["st"], params, sta["info"])
        torch.cuda.synchronize()
        for n in NAMES:
            assert torch.equal(ref[n], sta[n]), (M, k, n)
        assert torch.equal(ref["info"], sta["info"]), (M, k)
    assert b.read_cond_info(sta["info"]).applied == 1
    return sta


def test_static_scratch_step_matches_workspace_step_twice_in_a_row():
    p = b.cond_params()
    run_pair(200, 11, 3, p)           # ragged: M % 64 != 0, M % 32 != 0
    run_pair(96, 12, 3, p)            # smaller layer over the leftovers of the larger one
    run_pair(147, 13, 2, b.cond_params(gamma=1.0, beta=0.0))   # M % 4 != 0, no leak (Psi unused)


def test_static_scratch_step_rejects_sizes_beyond_its_array():
    M = b.FW_COND_STATIC_MAX_M + 64
    fake = 0x1000
    st = b.fw_cond_state(M, fake, fake, fake, fake, fake, fake, fake, fake)
    p = b.cond_params()
    assert b.lib.fw_cond_reduce_step_static(C.byref(st), C.byref(p), None, None) == b.FW_ERR_UNSUPPORTED
    st0 = b.fw_cond_state(0, fake, fake, fake, fake, fake, fake, fake, fake)
    assert b.lib.fw_cond_reduce_step_static(C.byref(st0), C.byref(p), None, None) == b.FW_ERR_INVALID_ARG
