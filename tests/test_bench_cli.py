"""Host-side checks of bench.py that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_default_run_covers_c2_c3_c4_and_the_sweep_is_selectable():
    sys.path.insert(0, ROOT)
    import bench
    a = bench.parse([])
    assert a.gpus == 1 and a.config == "all" and a.steps > 0 and a.warmup >= 0
    assert bench.parse(["--config", "c5"]).config == "c5"
    # the step the bench times names every export of the path, the refresh included
    assert bench.EXPORTS == ("cov_accumulate", "cov_finalize", "cond_state_refresh", "cond_reduce_step", "grad_transform")


def test_cond_state_keeps_its_tensors_alive():
    """The struct carries raw addresses only; the binding attaches the tensors so that a caller holding just the struct
    (a closure over it, say) does not hand the library memory that the allocator has already given away."""
    import gc
    import weakref

    import torch
    from paper_2010_01546_amd import binding as b
    M = 8
    ts = [torch.zeros(M, M) for _ in range(7)] + [torch.zeros(M)]
    Phi, T, Q, Qs, Py, Psi, lbar, xi2 = ts[0], ts[1], ts[2], ts[3], ts[4], ts[5], ts[6], ts[7]
    refs = [weakref.ref(t) for t in ts]
    ptrs = [t.data_ptr() for t in ts]
    st = b.cond_state(M, Phi, lbar, T, Q, Qs, Py, Psi, xi2)
    del ts, Phi, T, Q, Qs, Py, Psi, lbar, xi2
    gc.collect()
    assert all(r() is not None for r in refs)
    assert [st.Phi_x, st.T, st.Q, st.Qs, st.Phi_y, st.Psi, st.lambda_bar, st.xi2] == ptrs
    del st
    gc.collect()
    assert all(r() is None for r in refs)
