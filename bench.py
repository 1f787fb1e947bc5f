#!/usr/bin/env python3
"""Benchmark of the feature-whitening hot path on one MI355X.

One "step" is one whitened gradient update of one layer with block length L = 1 (the worst case: the paper amortises
everything but the moments and the gradient product over L batches): zero the block sums, fw_cov_accumulate on the
batch, fw_cov_finalize (alpha = 0.1), fw_cond_state_refresh (the block's new Phi_x invalidates Phi_y = T Phi_x T^T
and Psi = T Phi_x, which the recursive step keeps up to date only while Phi_x stands still), one fw_cond_reduce_step
with the paper's hyper-parameters, and fw_grad_transform of the layer's weight gradient.  Two different batches are
fed in turn, so Phi_x really moves from step to step.  Inputs are seeded synthetic activations and gradients, resident
in HBM before the timed region starts.

With no --config the three single-layer configurations C2, C3, C4 run one after the other in this process; the
top-level fields of the ONE JSON line are C4's (the largest state: all three roofs bind there), C2 and C3 sit under
"configs".  Every export of the step is bracketed by HIP events on the launch stream inside the timed region;
"rooflines" holds one entry per export, "roofline" repeats the entry of the export that takes the largest share of
the step.  `cpu_baseline` times the float64 numpy oracle on the host cores for updates of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"f32": 157.3e12, "bf16": 2.5e15}   # dense MFMA peaks of MI355X, flop/s
HBM_PEAK = 8.0e12

# HBM bytes (read, written) per call of an export, all its kernels.  NOT measured by this script: copied from rocprofv3
# --pmc FETCH_SIZE / WRITE_SIZE runs of `bench.py --config cN --no-cpu-baseline --no-extras --copy-calibration --steps 20
# --warmup 5` whose summary is profiles/whitened_update_step_hbm_traffic_counters.txt, each counter scaled by what it reads on
# a 256 MiB device copy appended to the same run.  Default layout (kkc) only.
PROFILED_TRAFFIC = {
    "c2": {"cov_accumulate": (156.7e6, 121.9e6), "cond_reduce_step": (12.6e6, 6.6e6), "cond_state_refresh": (28.6e6, 3.2e6),
           "grad_transform": (3.8e6, 0.1e6), "cov_finalize": (1.7e6, 1.3e6)},
    "c3": {"cov_accumulate": (195.3e6, 116.2e6), "cond_reduce_step": (189.3e6, 104.1e6), "cond_state_refresh": (408.7e6, 102.7e6),
           "grad_transform": (38.9e6, 2.3e6), "cov_finalize": (22.0e6, 21.3e6)},
    "c4": {"cov_accumulate": (499.7e6, 184.1e6), "cond_reduce_step": (748.7e6, 413.2e6), "cond_state_refresh": (1925.4e6, 410.3e6),
           "grad_transform": (272.0e6, 163.3e6), "cov_finalize": (85.5e6, 85.0e6)},
}
TRAFFIC_SOURCE = ("profiles/whitened_update_step_hbm_traffic_counters.txt (rocprofv3 counters of an earlier run of this command, "
                  "not measured by this run)")

# What a kernel of nothing but dense bfloat16 MFMAs on pseudo-random operands sustains on this chip (all 256 compute units
# busy: the matrix cores then run well below the 2.4 GHz of the published peak, under the chip's power limit).  Measured
# by every run with fw_mfma_rate_probe (measure_mfma_ceiling); the fallback is the figure of earlier runs.
SUSTAINED_BF16_MFMA = {"rate": 1.45e15, "source": "earlier runs of fw_mfma_rate_probe, not measured by this run"}


def measure_mfma_ceiling(torch, b):
    """Sustained bfloat16 matrix-core rate of this GPU: ten back-to-back launches of the library's measurement kernel
    (dense MFMAs on register operands, every compute unit busy) timed by events, for pseudo-random and for zero operands."""
    sink = torch.zeros(4, device="cuda:0")
    out = {}
    for name, zero in (("random_operands", 0), ("zero_operands", 1)):
        b.fw_mfma_rate_probe(zero, 400, sink); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = sum(b.fw_mfma_rate_probe(zero, 400, sink) for _ in range(10))
        e1.record(); torch.cuda.synchronize()
        out[name + "_TFLOPs"] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    out["kernel"] = "mfma_rate_kernel: 4096 wavefronts x 400 rounds x 16 v_mfma_f32_32x32x16_bf16, 10 launches"
    out["published_peak_TFLOPs"] = PEAK["bf16"] / 1e12
    SUSTAINED_BF16_MFMA["rate"] = out["random_operands_TFLOPs"] * 1e12
    SUSTAINED_BF16_MFMA["source"] = "fw_mfma_rate_probe with pseudo-random operands, measured by this run before the timed loops"
    return out

# What plain streaming kernels reach on this chip's HBM (published: 8 TB/s); measured by every run (measure_hbm_ceiling).
SUSTAINED_HBM = {"rate": 5.9e12, "source": "earlier runs (torch add over 1 GiB tensors), not measured by this run"}


def measure_hbm_ceiling(torch):
    """HBM rate of two plain streaming kernels of PyTorch over 1 GiB float32 tensors (far beyond the caches): a copy (one
    read, one write) and an addition (two reads, one write), ten launches each."""
    n = 256 * 1024 * 1024
    a, c = torch.ones(n, device="cuda:0"), torch.empty(n, device="cuda:0")
    bb = torch.ones(n, device="cuda:0")
    out = {}
    for name, fn, nbytes in (("copy", lambda: c.copy_(a), 8.0 * n), ("add", lambda: torch.add(a, bb, out=c), 12.0 * n)):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record(); torch.cuda.synchronize()
        out[name + "_GBs"] = 10 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    out["published_peak_GBs"] = HBM_PEAK / 1e9
    SUSTAINED_HBM["rate"] = max(out["copy_GBs"], out["add_GBs"]) * 1e9
    SUSTAINED_HBM["source"] = "the faster of a copy and an addition over 1 GiB tensors, measured by this run before the timed loops"
    del a, bb, c
    torch.cuda.empty_cache()
    return out


EXPORTS = ("cov_accumulate", "cov_finalize", "cond_state_refresh", "cond_reduce_step", "grad_transform")


def parse(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="all", choices=["all", "c1", "c2", "c3", "c4", "c5"],
                    help="all (default): C2, C3 and C4 in one process, C4 on top; c5 sweeps the 21 ResNet-18 layers and "
                         "reports the aggregate")
    ap.add_argument("--evd", action="store_true",
                    help="time one fw_whiten_evd call (outside the headline) even with --no-extras; the default run times it anyway")
    ap.add_argument("--layout", default="kkc", choices=["kkc", "nhwc", "nchw"],
                    help="kkc: NHWC tensor with channels-last feature order (ky,kx,c); nhwc/nchw: feature order (c,ky,kx)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the second timed loop (stationary Phi_x) and the companion exports (fused update, diagnostics, "
                         "per-channel variant): a profile of such a run holds the kernels of the step only")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, copy a 256 MiB tensor five times: the known-size kernel against which the\n"
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command are scaled")
    return ap.parse_args(argv)


def time_layer(layer, layout_name, steps, warmup, torch, b, wl, evd=False, extras=True):
    """One whitened layer: `steps` timed steps of the whole hot path, every export bracketed by events.  Returns a dict
    of timings and the step function (which keeps the layer's device state alive)."""
    dev = "cuda:0"
    d = layer.desc
    M, S, n_rows = d.M, layer.S, d.n_rows
    bf16 = layer.dtype == "bf16"
    dt = b.FW_BF16 if bf16 else b.FW_F32
    tdt = torch.bfloat16 if bf16 else torch.float32
    if layer.is_rows:
        lay = b.FW_LAYOUT_ROWS
        X0 = torch.as_tensor(layer.act).to(dev).to(tdt).contiguous()
        X1 = X0.flip(1).contiguous()            # a second batch: the same rows with the features in reverse order
    else:
        lay = {"kkc": b.FW_LAYOUT_NHWC_KKC, "nhwc": b.FW_LAYOUT_NHWC, "nchw": b.FW_LAYOUT_NCHW}[layout_name]
        X0 = torch.as_tensor(wl.to_layout(layer.act, lay)).to(dev).to(tdt).contiguous()
        X1 = X0.flip(3 if lay == b.FW_LAYOUT_NCHW else 2).contiguous()   # a second batch: the images mirrored left-right
    Xs = (X0, X1)
    desc = b.conv_desc(*d.astuple())
    G = torch.as_tensor(layer.G).to(dev)          # float32 gradient
    Gout = torch.empty_like(G)

    # raw sums of a block: A and s side by side in one buffer, so that starting a block is one fill
    off_s = (M * M + 3) // 4 * 4
    As = torch.zeros(off_s + M, device=dev)
    A, s = As[:M * M].view(M, M), As[off_s:]
    mu = torch.zeros(M, device=dev); Phi = torch.zeros(M, M, device=dev); phi = torch.zeros(M, device=dev)
    lbar = torch.zeros(4, device=dev)
    T, Q, Qs, Py, Psi = (torch.empty(M, M, device=dev) for _ in range(5))
    xi2 = torch.empty(M, device=dev)
    info = torch.zeros(8, dtype=torch.int32, device=dev)
    ws_cov = torch.empty(b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, M, 0, desc, dt), dtype=torch.uint8, device=dev)
    ws_cond = torch.empty(b.fw_workspace_bytes(b.FW_OP_COND_REDUCE_STEP, M), dtype=torch.uint8, device=dev)
    ws_ref = torch.empty(b.fw_workspace_bytes(b.FW_OP_COND_STATE_REFRESH, M), dtype=torch.uint8, device=dev)
    ws_grad = torch.empty(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S), dtype=torch.uint8, device=dev)
    prm = b.cond_params()                          # the paper's hyper-parameters (Sec. 6)
    alpha = 0.1
    st = b.cond_state(M, Phi, lbar, T, Q, Qs, Py, Psi, xi2)   # holds the nine tensors

    # first block: moments and initial state
    b.fw_cov_accumulate(X0, dt, lay, desc, A, s, ws_cov)
    b.fw_cov_finalize(A, s, n_rows, M, alpha, 1, mu, Phi, phi, lbar)
    b.fw_cond_state_init(st)
    torch.cuda.synchronize()
    counter = [0]

    def step(ev=None, refresh=True):
        X = Xs[counter[0] & 1] if refresh else X0   # without the refresh the same batch comes again: Phi_x stands still
        counter[0] += 1
        As.zero_()
        if ev is not None:
            ev[0].record()
        b.fw_cov_accumulate(X, dt, lay, desc, A, s, ws_cov)
        if ev is not None:
            ev[1].record()
        b.fw_cov_finalize(A, s, n_rows, M, alpha, 0, mu, Phi, phi, lbar)
        if ev is not None:
            ev[2].record()
        if refresh:
            b.fw_cond_state_refresh(st, ws_ref)   # full workspace: the products run on the bfloat16 pipe with split operands
        if ev is not None:
            ev[3].record()
        b.fw_cond_reduce_step(st, prm, info, ws_cond)
        if ev is not None:
            ev[4].record()
        b.fw_grad_transform(G, b.FW_F32, S, M, None, Qs, Gout, ws_grad)
        if ev is not None:
            ev[5].record()

    def timed(refresh):
        for _ in range(warmup):
            step(None, refresh)
        torch.cuda.synchronize()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(steps)]
        t0 = time.perf_counter()
        for k in range(steps):
            step(events[k], refresh)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        per = [sum(e[i].elapsed_time(e[i + 1]) for e in events) / steps for i in range(5)]
        return (t1 - t0) * 1e3 / steps, dict(zip(EXPORTS, per))

    ms_per_step, ex_ms = timed(True)
    assert torch.isfinite(Gout).all() and torch.isfinite(T).all() and torch.isfinite(Py).all()
    out = {"M": M, "S": S, "n_rows": n_rows, "bf16": bf16, "ms_per_step": ms_per_step, "export_ms": ex_ms,
           "gamma": prm.gamma, "act_bytes": float(X0.numel() * X0.element_size()), "step": step, "lay": lay, "extra_ms": {}}
    if extras:
        # Phi_x standing still (what a block of L > 1 batches sees between its boundaries, and the step as it was timed
        # before the refresh joined it): the same loop without fw_cond_state_refresh
        out["ms_per_step_stationary"], st_ms = timed(False)
        out["export_ms_stationary"] = st_ms

        # The same steps on two streams.  fw_cov_accumulate of batch k + 1 depends on that batch only, so a training loop
        # issues it (at forward time) while batch k's refresh, recursion and gradient product still run: here it goes to
        # a second stream and waits only for fw_cov_finalize of batch k to have read the sums.  Every export still runs
        # once per step; the first accumulation and the last step's tail have nothing to overlap with and are timed too.
        def timed_two_streams():
            main = torch.cuda.current_stream()
            side = torch.cuda.Stream()                 # default priority
            sums_read = torch.cuda.Event()
            sums_ready = torch.cuda.Event()

            def accumulate(k):
                with torch.cuda.stream(side):
                    side.wait_event(sums_read)
                    As.zero_()
                    b.fw_cov_accumulate(Xs[k & 1], dt, lay, desc, A, s, ws_cov)
                    sums_ready.record(side)

            def run(n):
                sums_read.record(main)
                accumulate(0)
                for k in range(n):
                    main.wait_event(sums_ready)
                    b.fw_cov_finalize(A, s, n_rows, M, alpha, 0, mu, Phi, phi, lbar)
                    sums_read.record(main)
                    if k + 1 < n:
                        accumulate(k + 1)
                    b.fw_cond_state_refresh(st, ws_ref)
                    b.fw_cond_reduce_step(st, prm, info, ws_cond)
                    b.fw_grad_transform(G, b.FW_F32, S, M, None, Qs, Gout, ws_grad)
                main.wait_stream(side)

            run(warmup)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(steps)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps
        out["ms_per_step_two_streams"] = timed_two_streams()

        def time_call(fn, reps=20):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn(); torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        # the companions outside the step: fused weight update (momentum 0.9, decay 5e-4: Sec. 6) and the whiteness figure
        Wt, Vt = torch.randn(S, M, device=dev), torch.zeros(S, M, device=dev)
        sgd = b.sgd_params(0.1, 0.9, 5e-4)
        diag_out = torch.zeros(4, device=dev)
        ws_diag = torch.empty(b.fw_workspace_bytes(b.FW_OP_DIAGNOSTICS, M), dtype=torch.uint8, device=dev)
        xm = out["extra_ms"]
        ws_sgd = torch.empty(b.fw_workspace_bytes(b.FW_OP_SGD_UPDATE, M, S), dtype=torch.uint8, device=dev)
        xm["sgd_update_fused"] = time_call(lambda: b.fw_sgd_update(G, b.FW_F32, S, M, 1, Qs, sgd, Wt, Vt, ws_sgd))
        xm["diagnostics_whiteness"] = time_call(lambda: b.fw_diagnostics(Py, None, M, diag_out, ws_diag))
        # the transform handed a raw T instead of Q: Q = T^T T is built in the workspace first (M^2 (M+1) flops)
        xm["grad_transform_from_raw_T"] = time_call(lambda: b.fw_grad_transform(G, b.FW_F32, S, M, T, None, Gout, ws_grad), reps=5)
        ws_probe = torch.empty(b.fw_workspace_bytes(b.FW_OP_COND_PROBE, M, 16), dtype=torch.uint8, device=dev)
        xm["cond_probe_16_steps"] = time_call(lambda: b.fw_cond_probe(Py, M, None, 16, diag_out, ws_probe), reps=5)
        if not layer.is_rows and d.kh * d.kw > 1:
            # per-channel variant of the same layer (whitening in front of the convolution, M = Cin): moments of the 1x1
            # "window" over the input pixels, and every tap's S x Cin gradient times the one Cin x Cin Q
            taps = d.kh * d.kw
            d1 = wl.ConvDesc(B=d.B, Cin=d.Cin, H=d.H, W=d.W, kh=1, kw=1, stride=1, pad=0)
            desc1 = b.conv_desc(*d1.astuple())
            A1 = torch.zeros(d.Cin, d.Cin, device=dev); s1 = torch.zeros(d.Cin, device=dev)
            ws1 = torch.empty(b.fw_workspace_bytes(b.FW_OP_COV_ACCUMULATE, d.Cin, 0, desc1, dt), dtype=torch.uint8, device=dev)
            Q1 = torch.eye(d.Cin, device=dev)
            G4 = torch.randn(S, d.Cin, taps, device=dev) * 0.03
            G4o = torch.empty_like(G4)
            ws4 = torch.empty(b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM_TAPS, d.Cin, S * taps), dtype=torch.uint8, device=dev)
            xm["per_channel_variant_cov_accumulate"] = time_call(lambda: b.fw_cov_accumulate(X0, dt, lay, desc1, A1, s1, ws1))
            xm["per_channel_variant_grad_transform_taps"] = time_call(
                lambda: b.fw_grad_transform_taps(G4, b.FW_F32, S, d.Cin, taps, Q1, G4o, ws4))
    if evd or extras:   # the EVD / ZCA reference construction replaces the recursive step; timed once, outside the headline
        ws_evd = torch.empty(b.fw_workspace_bytes(b.FW_OP_WHITEN_EVD, M), dtype=torch.uint8, device=dev)
        lam = torch.empty(M, device=dev)
        Te, Qe = torch.empty(M, M, device=dev), torch.empty(M, M, device=dev)
        b.fw_whiten_evd(Phi, M, b.evd_params(), Te, Qe, None, lam, ws_evd); torch.cuda.synchronize()
        te = time.perf_counter()
        b.fw_whiten_evd(Phi, M, b.evd_params(), Te, Qe, None, lam, ws_evd); torch.cuda.synchronize()
        out["extra_ms"]["whiten_evd"] = (time.perf_counter() - te) * 1e3
    return out


def rooflines_of(r, layer, b, cfg_key, layout_name):
    """One roofline entry per export of the step, from the event times of the timed region.

    a1: issued matrix-core flops / time against the MFMA peak of the type the product runs in (the shift-correlation form
    issues fewer flops than the dense lower triangle N_rows M (M+1); that dense-equivalent rate is reported beside it, it is a
    speed-up over the direct form, not a utilisation).  a2, refresh: issued flops of the form the call takes (float32, or
    three bfloat16 terms per multiplication on whole tiles) against the peak of that form.  a3: 16 M^2 (10 M^2 without leak) float32 words against the HBM peak; finalize: lower triangle of A and of the
    old Phi_x read, Phi_x written."""
    M, S, n_rows, bf16 = r["M"], r["S"], r["n_rows"], r["bf16"]
    d = layer.desc
    ex = r["export_ms"]
    plan = b.fw_cov_plan_query(b.FW_BF16 if bf16 else b.FW_F32, r["lay"], b.conv_desc(*d.astuple()))
    issued = plan.mfma_flops_issued
    dense = float(n_rows) * M * (M + 1)
    split = bool(plan.split_bf16)         # float32 input as hi + lo bfloat16 planes on the bfloat16 kernels
    peak = PEAK["bf16" if (bf16 or split) else "f32"]
    t = ex["cov_accumulate"] * 1e-3
    prof = PROFILED_TRAFFIC.get(cfg_key) if (layer.is_rows or layout_name == "kkc") else None

    def traffic_of(export):
        if not prof or export not in prof:
            return {"traffic": None}
        r_, w_ = prof[export]
        return {"traffic": r_ + w_, "traffic_read_written": [r_, w_], "traffic_source": TRAFFIC_SOURCE}
    shifted = bool(plan.shift)
    a1 = {"bound": "mfma", "export": "fw_cov_accumulate",
          "kernel": ((("pack_images + cov_bf16_tile + shift_tile_assemble + column_sums" if shifted else
                       "pack_images + cov_bf16_tile (+ tile_reduce) + column_sums") + (" + split_fold" if split else "")) if (bf16 or split) else
                     ("shift_partial_f32 + shift_region_reduce + shift_assemble" if shifted else
                      "cov_partial_f32v4 + cov_reduce")) + " = one fw_cov_accumulate",
          "achieved": issued / t / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s", "frac": issued / t / peak,
          "ms": ex["cov_accumulate"], "mfma_flops_issued": issued, "arithmetic": "bf16 hi+lo split of f32 input, f32 accumulate" if split else
          ("bf16 x bf16, f32 accumulate" if bf16 else "f32"),
          "note": "achieved = flops the matrix cores issue per call (padding included) / time of the call",
          "dense_equivalent_flops": dense, "dense_equivalent_rate_TFLOPs": dense / t / 1e12,
          "speedup_vs_direct_form_flops": dense / issued,
          "algorithmic_bytes": r["act_bytes"] + 4.0 * M * M,
          "plan": {"shift": plan.shift, "regions": plan.regions, "differences": plan.differences,
                   "workgroups": plan.workgroups, "ranges": plan.ranges, "split_bf16": plan.split_bf16}}
    a1.update(traffic_of("cov_accumulate"))
    t2 = ex["grad_transform"] * 1e-3
    gp = b.fw_grad_plan_query(b.FW_F32, S, M, b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, M, S))
    gpeak = PEAK["bf16" if gp.split else "f32"]
    a2 = {"bound": "mfma", "export": "fw_grad_transform",
          "kernel": ("2 x split_pack + gemm_split (bf16 hi/lo operands, 3 MFMA terms, contraction cut into runs) + split_reduce" if gp.split
                     else "grad_gemm_f32_strip"),
          "achieved": gp.mfma_flops_issued / t2 / 1e12, "peak": gpeak / 1e12, "unit": "TFLOP/s",
          "frac": gp.mfma_flops_issued / t2 / gpeak, "ms": ex["grad_transform"], "mfma_flops_issued": gp.mfma_flops_issued,
          "float32_equivalent_rate_TFLOPs": 2.0 * S * M * M / t2 / 1e12,
          "note": "achieved = matrix-core flops issued (whole tiles) / time of the call, packing and run-sum passes included"}
    a2.update(traffic_of("grad_transform"))
    words = 16 if r["gamma"] < 1.0 else 10
    t3 = ex["cond_reduce_step"] * 1e-3
    a3 = {"bound": "hbm", "export": "fw_cond_reduce_step", "kernel": "matvec_c + matvec_vt + matvec_u_vecmat + t_reduce_scalars + "
          "matvec + update + partial_sum", "achieved": words * 4.0 * M * M / t3 / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
          "frac": words * 4.0 * M * M / t3 / HBM_PEAK, "ms": ex["cond_reduce_step"], "algorithmic_bytes": words * 4.0 * M * M,
          "note": ("achieved = the algorithmic 16 M^2 words (10 without leak) / time; the update pass reads the symmetric matrices' "
                   "tiles once for both mirrored positions, so fewer bytes than that move") if M > 1152 else
                  "state of this size stays in the caches: launch- and latency-bound, no HBM fraction claimed"}
    a3.update(traffic_of("cond_reduce_step"))
    t4 = ex["cond_state_refresh"] * 1e-3
    rp = b.fw_cond_refresh_plan_query(M, b.fw_workspace_bytes(b.FW_OP_COND_STATE_REFRESH, M))
    rpeak = PEAK["bf16" if rp.split else "f32"]
    rf = {"bound": "mfma", "export": "fw_cond_state_refresh",
          "kernel": ("3 x split_pack + 2 x gemm_split (bf16 hi/lo operands, 3 MFMA terms per product) + mirror + row norms" if rp.split
                     else "2 x grad_gemm_f32_strip + mirror + row norms"),
          "achieved": rp.mfma_flops_issued / t4 / 1e12, "peak": rpeak / 1e12, "unit": "TFLOP/s",
          "frac": rp.mfma_flops_issued / t4 / rpeak, "ms": ex["cond_state_refresh"], "mfma_flops_issued": rp.mfma_flops_issued,
          "float32_equivalent_rate_TFLOPs": 4.0 * M ** 3 / t4 / 1e12,
          "note": "achieved = matrix-core flops issued for both products (whole tiles; the second product only on the lower "
                  "triangle) / time of the call, packing passes included"}
    rf.update(traffic_of("cond_state_refresh"))
    t5 = ex["cov_finalize"] * 1e-3
    fin_bytes = 4.0 * (M * (M + 1) + M * M)
    fn = {"bound": "hbm", "export": "fw_cov_finalize", "kernel": "finalize_phi64 + finalize_vec", "achieved": fin_bytes / t5 / 1e9,
          "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": fin_bytes / t5 / HBM_PEAK, "ms": ex["cov_finalize"]}
    fn.update(traffic_of("cov_finalize"))
    for e in (a3, fn):       # HBM-bound exports: the fraction of what plain streaming kernels reach, for context
        e["frac_of_sustained_hbm_rate"] = e["achieved"] * 1e9 / SUSTAINED_HBM["rate"]
        e["sustained_hbm_rate_GBs"] = SUSTAINED_HBM["rate"] / 1e9
        e["sustained_hbm_rate_source"] = SUSTAINED_HBM["source"]
    for e in (a1, a2, rf):   # bfloat16 products: the fraction of what the matrix cores sustain under the power limit, for context
        if e["peak"] == PEAK["bf16"] / 1e12:
            e["frac_of_sustained_mfma_rate"] = e["achieved"] * 1e12 / SUSTAINED_BF16_MFMA["rate"]
            e["sustained_mfma_rate_TFLOPs"] = SUSTAINED_BF16_MFMA["rate"] / 1e12
            e["sustained_mfma_rate_source"] = SUSTAINED_BF16_MFMA["source"]
    return {"a1_cov_accumulate": a1, "a1_cov_finalize": fn, "a2_grad_transform": a2, "a3_cond_reduce_step": a3,
            "a3_cond_state_refresh": rf}


def cpu_baseline_of(layer, np):
    """The oracle as it stands (float64 numpy) on a bounded sample: whole updates of the same workload, repeated until
    about 8 s have passed (at least one, at most 64); images beyond a memory bound are dropped and the moment terms,
    which are linear in the rows, scaled."""
    from oracle import fw_oracle as ora
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    d = layer.desc
    M = d.M
    alpha = 0.1
    Bs = d.B if layer.is_rows else max(1, min(d.B, int(4e9 // max(1, 8 * d.P * M))))
    scale = d.B / Bs
    reps, spent, secs = 0, 0.0, {"unfold": 0.0, "moments": 0.0, "cond_step": 0.0, "grad_transform": 0.0}
    while reps < 64 and spent < 8.0:
        tc0 = time.perf_counter()
        if layer.is_rows:
            Xr = np.asarray(layer.act[:Bs], dtype=np.float64)
        else:
            Xr = ora.patch_rows(layer.act[:Bs], Bs, d.Cin, d.H, d.W, d.kh, d.kw, d.stride, d.pad)
        tc1 = time.perf_counter()
        mu_o, Phi_o, phi_o, lb_o = ora.block_moments(Xr, alpha, True)
        del Xr
        tc2 = time.perf_counter()
        st_o, _ = ora.cond_reduce_step(ora.CondState.initial(Phi_o), lb_o, ora.CondParams())   # forms T Phi_x T^T explicitly
        tc3 = time.perf_counter()
        ora.grad_transform(layer.G, st_o.Qs)
        tc4 = time.perf_counter()
        for k, v in zip(secs, (tc1 - tc0, tc2 - tc1, tc3 - tc2, tc4 - tc3)):
            secs[k] += v
        reps += 1
        spent += tc4 - tc0
    secs = {k: v / reps for k, v in secs.items()}
    t_update = (secs["unfold"] + secs["moments"]) * scale + secs["cond_step"] + secs["grad_transform"]
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "unknown")
    except OSError:
        pass
    return {"value": 1.0 / t_update, "unit": "updates/s", "cores": int(cores), "cpu_model": cpu_model, "kind": "oracle",
            "sample": f"{reps} update(s) on {Bs} of {d.B} images (moment terms scaled by {scale:g}), "
                      f"float64 numpy, {spent:.1f} s of CPU work",
            "seconds_per_update": secs}


def config_record(cfg_key, args, torch, b, wl, np):
    """Everything reported for one single-layer configuration."""
    layer = {"c1": wl.config1, "c2": wl.config2, "c3": wl.config3, "c4": wl.config4}[cfg_key]()
    d = layer.desc
    r = time_layer(layer, args.layout, args.steps, args.warmup, torch, b, wl, evd=args.evd, extras=not args.no_extras)
    M, S, n_rows, bf16 = r["M"], r["S"], r["n_rows"], r["bf16"]
    roofs = rooflines_of(r, layer, b, cfg_key, args.layout)
    dominant = max(roofs.values(), key=lambda e: e["ms"])
    rec = {
        "metric": "whitened grad-updates/s per layer",
        "value": 1e3 / r["ms_per_step"],
        "unit": "updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not bf16 else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{layer.name}: M={M} S={S} N_rows={n_rows} layout={args.layout if not layer.is_rows else 'rows'}",
                   "batch": d.B, "block_length": 1,
                   "step": "zero sums, cov_accumulate, cov_finalize, cond_state_refresh, cond_reduce_step, grad_transform; "
                           "two batches fed in turn",
                   "cond_params": "gamma=0.99 beta=0.1 delta=0.25 alpha=0.1 (paper defaults, recursive variant)"},
        "roofline": dict(dominant, share_of_step=dominant["ms"] / r["ms_per_step"]),
        "rooflines": roofs,
        "breakdown_ms": dict(r["export_ms"]),
    }
    if "ms_per_step_stationary" in r:
        rec["ms_per_step_stationary_phi_x"] = r["ms_per_step_stationary"]
        rec["updates_per_s_stationary_phi_x"] = 1e3 / r["ms_per_step_stationary"]
    if "ms_per_step_two_streams" in r:
        rec["ms_per_step_two_streams"] = r["ms_per_step_two_streams"]
        rec["updates_per_s_two_streams"] = 1e3 / r["ms_per_step_two_streams"]
        rec["breakdown_ms_stationary_phi_x"] = r["export_ms_stationary"]
    if r["extra_ms"]:
        rec["companion_exports_ms"] = r["extra_ms"]
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline_of(layer, np)
    return rec


def run_c5(args, torch, b, wl):
    """ResNet-18 sweep: one whitened update of every layer per batch; aggregate = layers x steps / total time."""
    rows, total_ms, step_fns = [], 0.0, []
    for index in range(len(wl.RESNET18_LAYERS)):
        layer = wl.config5_layer(index)
        r = time_layer(layer, args.layout, args.steps, args.warmup, torch, b, wl, extras=False)
        total_ms += r["ms_per_step"]
        step_fns.append(r["step"])   # the closure holds every device tensor of the layer (the state struct holds its own)
        flops = float(r["n_rows"]) * r["M"] * (r["M"] + 1)
        plan = b.fw_cov_plan_query(b.FW_BF16, r["lay"], b.conv_desc(*layer.desc.astuple()))
        ex = r["export_ms"]
        rpl = b.fw_cond_refresh_plan_query(r["M"], b.fw_workspace_bytes(b.FW_OP_COND_STATE_REFRESH, r["M"]))
        gpl = b.fw_grad_plan_query(b.FW_F32, r["S"], r["M"], b.fw_workspace_bytes(b.FW_OP_GRAD_TRANSFORM, r["M"], r["S"]))
        rows.append({"layer": layer.name, "M": r["M"], "S": r["S"], "n_rows": r["n_rows"], "ms_per_step": round(r["ms_per_step"], 4),
                     "cov_ms": round(ex["cov_accumulate"], 4), "fin_ms": round(ex["cov_finalize"], 4),
                     "refresh_ms": round(ex["cond_state_refresh"], 4), "cond_ms": round(ex["cond_reduce_step"], 4),
                     "grad_ms": round(ex["grad_transform"], 4), "shift_form": int(plan.shift),
                     "cov_issued_frac_of_bf16_peak": round(plan.mfma_flops_issued / (ex["cov_accumulate"] * 1e-3) / PEAK["bf16"], 4),
                     "cov_dense_equivalent_TFLOPs": round(flops / (ex["cov_accumulate"] * 1e-3) / 1e12, 1),
                     # the other exports against their roofs: refresh and gradient product by the flops of the form taken
                     # over that form's MFMA peak; the recursive step by its 16 M^2 words over the HBM peak (only where
                     # the state does not sit in the caches)
                     "refresh_frac_of_mfma_peak": round(rpl.mfma_flops_issued / (ex["cond_state_refresh"] * 1e-3) /
                                                        PEAK["bf16" if rpl.split else "f32"], 4),
                     "refresh_form": "bf16 split" if rpl.split else "f32",
                     "grad_frac_of_mfma_peak": round(gpl.mfma_flops_issued / (ex["grad_transform"] * 1e-3) /
                                                     PEAK["bf16" if gpl.split else "f32"], 4),
                     "grad_form": "bf16 split" if gpl.split else "f32",
                     "cond_frac_of_hbm_peak": (round(64.0 * r["M"] ** 2 / (ex["cond_reduce_step"] * 1e-3) / HBM_PEAK, 4)
                                               if r["M"] > 1152 else None),
                     "issued": plan.mfma_flops_issued, "dense": flops})
        print(f"[c5] {layer.name}: {r['ms_per_step']:.3f} ms", file=sys.stderr, flush=True)
        del layer
    # The layers are independent: the same updates issued round-robin on four streams (default priority), so that
    # the launch- and latency-bound small layers run under the large ones.
    streams = [torch.cuda.Stream() for _ in range(4)]

    def sweep():
        for i, fn in enumerate(step_fns):
            with torch.cuda.stream(streams[i % 4]):
                fn()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        sweep()
    torch.cuda.synchronize()
    tc0 = time.perf_counter()
    for _ in range(args.steps):
        sweep()
    torch.cuda.synchronize()
    conc_ms = (time.perf_counter() - tc0) * 1e3 / args.steps
    issued = sum(x.pop("issued") for x in rows)
    dense = sum(x.pop("dense") for x in rows)
    cov_s = sum(x["cov_ms"] for x in rows) * 1e-3
    return {"metric": "whitened grad-updates/s per layer", "value": len(rows) * 1e3 / conc_ms, "unit": "updates/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": conc_ms,
            "ms_per_step_one_layer_at_a_time": total_ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "C5: ResNet-18 sweep, 21 layers at batch 256, one update of every layer per step",
                       "streams": 4, "block_length": 1,
                       "step": "zero sums, cov_accumulate, cov_finalize, cond_state_refresh, cond_reduce_step, grad_transform",
                       "cond_params": "gamma=0.99 beta=0.1 delta=0.25 alpha=0.1 (paper defaults, recursive variant)"},
            "roofline": {"bound": "mfma", "kernel": "fw_cov_accumulate over the 21 layers, one at a time",
                         "achieved": issued / cov_s / 1e12, "peak": PEAK["bf16"] / 1e12, "unit": "TFLOP/s",
                         "frac": issued / cov_s / PEAK["bf16"], "traffic": None,
                         "dense_equivalent_rate_TFLOPs": dense / cov_s / 1e12},
            "layers": rows}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import workloads as wl
    from paper_2010_01546_amd import binding as b

    assert torch.cuda.is_available(), "bench.py needs a GPU"

    # (left out with --no-extras, so that a profile of such a run holds the kernels of the step only)
    ceiling = None if args.no_extras else measure_mfma_ceiling(torch, b)
    hbm_ceiling = None if args.no_extras else measure_hbm_ceiling(torch)
    if args.config == "c5":
        rec = run_c5(args, torch, b, wl)
        rec["mfma_ceiling"] = ceiling
        rec["hbm_ceiling"] = hbm_ceiling
        print(json.dumps(rec))
        return
    if args.config == "all":
        recs = {}
        for key in ("c2", "c3", "c4"):
            recs[key] = config_record(key, args, torch, b, wl, np)
            print(f"[bench] {key}: {recs[key]['ms_per_step']:.3f} ms/step", file=sys.stderr, flush=True)
        out = recs.pop("c4")
        out["configs"] = recs
    else:
        out = config_record(args.config, args, torch, b, wl, np)

    out["mfma_ceiling"] = ceiling
    out["hbm_ceiling"] = hbm_ceiling
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, device="cuda:0")      # 256 MiB read + 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
