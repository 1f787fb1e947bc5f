#!/usr/bin/env python3
"""Benchmark of the feature-whitening hot path on one MI355X.

One "step" is one whitened gradient update of one layer: fw_cov_accumulate (+ fw_cov_finalize) on a batch, one
fw_cond_reduce_step, and fw_grad_transform of the layer's weight gradient -- block length L = 1, the worst case
(the paper amortises the recursive step over L batches).  Inputs are seeded synthetic activations and gradients,
resident in HBM before the timed region starts.

Prints ONE JSON line.  `roofline` describes the dominant kernel pair (the split-K covariance kernel and its reduce,
i.e. one fw_cov_accumulate call) timed with events on the launch stream inside the timed region; `cpu_baseline`
times the float64 numpy oracle on the host cores for one update of the same workload.
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

# HBM bytes (read + written) per fw_cov_accumulate call, all its kernels, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this script with --copy-calibration (summary: profiles/fw_cov_accumulate_hbm_traffic_counters.txt), each
# counter scaled by what it reads on a 256 MiB device copy (2 KiB per FETCH_SIZE count, 1 KiB per WRITE_SIZE count).
# Measured with the default layout (kkc); other layouts report null.
MEASURED_TRAFFIC = {"c2": {"read": 122.5e6, "written": 58.9e6},
                    "c3": {"read": 195.6e6, "written": 116.2e6},
                    "c4": {"read": 499.9e6, "written": 184.1e6}}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2", choices=["c1", "c2", "c3", "c4", "c5"],
                    help="c2 is the headline workload; c5 sweeps the 21 ResNet-18 layers and reports the aggregate")
    ap.add_argument("--evd", action="store_true", help="also time one fw_whiten_evd call (outside the headline)")
    ap.add_argument("--layout", default="kkc", choices=["kkc", "nhwc", "nchw"],
                    help="kkc: NHWC tensor with channels-last feature order (ky,kx,c); nhwc/nchw: feature order (c,ky,kx)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the timing of the companion exports (refresh, fused update, diagnostics, per-channel variant): "
                         "a profile of such a run holds the kernels of the step only")
    ap.add_argument("--c5-unlocked", action="store_true", help=argparse.SUPPRESS)   # only once the fault of the sweep is explained
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, copy a 256 MiB tensor five times: the known-size kernel against which the\n"
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command are scaled")
    return ap.parse_args()


def time_layer(layer, layout_name, steps, warmup, torch, b, wl, evd=False, extras=True):
    """One whitened layer: K timed steps of the whole hot path plus a per-export breakdown.  Returns a dict of timings."""
    dev = "cuda:0"
    d = layer.desc
    M, S, n_rows = d.M, layer.S, d.n_rows
    bf16 = layer.dtype == "bf16"
    dt = b.FW_BF16 if bf16 else b.FW_F32
    tdt = torch.bfloat16 if bf16 else torch.float32
    if layer.is_rows:
        lay = b.FW_LAYOUT_ROWS
        X = torch.as_tensor(layer.act).to(dev).to(tdt).contiguous()
    else:
        lay = {"kkc": b.FW_LAYOUT_NHWC_KKC, "nhwc": b.FW_LAYOUT_NHWC, "nchw": b.FW_LAYOUT_NCHW}[layout_name]
        X = torch.as_tensor(wl.to_layout(layer.act, lay)).to(dev).to(tdt).contiguous()
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
    prm = b.cond_params()                          # the paper's hyper-parameters (Sec. 6)
    alpha = 0.1
    st = b.cond_state(M, Phi, lbar, T, Q, Qs, Py, Psi, xi2)

    # first block: moments and initial state
    b.fw_cov_accumulate(X, dt, lay, desc, A, s, ws_cov)
    b.fw_cov_finalize(A, s, n_rows, M, alpha, 1, mu, Phi, phi, lbar)
    b.fw_cond_state_init(st)
    torch.cuda.synchronize()

    def step(ev=None):
        As.zero_()
        if ev is not None:
            ev[0].record()
        b.fw_cov_accumulate(X, dt, lay, desc, A, s, ws_cov)
        if ev is not None:
            ev[1].record()
        b.fw_cov_finalize(A, s, n_rows, M, alpha, 0, mu, Phi, phi, lbar)
        b.fw_cond_reduce_step(st, prm, info, ws_cond)
        b.fw_grad_transform(G, b.FW_F32, S, M, None, Qs, Gout)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):
        step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    cov_ms = sum(e0.elapsed_time(e1) for e0, e1 in events) / steps
    assert torch.isfinite(Gout).all() and torch.isfinite(T).all()

    # separate, untimed-for-the-headline breakdown of the other exports
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
    out = {"M": M, "S": S, "n_rows": n_rows, "bf16": bf16, "ms_per_step": ms_per_step, "cov_ms": cov_ms,
           "cond_ms": time_call(lambda: b.fw_cond_reduce_step(st, prm, info, ws_cond)),
           "grad_ms": time_call(lambda: b.fw_grad_transform(G, b.FW_F32, S, M, None, Qs, Gout)),
           "fin_ms": time_call(lambda: b.fw_cov_finalize(A, s, n_rows, M, alpha, 0, mu, Phi, phi, lbar)),
           "refresh_ms": time_call(lambda: b.fw_cond_state_refresh(st), reps=5) if extras else None,
           "sgd_ms": time_call(lambda: b.fw_sgd_update(G, b.FW_F32, S, M, 1, Qs, sgd, Wt, Vt)) if extras else None,
           "diag_ms": time_call(lambda: b.fw_diagnostics(Py, None, M, diag_out, ws_diag)) if extras else None,
           "gamma": prm.gamma, "act_bytes": float(X.numel() * X.element_size()), "step": step}
    if extras and not layer.is_rows and d.kh * d.kw > 1:
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
        out["per_channel_cov_ms"] = time_call(lambda: b.fw_cov_accumulate(X, dt, lay, desc1, A1, s1, ws1))
        out["per_channel_grad_ms"] = time_call(lambda: b.fw_grad_transform_taps(G4, b.FW_F32, S, d.Cin, taps, Q1, G4o, ws4))
    if evd:   # the EVD / ZCA reference construction replaces the recursive step; timed once, outside the headline
        ws_evd = torch.empty(b.fw_workspace_bytes(b.FW_OP_WHITEN_EVD, M), dtype=torch.uint8, device=dev)
        lam = torch.empty(M, device=dev)
        b.fw_whiten_evd(Phi, M, b.evd_params(), T, Q, None, lam, ws_evd); torch.cuda.synchronize()
        te = time.perf_counter()
        b.fw_whiten_evd(Phi, M, b.evd_params(), T, Q, None, lam, ws_evd); torch.cuda.synchronize()
        out["evd_ms"] = (time.perf_counter() - te) * 1e3
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if args.config == "c5" and not args.c5_unlocked:
        # One run of this sweep (default steps, fresh machine) ended with a GPU memory fault whose cause has not been
        # found; three runs of the same code before it were clean.  Until the cause is known the sweep does not run.
        print("bench.py --config c5 is switched off: a run of it ended in an unexplained GPU fault "
              "(the figures of its earlier clean runs are recorded in the design notes)", file=sys.stderr)
        sys.exit(3)
    import numpy as np
    import torch

    import workloads as wl
    from paper_2010_01546_amd import binding as b

    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if args.config == "c5":
        # ResNet-18 sweep: one whitened update of every layer per batch; aggregate = layers x steps / total time
        rows, total_ms, step_fns = [], 0.0, []
        for index in range(len(wl.RESNET18_LAYERS)):
            layer = wl.config5_layer(index)
            r = time_layer(layer, args.layout, args.steps, args.warmup, torch, b, wl)
            total_ms += r["ms_per_step"]
            step_fns.append(r["step"])   # keeps the layer's device state alive for the concurrent pass below
            flops = float(r["n_rows"]) * r["M"] * (r["M"] + 1)
            rows.append({"layer": layer.name, "M": r["M"], "S": r["S"], "n_rows": r["n_rows"], "ms_per_step": round(r["ms_per_step"], 4),
                         "cov_ms": round(r["cov_ms"], 4), "cov_frac_of_bf16_peak": round(flops / (r["cov_ms"] * 1e-3) / PEAK["bf16"], 4),
                         "cond_ms": round(r["cond_ms"], 4), "grad_ms": round(r["grad_ms"], 4)})
            del layer
        # The layers are independent: the same updates issued round-robin on four streams (default priority), so that
        # the launch- and latency-bound small layers run under the large ones.
        streams = [torch.cuda.Stream() for _ in range(4)]

        def sweep():
            for i, fn in enumerate(step_fns):
                with torch.cuda.stream(streams[i % 4]):
                    fn()
        for _ in range(args.warmup):
            sweep()
        torch.cuda.synchronize()
        tc0 = time.perf_counter()
        for _ in range(args.steps):
            sweep()
        torch.cuda.synchronize()
        conc_ms = (time.perf_counter() - tc0) * 1e3 / args.steps
        cov_flops = sum(float(x["n_rows"]) * x["M"] * (x["M"] + 1) for x in rows)
        cov_s = sum(x["cov_ms"] for x in rows) * 1e-3
        out = {"metric": "whitened grad-updates/s per layer", "value": len(rows) * 1e3 / conc_ms, "unit": "updates/s",
               "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": conc_ms,
               "ms_per_step_one_layer_at_a_time": total_ms,
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
               "config": {"workload": "C5: ResNet-18 sweep, 21 layers at batch 256, one update of every layer per step",
                          "streams": 4,
                          "block_length": 1, "cond_params": "gamma=0.99 beta=0.1 delta=0.25 (paper defaults)"},
               "roofline": {"bound": "mfma", "kernel": "fw_cov_accumulate over the 21 layers", "achieved": cov_flops / cov_s / 1e12,
                            "peak": PEAK["bf16"] / 1e12, "unit": "TFLOP/s", "frac": cov_flops / cov_s / PEAK["bf16"], "traffic": None},
               "layers": rows}
        print(json.dumps(out))
        return

    layer = {"c1": wl.config1, "c2": wl.config2, "c3": wl.config3, "c4": wl.config4}[args.config]()
    d = layer.desc
    r = time_layer(layer, args.layout, args.steps, args.warmup, torch, b, wl, evd=args.evd, extras=not args.no_extras)
    M, S, n_rows, bf16 = r["M"], r["S"], r["n_rows"], r["bf16"]
    ms_per_step, cov_ms, cond_ms, grad_ms, fin_ms = r["ms_per_step"], r["cov_ms"], r["cond_ms"], r["grad_ms"], r["fin_ms"]

    cov_flops = float(n_rows) * M * (M + 1)                 # lower triangle incl. diagonal, 2 flops per product
    achieved = cov_flops / (cov_ms * 1e-3)
    # A stride-1 window is accumulated through shift correlations: tap pairs with the same offset share one product, so
    # the matrix cores issue fewer flops than the algorithmic count (13 instead of 45 tap pairs for 3x3); report both.
    lay_id = b.FW_LAYOUT_ROWS if layer.is_rows else {"kkc": b.FW_LAYOUT_NHWC_KKC, "nhwc": b.FW_LAYOUT_NHWC, "nchw": b.FW_LAYOUT_NCHW}[args.layout]
    plan = b.fw_cov_plan_query(b.FW_BF16 if bf16 else b.FW_F32, lay_id, b.conv_desc(*d.astuple()))
    shifted, issued = bool(plan.shift), plan.mfma_flops_issued
    peak = PEAK[layer.dtype]
    tr = MEASURED_TRAFFIC.get(args.config) if (layer.is_rows or args.layout == "kkc") else None
    traffic = tr["read"] + tr["written"] if tr else None
    alg_bytes = r["act_bytes"] + 4.0 * M * M   # activation once + A once
    cond_words = 16 if r["gamma"] < 1.0 else 10
    cond_bytes = cond_words * M * M * 4.0
    out = {
        "metric": "whitened grad-updates/s per layer",
        "value": 1e3 / ms_per_step,
        "unit": "updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not bf16 else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{layer.name}: M={M} S={S} N_rows={n_rows} layout={args.layout if not layer.is_rows else 'rows'}",
                   "batch": d.B, "block_length": 1, "cond_params": "gamma=0.99 beta=0.1 delta=0.25 (paper defaults)"},
        "roofline": {"bound": "mfma",
                     "kernel": (("pack_images + cov_bf16_tile + shift_tile_assemble + column_sums" if shifted else
                                 "pack_images + cov_bf16_tile (+ tile_reduce) + column_sums") if bf16 else
                                ("shift_partial_f32 + shift_region_reduce + shift_assemble" if shifted else
                                 "cov_partial_f32v4 + cov_reduce")) + " = one fw_cov_accumulate",
                     "achieved": achieved / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": traffic, "traffic_unit": "bytes per fw_cov_accumulate call (HBM read + written, counters)",
                     "traffic_read_written": tr, "algorithmic_bytes": alg_bytes,
                     "note": "achieved = algorithmic flops N_rows*M*(M+1) per call / time of the call",
                     "mfma_flops_issued": issued, "issued_frac_of_peak": issued / (cov_ms * 1e-3) / peak,
                     "plan": {"shift": plan.shift, "regions": plan.regions, "differences": plan.differences,
                              "workgroups": plan.workgroups, "ranges": plan.ranges}},
        "breakdown_ms": {"cov_accumulate": cov_ms, "cov_finalize": fin_ms, "cond_reduce_step": cond_ms, "grad_transform": grad_ms},
        "cond_step_GBps": cond_bytes / (cond_ms * 1e-3) / 1e9,
        "grad_transform_TFLOPs": 2.0 * S * M * M / (grad_ms * 1e-3) / 1e12,
    }
    # once per block when the data (hence Phi_x) changes between blocks; the timed step feeds the same batch again, so
    # Phi_x is stationary there and the call is not part of the step
    if r["refresh_ms"] is not None:
        out["breakdown_ms"]["cond_state_refresh_per_block"] = r["refresh_ms"]
        out["breakdown_ms"]["sgd_update_fused"] = r["sgd_ms"]
        out["breakdown_ms"]["diagnostics_whiteness"] = r["diag_ms"]
        out["cond_state_refresh_TFLOPs"] = 4.0 * M * M * M / (r["refresh_ms"] * 1e-3) / 1e12
    if "per_channel_cov_ms" in r:
        out["breakdown_ms"]["per_channel_variant_cov_accumulate"] = r["per_channel_cov_ms"]
        out["breakdown_ms"]["per_channel_variant_grad_transform_taps"] = r["per_channel_grad_ms"]
    if "evd_ms" in r:
        out["breakdown_ms"]["whiten_evd"] = r["evd_ms"]
    alpha = 0.1
    dev = "cuda:0"

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, device=dev)      # 256 MiB read + 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        from oracle import fw_oracle as ora
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
        except Exception:
            cores = os.cpu_count() or 1
        # bounded sample: whole updates of the same workload by the oracle, repeated until about 10 s have passed
        # (at least one, at most 64 updates); images beyond a memory bound are dropped and the moment terms scaled,
        # which are linear in the rows
        Bs = d.B if layer.is_rows else max(1, min(d.B, int(4e9 // max(1, 8 * d.P * M))))
        scale = d.B / Bs
        reps, spent, secs = 0, 0.0, {"unfold": 0.0, "moments": 0.0, "cond_step": 0.0, "grad_transform": 0.0}
        while reps < 64 and spent < 10.0:
            tc0 = time.perf_counter()
            if layer.is_rows:
                Xr = np.asarray(layer.act[:Bs], dtype=np.float64)
            else:
                Xr = ora.patch_rows(layer.act[:Bs], Bs, d.Cin, d.H, d.W, d.kh, d.kw, d.stride, d.pad)
            tc1 = time.perf_counter()
            mu_o, Phi_o, phi_o, lb_o = ora.block_moments(Xr, alpha, True)
            del Xr
            tc2 = time.perf_counter()
            st_o, _ = ora.cond_reduce_step(ora.CondState.initial(Phi_o), lb_o, ora.CondParams())
            tc3 = time.perf_counter()
            ora.grad_transform(layer.G, st_o.Qs)
            tc4 = time.perf_counter()
            for k, v in zip(secs, (tc1 - tc0, tc2 - tc1, tc3 - tc2, tc4 - tc3)):
                secs[k] += v
            reps += 1
            spent += tc4 - tc0
        secs = {k: v / reps for k, v in secs.items()}
        t_update = (secs["unfold"] + secs["moments"]) * scale + secs["cond_step"] + secs["grad_transform"]
        out["cpu_baseline"] = {"value": 1.0 / t_update, "unit": "updates/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{reps} update(s) on {Bs} of {d.B} images (moment terms scaled by {scale:g}), "
                                         f"float64 numpy, {spent:.1f} s of CPU work",
                               "seconds_per_update": secs}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
