#!/usr/bin/env python3
"""Benchmark of the DWM forward convolution on one MI355X.

A "step" is one dwm_conv_forward (input transform + contraction/output transform) over one
synthetic batch that is already resident in HBM; the filter transform runs once before the
timed region (it is a function of the weights only).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config i] [--no-cpu-baseline]

--config picks one of the five layers of dwm_workloads.CONFIGS (default 2: the 7x7 stride-1
layer with 256 channels, the largest of the five, 161 GFLOP of direct convolution per step).
The headline line also carries `per_config`: every one of the five layers measured the same
way in the same run (the paper's runtime table, Table 4, is per layer as well), and under
`other_paths` the same layer's binary16 and bfloat16 forward pass and its two gradients, each
timed as its own mode of this script times it (--half, --bf16, --backward-data, --backward-filter).
--paper-layer KERNEL,HW,STRIDE runs one of the paper's own single-layer shapes instead
(Sec. 5: batch 256, same padding, 14x14 maps with 256 channels/filters or 28x28 with 128,
standard-normal inputs AND weights).

Stage times: each stage is timed as ONE pair of HIP events around `steps` back-to-back launches
of that stage on the stream the kernels run on, so the figure is the kernel's own average
duration (what a rocprofv3 kernel trace of the same command reports), not a launch plus the
idle gap before a dependent launch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "direct-conv-equivalent TFLOP/s of DWM conv (fp32, 1 GPU); MSE vs FP64 direct"
PEAK_MFMA_F32 = 157.3  # TFLOP/s, dense fp32 MFMA, MI355X
PEAK_HBM = 8000.0      # GB/s


def hbm_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from the rocprofv3 FETCH_SIZE / WRITE_SIZE
    summary under profiles/ (each counter scaled by what it reads for a plain copy of known
    size; the file states the build and commands it came from), or None if it has no such line."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                t = line.split()
                if len(t) >= 5 and not line.startswith("#") and t[0] == workload and t[1] == kernel:
                    return float(t[4])
    except OSError:
        pass
    return None


def cpu_baseline(x, w, L, target_s=12.0):
    """The FP64 direct-convolution oracle, as it stands, on a bounded sample of this
    workload's outputs: direct-equivalent TFLOP/s on the host cores."""
    import numpy as np
    import oracle
    import dwm_workloads as wl

    OH, OW = wl.out_hw(L)
    total = L.N * L.K * OH * OW
    rng = np.random.default_rng(7)
    per_out = 2.0 * L.C * L.R * L.S
    probe = min(total, 20000)
    idx = rng.choice(total, probe, replace=False)
    t0 = time.perf_counter()
    oracle.direct_f64_at(x, w, L.stride, L.pad, idx)
    dt = time.perf_counter() - t0
    n = int(min(total, max(probe, probe * target_s / max(dt, 1e-6))))
    idx = rng.choice(total, n, replace=False)
    t0 = time.perf_counter()
    oracle.direct_f64_at(x, w, L.stride, L.pad, idx)
    dt = time.perf_counter() - t0
    out = {"value": per_out * n / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
           "kind": "oracle", "seconds": round(dt, 2),
           "sample": "%d of %d outputs of %s drawn uniformly, FP64 direct convolution" % (n, total, L.name)}
    # the oracle's FP64 DWM (the paper's five steps, part by part) beside it: whole images of the
    # same layer, as many as fit the time
    per_img = 2.0 * L.K * L.C * L.R * L.S * OH * OW
    t0 = time.perf_counter()
    oracle.dwm_f64(x[:1], w, L.stride, L.pad)
    dt1 = time.perf_counter() - t0
    nimg = int(max(1, min(L.N, target_s / 2 / max(dt1, 1e-6))))
    if nimg > 1:
        t0 = time.perf_counter()
        oracle.dwm_f64(x[:nimg], w, L.stride, L.pad)
        dt1 = time.perf_counter() - t0
    out["dwm_f64"] = {"value": per_img * nimg / dt1 / 1e12, "unit": "TFLOP/s", "seconds": round(dt1, 2),
                      "sample": "%d of %d images of %s, FP64 DWM reference (direct-equivalent flops)" % (nimg, L.N, L.name)}
    return out


def bench_backward_data(args, L, x, w):
    """A step = one dwm_conv_backward_data on resident buffers (stride^2 stride-1 sub-convolutions of
    dy, or one kernel for layers with few input channels: --bwd-path 0 / 1 forces either); the
    filter transform of the flipped, phase-split weights runs once before."""
    import numpy as np
    import torch

    import dwm_workloads as wl
    import paper_2002_00552_amd as dwm

    OH, OW = wl.out_hw(L)
    dy = np.random.default_rng(3100).uniform(-1, 1, (L.N, L.K, OH, OW)).astype(np.float32)
    plan = dwm.dwm_bwd_data_plan_create(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    try:
        dwm.dwm_bwd_data_set_variant(plan, "path", args.bwd_path)
    except dwm.DwmError:
        raise SystemExit("bench.py: --bwd-path %d does not apply to %s" % (args.bwd_path, L.name))
    info = dwm.dwm_bwd_data_plan_info(plan)
    single = bool(info.single_kernel)
    dyd, wd = torch.from_numpy(dy).cuda(), torch.from_numpy(w).cuda()
    U = torch.empty(dwm.dwm_bwd_data_filter_bytes(plan) // 4, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(dwm.dwm_bwd_data_workspace_bytes(plan) // 4, 64), dtype=torch.float32, device="cuda")
    dx = torch.empty((L.N, L.C, L.H, L.W), dtype=torch.float32, device="cuda")
    dwm.dwm_bwd_data_set_workspace(plan, ws.data_ptr(), ws.numel() * 4)
    st = torch.cuda.current_stream().cuda_stream
    dwm.dwm_bwd_data_filter_transform(plan, wd.data_ptr(), U.data_ptr(), st)
    for _ in range(args.warmup):
        dwm.dwm_conv_backward_data(plan, dyd.data_ptr(), U.data_ptr(), dx.data_ptr(), st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dwm.dwm_conv_backward_data(plan, dyd.data_ptr(), U.data_ptr(), dx.data_ptr(), st)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    out = {
        "metric": "direct-conv-equivalent TFLOP/s of the DWM data gradient (fp32, 1 GPU); MSE vs FP64 definition",
        "value": info.direct_flops / dt / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": L.name + "_backward_data", "phases": info.n_phases, "subconvs": info.n_subconvs,
                   "path": "single kernel" if single else "sub-convolutions",
                   "direct_GFLOP": info.direct_flops / 1e9, "winograd_GFLOP": info.winograd_flops / 1e9},
        "roofline": {"kernel": "bwd_small_kernel" if single else "all sub-convolutions", "bound": "mfma", "achieved": info.winograd_flops / dt / 1e12,
                     "peak": PEAK_MFMA_F32, "unit": "TFLOP/s", "frac": info.winograd_flops / dt / 1e12 / PEAK_MFMA_F32,
                     "traffic": None},
    }
    if not args.no_check:
        import oracle
        got = dx.cpu().numpy()
        idx = np.random.default_rng(98).choice(got.size, min(got.size, 20000), replace=False)
        ref = oracle.backward_data_f64_at(dy, w, (L.N, L.C, L.H, L.W), L.stride, L.pad, idx)
        g = got.ravel()[idx].astype(np.float64)
        mse = float(np.mean((g - ref) ** 2))
        out["accuracy"] = {"max_rel_err": float(np.max(np.abs(g - ref)) / np.max(np.abs(ref))),
                           "mse_vs_fp64": mse, "log10_mse_plus_10": float(np.log10(mse) + 10),
                           "sampled_outputs": int(idx.size)}
    dwm.dwm_bwd_data_plan_destroy(plan)
    return out


def bench_backward_filter(args, L, x, w):
    """A step = one dwm_conv_backward_filter (input transform of x, A dY A^T, the per-plane GEMMs over
    the tiles, G^T (.) G) on resident buffers."""
    import numpy as np
    import torch

    import dwm_workloads as wl
    import paper_2002_00552_amd as dwm

    OH, OW = wl.out_hw(L)
    dy = np.random.default_rng(4100).uniform(-1, 1, (L.N, L.K, OH, OW)).astype(np.float32)
    plan = dwm.dwm_bwd_filter_plan_create(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    info = dwm.dwm_bwd_filter_plan_info(plan)
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    ws = torch.empty(dwm.dwm_bwd_filter_workspace_bytes(plan) // 4, dtype=torch.float32, device="cuda")
    dw = torch.empty((L.K, L.C, L.R, L.S), dtype=torch.float32, device="cuda")
    dwm.dwm_bwd_filter_set_workspace(plan, ws.data_ptr(), ws.numel() * 4)
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(args.warmup):
        dwm.dwm_conv_backward_filter(plan, xd.data_ptr(), dyd.data_ptr(), dw.data_ptr(), st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dwm.dwm_conv_backward_filter(plan, xd.data_ptr(), dyd.data_ptr(), dw.data_ptr(), st)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    out = {
        "metric": "direct-conv-equivalent TFLOP/s of the DWM filter gradient (fp32, 1 GPU); MSE vs FP64 definition",
        "value": info.direct_flops / dt / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": L.name + "_backward_filter", "planes": info.n_planes, "tiles": info.n_tiles,
                   "splits": info.splits, "direct_GFLOP": info.direct_flops / 1e9,
                   "winograd_GFLOP": info.winograd_flops / 1e9, "workspace_MB": ws.numel() * 4 / 1e6},
        "roofline": {"kernel": "wgrad_gemm_kernel (whole step timed)", "bound": "mfma",
                     "achieved": info.winograd_flops / dt / 1e12, "peak": PEAK_MFMA_F32, "unit": "TFLOP/s",
                     "frac": info.winograd_flops / dt / 1e12 / PEAK_MFMA_F32, "traffic": None},
    }
    if not args.no_check:
        import oracle
        ks = sorted({0, L.K - 1})
        ref = oracle.backward_filter_f64(x, np.ascontiguousarray(dy[:, ks]), (len(ks), L.C, L.R, L.S), L.stride, L.pad)
        g = dw.cpu().numpy()[ks].astype(np.float64)
        mse = float(np.mean((g - ref) ** 2))
        out["accuracy"] = {"max_rel_err": float(np.max(np.abs(g - ref)) / np.max(np.abs(ref))),
                           "mse_vs_fp64": mse, "log10_mse_plus_10": float(np.log10(mse) + 10),
                           "checked_filters": len(ks)}
    dwm.dwm_bwd_filter_plan_destroy(plan)
    return out


def bench_half(args, L, x, w, bf16=False):
    """A step = one dwm_f16_conv_forward (binary16 x, U, V, y; FP16 MFMA with FP32 accumulation) or,
    with bf16, one dwm_bf16_conv_forward (the same with bfloat16) on resident buffers; the filter
    transform runs once before.  With 16-bit operands the contraction's arithmetic intensity (about
    200 flop per byte of V, U and y) is below the chip's balance of 2.5 PFLOP/s : 8 TB/s, so both
    stages are priced against the HBM roofline."""
    import numpy as np
    import torch

    import paper_2002_00552_amd as dwm

    PEAK_MFMA_F16 = 2500.0
    tdt = torch.bfloat16 if bf16 else torch.float16
    fn = lambda name: getattr(dwm, ("dwm_bf16_" if bf16 else "dwm_f16_") + name)  # noqa: E731
    xd, wd = torch.from_numpy(x).to(tdt).cuda(), torch.from_numpy(w).to(tdt).cuda()
    x16, w16 = xd.float().cpu().numpy(), wd.float().cpu().numpy()  # the 16-bit values, as float32
    plan = fn("plan_create")(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    if args.contract_variant >= 0:
        fn("set_variant")(plan, "contract", args.contract_variant)
    if args.forward_variant >= 0:
        fn("set_variant")(plan, "forward", args.forward_variant)
    info = fn("plan_info")(plan)
    single = info.forward_path == 1
    U = torch.empty(fn("filter_bytes")(plan) // 2, dtype=tdt, device="cuda")
    ws = torch.empty(max(fn("workspace_bytes")(plan), 256), dtype=torch.uint8, device="cuda")
    y = torch.empty((L.N, L.K, info.OH, info.OW), dtype=tdt, device="cuda")
    fn("set_workspace")(plan, ws.data_ptr(), ws.numel())
    st = torch.cuda.current_stream().cuda_stream
    xp, Up, yp = xd.data_ptr(), U.data_ptr(), y.data_ptr()
    fn("filter_transform")(plan, wd.data_ptr(), Up, st)
    for _ in range(args.warmup):
        fn("conv_forward")(plan, xp, Up, yp, st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fn("conv_forward")(plan, xp, Up, yp, st)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps

    def timed(call):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    x_bytes, y_bytes = 2.0 * x.size, 2.0 * y.numel()
    if single:
        # one kernel: x and y cross HBM once, V never leaves the registers
        k_ms = timed(lambda: fn("conv_forward")(plan, xp, Up, yp, st))
        stages = {
            "fused16_forward": {"ms": k_ms, "bound": "hbm", "algorithmic_bytes": x_bytes + y_bytes,
                                "achieved_GBps": (x_bytes + y_bytes) / k_ms / 1e6,
                                "frac_of_hbm_peak": (x_bytes + y_bytes) / k_ms / 1e6 / PEAK_HBM,
                                "algorithmic_flops": info.winograd_flops,
                                "achieved_TFLOPs": info.winograd_flops / k_ms / 1e9,
                                "frac_of_f16_mfma_peak": info.winograd_flops / k_ms / 1e9 / PEAK_MFMA_F16},
        }
        dom = "fused16_forward"
    else:
        in_ms = timed(lambda: fn("input_transform")(plan, xp, st))
        ct_ms = timed(lambda: fn("contract_output")(plan, Up, yp, st))
        v_bytes = 2.0 * info.mults_per_tile * L.C * info.T
        u_bytes = 2.0 * info.mults_per_tile * L.C * L.K
        ct_bytes = v_bytes + u_bytes + y_bytes
        stages = {
            "input_transform": {"ms": in_ms, "bound": "hbm", "algorithmic_bytes": x_bytes + v_bytes,
                                "achieved_GBps": (x_bytes + v_bytes) / in_ms / 1e6,
                                "frac_of_hbm_peak": (x_bytes + v_bytes) / in_ms / 1e6 / PEAK_HBM},
            "contract_output": {"ms": ct_ms, "bound": "hbm", "algorithmic_bytes": ct_bytes,
                                "achieved_GBps": ct_bytes / ct_ms / 1e6, "frac_of_hbm_peak": ct_bytes / ct_ms / 1e6 / PEAK_HBM,
                                "algorithmic_flops": info.winograd_flops,
                                "achieved_TFLOPs": info.winograd_flops / ct_ms / 1e9,
                                "frac_of_f16_mfma_peak": info.winograd_flops / ct_ms / 1e9 / PEAK_MFMA_F16},
        }
        dom = "contract_output" if ct_ms >= in_ms else "input_transform"
    out = {
        "metric": "direct-conv-equivalent TFLOP/s of DWM conv (%s storage, FP32 accumulation, 1 GPU); "
                  "MSE vs FP64 direct" % ("bfloat16" if bf16 else "binary16"),
        "value": info.direct_flops / dt / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f16", "data": "synthetic",
        "config": {"workload": L.name + ("_bf16" if bf16 else "_half"), "path": "single kernel" if single else "staged",
                   "parts": info.n_parts, "mults_per_tile": info.mults_per_tile,
                   "direct_GFLOP": info.direct_flops / 1e9, "winograd_GFLOP": info.winograd_flops / 1e9},
        "roofline": {"kernel": {"contract_output": "contract16_kernel", "input_transform": "input_transform_f16_kernel",
                                "fused16_forward": "fused16_forward_kernel"}[dom],
                     "bound": "hbm", "achieved": stages[dom]["achieved_GBps"], "peak": PEAK_HBM, "unit": "GB/s",
                     "frac": stages[dom]["frac_of_hbm_peak"], "traffic": None},
        "stages": stages,
    }
    if not args.no_check:
        import oracle
        yh = y.float().cpu().numpy()
        idx = np.random.default_rng(99).choice(yh.size, min(yh.size, 40000), replace=False)
        ref = oracle.direct_f64_at(x16.astype(np.float32), w16.astype(np.float32), L.stride, L.pad, idx)
        got = yh.ravel()[idx].astype(np.float64)
        mse = float(np.mean((got - ref) ** 2))
        out["accuracy"] = {"max_rel_err": float(np.max(np.abs(got - ref)) / np.max(np.abs(ref))),
                           "mse_vs_fp64_direct": mse, "log10_mse_plus_10": float(np.log10(mse) + 10),
                           "sampled_outputs": int(idx.size)}
    fn("plan_destroy")(plan)
    return out


def measure_forward(L, index, steps, warmup, args, check=True):
    """One layer through dwm_conv_forward: whole-step time, per-stage kernel times, accuracy."""
    import numpy as np
    import torch

    import dwm_workloads as wl
    import paper_2002_00552_amd as dwm

    if args.paper_layer:
        x, w = wl.make_layer_tensors(L, index)
    else:
        x, w = wl.make_layer_tensors(L, index)
    plan = dwm.dwm_plan_create(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    info = dwm.dwm_plan_info(plan)
    if args.contract_variant >= 0:
        dwm.dwm_plan_set_variant(plan, "contract", args.contract_variant)
    if args.input_variant >= 0:
        dwm.dwm_plan_set_variant(plan, "input", args.input_variant)
    if args.input_cg >= 0:
        dwm.dwm_plan_set_variant(plan, "input_cg", args.input_cg)
    if args.split_mode >= 0:
        dwm.dwm_plan_set_variant(plan, "split", args.split_mode)
    if args.forward_variant >= 0:
        dwm.dwm_plan_set_variant(plan, "forward", args.forward_variant)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    U = torch.empty(dwm.dwm_plan_filter_bytes(plan) // 4, dtype=torch.float32, device="cuda")
    ws = torch.empty(dwm.dwm_plan_workspace_bytes(plan) // 4, dtype=torch.float32, device="cuda")
    y = torch.empty((L.N, L.K, info.OH, info.OW), dtype=torch.float32, device="cuda")
    dwm.dwm_plan_set_workspace(plan, ws.data_ptr(), ws.numel() * 4)
    st = torch.cuda.current_stream().cuda_stream
    xp, Up, yp = xd.data_ptr(), U.data_ptr(), y.data_ptr()

    def event():
        return torch.cuda.Event(enable_timing=True)

    def timed(fn, n):
        """average ms of n back-to-back calls of fn between one pair of events on the kernels' stream"""
        e0, e1 = event(), event()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    dwm.dwm_filter_transform(plan, wd.data_ptr(), Up, st)  # first call: code object load
    filter_ms = timed(lambda: dwm.dwm_filter_transform(plan, wd.data_ptr(), Up, st), 1)

    for _ in range(warmup):
        dwm.dwm_conv_forward(plan, xp, Up, yp, st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        dwm.dwm_conv_forward(plan, xp, Up, yp, st)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3

    path = dwm.dwm_plan_info(plan).forward_path
    v_bytes = 4.0 * info.mults_per_tile * L.C * info.T
    x_bytes, y_bytes = 4.0 * x.size, 4.0 * y.numel()
    if path != 0:
        kname = "fused_forward_kernel"
        f_ms = timed(lambda: dwm.dwm_conv_forward(plan, xp, Up, yp, st), steps)
        stages = {
            "fused_forward": {"ms": f_ms, "algorithmic_flops": info.winograd_flops,
                              "achieved_TFLOPs": info.winograd_flops / f_ms / 1e9,
                              "frac_of_mfma_peak": info.winograd_flops / f_ms / 1e9 / PEAK_MFMA_F32,
                              "hbm_GBps_on_x_y": (x_bytes + y_bytes) / f_ms / 1e6,
                              "frac_of_hbm_peak": (x_bytes + y_bytes) / f_ms / 1e6 / PEAK_HBM},
            "filter_transform_once": {"ms": filter_ms},
        }
        roofline = {"kernel": kname, "bound": "mfma",
                    "achieved": info.winograd_flops / f_ms / 1e9, "peak": PEAK_MFMA_F32, "unit": "TFLOP/s",
                    "frac": info.winograd_flops / f_ms / 1e9 / PEAK_MFMA_F32,
                    "traffic": hbm_traffic(L.name, kname)}
    else:
        in_ms = timed(lambda: dwm.dwm_input_transform(plan, xp, st), steps)
        ct_ms = timed(lambda: dwm.dwm_contract_output(plan, Up, yp, st), steps)
        stages = {
            "input_transform": {"ms": in_ms, "bound": "hbm", "algorithmic_bytes": x_bytes + v_bytes,
                                "achieved_GBps": (x_bytes + v_bytes) / in_ms / 1e6,
                                "frac_of_hbm_peak": (x_bytes + v_bytes) / in_ms / 1e6 / PEAK_HBM},
            "contract_output": {"ms": ct_ms, "bound": "mfma", "algorithmic_flops": info.winograd_flops,
                                "achieved_TFLOPs": info.winograd_flops / ct_ms / 1e9,
                                "frac_of_mfma_peak": info.winograd_flops / ct_ms / 1e9 / PEAK_MFMA_F32,
                                "hbm_GBps_on_V_U_y": (v_bytes + y_bytes + 4.0 * U.numel()) / ct_ms / 1e6},
            "filter_transform_once": {"ms": filter_ms},
        }
        if ct_ms >= in_ms:
            roofline = {"kernel": "contract_kernel", "bound": "mfma",
                        "achieved": info.winograd_flops / ct_ms / 1e9, "peak": PEAK_MFMA_F32, "unit": "TFLOP/s",
                        "frac": info.winograd_flops / ct_ms / 1e9 / PEAK_MFMA_F32,
                        "traffic": hbm_traffic(L.name, "contract_kernel")}
        else:
            roofline = {"kernel": "input_transform_lds_kernel", "bound": "hbm",
                        "achieved": (x_bytes + v_bytes) / in_ms / 1e6, "peak": PEAK_HBM, "unit": "GB/s",
                        "frac": (x_bytes + v_bytes) / in_ms / 1e6 / PEAK_HBM,
                        "traffic": hbm_traffic(L.name, "input_transform_lds_kernel")}
    res = {
        "workload": L.name, "ms_per_step": ms_per_step,
        "value": info.direct_flops / (dt / steps) / 1e12,
        "config": {"workload": L.name, "N": L.N, "C": L.C, "H": L.H, "W": L.W, "K": L.K, "R": L.R, "S": L.S,
                   "stride": L.stride, "pad": L.pad, "parts": info.n_parts,
                   "mults_per_tile": info.mults_per_tile, "direct_GFLOP": info.direct_flops / 1e9,
                   "winograd_GFLOP": info.winograd_flops / 1e9},
        "roofline": roofline, "stages": stages,
        "path": ["input transform + contraction", "single kernel (V in registers)"][path],
    }
    if check:
        import oracle
        y.fill_(float("nan"))
        dwm.dwm_conv_forward(plan, xp, Up, yp, st)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        rng = np.random.default_rng(99)
        idx = rng.choice(yh.size, min(yh.size, 40000), replace=False)
        ref = oracle.direct_f64_at(x, w, L.stride, L.pad, idx)
        got = yh.ravel()[idx].astype(np.float64)
        mse = float(np.mean((got - ref) ** 2))
        res["accuracy"] = {"max_rel_err": float(np.max(np.abs(got - ref)) / np.max(np.abs(ref))),
                           "mse_vs_fp64_direct": mse, "log10_mse_plus_10": float(np.log10(mse) + 10),
                           "sampled_outputs": int(idx.size)}
    dwm.dwm_plan_destroy(plan)
    del xd, wd, U, ws, y
    torch.cuda.empty_cache()
    return res, x, w


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--paper-layer", type=str, default="", help="KERNEL,HW,STRIDE[,BATCH] e.g. 7,14,1")
    ap.add_argument("--contract-variant", type=int, default=-1)
    ap.add_argument("--input-variant", type=int, default=-1)
    ap.add_argument("--split-mode", type=int, default=-1)
    ap.add_argument("--input-cg", type=int, default=-1)
    ap.add_argument("--forward-variant", type=int, default=-1, help="0 staged, 1 single kernel, -1 planner")
    ap.add_argument("--backward-data", action="store_true",
                    help="time the gradient with respect to the input of the same layer instead of the forward pass")
    ap.add_argument("--bwd-path", type=int, default=-1, help="data gradient: 0 sub-convolutions, 1 single kernel, -1 planner")
    ap.add_argument("--backward-filter", action="store_true",
                    help="time the gradient with respect to the filter of the same layer instead of the forward pass")
    ap.add_argument("--half", action="store_true",
                    help="time the half-precision forward path (dwm_f16_*) of the same layer")
    ap.add_argument("--bf16", action="store_true",
                    help="time the bfloat16 forward path (dwm_bf16_*) of the same layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="measure the chosen layer only (the default also measures the other four)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "use --gpus 1. The forward path would shard over the batch with no exchange.")

    import torch

    import dwm_workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if args.paper_layer:
        vals = [int(v) for v in args.paper_layer.split(",")]
        kern, hw, stride = vals[:3]
        L = wl.paper_layer(kern, hw, stride, *vals[3:4])  # optional fourth value: batch size (the paper's is 256)
        index = 100 * kern + hw + stride
    else:
        L = wl.CONFIGS[args.config]
        index = args.config

    if args.backward_data or args.backward_filter or args.half or args.bf16:
        x, w = wl.make_layer_tensors(L, index)
        if args.backward_data:
            out = bench_backward_data(args, L, x, w)
        elif args.backward_filter:
            out = bench_backward_filter(args, L, x, w)
        else:
            out = bench_half(args, L, x, w, bf16=args.bf16)
        print(json.dumps(out))
        return

    res, x, w = measure_forward(L, index, args.steps, args.warmup, args, check=not args.no_check)
    out = {
        "metric": METRIC, "value": res["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": res["config"], "roofline": res["roofline"], "stages": res["stages"], "path": res["path"],
    }
    if "accuracy" in res:
        out["accuracy"] = res["accuracy"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x, w, L)
    del x, w
    if not args.no_per_config and not args.paper_layer:
        # all five layers, each measured like the headline one (its own entry is repeated here)
        per = []
        for i, Li in enumerate(wl.CONFIGS):
            r = res if i == args.config else measure_forward(Li, i, min(args.steps, 100), min(args.warmup, 30), args,
                                                             check=not args.no_check)[0]
            e = {"workload": r["workload"], "ms_per_step": r["ms_per_step"], "direct_equiv_TFLOPs": r["value"],
                 "path": r["path"], "kernel": r["roofline"]["kernel"], "bound": r["roofline"]["bound"],
                 "frac": r["roofline"]["frac"],
                 "stage_ms": {k: v["ms"] for k, v in r["stages"].items()}}
            if "input_transform" in r["stages"]:
                e["input_transform_frac_of_hbm_peak"] = r["stages"]["input_transform"]["frac_of_hbm_peak"]
            if "accuracy" in r:
                e["max_rel_err"] = r["accuracy"]["max_rel_err"]
                e["log10_mse_plus_10"] = r["accuracy"]["log10_mse_plus_10"]
            # the other paths of the same layer, each timed like its own mode of this script
            import copy
            a2 = copy.copy(args)
            a2.steps, a2.warmup = min(args.steps, 100), min(args.warmup, 30)
            a2.forward_variant = a2.contract_variant = a2.input_variant = a2.bwd_path = -1
            xi, wi = wl.make_layer_tensors(Li, i)
            other = {}
            for name, fn in (("binary16_forward", lambda: bench_half(a2, Li, xi, wi)),
                             ("bfloat16_forward", lambda: bench_half(a2, Li, xi, wi, bf16=True)),
                             ("backward_data", lambda: bench_backward_data(a2, Li, xi, wi)),
                             ("backward_filter", lambda: bench_backward_filter(a2, Li, xi, wi))):
                o = fn()
                other[name] = {"ms_per_step": o["ms_per_step"], "path": o["config"].get("path"),
                               "max_rel_err": o.get("accuracy", {}).get("max_rel_err")}
            del xi, wi
            e["other_paths"] = other
            per.append(e)
        out["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
