#!/usr/bin/env python3
"""Benchmark of the dft3d hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all]

One "step" is one whole transform (dft3d_exec: every kernel of the path) of one seeded
synthetic tensor that is already resident in HBM.  The default run (`--workload all`) times the
largest single-GPU configuration, the 2048^3 KDFT, for exactly K steps after W warm-up steps --
that is the headline `value` -- and then, with step counts of their own, the other
configurations (32^3, 256^3, 512^3 FFT formulation, nonuniform 128^3, 2048^3 FFT formulation),
which it reports in the `configs` table of the same single JSON line.  Every entry carries the
time per transform, the effective GFLOP/s (5 E log2 E convention), the roofline of its dominant
kernel measured with HIP events recorded by the library on the exec stream inside the timed
region, and the relative L2 distance from the CPU oracle on a sample of its outputs.  The oracle
is also timed on the host cores on a bounded sample of the headline workload (`cpu_baseline`).

`--workload <name>` runs one configuration alone (the form the rocprofv3 summaries under
profiles/ are made with).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time
from types import SimpleNamespace

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3      # 256 CU x 256 flop/clk x 2.4 GHz
PEAK_MFMA_BF16_TFLOPS = 2500.0    # dense bf16 matrix-core peak
PEAK_MFMA_F64_TFLOPS = 78.6
# fp32 vector units without the packed forms (this library is built with them switched off):
# 256 CU x 4 SIMD x 16 lanes x 2 flop (one FMA) x 2.4 GHz
PEAK_VALU_F32_TFLOPS = 78.6
PEAK_HBM_GBS = 8000.0

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.md")

# step counts of the configurations in the `configs` table of the default run (the headline
# configuration takes --steps / --warmup)
TABLE_RUNS = (
    ("cfg1", 200, 20),
    ("cfg2", 100, 10),
    ("cfg3", 100, 10),
    ("cfg4", 200, 20),
    ("cfg5-fft", 20, 3),
)
HEADLINE = "cfg5-kdft"


def log(msg: str) -> None:
    """Progress line on stderr (stdout carries the one JSON line)."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def effective_flop(E: int) -> float:
    return 5.0 * E * math.log2(E)


def measured_traffic(key: str):
    """HBM bytes per launch of the dominant kernel of a workload, from the committed counter table
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by the copy-kernel calibration); None if
    the table has no row for it."""
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 5 and cells[0] == key:
                    return float(cells[-1])
    except (OSError, ValueError):
        pass
    return None


def cpu_baseline(w, wl, budget_macs: float = 3.0e10):
    """Time the fp64 oracle on the host cores; full transform if small, else per-mode slabs."""
    import numpy as np
    from oracle import dft3d_oracle as orc

    n1, n2, n3 = w.shape
    E = w.elements
    total_macs = E * (n1 + n2 + n3)
    coords = wl.make_coords(w)
    if total_macs <= budget_macs:
        x = wl.make_input(w)
        t0 = time.perf_counter()
        orc.dft3d(x, coords)
        t = time.perf_counter() - t0
        sample = f"full {n1}x{n2}x{n3} transform, 1 run"
    else:
        # same sums on slabs of the tensor, one mode at a time, extrapolated linearly in the
        # number of independent rows (each mode's cost is exactly proportional to it)
        per_mode = budget_macs / 3
        t = 0.0
        parts = []
        for axis, n in enumerate(w.shape):
            other = E // n
            rows = max(1, min(other, int(per_mode / (n * n))))   # independent 1-D transforms
            # build a sample tensor whose `axis` has full length and the rest holds `rows` lines
            if axis == 0:
                shape = (n, 1, rows)
            elif axis == 1:
                shape = (1, n, rows)
            else:
                shape = (1, rows, n)
            xs = wl.draw_complex(shape, w.dist, w.seed + 17 * axis).astype(np.complex128)
            M = orc.dft_matrix(n, coords[axis])
            t0 = time.perf_counter()
            orc.mode_contract(M, xs, axis)
            dt = time.perf_counter() - t0
            t += dt * (other / rows)
            parts.append(f"mode {axis}: {rows} of {other} lines")
        sample = "per-mode direct sums on line samples, extrapolated: " + "; ".join(parts)
    return {
        "value": effective_flop(E) / t / 1e9,
        "unit": "GFLOP/s (5*E*log2(E))",
        "seconds_full_transform": t,
        "cores": orc.num_threads(),
        "kind": "oracle",
        "sample": sample,
    }


def download(x_dev):
    """Host copy of a device tensor, plane chunk by plane chunk (no second device buffer)."""
    import numpy as np
    import torch

    host = np.empty(tuple(x_dev.shape), dtype=np.complex64)
    ht = torch.from_numpy(host)
    chunk = max(1, (1 << 28) // max(1, x_dev.shape[1] * x_dev.shape[2]))
    for i in range(0, x_dev.shape[0], chunk):
        ht[i:i + chunk].copy_(x_dev[i:i + chunk])
    torch.cuda.synchronize()
    return host


def oracle_reference(w, wl, x_host, budget_macs: float = 3.0e10):
    """The oracle's values on a sample of the outputs of workload w (all of them when the whole
    fp64 transform is affordable, else a few output pencils along the first axis).  Returns
    (description, selector, reference) with selector(out_device_tensor) -> numpy sample."""
    import numpy as np
    from oracle import dft3d_oracle as orc

    n1, n2, n3 = w.shape
    coords = wl.make_coords(w)
    if w.elements * (n1 + n2 + n3) <= budget_macs:
        want = orc.dft3d(x_host, coords)
        return "every output", (lambda out: out.cpu().numpy()), want
    k2s = sorted({0, n2 - 1, 777 % n2})
    k3s = sorted({5 % n3, n3 // 2})
    want = orc.dft3d_pencils(x_host, k2s, k3s, coords)
    desc = f"output pencils X[:, k2, k3] for k2 in {k2s}, k3 in {k3s} ({want.size} outputs)"
    return desc, (lambda out: out[:, k2s][:, :, k3s].cpu().numpy()), want


def parity_entry(desc, got, want):
    import numpy as np

    got = np.asarray(got, dtype=np.complex128)
    err = np.abs(got - want)
    rms = float(np.sqrt(np.mean(np.abs(want) ** 2)))
    return {
        "rel_l2_vs_oracle": float(np.linalg.norm(err.ravel()) / max(np.linalg.norm(want.ravel()), 1e-300)),
        "max_abs_err_over_rms_ref": float(err.max() / max(rms, 1e-300)),
        "sample": desc,
        "tolerance": 2e-5,
    }


def resolve(name, wl, dft):
    """(workload, formulation) of a --workload name."""
    if name.startswith("shape:"):
        # any other size, e.g. shape:1024x1024x1024:fft or shape:1x4096x4096:fft:0,64,64 (first factors, 0 = the
        # library's default) or shape:384x384x384:kdft -- N(0,1) input, not one of the named configurations
        parts = name.split(":")
        shape = tuple(int(v) for v in parts[1].split("x"))
        form = dft.FFT if (len(parts) > 2 and parts[2] == "fft") else dft.KDFT
        splits = None
        if len(parts) > 3:
            first = [int(v) for v in parts[3].split(",")]
            splits = tuple((a, n // a) if a > 0 else (0, 0) for a, n in zip(first, shape))
        if len(shape) != 3 or min(shape) < 1:
            raise SystemExit("bench.py: shape:NXxNYxNZ[:fft|kdft[:a,b,c]]")
        return wl.Workload("shape_" + parts[1], 7, shape, form, "normal", splits=splits), form, True
    if name.startswith("cfg5") or name.startswith("2d-8192"):
        form = dft.FFT if name.endswith("fft") else dft.KDFT
        w = wl.WORKLOADS["cfg5"] if name.startswith("cfg5") else wl.EXTRA_WORKLOADS["2d-8192"]
        return w, form, True
    w = wl.WORKLOADS[name]
    return w, w.formulation, False


def measure(name, steps, warmup, settle_s, opts, mods, buffers=None, want_parity=False, x_host=None):
    """Times `steps` transforms of one workload and prices its dominant kernel.  Returns the result
    dictionary (the fields of the JSON line).  buffers = (x, out, workspace) device tensors to use
    instead of allocating; x_host = host copy of x for the oracle sample."""
    torch, wl, dft = mods.torch, mods.wl, mods.dft
    w, form, named_form = resolve(name, wl, dft)
    big = w.elements > (1 << 30)
    coords = wl.make_coords(w)
    # (opts.split_first: first-stage lengths that replace the workload's own split, e.g. the 32 x 64 split the
    # 2048^3 configuration is named with, next to the library's default 16 x 128)
    splits = w.splits
    if getattr(opts, "split_first", None) and form == dft.FFT:
        splits = tuple((a, n // a) for a, n in zip(opts.split_first, w.shape))
    split = [a for a, _ in splits] if (form == dft.FFT and splits) else None
    flags = 0
    if opts.unfused and form == dft.FFT:
        flags = dft.FLAG_UNFUSED     # 10 passes
    if opts.three_m and form == dft.KDFT:
        flags |= dft.FLAG_3M
    if opts.bf16x3 and form == dft.KDFT:
        flags |= dft.FLAG_BF16X3
    c128 = opts.complex128
    if c128:
        if big:
            raise SystemExit("bench.py: a complex128 tensor of this workload, its output and the workspace do not fit one GPU")
        flags = dft.FLAG_COMPLEX128
    plan = dft.Plan(w.shape, form, coords=coords, split=split, flags=flags)
    if form == dft.FFT:
        splits = tuple(plan.split(ax) for ax in range(3))      # (what the plan chose where none was named)
    axis_passes = [plan.mode_kernel(ax) for ax in range(3)]   # kernel family (KDFT) / pass structure (FFT) per axis
    if buffers is not None:
        x, out, ws = buffers
        if plan.workspace_bytes():
            plan.set_workspace(ws)
    else:
        if c128:
            x = torch.from_numpy(wl.draw_complex128(w.shape, w.seed)).to("cuda")
        elif big:
            x = wl.make_input_device(w)
        else:
            if x_host is None:
                x_host = wl.make_input(w)
            x = torch.from_numpy(x_host).to("cuda")
        out = torch.empty_like(x)
        plan.ensure_workspace()
    stream = torch.cuda.current_stream()

    # The shader clock of an idle MI355X takes some tenths of a second of load to reach its sustained
    # value (counted inside the 256^3 contraction kernel: 2.09 GHz in the first milliseconds, 2.35 GHz
    # sustained), so sub-millisecond workloads run the same step untimed for settle_s before the
    # warmup steps; the seconds-long workloads need none.
    # What a caller sees who starts from an idle chip: the same loop after half a second of idleness with
    # nothing but the warm-up steps before it (reported next to the settled time, never instead of it).
    ms_cold = None
    if settle_s > 0 and not opts.graph:
        torch.cuda.synchronize()
        time.sleep(0.5)
        for _ in range(warmup):
            plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
        tc = time.perf_counter()
        for _ in range(steps):
            plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
        ms_cold = (time.perf_counter() - tc) * 1e3 / steps
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < settle_s:
        for _ in range(20):
            plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
    for _ in range(warmup):
        plan.exec(x, out, stream=stream)
    torch.cuda.synchronize()

    if opts.graph:
        if big:
            raise SystemExit("bench.py: --graph is meant for the small workloads")
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            plan.exec(x, out)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        plan.enable_profiling(steps)
        te = time.perf_counter()
        for _ in range(steps):
            plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
        ms_with_events = (time.perf_counter() - te) * 1e3 / steps
    elif big:
        # seconds-long passes: the library's per-pass events sit inside the timed region
        plan.enable_profiling(steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_with_events = (t1 - t0) * 1e3 / steps
    else:
        # Small transforms: two event records per pass cost more than the passes are apart (32^3: 7.9 us
        # per transform without them, 15.3 us with them; 128^3: 64 against 87 us), so the timed region
        # runs the transform as a caller does, without per-pass timing, and the same number of steps is
        # repeated right after it with the events on for the per-kernel durations.
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        plan.enable_profiling(steps)
        te = time.perf_counter()
        for _ in range(steps):
            plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
        ms_with_events = (time.perf_counter() - te) * 1e3 / steps

    ms_per_step = (t1 - t0) * 1e3 / steps
    E = w.elements
    value = effective_flop(E) / (ms_per_step * 1e-3) / 1e9

    # per-pass kernel durations from the events the library recorded inside the timed region
    per_exec = [plan.read_profile(i) for i in range(steps)]
    npass = len(per_exec[0])
    pass_ms = [sum(p[i] for p in per_exec) / steps for i in range(npass)]
    kernel_note = None

    if form == dft.KDFT and npass == 1 and max(w.shape) <= 32 and not c128:
        # every axis at most 32 long: the whole transform is one launch
        pass_names = ["whole_transform"]
        dom_ms = pass_ms[0]
        flops = 8.0 * (w.shape[0] + w.shape[1] + w.shape[2]) * E
        roofline = {
            "bound": "alu", "kernel": "k_kdft_small (all three modes in one launch: x in fp32 vector arithmetic, z and y on fp32 MFMA)",
            "achieved": flops / (dom_ms * 1e-3) / 1e12, "peak": PEAK_VALU_F32_TFLOPS,
            "unit": "TFLOP/s", "avg_launch_ms": dom_ms, "flop_per_launch": flops,
            "note": "launch latency, not arithmetic, sets the time at this size: the fraction says nothing about the kernel",
        }
    elif form == dft.KDFT:
        # one pass per axis of length > 1, in the order z, y, x
        live = [ax for ax in (2, 1, 0) if w.shape[ax] > 1] or [2]
        pass_names = [f"mode_{'xyz'[ax]}({'contiguous' if ax == 2 else 'strided'})" for ax in live]
        # the strided contraction kernel runs all passes but the first: the dominant kernel
        dom = [i for i, ax in enumerate(live) if ax != 2] or [0]
        dom_ms = sum(pass_ms[i] for i in dom) / len(dom)
        n_dom = sum(w.shape[live[i]] for i in dom) / len(dom)     # contracted length of those passes
        # 4 (or, with --three-m, 3) real products per complex multiply-add
        flops = (6.0 if opts.three_m else 8.0) * n_dom * E
        roofline = {
            "bound": "mfma", "kernel": "k_contract_s (strided mode contraction, fp32 MFMA)",
            "achieved": flops / (dom_ms * 1e-3) / 1e12, "peak": PEAK_MFMA_F32_TFLOPS,
            "unit": "TFLOP/s", "avg_launch_ms": dom_ms,
            "flop_per_launch": flops,
        }
        if (not c128 and not opts.bf16x3 and not opts.three_m
                and all(w.shape[live[i]] in (16, 32, 64) for i in dom) and w.shape[2] % 16 == 0):
            # small square matrices run the streaming kernel, which uses three real products per complex one
            flops = 6.0 * n_dom * E
            roofline.update({"kernel": "k_contract_sr (streaming strided mode contraction, fp32 MFMA, 3M)",
                             "achieved": flops / (dom_ms * 1e-3) / 1e12, "flop_per_launch": flops})
        if c128:
            roofline.update({"kernel": "k_contract_f64 (strided mode contraction, fp64 MFMA)",
                             "peak": PEAK_MFMA_F64_TFLOPS})
        elif opts.bf16x3:
            # each real fp32 product becomes six bf16 products (level pairs of total order <= 2) and the
            # bf16 kernel takes three real products per complex one: priced in bf16 flops against the bf16 peak
            flops = 6.0 * 6.0 * n_dom * E
            roofline.update({"kernel": "k_contract_bf16x3 (strided mode contraction, bf16 MFMA, 3 real x 6 level products)",
                             "achieved": flops / (dom_ms * 1e-3) / 1e12, "peak": PEAK_MFMA_BF16_TFLOPS,
                             "flop_per_launch": flops,
                             "fp32_equivalent_tflops": 8.0 * n_dom * E / (dom_ms * 1e-3) / 1e12})
    else:
        pass_names = ["z_stage1+twiddle", "z_stage2", "y_stage1+twiddle", "y_stage2+reorder",
                      "x_stage1+twiddle", "x_stage2+reorder", "z_reorder"]
        if opts.unfused:
            pass_names = [f"{ax}_{st}" for ax in "zyx" for st in ("stage1", "phase", "stage2")] + ["reorder_xyz"]
        elif w.shape[0] == 1:
            pass_names = pass_names[0:4] + ["z_reorder"]          # no pass for the axis of length 1
        elif npass == 5:
            pass_names = ["z_fused_axis"] + pass_names[2:6]
        elif npass == 3:
            # (plans with 2048 points along x run the x pass first)
            pass_names = [f"{'xyz'[ax]}_fused_axis" for ax in plan.axis_order()]
        if w.name.startswith("shape_") and not (npass == 3 and min(w.shape) > 1):
            # an ad-hoc size: the pass structure is the plan's business; the passes are numbered and the slowest
            # one is priced by its bytes only
            pass_names = [f"pass{i}" for i in range(npass)]
        dom = max(range(npass), key=lambda i: pass_ms[i])
        dom_ms = pass_ms[dom]
        dom_name = pass_names[dom] if dom < len(pass_names) else f"pass{dom}"
        if (npass == 3 and not c128 and splits and splits[0] == splits[1] and pass_names[dom][0] in "xy"):
            # the y and the x pass are two launches of one kernel: the roofline of that kernel
            # uses its average launch duration, which is what a per-kernel profile reports
            dom_ms = 0.5 * sum(pass_ms[i] for i in range(3) if pass_names[i][0] in "xy")
            dom_name = "y_and_x_fused_axis"
            kernel_note = "fused strided-axis kernel, average of its two launches (y pass and x pass)"
        nbytes = (32.0 if c128 else 16.0) * E
        mfma_peak = PEAK_MFMA_F64_TFLOPS if c128 else PEAK_MFMA_F32_TFLOPS
        # flop of that pass: 8 per complex multiply-add of its stage matrices (+6 for a fused twiddle);
        # complex128 plans run staged passes with four real products throughout
        ax = {"z": 2, "y": 1, "x": 0}.get(dom_name[0])
        flops = 0.0
        if ax is not None and splits and "reorder_xyz" not in dom_name and "z_reorder" != dom_name and "phase" not in dom_name:
            A, B = splits[ax]
            if "fused" in dom_name:
                # fused kernels with three real products per complex product: 16x16 on every axis, 32x64 on
                # the contiguous axis; the others use four
                three = (A == 16 and B == 16)
                per_cmac = 6.0 if three else 8.0
                flops = (per_cmac * (A + B) + 6.0) * E
                nested = (A == 16 and B in (32, 64, 128)) or (A, B) == (32, 64)
                if ax == 2 and nested:
                    # second factor split once more inside the kernel (B = C*16): an A-point and a 16-point
                    # matrix stage with three real products each; the C-point butterflies and both twiddles
                    # are vector arithmetic and are not counted as matrix-core work
                    flops = 6.0 * (A + 16) * E
                elif ax != 2 and nested:
                    # the same on a strided axis: three real products in the first stage, four in the last
                    # (whose accumulators are the resident output tile)
                    flops = (6.0 * A + 8.0 * 16) * E
            elif "stage1" in dom_name and A in (2, 4, 8) and not c128 and not opts.unfused:
                # butterflies and twiddle in vector arithmetic: an element-wise, memory-bound pass
                flops = 0.0
            elif "stage2" in dom_name and A in (2, 4, 8) and B in (512, 1024, 2048) and not c128 and not opts.unfused:
                # the B-point stage on the fused kernels (B = 16 x (C*16)): two 16-point matrix stages, three real
                # products each on the contiguous axis, three and four on a strided one
                flops = (6.0 * 32 if ax == 2 else 6.0 * 16 + 8.0 * 16) * E
            elif "stage1" in dom_name:
                # strided stages with a 16 / 32 / 64 matrix run the three-product streaming kernel, and
                # every stage of 128 points or more takes the three-product scheme
                per_cmac = 6.0 if (not c128 and ((ax != 2 and A in (16, 32, 64)) or A >= 128 or
                                                  (A == 64 and not opts.unfused))) else 8.0
                flops = (per_cmac * A + (0.0 if opts.unfused else 6.0)) * E
            elif "stage2" in dom_name:
                per_cmac = 6.0 if (not c128 and ((ax != 2 and B in (16, 32, 64)) or B >= 128)) else 8.0
                flops = per_cmac * B * E
        hbm_frac = nbytes / (dom_ms * 1e-3) / 1e9 / PEAK_HBM_GBS
        mfma_frac = flops / (dom_ms * 1e-3) / 1e12 / mfma_peak
        # the pass is bound by whichever of the two takes longer at its peak rate
        if mfma_frac > hbm_frac:
            roofline = {
                "bound": "mfma", "kernel": dom_name,
                "achieved": flops / (dom_ms * 1e-3) / 1e12, "peak": mfma_peak, "unit": "TFLOP/s",
                "avg_launch_ms": dom_ms, "flop_per_launch": flops, "bytes_per_launch": nbytes,
                "hbm_frac": hbm_frac,
            }
        else:
            roofline = {
                "bound": "hbm", "kernel": dom_name,
                "achieved": nbytes / (dom_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "avg_launch_ms": dom_ms, "bytes_per_launch": nbytes, "flop_per_launch": flops,
                "mfma_frac": mfma_frac,
            }
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    if kernel_note:
        roofline["kernel_note"] = kernel_note
    variant = ("+complex128" if c128 else "") + ("+bf16x3" if (opts.bf16x3 and form == dft.KDFT) else "") + \
              ("+3m" if (opts.three_m and form == dft.KDFT) else "") + ("+unfused" if opts.unfused else "") + \
              ("+split" if (getattr(opts, "split_first", None) and form == dft.FFT) else "")
    roofline["traffic"] = measured_traffic(name + variant)
    if opts.three_m and form == dft.KDFT and not c128:
        roofline["complex_scheme"] = "3M"
    roofline["passes_ms"] = {(pass_names[i] if i < len(pass_names) else f"pass{i}"): round(pass_ms[i], 5)
                             for i in range(npass)}
    if opts.unfused and form == dft.FFT:
        # the memory-bound exhibits: every twiddle pass and the re-ordering pass move 16 bytes per element
        nb = 16.0 * E
        ph = [pass_ms[i] for i in range(npass) if i < len(pass_names) and pass_names[i].endswith("_phase")]
        ro = [pass_ms[i] for i in range(npass) if i < len(pass_names) and pass_names[i] == "reorder_xyz"]
        roofline["memory_bound_passes"] = {
            kname: {"avg_launch_ms": sum(v) / len(v), "achieved_GBs": nb / (sum(v) / len(v) * 1e-3) / 1e9,
                    "frac_of_hbm_peak": nb / (sum(v) / len(v) * 1e-3) / 1e9 / PEAK_HBM_GBS}
            for kname, v in (("k_phase", ph), ("k_reorder_rows", ro)) if v}

    result = {
        "metric": "dft3d_effective_gflops",
        "value": value,
        "unit": "GFLOP/s (5*E*log2(E), E = total points)",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64" if c128 else "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name + ("" if not named_form else ("_fft" if form == dft.FFT else "_kdft")),
            "clock_settle_s": settle_s,
            "ms_per_step_from_idle": ms_cold,
            "launch": "hip graph replay" if opts.graph else "eager",
            "per_pass_events": ("in the timed region" if (big and not opts.graph) else
                                "in a second loop of the same steps, %.5f ms per step there" % ms_with_events),
            "formulation": "FFT" if form == dft.FFT else "KDFT",
            "complex_scheme": "3M" if ((opts.three_m or opts.bf16x3) and form == dft.KDFT) else "4M",
            "arithmetic": "fp64 MFMA" if c128 else
                          "bf16x3 split on bf16 MFMA, fp32 accumulate" if (opts.bf16x3 and form == dft.KDFT)
                          else "fp32 MFMA",
            "shape": list(w.shape), "input": f"{'complex128' if c128 else 'complex64'}, iid {w.dist}, seed {w.seed}",
            "nonuniform": w.nonuniform,
            "split": [list(s) for s in splits] if (form == dft.FFT and splits) else None,
            "axes_xyz": axis_passes,
        },
        "roofline": roofline,
    }
    if want_parity and not c128:
        if x_host is None:
            x_host = download(x)
        ref = want_parity if isinstance(want_parity, tuple) else oracle_reference(w, wl, x_host)
        desc, select, want = ref
        plan.exec(x, out, stream=stream)
        torch.cuda.synchronize()
        result["parity"] = parity_entry(desc, select(out), want)
    plan.destroy()
    return result


PAPER_CONTEXT = {"hardware": "full TPU v3 Pod, 2048 cores (another machine, inter-core communication included)",
                 "size": "8192^3", "kdft_seconds": 12.66, "fft_seconds": 8.30,
                 "size_2048": {"kdft_seconds": 0.120, "fft_seconds": 0.118}}


def table_entry(r):
    """The fields of a `configs` table row, from a full result dictionary."""
    ro = r["roofline"]
    e = {
        "workload": r["config"]["workload"], "formulation": r["config"]["formulation"],
        "steps": r["steps"], "warmup": r["warmup"], "clock_settle_s": r["config"]["clock_settle_s"],
        "ms_per_step": r["ms_per_step"], "ms_per_step_from_idle": r["config"]["ms_per_step_from_idle"],
        "effective_gflops": r["value"],
        "dominant_kernel": ro["kernel"], "bound": ro["bound"], "avg_launch_ms": ro["avg_launch_ms"],
        "achieved": ro["achieved"], "peak": ro["peak"], "unit": ro["unit"], "frac": ro["frac"],
        "traffic": ro["traffic"], "passes_ms": ro["passes_ms"],
    }
    if r["config"].get("split"):
        e["split"] = r["config"]["split"]
    for k in ("hbm_frac", "mfma_frac", "note", "kernel_note"):
        if k in ro:
            e[k] = ro[k]
    if "parity" in r:
        e["parity"] = r["parity"]
    return e


def run_all(args, opts, mods):
    """The default run: headline 2048^3 KDFT with --steps / --warmup, then the configs table."""
    torch, wl, dft = mods.torch, mods.wl, mods.dft
    steps = args.steps if args.steps is not None else 5
    warmup = args.warmup if args.warmup is not None else 1
    w5 = wl.WORKLOADS["cfg5"]
    free, _total = torch.cuda.mem_get_info()
    need = 3 * w5.elements * 8 + (2 << 30)
    if free < need:
        raise SystemExit(f"bench.py: the 2048^3 configuration needs {need >> 30} GiB of free HBM "
                         f"(input, output, workspace), {free >> 30} GiB available")
    t_start = time.perf_counter()
    log("generating the 2048^3 input on the device")
    x = wl.make_input_device(w5)
    out = torch.empty_like(x)
    ws = torch.empty_like(x)
    torch.cuda.synchronize()
    log(f"{HEADLINE}: {warmup} warm-up + {steps} timed steps")
    head = measure(HEADLINE, steps, warmup, 0.0 if args.settle is None else args.settle, opts, mods,
                   buffers=(x, out, ws))
    # sample of the headline outputs against the oracle (needs the whole input on the host)
    parity_on = not args.no_parity
    ref5 = None
    log(f"{HEADLINE}: {head['ms_per_step']:.1f} ms per step")
    if parity_on:
        log("copying the input to the host for the oracle sample")
        x_host = download(x)
        log("oracle: sampled output pencils of the 2048^3 transform")
        ref5 = oracle_reference(w5, wl, x_host)
        del x_host
        desc, select, want = ref5
        head["parity"] = parity_entry(desc, select(out), want)   # `out` still holds the last timed step's result
    table = {HEADLINE: table_entry(head)}
    log("cfg5-fft")
    r = measure("cfg5-fft", 20, 3, 0.0, opts, mods, buffers=(x, out, ws), want_parity=ref5 if parity_on else False)
    table["cfg5-fft"] = table_entry(r)
    if parity_on:
        a, b = table[HEADLINE]["parity"], table["cfg5-fft"]["parity"]
        a["note"] = b["note"] = "the two formulations are compared on the same outputs of the same input"
    # the opt-in arithmetic variants of the contraction, on the same buffers and the same oracle sample
    variants = {}

    def with_flag(**kw):
        o = argparse.Namespace(**vars(opts))
        for key, val in kw.items():
            setattr(o, key, val)
        return o

    for label, kw in (("cfg5-kdft+3m", {"three_m": True}), ("cfg5-kdft+bf16x3", {"bf16x3": True})):
        log(label)
        r = measure(HEADLINE, 5, 1, 0.0, with_flag(**kw), mods, buffers=(x, out, ws),
                    want_parity=ref5 if parity_on else False)
        variants[label] = table_entry(r)
    # the FFT formulation with the split the configuration is named with (2048 = 32 x 64); the library's own
    # default, 16 x 128 with the second factor split once more inside the kernels, is the cfg5-fft entry
    log("cfg5-fft, split 32 x 64")
    r = measure("cfg5-fft", 10, 2, 0.0, with_flag(split_first=(32, 32, 32)), mods, buffers=(x, out, ws),
                want_parity=ref5 if parity_on else False)
    variants["cfg5-fft, split 32x64"] = table_entry(r)
    del x, out, ws, ref5
    torch.cuda.empty_cache()
    for label, kw in (("cfg2+3m", {"three_m": True}), ("cfg2+bf16x3", {"bf16x3": True}),
                      ("cfg2+complex128", {"complex128": True})):
        log(label)
        r = measure("cfg2", 100, 10, 0.3 if args.settle is None else args.settle, with_flag(**kw), mods,
                    want_parity=parity_on and "complex128" not in kw)
        variants[label] = table_entry(r)
    for name, k, wu in TABLE_RUNS:
        if name == "cfg5-fft":
            continue
        log(name)
        r = measure(name, k, wu, 0.3 if args.settle is None else args.settle, opts, mods, want_parity=parity_on)
        table[name] = table_entry(r)
    # the paper's two-dimensional size (8192 x 8192, the 2-D strong-scaling figure of Section V): not one of the
    # five configurations, reported beside them
    two_d = {}
    for name, k, wu in (("2d-8192-kdft", 10, 2), ("2d-8192-fft", 100, 10)):
        log(name)
        r = measure(name, k, wu, 0.3 if args.settle is None else args.settle, opts, mods, want_parity=parity_on)
        two_d[name] = table_entry(r)
    head["configs"] = {k: table[k] for k in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5-kdft", "cfg5-fft")}
    head["two_dimensional"] = two_d
    head["variants"] = variants
    head["paper_context"] = PAPER_CONTEXT
    if not args.no_cpu_baseline:
        log("cpu_baseline: the oracle on line samples of the 2048^3 workload")
        head["cpu_baseline"] = cpu_baseline(w5, wl)
    head["bench_wall_s"] = time.perf_counter() - t_start
    return head


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="all",
                    help="all (default: headline cfg5-kdft = KDFT 2048^3 plus a table of every configuration), "
                         "or one of cfg1..cfg4, cfg5-kdft, cfg5-fft, 2d-8192-kdft, 2d-8192-fft, copy, "
                         "or shape:NXxNYxNZ:fft|kdft[:first factors] for any other size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle samples of the default run")
    ap.add_argument("--parity", action="store_true", help="single workload: add the oracle sample")
    ap.add_argument("--three-m", action="store_true",
                    help="KDFT: three real products per complex product (DFT3D_FLAG_3M)")
    ap.add_argument("--bf16x3", action="store_true",
                    help="KDFT: fp32 accuracy from three bf16 levels on the bf16 matrix cores (DFT3D_FLAG_BF16X3)")
    ap.add_argument("--complex128", action="store_true",
                    help="KDFT: complex128 tensors on the fp64 matrix cores (DFT3D_FLAG_COMPLEX128)")
    ap.add_argument("--settle", type=float, default=None,
                    help="seconds of untimed steps before the warmup (default 0.3 for the sub-second "
                         "workloads, 0 for the seconds-long ones; 0 for counter collection runs)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one HIP graph that holds one exec (for the small, launch-bound "
                         "workloads); the per-kernel durations of the roofline then come from profiled "
                         "eager steps run right after the timed region")
    ap.add_argument("--unfused", action="store_true",
                    help="FFT: run the twiddle and the re-ordering as separate memory-bound kernels")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one MI355X holds the whole "
              "problem); --gpus must be 1", file=sys.stderr)
        return 2

    import torch

    import dft3d_workloads as wl
    import paper_2002_03260_amd as dft

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dft.load_library()
    torch.cuda.set_device(0)
    mods = SimpleNamespace(torch=torch, wl=wl, dft=dft)
    opts = SimpleNamespace(three_m=args.three_m, bf16x3=args.bf16x3, complex128=args.complex128,
                           unfused=args.unfused, graph=args.graph)

    name = args.workload
    if name == "copy":
        # bandwidth reference / counter calibration: plain copy of a 1 GiB tensor (the size of one
        # 512^3 complex64 tensor), traffic exactly 2 GiB per launch
        steps = args.steps if args.steps is not None else 20
        warmup = args.warmup if args.warmup is not None else 3
        n = (1 << 30) // 8
        a = torch.empty(n, dtype=torch.complex64, device="cuda").normal_()
        b = torch.empty_like(a)

        def timed(variant):
            for _ in range(warmup):
                dft.device_copy(a, b, variant)
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            t0 = time.perf_counter()
            ev[0].record()
            for _ in range(steps):
                dft.device_copy(a, b, variant)
            ev[1].record()
            torch.cuda.synchronize()
            return ev[0].elapsed_time(ev[1]) / steps, (time.perf_counter() - t0) * 1e3 / steps

        ms, wall_ms = timed(1)                  # plain accesses (the counter calibration kernel)
        ms_stream, _ = timed(101)               # streaming hint on loads and stores
        gbs = 2 * n * 8 / (ms * 1e-3) / 1e9
        print(json.dumps({"metric": "device_copy_bandwidth", "value": gbs, "unit": "GB/s", "n_gpus": 1,
                          "steps": steps, "warmup": warmup, "ms_per_step": wall_ms,
                          "higher_is_better": True, "dtype": "u8", "data": "synthetic",
                          "config": {"workload": "copy_1GiB"},
                          "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                       "frac": gbs / PEAK_HBM_GBS, "avg_launch_ms": ms,
                                       "bytes_per_launch": 2.0 * n * 8,
                                       "streaming_hint_GBs": 2 * n * 8 / (ms_stream * 1e-3) / 1e9}}), flush=True)
        return 0

    if name == "all":
        if args.complex128 or args.graph or args.unfused or args.three_m or args.bf16x3:
            print("bench.py: variant flags go with a single --workload", file=sys.stderr)
            return 2
        result = run_all(args, opts, mods)
        print(json.dumps(result), flush=True)
        return 0

    w, form, _ = resolve(name, wl, dft)
    big = w.elements > (1 << 30)
    steps = args.steps if args.steps is not None else (3 if (big and form == dft.KDFT) else 100)
    warmup = args.warmup if args.warmup is not None else (1 if big else 10)
    settle_s = args.settle if args.settle is not None else (0.0 if big else 0.3)
    result = measure(name, steps, warmup, settle_s, opts, mods, want_parity=args.parity)
    result["paper_context"] = PAPER_CONTEXT
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, wl)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
