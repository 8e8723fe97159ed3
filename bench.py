#!/usr/bin/env python3
"""Benchmark of the deep BLSTM training pass (forward + back-propagation through time).

One "step" = one blstm_stack_fwd_bwd call on one minibatch of synthetic,
speech-shaped input that is already resident in HBM: all layers, both
directions, gradients of every parameter.  Prints ONE JSON line:
frames/s over valid (unpadded) frames, plus a roofline object for the
dominant kernel (timed live with HIP events on its launch stream by the
library's profiling hooks) and the CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config3|config2]
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

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0    # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0
# fp32 operands multiplied as three bf16 parts each (the library's default): six bf16 matrix instructions do the work
# of one fp32 product, so a counted TFLOP/s of such a product is priced against a sixth of the bf16 peak
PEAK_F32_AS_3XBF16_TFLOPS = PEAK_BF16_MFMA_TFLOPS / 6.0
PRODUCT_KERNELS = ("input_projection", "input_gradient", "weight_gradient", "recurrent_weight_gradient", "output_layer_product")


def products_note(operand_dtype, gemm_variant):
    """How the whole-minibatch matrix products of a run were computed (the recurrent steps: matrix instructions of the
    operand type, fp32 accumulation)."""
    if operand_dtype == 1:
        return "operands rounded to bf16, bf16 matrix instructions, fp32 accumulation"
    if not gemm_variant:
        return ("fp32 operands, each cut exactly into three bf16 parts; six bf16 matrix instructions per product, fp32 "
                "accumulation; as close to an fp64 product as the fp32 matrix instructions (gemm_variant 3 selects those)")
    return "fp32 operands, fp32 matrix instructions"


def mfma_peak(kernel, operand_dtype, gemm_variant, recurrent_form=0):
    """(peak TFLOP/s, what it is) for the counted FLOP of one of the library's kernel groups.  recurrent_form: the plan's
    form of the recurrent product's operands (2: three bf16 parts)."""
    if operand_dtype == 1:
        return PEAK_BF16_MFMA_TFLOPS, "bf16 matrix instructions"
    if kernel in ("recurrent_forward", "recurrent_backward") and recurrent_form == 2:
        return PEAK_F32_AS_3XBF16_TFLOPS, "bf16 matrix instructions, six per fp32 product (operands exchanged and kept as three bf16 parts)"
    if kernel in PRODUCT_KERNELS and not gemm_variant:
        return PEAK_F32_AS_3XBF16_TFLOPS, "bf16 matrix instructions, six per fp32 product (operands cut into three bf16 parts)"
    return PEAK_FP32_MFMA_TFLOPS, "fp32 matrix instructions"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def clock_state():
    """Clock and power state of the first GPU as the amdgpu driver's sysfs files report it (a short string; None
    where they cannot be read).  Files are read directly: no other program is started from this process."""
    import glob

    def first_line(path, star_only=False):
        try:
            with open(path) as fh:
                lines = [ln.strip() for ln in fh.read().splitlines() if ln.strip()]
        except OSError:
            return None
        if star_only:
            lines = [ln for ln in lines if ln.endswith("*")] or lines[:1]
        return lines[0] if lines else None

    out = []
    for dev_dir in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        if first_line(os.path.join(dev_dir, "vendor")) != "0x1002":
            continue
        for name, star in (("pp_dpm_sclk", True), ("pp_dpm_mclk", True), ("pp_dpm_fclk", True),
                           ("power_dpm_force_performance_level", False)):
            v = first_line(os.path.join(dev_dir, name), star)
            if v is not None:
                out.append(f"{name} {v}")
        for hw in sorted(glob.glob(os.path.join(dev_dir, "hwmon", "hwmon*"))):
            for name in ("power1_average", "power1_input"):
                v = first_line(os.path.join(hw, name))
                if v is not None:
                    out.append(f"{name} {int(v) / 1e6:.0f} W")
                    break
        break
    return "; ".join(out) if out else None


def recorded_traffic(workload, kernel, version, plan=None):
    """HBM bytes per launch of `kernel` from the rocprofv3 counter runs recorded in profiles/hbm_traffic.json, or
    (None, why) when the record was made with other kernels than the ones this run launched (another library
    version or another layout of the recurrent passes): a stale figure is worse than none."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as fh:
            rec = json.load(fh)["workloads"].get(workload)
    except (OSError, ValueError, KeyError) as ex:
        return None, f"no usable traffic record ({type(ex).__name__})"
    if rec is None:
        return None, "no counter run recorded for this workload"
    if rec.get("library_version") != version:
        return None, (f"counter run was made with library version {rec.get('library_version')} (commit {rec.get('commit')}), "
                      f"this is {version}: not reported")
    if plan is not None and rec.get("plan") is not None and rec["plan"] != plan:
        return None, "counter run was made with another layout of the recurrent passes: not reported"
    v = rec["bytes_per_launch"].get(kernel)
    return v, f"{rec['source']} (commit {rec.get('commit')}, {rec.get('date')})"


def time_steps(step, steps, rl, torch):
    """The timing protocol of every workload: `steps` calls between device synchronisations with the library's event
    hooks off, each call also bracketed by a pair of events on the current stream (median / minimum); then a loop of at
    most 5 calls with the hooks on, from which the per-kernel figures come.  Returns a dict."""
    rl.rlstm_profile_enable(False)
    rl.rlstm_profile_read()
    step_events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    clocks = clock_state()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in step_events:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_ms = sorted(e0.elapsed_time(e1) for e0, e1 in step_events)
    hook_steps = max(1, min(steps, 5))
    rl.rlstm_profile_enable(True)
    torch.cuda.synchronize()
    th0 = time.perf_counter()
    for _ in range(hook_steps):
        step()
    torch.cuda.synchronize()
    th1 = time.perf_counter()
    rl.rlstm_profile_enable(False)
    prof = rl.rlstm_profile_read(1 << 16)
    return {"ms_per_step": (t1 - t0) * 1e3 / steps, "ms_per_step_median": step_ms[len(step_ms) // 2],
            "ms_per_step_min": step_ms[0], "ms_per_step_with_timing_hooks": (th1 - th0) * 1e3 / hook_steps,
            "hook_steps": hook_steps, "prof": prof, "clock_state": clocks,
            "timing": "value and ms_per_step: K steps between device synchronisations, the library's event hooks off; "
                      "median / min: per-step event pairs in that same loop; the per-kernel figures come from a separate "
                      f"loop of {hook_steps} steps with the hooks on (ms_per_step_with_timing_hooks)"}


def rec_bytes(kind, wl, steps):
    """Algorithmic HBM bytes of `steps` recurrent steps (both directions), fp32: forward reads Z and writes
    gates, y, c; backward reads gates, c (twice), dy and writes dz; the recurrent matrix is read once per launch."""
    per_slot_dir = 4 * ((4 + 4 + 1 + 1) * wl.H) if kind == 1 else 4 * ((4 + 2 + 1 + 4) * wl.H)
    return 2.0 * steps * wl.B * per_slot_dir


def cpu_baseline(wl_full, seconds_budget=20.0, output_layer=None):
    """Times the oracle (as it is, numpy fp64) on a bounded sample of the same workload:
    the same network on the first Ts frames of the minibatch.  output_layer = (Wo, bo, labels): the
    sample is a whole training step (output layer between the passes, Adam update of every parameter)."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import blstm_stack_backward, blstm_stack_forward
    from paper_1608_00895_amd import synth

    # frames of the slice: sized so that the oracle runs for some tens of seconds (config 4: 6 x 1000 units, B = 64)
    Ts = 64 if wl_full.H >= 1000 else (512 if wl_full.H >= 400 else 500)
    Ts = min(Ts, wl_full.T)
    lens = np.minimum(wl_full.seq_lens, Ts).astype(np.int32)
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl_full.params]
    x = wl_full.x[:Ts].astype(np.float64)
    G = wl_full.G[:Ts].astype(np.float64)
    what = "forward+backward"
    t0 = time.perf_counter()
    y, caches = blstm_stack_forward(x, params, lens)
    if output_layer is None:
        blstm_stack_backward(caches, G)
    else:
        from oracle import adam_step, softmax_ce_backward, softmax_ce_forward
        Wo, bo, labels = output_layer
        g = softmax_ce_backward(softmax_ce_forward(y, Wo, bo, labels[:Ts], lens))
        grads, _ = blstm_stack_backward(caches, g["dy"])
        flat_p = [a for layer in params for p in layer for a in p] + [Wo.astype(np.float64), bo.astype(np.float64)]
        flat_g = [grads[l][d][k] for l in range(wl_full.L) for d in range(2) for k in ("dW", "dR", "db")] + [g["dWo"], g["dbo"]]
        for p, gr in zip(flat_p, flat_g):
            adam_step(p, gr, np.zeros_like(p), np.zeros_like(p), 1e-5, 0.9, 0.999, 1e-8, 1)
        what = "training step (forward, softmax/cross-entropy, backward, Adam)"
    dt = time.perf_counter() - t0
    threads = max([i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"] or [1])
    frames = int(lens.sum())
    return {"value": frames / dt, "unit": "frames/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{wl_full.name}: same {wl_full.L}-layer network, first {Ts} frames of all {wl_full.B} "
                      f"sequences ({frames} frames), numpy fp64 {what}, {dt:.1f} s"}


def bench_config5(args):
    """The two-dimensional LSTM layer (four scan directions) on config 5: one step = mdlstm_fwd + mdlstm_bwd
    on one batch of 8 images resident in HBM, gradients of every parameter, no dx (the layer is the bottom one)."""
    import numpy as np
    import torch
    from paper_1608_00895_amd import binding as rl
    from paper_1608_00895_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    wl = synth.config5()
    log(f"workload {wl.name}: Hh={wl.Hh} Ww={wl.Ww} B={wl.B} D={wl.D} H={wl.H} pixels={wl.pixels}")
    desc = rl.rmdlstm_desc(Hh=wl.Hh, Ww=wl.Ww, B=wl.B, D=wl.D, H=wl.H, operand_dtype=0)
    x = torch.from_numpy(wl.x).to(dev)
    widths = torch.from_numpy(wl.widths).to(dev)
    params = [torch.from_numpy(a).to(dev) for p in wl.params for a in p]
    grads = [torch.empty_like(p) for p in params]
    G = torch.from_numpy(wl.G).to(dev)
    y = torch.empty((wl.Hh, wl.Ww, wl.B, 4 * wl.H), device=dev)
    reserve = torch.empty(rl.rmdlstm_reserve_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(rl.rmdlstm_workspace_bytes(desc), dtype=torch.uint8, device=dev)

    def step():
        rl.mdlstm_fwd(desc, x, params, widths, y, reserve, ws)
        rl.mdlstm_bwd(desc, x, params, widths, reserve, G, None, grads, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    tm = time_steps(step, args.steps, rl, torch)
    prof, hook_steps = tm["prof"], tm["hook_steps"]
    if args.calibration_copy:
        n = 1 << 28
        src = torch.ones(n, device=dev)
        dst = torch.empty(n, device=dev)
        rl.rlstm_copy_f32(dst, src, n)
        torch.cuda.synchronize()
    ms_per_step = tm["ms_per_step"]
    by_kind = {}
    for kind, layer, ndir, ms, nsteps, flop in prof:
        d = by_kind.setdefault(kind, {"ms": 0.0, "launches": 0, "flop": 0.0, "rsteps": 0})
        d["ms"] += ms; d["launches"] += 1; d["flop"] += flop; d["rsteps"] += nsteps
    names = {0: "input_projection", 1: "mdlstm_forward_scan", 2: "mdlstm_backward_scan", 3: "input_gradient",
             4: "weight_gradient", 5: "recurrent_weight_gradient"}
    kernels = []
    # the scans only do arithmetic inside the images: price them with the valid pixels, not the padded slots
    valid_frac = wl.pixels / float(wl.Hh * wl.Ww * wl.B)
    for kind, d in sorted(by_kind.items()):
        flop = d["flop"] * (valid_frac if kind in (1, 2) else 1.0)
        e = {"kernel": names[kind], "launches_per_step": d["launches"] / hook_steps, "avg_ms": d["ms"] / d["launches"],
             "ms_per_step": d["ms"] / hook_steps, "tflops": flop / (d["ms"] * 1e-3) / 1e12}
        if kind in (1, 2):
            e["diagonals_per_launch"] = d["rsteps"] / d["launches"]
            e["diagonal_us"] = 1e3 * d["ms"] / d["rsteps"]
        kernels.append(e)
        log(e)
    dom = max(kernels, key=lambda e: e["ms_per_step"])
    # HBM bytes per launch from the rocprofv3 FETCH_SIZE + WRITE_SIZE runs at this workload, scaled by a copy kernel
    traffic, traffic_source = recorded_traffic("config5", dom["kernel"], rl.version())
    roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["tflops"] / PEAK_FP32_MFMA_TFLOPS, "traffic": traffic,
                "traffic_source": traffic_source,
                "avg_launch_ms": dom["avg_ms"],
                "note": "one workgroup per (scan direction, image, band of 16 rows): 128 of the 256 CUs work, and the chain of "
                        "anti-diagonals is serial (a step's MFMAs alone take a CU 0.53 us of the measured step); priced against "
                        "the whole chip's fp32 MFMA peak with 2 * 2H * 5H FLOP per valid pixel and direction"}
    out = {"metric": "MDLSTM train pixels/sec (fwd+bwd), 4 scan directions", "value": wl.pixels / (ms_per_step * 1e-3),
           "unit": "pixels/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "ms_per_step_median": tm["ms_per_step_median"], "ms_per_step_min": tm["ms_per_step_min"],
           "ms_per_step_with_timing_hooks": tm["ms_per_step_with_timing_hooks"], "timing": tm["timing"],
           "clock_state": tm["clock_state"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": wl.name, "height": wl.Hh, "padded_width": wl.Ww, "images": wl.B,
                      "units_per_direction": wl.H, "valid_pixels": wl.pixels,
                      "padded_pixel_slots": wl.Hh * wl.Ww * wl.B},
           "roofline": roofline, "kernels": kernels}
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        from oracle import mdlstm4_backward, mdlstm4_forward
        wc = 400                                   # the oracle on the first 400 columns of every image (about 10 s)
        p64 = [tuple(a.astype(np.float64) for a in p) for p in wl.params]
        wcrop = np.minimum(wl.widths, wc)
        t0 = time.perf_counter()
        yc, fw = mdlstm4_forward(wl.x[:, :wc].astype(np.float64), p64, wcrop)
        mdlstm4_backward(fw, wl.G[:, :wc].astype(np.float64))
        dt = time.perf_counter() - t0
        threads = max([i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"] or [1])
        px = int(wcrop.sum()) * wl.Hh
        out["cpu_baseline"] = {"value": px / dt, "unit": "pixels/s", "cores": int(threads), "kind": "oracle",
                               "sample": f"{wl.name}: first {wc} columns of all {wl.B} images ({px} pixels), "
                                         f"numpy fp64 forward+backward, {dt:.1f} s"}
    print(json.dumps(out), flush=True)


def bench_gemm(args):
    """The whole-minibatch matrix products alone, at the shapes of config 3 and of the paper's batch: one step = one
    launch of every shape; reports TFLOP/s per shape for the kernel the library picks for fp32 operands (three bf16
    parts per operand, six bf16 matrix instructions per product: priced against a sixth of the bf16 peak) and for the
    kernels on the fp32 matrix instructions (pipelined where the operands allow, and plain)."""
    import torch
    from paper_1608_00895_amd import binding as rl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    shapes = [("config3 projection X W (NN)", 0, 0, 32000, 2000, 1000), ("config3 input gradient dZ W^T (NT)", 0, 1, 32000, 500, 2000),
              ("config3 weight gradient X^T dZ (TN)", 1, 0, 1000, 2000, 32000), ("config3 recurrent weight gradient (TN)", 1, 0, 500, 2000, 31968),
              ("paper batch projection (NN)", 0, 0, 20250, 2048, 1024), ("paper batch input gradient (NT)", 0, 1, 20250, 512, 2048),
              ("paper batch weight gradient (TN)", 1, 0, 1024, 2048, 20250), ("paper batch output layer logits (NN)", 0, 0, 20250, 1504, 1024),
              ("square 8192 (NN)", 0, 0, 8192, 8192, 8192)]
    sk = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    kernels, total_flop, total_ms = [], 0.0, 0.0
    # bring the clocks up before the first timed shape
    Aw, Bw, Cw = torch.randn((4096, 4096), device=dev), torch.randn((4096, 4096), device=dev), torch.empty((4096, 4096), device=dev)
    for _ in range(40):
        rl.rlstm_gemm_f32(0, 0, 4096, 4096, 4096, Aw, 4096, Bw, 4096, Cw, 4096, None, None)
    torch.cuda.synchronize()
    for name, ta, tb, M, N, K in shapes:
        A = torch.randn((K, M) if ta else (M, K), device=dev)
        B = torch.randn((N, K) if tb else (K, N), device=dev)
        C = torch.empty((M, N), device=dev)
        lda, ldb = (M if ta else K), (K if tb else N)
        res = {}
        for variant, tag in ((0, "picked"), (3, "fp32_instructions"), (2, "plain")):
            for _ in range(args.warmup):
                rl.rlstm_gemm_f32(ta, tb, M, N, K, A, lda, B, ldb, C, N, None, sk, variant=variant)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                rl.rlstm_gemm_f32(ta, tb, M, N, K, A, lda, B, ldb, C, N, None, sk, variant=variant)
            e1.record()
            torch.cuda.synchronize()
            res[tag] = e0.elapsed_time(e1) / args.steps
        flop = 2.0 * M * N * K
        kernels.append({"kernel": name, "M": M, "N": N, "K": K, "avg_ms": res["picked"], "tflops": flop / res["picked"] / 1e9,
                        "frac_of_mfma_peak": flop / res["picked"] / 1e9 / PEAK_F32_AS_3XBF16_TFLOPS,
                        "fp32_instruction_kernel_ms": res["fp32_instructions"],
                        "fp32_instruction_kernel_tflops": flop / res["fp32_instructions"] / 1e9,
                        "plain_kernel_ms": res["plain"], "plain_kernel_tflops": flop / res["plain"] / 1e9})
        log(kernels[-1])
        total_flop += flop; total_ms += res["picked"]
    # the bf16-operand products at config 4's shapes: operands read as fp32 and rounded on the way into LDS (operands in the
    # layouts the layer holds them in) against bf16 copies laid out along k (what the stack's large products run on)
    bf16_kernels = []
    shapes16 = [("config4 projection X W (NN)", 0, 0, 96000, 4000, 2000), ("config4 input gradient of both directions, K = 8H (NT)", 0, 1, 96000, 2000, 8000),
                ("config4 weight gradient X^T dZ (TN)", 1, 0, 2000, 4000, 96000), ("config4 recurrent weight gradient (TN)", 1, 0, 1000, 4000, 95936)]
    sk16 = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    for name, ta, tb, M, N, K in shapes16:
        A = torch.randn((K, M) if ta else (M, K), device=dev)
        B = torch.randn((N, K) if tb else (K, N), device=dev)
        C = torch.empty((M, N), device=dev)
        Ak = torch.empty((M, K), dtype=torch.int16, device=dev)
        Bk = torch.empty((N, K), dtype=torch.int16, device=dev)
        if ta:
            rl.rlstm_to_bf16_2d(None, Ak, A, K, M, M)
        else:
            rl.rlstm_to_bf16(Ak, A)
        if tb:
            rl.rlstm_to_bf16(Bk, B)
        else:
            rl.rlstm_to_bf16_2d(None, Bk, B, K, N, N)
        lda, ldb = A.shape[1], B.shape[1]
        res = {}
        for tag, fn in (("fp32_operands", lambda: rl.rlstm_gemm_bf16(ta, tb, M, N, K, A, lda, B, ldb, C, N, None, sk16)),
                        ("bf16_copies", lambda: rl.rlstm_gemm_bf16_mem(0, 1, M, N, K, Ak, K, Bk, K, C, N, None, sk16))):
            for _ in range(args.warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            res[tag] = e0.elapsed_time(e1) / args.steps
        flop = 2.0 * M * N * K
        bf16_kernels.append({"kernel": name, "M": M, "N": N, "K": K, "avg_ms": res["bf16_copies"], "tflops": flop / res["bf16_copies"] / 1e9,
                             "frac_of_bf16_peak": flop / res["bf16_copies"] / 1e9 / PEAK_BF16_MFMA_TFLOPS,
                             "fp32_operands_ms": res["fp32_operands"], "fp32_operands_tflops": flop / res["fp32_operands"] / 1e9})
        log(bf16_kernels[-1])
        del A, B, C, Ak, Bk
    dom = kernels[0]
    out = {"metric": "fp32 matrix products alone, TFLOP/s over all shapes", "value": total_flop / total_ms / 1e9, "unit": "TFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": total_ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "matrix products at the shapes of config 3 and of the paper's batch"},
           "roofline": {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_F32_AS_3XBF16_TFLOPS,
                        "unit": "TFLOP/s", "frac": dom["tflops"] / PEAK_F32_AS_3XBF16_TFLOPS, "traffic": None,
                        "note": "fp32 operands cut into three bf16 parts, six bf16 matrix instructions per product: "
                                "the peak is a sixth of the bf16 matrix peak"},
           "kernels": kernels, "bf16_kernels": bf16_kernels}
    print(json.dumps(out), flush=True)


def bench_stream(args):
    """The streaming mode on whole sequences: one step = one lstm_stream_fwd_bwd call (all segments, forward and
    truncated backward, gradients of every parameter) on sequences resident in HBM."""
    import numpy as np
    import torch
    from paper_1608_00895_amd import binding as rl
    from paper_1608_00895_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    wl = synth.paper_stream()
    log(f"workload {wl.name}: L={wl.L} S={wl.S} Tc={wl.Tc} B={wl.B} D={wl.D} H={wl.H} frames={wl.frames}")
    desc = rl.rlstm_stream_desc(L=wl.L, S=wl.S, Tc=wl.Tc, B=wl.B, D=wl.D, H=wl.H, operand_dtype=0, engine=args.engine,
                                batch_groups=args.batch_groups or 0, bwd_exchange=args.bwd_exchange or 0)
    x = torch.from_numpy(wl.x).to(dev)
    sl = torch.from_numpy(wl.seq_lens).to(dev)
    params = [torch.from_numpy(a).to(dev) for p in wl.params for a in p]
    grads = [torch.empty_like(p) for p in params]
    G = torch.from_numpy(wl.G).to(dev)
    y = torch.empty((wl.S * wl.Tc, wl.B, wl.H), device=dev)
    state = torch.zeros((wl.L, 2, wl.B, wl.H), device=dev)
    reserve = torch.empty(rl.rlstm_stream_reserve_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(rl.rlstm_stream_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    stream_b = None if args.one_stream else torch.cuda.Stream()      # takes the weight gradients

    def step():
        state.zero_()
        rl.lstm_stream_fwd_bwd(desc, x, params, sl, G, y, grads, None, state, reserve, ws, stream_b=stream_b)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert rl.rlstm_last_timeout(ws) == 0
    tm = time_steps(step, args.steps, rl, torch)
    prof, hook_steps = tm["prof"], tm["hook_steps"]
    assert rl.rlstm_last_timeout(ws) == 0
    if args.calibration_copy:
        n = 1 << 28
        src = torch.ones(n, device=dev)
        dst = torch.empty(n, device=dev)
        rl.rlstm_copy_f32(dst, src, n)
        torch.cuda.synchronize()
    ms_per_step = tm["ms_per_step"]
    by_kind = {}
    for kind, layer, ndir, ms, nsteps, flop in prof:
        d = by_kind.setdefault(kind, {"ms": 0.0, "launches": 0, "flop": 0.0, "rsteps": 0})
        d["ms"] += ms; d["launches"] += 1; d["flop"] += flop; d["rsteps"] += nsteps
    kernels = []
    for kind, d in sorted(by_kind.items()):
        e = {"kernel": rl.PROFILE_KINDS[kind], "launches_per_step": d["launches"] / hook_steps,
             "avg_ms": d["ms"] / d["launches"], "ms_per_step": d["ms"] / hook_steps,
             "tflops": d["flop"] / (d["ms"] * 1e-3) / 1e12}
        e["mfma_peak_tflops"], e["mfma_path"] = mfma_peak(e["kernel"], 0, args.gemm_variant)
        e["frac_of_mfma_peak"] = e["tflops"] / e["mfma_peak_tflops"]
        if kind in (1, 2):
            e["steps_per_launch"] = d["rsteps"] / d["launches"]
            e["step_us"] = 1e3 * d["ms"] / d["rsteps"]
        kernels.append(e)
        log(e)
    dom = max(kernels, key=lambda e: e["ms_per_step"])
    # bytes per launch from the rocprofv3 FETCH_SIZE + WRITE_SIZE runs (profiles/lstm_stream_paper_stream_hbm_counters.md)
    traffic, traffic_source = recorded_traffic("paper_stream", dom["kernel"], rl.version())
    if args.batch_groups is not None or args.bwd_exchange is not None or args.engine != 0:
        traffic, traffic_source = None, "not reported with non-default settings"
    roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["tflops"] / PEAK_FP32_MFMA_TFLOPS, "traffic": traffic,
                "traffic_source": traffic_source,
                "avg_launch_ms": dom["avg_ms"], "steps_per_launch": dom.get("steps_per_launch"), "step_us": dom.get("step_us"),
                "note": "the recurrent kernels are bound by the serial chain of dependent steps (see step_us); priced "
                        "against the fp32 MFMA peak with 2*B*H*4H FLOP per step"}
    slots = wl.S * wl.Tc * wl.B
    out = {"metric": "LSTM streaming train frames/sec (segments chained by final states, truncated BPTT)",
           "value": wl.frames / (ms_per_step * 1e-3), "unit": "frames/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step,
           "ms_per_step_median": tm["ms_per_step_median"], "ms_per_step_min": tm["ms_per_step_min"],
           "ms_per_step_with_timing_hooks": tm["ms_per_step_with_timing_hooks"], "timing": tm["timing"],
           "clock_state": tm["clock_state"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": wl.name, "layers": wl.L, "units": wl.H, "sequences": wl.B, "segments": wl.S,
                      "segment_frames": wl.Tc, "valid_frames": wl.frames, "padded_slots": slots,
                      "engine": "persistent" if args.engine in (0, 1) else "stepwise",
                      "products": products_note(0, args.gemm_variant)},
           "roofline": roofline, "kernels": kernels}
    try:
        out["config"]["plan"] = rl.rblstm_plan(rl.rblstm_desc(L=wl.L, T=wl.Tc, B=wl.B, D=wl.D, H=wl.H, operand_dtype=0,
                                                              engine=args.engine))
        out["config"]["plan_note"] = "plan of a bidirectional stack of the same shape, for reference only"
    except rl.RlstmError:
        pass
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        from oracle import lstm_stream_forward_backward
        Tc, S2 = wl.Tc, 4                          # the oracle on the first 4 of the 6 segments (about 10 s)
        p64 = [tuple(a.astype(np.float64) for a in p) for p in wl.params]
        lens = np.minimum(wl.seq_lens, Tc * S2)
        t0 = time.perf_counter()
        lstm_stream_forward_backward(wl.x[:Tc * S2].astype(np.float64), p64, lens, wl.G[:Tc * S2].astype(np.float64), Tc)
        dt = time.perf_counter() - t0
        threads = max([i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"] or [1])
        out["cpu_baseline"] = {"value": int(lens.sum()) / dt, "unit": "frames/s", "cores": int(threads), "kind": "oracle",
                               "sample": f"{wl.name}: same network, first {S2} segments of {Tc} frames of all {wl.B} "
                                         f"sequences ({int(lens.sum())} frames), numpy fp64, {dt:.1f} s"}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config3", choices=["config2", "config3", "config4", "config5", "paper_chunks", "paper_train", "paper_stream", "gemm"])
    ap.add_argument("--engine", type=int, default=0)
    ap.add_argument("--one-stream", action="store_true")
    ap.add_argument("--first-piece", type=int, default=None,
                    help="steps of the first piece the recurrent passes are cut into (library default if omitted; -1 = uncut)")
    ap.add_argument("--batch-groups", type=int, default=None,
                    help="groups the sequences are dealt out to per direction (library default if omitted)")
    ap.add_argument("--overlap-mode", type=int, default=None,
                    help="1 serial, 2 products share CUs with the recurrent kernels (chosen per shape if omitted)")
    ap.add_argument("--bwd-exchange", type=int, default=None,
                    help="exchanges per step of the backward recurrent kernel: 1 two, 2 one where it applies (library default if omitted)")
    ap.add_argument("--gemm-variant", type=int, default=None,
                    help="matrix-product kernel choice (the descriptors' gemm_variant; library default if omitted)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, run one plain 1 GiB copy kernel (known HBM traffic) "
                         "so that a counter-collecting profiler run can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "config5":
        return bench_config5(args)
    if args.workload == "paper_stream":
        return bench_stream(args)
    if args.workload == "gemm":
        return bench_gemm(args)

    import numpy as np
    import torch
    from paper_1608_00895_amd import binding as rl
    from paper_1608_00895_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    chunking = None
    if args.workload in ("paper_chunks", "paper_train"):
        # the batch is cut from the corpus by the library: segment table on the host, gather kernel on the device
        cx, clens = synth.paper_corpus()
        size, nb = synth.PAPER_SEGMENT_FRAMES, synth.PAPER_BATCH_SEGMENTS
        cseq, cstart, clen = rl.rlstm_chunk_plan(clens, size, size)
        cxd = torch.from_numpy(cx).to(dev)
        tab = [torch.from_numpy(a[:nb].copy()).to(dev) for a in (cseq, cstart, clen)]
        x = torch.empty((size, nb, cx.shape[2]), device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        rl.rlstm_chunk_gather(cxd, tab[0], tab[1], tab[2], size, x)
        e0.record()
        rl.rlstm_chunk_gather(cxd, tab[0], tab[1], tab[2], size, x)
        e1.record()
        torch.cuda.synchronize()
        wl = synth.paper_workload(x.cpu().numpy(), clen[:nb])
        sl = tab[2]
        chunking = {"corpus_sequences": int(len(clens)), "corpus_frames": int(clens.sum()), "segments": int(len(cseq)),
                    "segment_frames": size, "gather_ms": e0.elapsed_time(e1)}
    else:
        wl = {"config2": synth.config2, "config3": synth.config3, "config4": synth.config4}[args.workload]()
        x = torch.from_numpy(wl.x).to(dev)
        sl = torch.from_numpy(wl.seq_lens).to(dev)
    log(f"workload {wl.name}: L={wl.L} T={wl.T} B={wl.B} D={wl.D} H={wl.H} frames={wl.frames} slots={wl.T * wl.B}")
    tuning = dict(first_piece=args.first_piece or 0, batch_groups=args.batch_groups or 0, overlap_mode=args.overlap_mode or 0,
                  bwd_exchange=args.bwd_exchange or 0, gemm_variant=args.gemm_variant or 0)
    desc = rl.rblstm_desc(L=wl.L, T=wl.T, B=wl.B, D=wl.D, H=wl.H, operand_dtype=wl.operand_dtype, engine=args.engine, **tuning)
    train = None
    host_params = [a for layer in wl.params for p in layer for a in p]
    if args.workload == "paper_train":
        # a whole training step: the 1501-class softmax / cross-entropy layer on top (Sec. 6) and an Adam update of
        # every parameter; parameters, gradients and Adam's two moments live in one flat buffer each
        C = 1501
        Wo, bo, labels = synth.output_layer(wl.T, wl.B, 2 * wl.H, C, seed=67, wscale=0.05)
        host_params = host_params + [Wo, bo]
        train = {"C": C, "Wo": Wo, "bo": bo, "labels": labels}
    n_all = sum(a.size for a in host_params)
    flat_p = torch.empty(n_all, device=dev)
    flat_g = torch.zeros(n_all, device=dev)
    params, grads, o = [], [], 0
    for a in host_params:
        flat_p[o:o + a.size] = torch.from_numpy(a).reshape(-1).to(dev)
        params.append(flat_p[o:o + a.size].view(a.shape))
        grads.append(flat_g[o:o + a.size].view(a.shape))
        o += a.size
    if train:
        train.update(dWo=grads[-2], dbo=grads[-1], dev_Wo=params[-2], dev_bo=params[-1],
                     labels_dev=torch.from_numpy(labels).to(dev), m=torch.zeros(n_all, device=dev),
                     v=torch.zeros(n_all, device=dev), loss=torch.zeros(1, device=dev),
                     errors=torch.zeros(1, dtype=torch.int32, device=dev),
                     dy=torch.empty((wl.T, wl.B, 2 * wl.H), device=dev),
                     ws=torch.empty(rl.rlstm_ce_workspace_bytes(wl.T, wl.B, 2 * wl.H, C), dtype=torch.uint8, device=dev),
                     step=0)
        params, grads = params[:-2], grads[:-2]
    G = torch.from_numpy(wl.G).to(dev)
    y_top = torch.empty((wl.T, wl.B, 2 * wl.H), device=dev)
    reserve = torch.empty(rl.rblstm_reserve_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(rl.rblstm_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    sa = torch.cuda.current_stream()
    sb = None if args.one_stream else torch.cuda.Stream()

    def step(desc=desc):
        # the bottom layer's input gradient is not needed for training and is skipped (dx = null)
        if train is None:
            rl.blstm_stack_fwd_bwd(desc, x, params, sl, G, y_top, grads, None, reserve, ws, sa, sb)
            return
        F = 2 * wl.H
        rl.blstm_stack_fwd(desc, x, params, sl, y_top, reserve, ws, sa)
        rl.softmax_ce_fwd_bwd(wl.T, wl.B, F, train["C"], wl.operand_dtype, y_top, train["dev_Wo"], train["dev_bo"],
                              train["labels_dev"], sl, train["loss"], train["errors"], train["dy"], train["dWo"],
                              train["dbo"], train["ws"], sa)
        rl.blstm_stack_bwd(desc, x, params, sl, train["dy"], y_top, grads, None, reserve, ws, sa, sb)
        train["step"] += 1
        rl.rlstm_adam_step(flat_p, flat_g, train["m"], train["v"], 1e-5, 0.9, 0.999, 1e-8, train["step"], sa)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert rl.rlstm_last_timeout(ws) == 0
    rl.rlstm_profile_enable(False)
    rl.rlstm_profile_read()
    # Timed region: exactly K steps between device synchronisations, the library's timing hooks off.  Every step is
    # also bracketed by a pair of events on stream a (a call returns with stream a waiting for stream b), which
    # gives the per-step times behind the median and the minimum.
    step_events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    clocks_before = clock_state()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in step_events:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert rl.rlstm_last_timeout(ws) == 0
    step_ms = sorted(e0.elapsed_time(e1) for e0, e1 in step_events)
    # A loop of its own with the hooks on: every kernel group bracketed by events on its launch stream.
    hook_steps = max(1, min(args.steps, 5))
    rl.rlstm_profile_enable(True)
    torch.cuda.synchronize()
    th0 = time.perf_counter()
    for _ in range(hook_steps):
        step()
    torch.cuda.synchronize()
    th1 = time.perf_counter()
    rl.rlstm_profile_enable(False)
    prof = rl.rlstm_profile_read(1 << 16)
    assert rl.rlstm_last_timeout(ws) == 0
    ms_per_step_hooks = (th1 - th0) * 1e3 / hook_steps
    if args.calibration_copy:
        n = 1 << 28
        src = torch.ones(n, device=dev)
        dst = torch.empty(n, device=dev)
        rl.rlstm_copy_f32(dst, src, n)
        torch.cuda.synchronize()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    frames_per_s = wl.frames / (ms_per_step * 1e-3)

    # per-kernel-group summary from the HIP events recorded inside the timed region
    by_kind = {}
    for kind, layer, ndir, ms, nsteps, flop in prof:
        d = by_kind.setdefault(kind, {"ms": 0.0, "launches": 0, "flop": 0.0, "rsteps": 0})
        d["ms"] += ms
        d["launches"] += 1
        d["flop"] += flop
        d["rsteps"] += nsteps
    try:
        plan_now = rl.rblstm_plan(desc) if args.engine in (0, 1) else None
    except rl.RlstmError:
        plan_now = None
    rec_form = plan_now["recurrent_operand_form"] if plan_now else 0
    kernels = []
    for kind, d in sorted(by_kind.items()):
        e = {"kernel": rl.PROFILE_KINDS[kind], "launches_per_step": d["launches"] / hook_steps,
             "avg_ms": d["ms"] / d["launches"], "ms_per_step": d["ms"] / hook_steps,
             "tflops": d["flop"] / (d["ms"] * 1e-3) / 1e12}
        # fraction of the matrix cores' peak for the instructions the kernel runs on (MFMA utilisation by throughput)
        e["mfma_peak_tflops"], e["mfma_path"] = mfma_peak(e["kernel"], wl.operand_dtype, args.gemm_variant, rec_form)
        e["frac_of_mfma_peak"] = e["tflops"] / e["mfma_peak_tflops"]
        if kind in (1, 2):
            # a pass over the T steps may be cut into several launches
            e["steps_per_launch"] = d["rsteps"] / d["launches"]
            e["step_us"] = 1e3 * d["ms"] / d["rsteps"]
            e["hbm_gbs"] = rec_bytes(kind, wl, d["rsteps"]) / (d["ms"] * 1e-3) / 1e9
        kernels.append(e)
        log(e)
    dom = max(kernels, key=lambda e: e["ms_per_step"])
    # bytes per launch at the L2-to-fabric interface, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs recorded in
    # profiles/hbm_traffic.json (default settings only; scaled by the copy kernel)
    default_knobs = (args.first_piece is None and args.batch_groups is None and not args.one_stream and args.engine == 0
                     and args.overlap_mode is None and args.bwd_exchange is None and args.gemm_variant is None)
    if default_knobs:
        traffic, traffic_source = recorded_traffic(args.workload, dom["kernel"], rl.version(), plan_now)
    else:
        traffic, traffic_source = None, "not reported with non-default settings"
    peak = dom["mfma_peak_tflops"]
    roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": peak, "mfma_path": dom["mfma_path"],
                "unit": "TFLOP/s", "frac": dom["tflops"] / peak,
                "traffic": traffic, "traffic_source": traffic_source,
                "avg_launch_ms": dom["avg_ms"],
                "steps_per_launch": dom.get("steps_per_launch"),
                "note": "the recurrent kernels are bound by the serial chain of T dependent steps "
                        "(see step_us), not by MFMA or HBM throughput; priced here against the MFMA "
                        "peak of the operand type with 2*B*H*4H FLOP per step and direction; a pass over the T steps "
                        "is cut into several launches (steps_per_launch)"}

    # The same recurrent kernels with nothing beside them: two calls with the products in serial order on one
    # stream (outside the timed region), for the step time the kernels reach alone.
    if args.engine in (0, 1) and train is None and not args.one_stream and args.overlap_mode is None:
        serial = rl.rblstm_desc(L=wl.L, T=wl.T, B=wl.B, D=wl.D, H=wl.H, operand_dtype=wl.operand_dtype, engine=args.engine,
                                **dict(tuning, overlap_mode=1))
        if True:
            step(serial)
            torch.cuda.synchronize()
            rl.rlstm_profile_read()
            rl.rlstm_profile_enable(True)
            step(serial)
            torch.cuda.synchronize()
            rl.rlstm_profile_enable(False)
            alone = {}
            for kind, layer, ndir, ms, nsteps, flop in rl.rlstm_profile_read(1 << 16):
                if kind in (1, 2):
                    a = alone.setdefault(kind, [0.0, 0])
                    a[0] += ms; a[1] += nsteps
            for e in kernels:
                for kind, nm in ((1, "recurrent_forward"), (2, "recurrent_backward")):
                    if e["kernel"] == nm and kind in alone and alone[kind][1]:
                        e["step_us_alone"] = 1e3 * alone[kind][0] / alone[kind][1]
            if "step_us_alone" in dom:
                roofline["step_us_alone"] = dom["step_us_alone"]

    # Floor of the step chain: the bare exchange of one hop (store, acknowledge, flag, poll, load; no
    # arithmetic) timed live at the same group shape.  Forward: one hop per step (h_t); backward: two
    # (d a_t, then the partial tiles, which the kernel sends as tagged words; timed here with flags).
    if args.engine in (0, 1):
        try:
            plan = rl.rblstm_plan(desc)
            es = 2 if wl.operand_dtype == 1 else (6 if plan["recurrent_operand_form"] == 2 else 4)
            ng, bp, u = plan["groups"], max(16, plan["rows"]), plan["units_per_workgroup"]
            def floor(members, tile, read):
                wsf = torch.empty(rl.rlstm_exchange_floor_bytes(ng, members, tile), dtype=torch.uint8, device=dev)
                return rl.rlstm_exchange_floor(ng, members, tile, read, 2000, wsf)
            f_fwd = floor(plan["members_fwd"], bp * u * es, plan["members_fwd"] * bp * u * es)
            if plan["bwd_exchanges_per_step"] == 1:
                # one exchange: every workgroup writes a [16 x padded H] tile and reads its piece of every producer's
                f_bwd = floor(plan["members_bwd"], 16 * plan["Hq"] * 4, plan["members_bwd"] * 16 * u * 4)
            else:
                f_dz = floor(plan["members_bwd"], bp * u * 4 * es, plan["members_bwd"] * bp * u * es)
                f_bwd = f_dz + floor(plan["members_bwd"], bp * 4 * u * 8, 4 * bp * u * 8)
            for e in kernels:
                if e["kernel"] == "recurrent_forward":
                    e["exchange_floor_us"] = f_fwd
                if e["kernel"] == "recurrent_backward":
                    e["exchange_floor_us"] = f_bwd
            roofline["plan"] = plan
            if dom["kernel"] in ("recurrent_forward", "recurrent_backward"):
                roofline["step_us"] = dom["step_us"]
                roofline["exchange_floor_us"] = dom["exchange_floor_us"]
        except rl.RlstmError as ex:
            log("exchange floor not measured:", ex)

    out = {
        "metric": "BLSTM train frames/sec (fwd+bwd)", "value": frames_per_s, "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": step_ms[len(step_ms) // 2], "ms_per_step_min": step_ms[0],
        "ms_per_step_with_timing_hooks": ms_per_step_hooks,
        "timing": "value and ms_per_step: K steps between device synchronisations, the library's event hooks off; median / min: "
                  "per-step event pairs on stream a in that same loop; the per-kernel figures come from a separate loop of "
                  f"{hook_steps} steps with the hooks on (ms_per_step_with_timing_hooks)",
        "clock_state": clocks_before,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.operand_dtype == 0 else "bf16 operands, f32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.L, "units_per_direction": wl.H, "batch": wl.B,
                   "T_padded": wl.T, "valid_frames": wl.frames, "padded_slots": wl.T * wl.B,
                   "padded_slots_per_s": wl.T * wl.B / (ms_per_step * 1e-3),
                   "engine": "persistent" if args.engine in (0, 1) else "stepwise",
                   "streams": 1 if args.one_stream else 2,
                   "products": products_note(wl.operand_dtype, args.gemm_variant)},
        "roofline": roofline,
        "kernels": kernels,
    }
    if chunking:
        out["config"]["chunking"] = chunking
    if train:
        out["metric"] = "BLSTM train frames/sec (whole training step: fwd, softmax/CE, bwd, Adam)"
        out["config"].update(classes=train["C"], update="adam", parameters=int(n_all),
                             loss_per_frame=float(train["loss"].item()) / wl.frames,
                             frame_error_rate=int(train["errors"].item()) / wl.frames)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, output_layer=(train["Wo"], train["bo"], train["labels"]) if train else None)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
