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


def log(*a):
    print(*a, file=sys.stderr, flush=True)


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

    Ts = 512 if wl_full.H >= 400 else 500
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
    rl.rlstm_profile_read()
    rl.rlstm_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    rl.rlstm_profile_enable(False)
    prof = rl.rlstm_profile_read(1 << 16)
    if args.calibration_copy:
        n = 1 << 28
        src = torch.ones(n, device=dev)
        dst = torch.empty(n, device=dev)
        rl.rlstm_copy_f32(dst, src, n)
        torch.cuda.synchronize()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
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
        e = {"kernel": names[kind], "launches_per_step": d["launches"] / args.steps, "avg_ms": d["ms"] / d["launches"],
             "ms_per_step": d["ms"] / args.steps, "tflops": flop / (d["ms"] * 1e-3) / 1e12}
        if kind in (1, 2):
            e["diagonals_per_launch"] = d["rsteps"] / d["launches"]
            e["diagonal_us"] = 1e3 * d["ms"] / d["rsteps"]
        kernels.append(e)
        log(e)
    dom = max(kernels, key=lambda e: e["ms_per_step"])
    # HBM bytes per launch from the rocprofv3 FETCH_SIZE + WRITE_SIZE runs at this workload, scaled by a copy kernel
    measured_traffic = {"mdlstm_forward_scan": 0.046e9 + 1.669e9, "mdlstm_backward_scan": 1.134e9 + 1.135e9}
    roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["tflops"] / PEAK_FP32_MFMA_TFLOPS, "traffic": measured_traffic.get(dom["kernel"]),
                "avg_launch_ms": dom["avg_ms"],
                "note": "one workgroup per (scan direction, image, band of 16 rows): 128 of the 256 CUs work, and the chain of "
                        "anti-diagonals is serial (a step's MFMAs alone take a CU 0.53 us of the measured step); priced against "
                        "the whole chip's fp32 MFMA peak with 2 * 2H * 5H FLOP per valid pixel and direction"}
    out = {"metric": "MDLSTM train pixels/sec (fwd+bwd), 4 scan directions", "value": wl.pixels / (ms_per_step * 1e-3),
           "unit": "pixels/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": wl.name, "height": wl.Hh, "padded_width": wl.Ww, "images": wl.B,
                      "units_per_direction": wl.H, "valid_pixels": wl.pixels,
                      "padded_pixel_slots": wl.Hh * wl.Ww * wl.B},
           "roofline": roofline, "kernels": kernels}
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        from oracle import mdlstm4_backward, mdlstm4_forward
        wc = 24                                    # the oracle on the first 24 columns of every image
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
    launch of every shape; reports TFLOP/s per shape (fp32 MFMA roofline) for the kernel variant the library picks
    and for the plain kernel."""
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
        for variant, tag in ((0, "picked"), (2, "plain")):
            rl.rlstm_set_gemm_variant(variant)
            for _ in range(args.warmup):
                rl.rlstm_gemm_f32(ta, tb, M, N, K, A, lda, B, ldb, C, N, None, sk)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                rl.rlstm_gemm_f32(ta, tb, M, N, K, A, lda, B, ldb, C, N, None, sk)
            e1.record()
            torch.cuda.synchronize()
            res[tag] = e0.elapsed_time(e1) / args.steps
        rl.rlstm_set_gemm_variant(0)
        flop = 2.0 * M * N * K
        kernels.append({"kernel": name, "M": M, "N": N, "K": K, "avg_ms": res["picked"], "tflops": flop / res["picked"] / 1e9,
                        "plain_kernel_ms": res["plain"], "plain_kernel_tflops": flop / res["plain"] / 1e9})
        log(kernels[-1])
        total_flop += flop; total_ms += res["picked"]
    dom = kernels[0]
    out = {"metric": "fp32 matrix products alone, TFLOP/s over all shapes", "value": total_flop / total_ms / 1e9, "unit": "TFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": total_ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "matrix products at the shapes of config 3 and of the paper's batch"},
           "roofline": {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS,
                        "unit": "TFLOP/s", "frac": dom["tflops"] / PEAK_FP32_MFMA_TFLOPS, "traffic": None},
           "kernels": kernels}
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
    desc = rl.rlstm_stream_desc(L=wl.L, S=wl.S, Tc=wl.Tc, B=wl.B, D=wl.D, H=wl.H, operand_dtype=0, engine=args.engine)
    x = torch.from_numpy(wl.x).to(dev)
    sl = torch.from_numpy(wl.seq_lens).to(dev)
    params = [torch.from_numpy(a).to(dev) for p in wl.params for a in p]
    grads = [torch.empty_like(p) for p in params]
    G = torch.from_numpy(wl.G).to(dev)
    y = torch.empty((wl.S * wl.Tc, wl.B, wl.H), device=dev)
    state = torch.zeros((wl.L, 2, wl.B, wl.H), device=dev)
    reserve = torch.empty(rl.rlstm_stream_reserve_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(rl.rlstm_stream_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    if args.batch_groups is not None:
        rl.rlstm_set_batch_groups(args.batch_groups)

    def step():
        state.zero_()
        rl.lstm_stream_fwd_bwd(desc, x, params, sl, G, y, grads, None, state, reserve, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert rl.rlstm_last_timeout(ws) == 0
    rl.rlstm_profile_read()
    rl.rlstm_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    rl.rlstm_profile_enable(False)
    prof = rl.rlstm_profile_read(1 << 16)
    assert rl.rlstm_last_timeout(ws) == 0
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    by_kind = {}
    for kind, layer, ndir, ms, nsteps, flop in prof:
        d = by_kind.setdefault(kind, {"ms": 0.0, "launches": 0, "flop": 0.0, "rsteps": 0})
        d["ms"] += ms; d["launches"] += 1; d["flop"] += flop; d["rsteps"] += nsteps
    kernels = []
    for kind, d in sorted(by_kind.items()):
        e = {"kernel": rl.PROFILE_KINDS[kind], "launches_per_step": d["launches"] / args.steps,
             "avg_ms": d["ms"] / d["launches"], "ms_per_step": d["ms"] / args.steps,
             "tflops": d["flop"] / (d["ms"] * 1e-3) / 1e12}
        if kind in (1, 2):
            e["steps_per_launch"] = d["rsteps"] / d["launches"]
            e["step_us"] = 1e3 * d["ms"] / d["rsteps"]
        kernels.append(e)
        log(e)
    dom = max(kernels, key=lambda e: e["ms_per_step"])
    # bytes per launch from the rocprofv3 FETCH_SIZE + WRITE_SIZE runs (profiles/lstm_stream_paper_stream_hbm_counters.md)
    measured_traffic = {"recurrent_forward": 0.397e9 + 0.393e9, "recurrent_backward": 1.088e9 + 0.655e9}
    roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["tflops"] / PEAK_FP32_MFMA_TFLOPS, "traffic": measured_traffic.get(dom["kernel"]),
                "avg_launch_ms": dom["avg_ms"], "steps_per_launch": dom.get("steps_per_launch"), "step_us": dom.get("step_us"),
                "note": "the recurrent kernels are bound by the serial chain of dependent steps (see step_us); priced "
                        "against the fp32 MFMA peak with 2*B*H*4H FLOP per step"}
    slots = wl.S * wl.Tc * wl.B
    out = {"metric": "LSTM streaming train frames/sec (segments chained by final states, truncated BPTT)",
           "value": wl.frames / (ms_per_step * 1e-3), "unit": "frames/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": wl.name, "layers": wl.L, "units": wl.H, "sequences": wl.B, "segments": wl.S,
                      "segment_frames": wl.Tc, "valid_frames": wl.frames, "padded_slots": slots,
                      "engine": "persistent" if args.engine in (0, 1) else "stepwise"},
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
        Tc, S2 = 100, 2                            # the oracle on the first 2 segments of 100 frames
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
                    help="steps of the first piece the recurrent passes are cut into (library default if omitted; 0 = uncut)")
    ap.add_argument("--batch-groups", type=int, default=None,
                    help="groups the sequences are dealt out to per direction (library default if omitted)")
    ap.add_argument("--overlap-mode", type=int, default=None,
                    help="-1 per shape (library default), 0 serial, 1 products share CUs with the recurrent kernels")
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
    wl = {"config2": synth.config2, "config3": synth.config3, "config4": synth.config4,
          "paper_chunks": synth.paper_chunks, "paper_train": synth.paper_chunks}[args.workload]()
    log(f"workload {wl.name}: L={wl.L} T={wl.T} B={wl.B} D={wl.D} H={wl.H} frames={wl.frames} slots={wl.T * wl.B}")

    desc = rl.rblstm_desc(L=wl.L, T=wl.T, B=wl.B, D=wl.D, H=wl.H, operand_dtype=wl.operand_dtype, engine=args.engine)
    x = torch.from_numpy(wl.x).to(dev)
    sl = torch.from_numpy(wl.seq_lens).to(dev)
    chunking = None
    if args.workload in ("paper_chunks", "paper_train"):
        # the batch is cut from the corpus on the device: segment table on the host, gather kernel
        cx, clens = synth.paper_corpus()
        cseq, cstart, clen = rl.rlstm_chunk_plan(clens, wl.T, wl.T)
        cxd = torch.from_numpy(cx).to(dev)
        tab = [torch.from_numpy(a[:wl.B].copy()).to(dev) for a in (cseq, cstart, clen)]
        x = torch.empty((wl.T, wl.B, wl.D), device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        rl.rlstm_chunk_gather(cxd, tab[0], tab[1], tab[2], wl.T, x)
        e0.record()
        rl.rlstm_chunk_gather(cxd, tab[0], tab[1], tab[2], wl.T, x)
        e1.record()
        torch.cuda.synchronize()
        assert np.array_equal(x.cpu().numpy(), wl.x) and np.array_equal(clen[:wl.B], wl.seq_lens)
        sl = tab[2]
        chunking = {"corpus_sequences": int(len(clens)), "corpus_frames": int(clens.sum()), "segments": int(len(cseq)),
                    "segment_frames": wl.T, "gather_ms": e0.elapsed_time(e1)}
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
    if args.overlap_mode is not None:
        rl.rlstm_set_overlap_mode(args.overlap_mode)
    if args.first_piece is not None:
        rl.rlstm_set_first_piece(args.first_piece)
    if args.batch_groups is not None:
        rl.rlstm_set_batch_groups(args.batch_groups)

    def step():
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
    rl.rlstm_profile_read()
    rl.rlstm_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    rl.rlstm_profile_enable(False)
    prof = rl.rlstm_profile_read(1 << 16)
    assert rl.rlstm_last_timeout(ws) == 0
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
    kernels = []
    for kind, d in sorted(by_kind.items()):
        e = {"kernel": rl.PROFILE_KINDS[kind], "launches_per_step": d["launches"] / args.steps,
             "avg_ms": d["ms"] / d["launches"], "ms_per_step": d["ms"] / args.steps,
             "tflops": d["flop"] / (d["ms"] * 1e-3) / 1e12}
        if kind in (1, 2):
            # a pass over the T steps may be cut into several launches
            e["steps_per_launch"] = d["rsteps"] / d["launches"]
            e["step_us"] = 1e3 * d["ms"] / d["rsteps"]
            e["hbm_gbs"] = rec_bytes(kind, wl, d["rsteps"]) / (d["ms"] * 1e-3) / 1e9
        kernels.append(e)
        log(e)
    dom = max(kernels, key=lambda e: e["ms_per_step"])
    # bytes per launch at the L2-to-fabric interface, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
    # summarised in profiles/blstm_stack_config3_hbm_counters.md (config 3 with the library's default cut of
    # the passes and groups of sequences only; scaled by the copy kernel)
    measured_traffic = {"recurrent_forward": 0.391e9 + 0.481e9, "recurrent_backward": 1.074e9 + 0.713e9,
                        "input_projection": 0.135e9 + 0.070e9, "input_gradient": 0.112e9 + 0.017e9,
                        "weight_gradient": 0.572e9 + 0.062e9, "recurrent_weight_gradient": 0.572e9 + 0.062e9}
    # the same for the paper's batch shape (profiles/train_step_paper_shape_hbm_counters.md)
    paper_shape_traffic = {"recurrent_forward": 0.948e9 + 0.913e9, "recurrent_backward": 2.764e9 + 2.257e9}
    default_knobs = args.first_piece is None and args.batch_groups is None and not args.one_stream and args.engine == 0
    peak = PEAK_FP32_MFMA_TFLOPS if wl.operand_dtype == 0 else PEAK_BF16_MFMA_TFLOPS
    roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": peak,
                "unit": "TFLOP/s", "frac": dom["tflops"] / peak,
                "traffic": (measured_traffic if args.workload == "config3" else paper_shape_traffic).get(dom["kernel"])
                if args.workload in ("config3", "paper_chunks", "paper_train") and default_knobs else None,
                "avg_launch_ms": dom["avg_ms"],
                "steps_per_launch": dom.get("steps_per_launch"),
                "note": "the recurrent kernels are bound by the serial chain of T dependent steps "
                        "(see step_us), not by MFMA or HBM throughput; priced here against the fp32 MFMA "
                        "peak with 2*B*H*4H FLOP per step and direction; a pass over the T steps is cut "
                        "into several launches (steps_per_launch)"}

    # The same recurrent kernels with nothing beside them: two calls with the products in serial order on one
    # stream (outside the timed region), for the step time the kernels reach alone.
    if args.engine in (0, 1) and train is None and not args.one_stream and args.overlap_mode is None:
        rl.rlstm_set_overlap_mode(0)
        try:
            step()
            torch.cuda.synchronize()
            rl.rlstm_profile_read()
            rl.rlstm_profile_enable(True)
            step()
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
        finally:
            rl.rlstm_set_overlap_mode(-1)

    # Floor of the step chain: the bare exchange of one hop (store, acknowledge, flag, poll, load; no
    # arithmetic) timed live at the same group shape.  Forward: one hop per step (h_t); backward: two
    # (d a_t, then the partial tiles, which the kernel sends as tagged words; timed here with flags).
    if args.engine in (0, 1):
        try:
            plan = rl.rblstm_plan(desc)
            es = 2 if wl.operand_dtype == 1 else 4
            ng, bp, u = plan["groups"], max(16, plan["rows"]), plan["units_per_workgroup"]
            def floor(members, tile, read):
                wsf = torch.empty(rl.rlstm_exchange_floor_bytes(ng, members, tile), dtype=torch.uint8, device=dev)
                return rl.rlstm_exchange_floor(ng, members, tile, read, 2000, wsf)
            f_fwd = floor(plan["members_fwd"], bp * u * es, plan["members_fwd"] * bp * u * es)
            f_dz = floor(plan["members_bwd"], bp * u * 4 * es, plan["members_bwd"] * bp * u * es)
            f_part = floor(plan["members_bwd"], bp * 4 * u * 8, 4 * bp * u * 8)
            for e in kernels:
                if e["kernel"] == "recurrent_forward":
                    e["exchange_floor_us"] = f_fwd
                if e["kernel"] == "recurrent_backward":
                    e["exchange_floor_us"] = f_dz + f_part
            roofline["plan"] = plan
            if dom["kernel"] in ("recurrent_forward", "recurrent_backward"):
                roofline["step_us"] = dom["step_us"]
                roofline["exchange_floor_us"] = dom["exchange_floor_us"]
        except rl.RlstmError as ex:
            log("exchange floor not measured:", ex)

    out = {
        "metric": "BLSTM train frames/sec (fwd+bwd)", "value": frames_per_s, "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.operand_dtype == 0 else "bf16 operands, f32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.L, "units_per_direction": wl.H, "batch": wl.B,
                   "T_padded": wl.T, "valid_frames": wl.frames, "padded_slots": wl.T * wl.B,
                   "padded_slots_per_s": wl.T * wl.B / (ms_per_step * 1e-3),
                   "engine": "persistent" if args.engine in (0, 1) else "stepwise",
                   "streams": 1 if args.one_stream else 2},
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
    if not args.no_cpu_baseline and args.workload != "config4":
        out["cpu_baseline"] = cpu_baseline(wl, output_layer=(train["Wo"], train["bo"], train["labels"]) if train else None)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
