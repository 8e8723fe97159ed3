#!/usr/bin/env python3
"""Writes tests/golden/config3_oracle_samples.npz: sampled outputs of the CPU oracle on the
full-size benchmark workload (config 3: 4-layer BLSTM, H=500 per direction, B=32, T=1000).

Only the oracle and the seeded input generator are used; nothing here touches the HIP path.
For every output tensor (y_top, dx, and dW, dR, db of every layer and direction) it stores the
flat indices of a seeded random sample, the oracle's float64 values there, and the tensor's
largest absolute value (the tolerances are relative to it).  Uniform samples rarely land where a
kernel that cuts the time axis into pieces, pads H and deals the sequences out to groups can go
wrong, so it also stores (as float32, which is exact to 6e-8 of a value against bars of 1e-5 / 1e-4):
whole [B, 2H] slabs of y_top and [B, D] slabs of dx at the frames on either side of every place the
passes can be cut (steps 128, 256, 512 from either end) and at both ends; for every sequence its last
valid and its first padded frame; of every dW and dR the last four rows and the columns of the last
two units of every gate (next to the padding of H = 500 to a multiple of 16); every db whole.
Takes a few minutes and ~12 GB.

    python tests/golden/make_config3_golden.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import blstm_stack_backward, blstm_stack_forward  # noqa: E402
from paper_1608_00895_amd import synth  # noqa: E402


def main():
    wl = synth.config3()
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    t0 = time.time()
    y, caches = blstm_stack_forward(wl.x.astype(np.float64), params, wl.seq_lens)
    print(f"oracle forward done in {time.time() - t0:.0f} s", flush=True)
    grads, dx = blstm_stack_backward(caches, wl.G.astype(np.float64))
    print(f"oracle backward done in {time.time() - t0:.0f} s", flush=True)
    rng = np.random.Generator(np.random.Philox(20160800895))
    out = {}

    def put(name, arr, n):
        flat = arr.reshape(-1)
        idx = np.sort(rng.choice(flat.size, size=min(n, flat.size), replace=False)).astype(np.int64)
        out[name + "_idx"] = idx
        out[name + "_val"] = flat[idx].astype(np.float64)
        out[name + "_max"] = np.float64(np.abs(flat).max())

    put("y", y, 4096)
    put("dx", dx, 2048)
    for l in range(wl.L):
        for d in range(2):
            for nm in ("dW", "dR", "db"):
                put(f"{nm}_{l}_{d}", grads[l][d][nm], 512)
    out["seq_lens"] = wl.seq_lens
    T, B, H = wl.T, wl.B, wl.H
    cuts = [128, 256, 512]
    frames = sorted({0, T - 1} | {c - 1 for c in cuts} | set(cuts) | {T - c for c in cuts} | {T - c - 1 for c in cuts})
    frames = np.array([t for t in frames if 0 <= t < T], np.int64)
    out["frames"] = frames
    out["y_slab"] = y[frames].astype(np.float32)
    out["dx_slab"] = dx[frames].astype(np.float32)
    y_end = np.zeros((B, 2, 2 * H), np.float32)      # [n, 0] = frame len-1, [n, 1] = frame len (zeros if len == T)
    dx_end = np.zeros((B, 2, wl.D), np.float32)
    for n in range(B):
        ln = int(wl.seq_lens[n])
        y_end[n, 0], dx_end[n, 0] = y[ln - 1, n], dx[ln - 1, n]
        if ln < T:
            y_end[n, 1], dx_end[n, 1] = y[ln, n], dx[ln, n]
    out["y_end"], out["dx_end"] = y_end, dx_end
    cols = np.concatenate([g * H + np.arange(H - 2, H) for g in range(4)]).astype(np.int64)
    out["cols"] = cols
    for l in range(wl.L):
        for d in range(2):
            for nm in ("dW", "dR"):
                out[f"{nm}_{l}_{d}_lastrows"] = grads[l][d][nm][-4:, :].astype(np.float32)
                out[f"{nm}_{l}_{d}_lastcols"] = grads[l][d][nm][:, cols].astype(np.float32)
            out[f"db_{l}_{d}_whole"] = grads[l][d]["db"].astype(np.float64)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config3_oracle_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
