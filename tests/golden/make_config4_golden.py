#!/usr/bin/env python3
"""Writes tests/golden/config4_oracle_samples.npz from the CPU oracle only.

Config 4 (6-layer BLSTM, H=1000 per direction, B=64, T=1500) is too large for the oracle to hold
whole (its per-frame caches alone would need ~80 GB), so two things are stored:
  (a) the same network on short sequences (synth.config4_short): sampled entries of every output;
  (b) the full-length workload, run through the oracle in groups of 8 sequences.  Sequences of a
      minibatch do not influence each other and the weight gradients are plain sums over the
      sequences (Sec. 4.3; both are pins of the oracle: padding invariance, additivity over
      sequences), so y_top and dx of a group are those of the minibatch and the groups' dW, dR, db
      add up to the minibatch's.  A group is run on its own padded length max(len) <= T (frames
      past every sequence of the group are padding and hold zeros).  Stored: for every sequence
      random samples of y_top and dx, whole [B, 2H] / [B, D] slabs at the first and last frame, each
      sequence's last valid and first padded frame; for every layer and direction random samples of
      dW, dR, the whole db, and the rows / columns of dW, dR that belong to the last units (next to
      the padding the kernels add to H = 1000).

Takes about an hour and ~16 GB.

    python tests/golden/make_config4_golden.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import blstm_stack_backward, blstm_stack_forward  # noqa: E402
from paper_1608_00895_amd import synth  # noqa: E402

GROUP = 8


def last_unit_columns(H, n=2):
    """Columns of a [*, 4H] matrix that belong to the last n units of every gate block."""
    return np.concatenate([g * H + np.arange(H - n, H) for g in range(4)]).astype(np.int64)


def main():
    out = {}
    rng = np.random.Generator(np.random.Philox(4160800895))

    def put(name, arr, n):
        flat = arr.reshape(-1)
        idx = np.sort(rng.choice(flat.size, size=min(n, flat.size), replace=False)).astype(np.int64)
        out[name + "_idx"] = idx
        out[name + "_val"] = flat[idx].astype(np.float64)
        out[name + "_max"] = np.float64(np.abs(flat).max())

    t0 = time.time()
    wl = synth.config4_short()
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    y, caches = blstm_stack_forward(wl.x.astype(np.float64), params, wl.seq_lens)
    grads, dx = blstm_stack_backward(caches, wl.G.astype(np.float64))
    del caches
    put("short_y", y, 4096)
    put("short_dx", dx, 2048)
    for l in range(wl.L):
        for d in range(2):
            for nm in ("dW", "dR", "db"):
                put(f"short_{nm}_{l}_{d}", grads[l][d][nm], 512)
    out["short_seq_lens"] = wl.seq_lens
    print(f"short workload done in {time.time() - t0:.0f} s", flush=True)

    wl = synth.config4()
    T, B, D, H, L = wl.T, wl.B, wl.D, wl.H, wl.L
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    out["full_seq_lens"] = wl.seq_lens
    frames = np.array([0, T - 1], np.int64)
    out["full_frames"] = frames
    y_slab = np.zeros((len(frames), B, 2 * H))
    dx_slab = np.zeros((len(frames), B, D))
    y_end = np.zeros((B, 2, 2 * H))          # [n, 0] = frame len-1, [n, 1] = frame len (zeros if len == T)
    dx_end = np.zeros((B, 2, D))
    y_idx, y_val, dx_idx, dx_val = [], [], [], []
    y_max = dx_max = 0.0
    gsum = None
    for n0 in range(0, B, GROUP):
        ns = np.arange(n0, min(n0 + GROUP, B))
        lens = wl.seq_lens[ns]
        Tg = int(lens.max())
        y, caches = blstm_stack_forward(wl.x[:Tg, ns].astype(np.float64), params, lens)
        grads, dx = blstm_stack_backward(caches, wl.G[:Tg, ns].astype(np.float64))
        del caches
        if gsum is None:
            gsum = [[{nm: grads[l][d][nm].copy() for nm in ("dW", "dR", "db")} for d in range(2)] for l in range(L)]
        else:
            for l in range(L):
                for d in range(2):
                    for nm in ("dW", "dR", "db"):
                        gsum[l][d][nm] += grads[l][d][nm]
        del grads
        y_max = max(y_max, float(np.abs(y).max()))
        dx_max = max(dx_max, float(np.abs(dx).max()))
        for k, t in enumerate(frames):
            if t < Tg:
                y_slab[k, ns] = y[t]
                dx_slab[k, ns] = dx[t]
        for j, n in enumerate(ns):
            ln = int(lens[j])
            y_end[n, 0] = y[ln - 1, j]
            dx_end[n, 0] = dx[ln - 1, j]
            if ln < Tg:
                y_end[n, 1] = y[ln, j]
                dx_end[n, 1] = dx[ln, j]
        # random samples inside the group, stored with their flat index in the minibatch's [T, B, .] tensors
        for arr, width, nsamp, idxs, vals in ((y, 2 * H, 2048, y_idx, y_val), (dx, D, 512, dx_idx, dx_val)):
            loc = np.sort(rng.choice(arr.size, size=nsamp, replace=False))
            t_, j_, c_ = np.unravel_index(loc, arr.shape)
            idxs.append((t_ * B + ns[j_]) * width + c_)
            vals.append(arr.reshape(-1)[loc])
        print(f"sequences {ns[0]}..{ns[-1]} (padded length {Tg}) done at {time.time() - t0:.0f} s", flush=True)
        del y, dx

    out["full_y_idx"] = np.concatenate(y_idx).astype(np.int64)
    out["full_y_val"] = np.concatenate(y_val)
    out["full_y_max"] = np.float64(y_max)
    out["full_dx_idx"] = np.concatenate(dx_idx).astype(np.int64)
    out["full_dx_val"] = np.concatenate(dx_val)
    out["full_dx_max"] = np.float64(dx_max)
    out["full_y_slab"] = y_slab.astype(np.float32)
    out["full_dx_slab"] = dx_slab.astype(np.float32)
    out["full_y_end"] = y_end.astype(np.float32)
    out["full_dx_end"] = dx_end.astype(np.float32)
    cols = last_unit_columns(H)
    out["full_cols"] = cols
    for l in range(L):
        for d in range(2):
            g = gsum[l][d]
            for nm in ("dW", "dR"):
                put(f"full_{nm}_{l}_{d}", g[nm], 1024)
                out[f"full_{nm}_{l}_{d}_lastrows"] = g[nm][-4:, :].astype(np.float32)
                out[f"full_{nm}_{l}_{d}_lastcols"] = g[nm][:, cols].astype(np.float32)
            out[f"full_db_{l}_{d}"] = g["db"].astype(np.float64)

    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config4_oracle_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
