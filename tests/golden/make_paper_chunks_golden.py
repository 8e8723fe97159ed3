#!/usr/bin/env python3
"""Writes tests/golden/paper_chunks_oracle_samples.npz: sampled outputs of the CPU oracle on the
paper-shaped workload (81 segments of 250 frames, 45 values per frame, 3-layer BLSTM, H=512 per direction).

Only the oracle and the seeded input generator are used; nothing here touches the HIP path.
For every output tensor (y_top, dx, and dW, dR, db of every layer and direction) it stores the
flat indices of a seeded random sample, the oracle's float64 values there, and the tensor's
largest absolute value (the tolerances are relative to it); and, as float32, whole [B, 2H] / [B, D] slabs of
y_top and dx at the first and the last frame, every segment's last valid and first padded frame, the last four
rows and the last two units' columns of every dW and dR, and every db whole.  The minibatch is cut from the
corpus by the oracle (oracle.chunk_batch).  Takes a minute or two.

    python tests/golden/make_paper_chunks_golden.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import blstm_stack_backward, blstm_stack_forward, chunk_batch  # noqa: E402
from paper_1608_00895_amd import synth  # noqa: E402


def main():
    cx, clens = synth.paper_corpus()
    xc, (_, _, clen) = chunk_batch(cx, clens, synth.PAPER_SEGMENT_FRAMES, synth.PAPER_SEGMENT_FRAMES)
    nb = synth.PAPER_BATCH_SEGMENTS
    wl = synth.paper_workload(xc[:, :nb], clen[:nb])      # the first 81 segments of the corpus, cut by the oracle
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    t0 = time.time()
    y, caches = blstm_stack_forward(wl.x.astype(np.float64), params, wl.seq_lens)
    print(f"oracle forward done in {time.time() - t0:.0f} s", flush=True)
    grads, dx = blstm_stack_backward(caches, wl.G.astype(np.float64))
    print(f"oracle backward done in {time.time() - t0:.0f} s", flush=True)
    rng = np.random.Generator(np.random.Philox(60160800895))
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
    frames = np.array([0, T - 1], np.int64)
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
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_chunks_oracle_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
