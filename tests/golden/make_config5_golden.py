#!/usr/bin/env python3
"""Writes tests/golden/config5_oracle_samples.npz from the CPU oracle only.

Config 5 (two-dimensional LSTM, four scan directions, 8 images of 64 x up to 800 pixels, H = 32 per
direction): sampled entries (flat indices, float64 values, tensor max-abs) of every output of the oracle on
the full-size workload, so that the GPU test can check the full-size run without re-running the oracle
(minutes of CPU time).

    python tests/golden/make_config5_golden.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import mdlstm4_backward, mdlstm4_forward  # noqa: E402
from paper_1608_00895_amd import synth  # noqa: E402


def main():
    t0 = time.time()
    wl = synth.config5()
    params = [tuple(a.astype(np.float64) for a in p) for p in wl.params]
    y, fwds = mdlstm4_forward(wl.x.astype(np.float64), params, wl.widths)
    print(f"forward done at {time.time() - t0:.0f} s", flush=True)
    grads, dx = mdlstm4_backward(fwds, wl.G.astype(np.float64))
    print(f"backward done at {time.time() - t0:.0f} s", flush=True)
    out = {"widths": wl.widths}
    rng = np.random.Generator(np.random.Philox(5160800895))

    def put(name, arr, n):
        flat = arr.reshape(-1)
        idx = np.sort(rng.choice(flat.size, size=min(n, flat.size), replace=False)).astype(np.int64)
        out[name + "_idx"] = idx
        out[name + "_val"] = flat[idx].astype(np.float64)
        out[name + "_max"] = np.float64(np.abs(flat).max())

    put("y", y, 8192)
    put("dx", dx, 4096)
    for d in range(4):
        for k in ("dW", "dRu", "dRv", "db"):
            put(f"{k}_{d}", grads[d][k], 4096)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config5_oracle_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
