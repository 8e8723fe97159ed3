#!/usr/bin/env python3
"""Writes tests/golden/paper_stream_oracle_samples.npz: sampled outputs of the CPU oracle of the streaming mode on
its full-size workload (64 sequences of the paper's length statistics, segments of 250 frames, three unidirectional
layers of 512 units; synth.paper_stream).

Only the oracle and the seeded input generator are used; nothing here touches the HIP path.  For every output
(y_top, dx, the final state and dW, dR, db of every layer) it stores the flat indices of a seeded random sample,
the oracle's float64 values there, and the tensor's largest absolute value.  Takes a few minutes.

    python tests/golden/make_paper_stream_golden.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import lstm_stream_forward_backward  # noqa: E402
from paper_1608_00895_amd import synth  # noqa: E402


def main():
    wl = synth.paper_stream()
    params = [tuple(a.astype(np.float64) for a in p) for p in wl.params]
    t0 = time.time()
    y, grads, dx, state = lstm_stream_forward_backward(wl.x.astype(np.float64), params, wl.seq_lens, wl.G.astype(np.float64), wl.Tc)
    print(f"oracle done in {time.time() - t0:.0f} s", flush=True)
    rng = np.random.Generator(np.random.Philox(80160800895))
    out = {}

    def put(name, arr, n):
        flat = arr.reshape(-1)
        idx = np.sort(rng.choice(flat.size, size=min(n, flat.size), replace=False)).astype(np.int64)
        out[name + "_idx"] = idx
        out[name + "_val"] = flat[idx].astype(np.float64)
        out[name + "_max"] = np.float64(np.abs(flat).max())

    put("y", y, 4096)
    put("dx", dx, 2048)
    put("state", np.stack([np.stack(s) for s in state]), 2048)
    for l in range(wl.L):
        for nm in ("dW", "dR", "db"):
            put(f"{nm}_{l}", grads[l][nm], 512)
    out["seq_lens"] = wl.seq_lens
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_stream_oracle_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
