#!/usr/bin/env python3
"""Writes tests/golden/config4_oracle_samples.npz from the CPU oracle only.

Config 4 (6-layer BLSTM, H=1000 per direction, B=64, T=1500) is too large for the oracle to run
whole (its per-frame caches alone would need ~80 GB), so two things are stored:
  (a) the same network on short sequences (synth.config4_short): sampled entries of every output;
  (b) the full-length workload for two single sequences, each run alone through the whole stack
      (sequences in a minibatch do not influence each other): sampled entries of y_top[:, n, :]
      and dx[:, n, :].  Weight gradients are sums over the minibatch and cannot be sampled this way.

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
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    out["full_seq_lens"] = wl.seq_lens
    picks = [0, int(np.argmin(wl.seq_lens))]
    out["full_picks"] = np.array(picks, np.int64)
    for n in picks:
        ln = int(wl.seq_lens[n])
        y, caches = blstm_stack_forward(wl.x[:ln, n:n + 1].astype(np.float64), params, np.array([ln]))
        _, dx = blstm_stack_backward(caches, wl.G[:ln, n:n + 1].astype(np.float64))
        del caches
        put(f"full_y_seq{n}", y, 4096)          # indices into the [len, 1, 2H] array of that sequence
        put(f"full_dx_seq{n}", dx, 2048)
        print(f"full-length sequence {n} (len {ln}) done at {time.time() - t0:.0f} s", flush=True)

    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config4_oracle_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
