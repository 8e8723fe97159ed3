#!/usr/bin/env python3
"""Writes tests/golden/paper_train_oracle_samples.npz: the CPU oracle's training step at full size on the batch
shape the paper's experiments time (81 segments of 250 frames, 3-layer BLSTM with 512 units per direction, softmax /
cross-entropy over 1501 classes): loss, frame errors, the smallest gap between the two largest logits of a valid
frame, and sampled entries of every gradient (output layer and stack) and of the Adam-updated parameters.

Only the oracle and the seeded input generators are used; nothing here touches the HIP path.  Takes a few minutes.

    python tests/golden/make_paper_train_golden.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import adam_step, blstm_stack_backward, blstm_stack_forward, chunk_batch, softmax_ce_backward, softmax_ce_forward  # noqa: E402
from paper_1608_00895_amd import synth  # noqa: E402

CLASSES, LABEL_SEED, WSCALE = 1501, 67, 0.05
ADAM = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)


def main():
    cx, clens = synth.paper_corpus()
    xc, (_, _, clen) = chunk_batch(cx, clens, synth.PAPER_SEGMENT_FRAMES, synth.PAPER_SEGMENT_FRAMES)
    nb = synth.PAPER_BATCH_SEGMENTS
    wl = synth.paper_workload(xc[:, :nb], clen[:nb])      # the first 81 segments of the corpus, cut by the oracle
    Wo, bo, labels = synth.output_layer(wl.T, wl.B, 2 * wl.H, CLASSES, seed=LABEL_SEED, wscale=WSCALE)
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    t0 = time.time()
    y, caches = blstm_stack_forward(wl.x.astype(np.float64), params, wl.seq_lens)
    print(f"stack forward done in {time.time() - t0:.0f} s", flush=True)
    f = softmax_ce_forward(y, Wo, bo, labels, wl.seq_lens)
    g = softmax_ce_backward(f)
    print(f"output layer done in {time.time() - t0:.0f} s: loss {f['loss']:.6f}, errors {f['errors']}", flush=True)
    grads, _ = blstm_stack_backward(caches, g["dy"])
    print(f"stack backward done in {time.time() - t0:.0f} s", flush=True)
    # how close the decision "arg max == label" comes to a tie on any valid frame (float32 parity of the error count)
    z = y @ Wo.astype(np.float64) + bo.astype(np.float64)
    top2 = np.sort(z, axis=2)[:, :, -2:]
    valid = np.arange(wl.T)[:, None] < wl.seq_lens[None, :]
    gap = (top2[:, :, 1] - top2[:, :, 0])[valid]
    rng = np.random.Generator(np.random.Philox(67160800895))
    out = dict(loss=np.float64(f["loss"]), errors=np.int64(f["errors"]), min_top2_gap=np.float64(gap.min()),
               frames_with_gap_below_1e_5=np.int64((gap < 1e-5).sum()), max_abs_logit=np.float64(np.abs(z[valid]).max()),
               seq_lens=wl.seq_lens)

    def put(name, arr, n):
        flat = np.asarray(arr).reshape(-1)
        idx = np.sort(rng.choice(flat.size, size=min(n, flat.size), replace=False)).astype(np.int64)
        out[name + "_idx"] = idx
        out[name + "_val"] = flat[idx].astype(np.float64)
        out[name + "_max"] = np.float64(np.abs(flat).max())
        return idx

    put("dy", g["dy"], 4096)
    flat_p = [a for layer in params for p in layer for a in p] + [Wo.astype(np.float64), bo.astype(np.float64)]
    flat_g = [grads[l][d][k] for l in range(wl.L) for d in range(2) for k in ("dW", "dR", "db")] + [g["dWo"], g["dbo"]]
    for i, (p, gr) in enumerate(zip(flat_p, flat_g)):
        idx = put(f"grad_{i}", gr, 512)
        newp, _, vhat_src = adam_step(p, gr, np.zeros_like(p), np.zeros_like(p), ADAM["lr"], ADAM["beta1"], ADAM["beta2"],
                                      ADAM["eps"], 1)
        out[f"param_{i}_val"] = newp.reshape(-1)[idx]                 # updated parameters at the same sample
        out[f"param_{i}_old"] = p.reshape(-1)[idx]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_train_oracle_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
