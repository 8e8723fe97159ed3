"""CPU oracle for chunking: cutting the sequences of a corpus into segments of constant length.

THIS IS TEST INFRASTRUCTURE (see lstm_oracle.py); plain Python loops, no code shared with the HIP path.

What the paper fixes (RETURNN, arXiv 1608.00895): Sec. 4 — sequences can be cut into possibly overlapping
segments of constant length so that batches carry little zero padding; Sec. 6 — the experiments use segments
of 250 frames, with zero frames appended where a sequence ends inside a segment, 81 segments per batch.
Reading where the paper is silent: a sequence of n frames yields the segments starting at frames
0, step, 2*step, ... as long as the start lies inside the sequence; a segment holds ``size`` frames or, at
the end of the sequence, the frames that are left (the rest of its slot in the batch is zero padding);
segments are listed sequence by sequence, starts ascending.
"""
from __future__ import annotations

import numpy as np


def chunk_table(seq_lens, size: int, step: int):
    """(seq, start, length) of every segment, as three int32 arrays."""
    assert size > 0 and step > 0
    seq, start, length = [], [], []
    for b, n in enumerate(seq_lens):
        t = 0
        while t < int(n):
            seq.append(b)
            start.append(t)
            length.append(min(size, int(n) - t))
            t += step
    return np.array(seq, np.int32), np.array(start, np.int32), np.array(length, np.int32)


def chunk_batch(x: np.ndarray, seq_lens, size: int, step: int):
    """x [T, B, D] -> (xc [size, K, D] with zeros past each segment's length, the segment table)."""
    seq, start, length = chunk_table(seq_lens, size, step)
    xc = np.zeros((size, len(seq), x.shape[2]), x.dtype)
    for k in range(len(seq)):
        for t in range(int(length[k])):
            xc[t, k, :] = x[start[k] + t, seq[k], :]
    return xc, (seq, start, length)
