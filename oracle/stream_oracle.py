"""CPU oracle for the streaming mode: a unidirectional LSTM stack that reads its sequences segment by
segment, each segment starting from the final state of the one before (state hand-off), with
back-propagation through time truncated at the segment boundaries.

THIS IS TEST INFRASTRUCTURE (see lstm_oracle.py); numpy float64, no code shared with the HIP path.

What the paper fixes (RETURNN, arXiv 1608.00895): Sec. 3.2 — recurrent layers can be connected by passing
the final state of one on to another; Sec. 4 — cutting sequences into segments of constant length gives
up the context that the end states of the segments hold.  This mode keeps that context: it is the
composition "final state of segment s = initial state of segment s + 1" of the layer of Sec. 4.2, so the
oracle is that composition written out with the layer oracle (lstm_forward / lstm_backward), nothing else.
Readings where the paper is silent: the stack is unidirectional (direction +1; a backward-in-time layer
would need the segments that have not been read yet); segment s holds frames [s Tc, (s + 1) Tc) of every
sequence, so sequence n has clamp(len_n - s Tc, 0, Tc) valid frames in it, and a sequence that has ended
carries its state unchanged (the masking rule of the layer); the backward pass of a segment treats the
segment's initial state as a constant (no gradient flows into the previous segment), and the gradients of
the segments are summed.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from .lstm_oracle import lstm_backward, lstm_forward

F64 = np.float64
LayerParams = Sequence[Tuple[np.ndarray, np.ndarray, np.ndarray]]     # per layer (W, R, b)


def segment_lengths(seq_lens, s: int, Tc: int) -> np.ndarray:
    """Valid frames of every sequence inside segment s."""
    return np.clip(np.asarray(seq_lens).astype(np.int64) - s * Tc, 0, Tc)


def lstm_stream_forward_backward(x, params: LayerParams, seq_lens, G, Tc: int, state0=None):
    """x [S*Tc,B,D]; params: per layer (W [D_l,4H], R [H,4H], b [4H]), D_0 = D, D_l = H; G [S*Tc,B,H]: gradient of
    the loss w.r.t. the top layer's output; state0: per layer (h [B,H], c [B,H]) or None (zeros).
    Returns y_top [S*Tc,B,H], grads (per layer dict dW, dR, db: sums over the segments), dx [S*Tc,B,D] and
    the final state per layer."""
    x = np.asarray(x, F64)
    G = np.asarray(G, F64)
    Ttot, B, _ = x.shape
    assert Ttot % Tc == 0
    S = Ttot // Tc
    L = len(params)
    H = params[0][1].shape[0]
    state = [(np.zeros((B, H), F64), np.zeros((B, H), F64)) for _ in range(L)] if state0 is None else \
            [(np.asarray(h, F64), np.asarray(c, F64)) for h, c in state0]
    y_top = np.zeros((Ttot, B, H), F64)
    dx = np.zeros_like(x)
    grads = [dict(dW=np.zeros_like(np.asarray(W, F64)), dR=np.zeros_like(np.asarray(R, F64)),
                  db=np.zeros_like(np.asarray(b, F64))) for W, R, b in params]
    for s in range(S):
        lens = segment_lengths(seq_lens, s, Tc)
        inp = x[s * Tc:(s + 1) * Tc]
        fwds = []
        for l, (W, R, b) in enumerate(params):
            f = lstm_forward(inp, W, R, b, lens, 1, state[l][0], state[l][1])
            fwds.append(f)
            state[l] = (f["hT"], f["cT"])
            inp = f["y"]
        y_top[s * Tc:(s + 1) * Tc] = inp
        d = G[s * Tc:(s + 1) * Tc]
        for l in range(L - 1, -1, -1):
            g = lstm_backward(fwds[l], d)                  # no gradient arrives at the segment's final state
            for k in ("dW", "dR", "db"):
                grads[l][k] += g[k]
            d = g["dx"]                                    # dh0 / dc0 are dropped: the truncation
        dx[s * Tc:(s + 1) * Tc] = d
    return y_top, grads, dx, state
