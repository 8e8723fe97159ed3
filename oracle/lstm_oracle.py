"""CPU oracle for the LSTM layer's forward recurrence and back-propagation
through time, one direction, both directions, and the stacked deep BLSTM.

THIS IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the HIP
library is checked against; nothing in the product path may import it.  It
shares no code with the HIP path and never falls back to it.

Everything is numpy float64.  There is no blocking, fusion or reordering:
each time step evaluates the definition below once, with ``@`` (a library
matrix product) as the only non-elementwise step.

What the paper fixes (RETURNN, arXiv 1608.00895)
------------------------------------------------
* Sec. 1 names the cell by citation only (the LSTM of Hochreiter &
  Schmidhuber); the paper prints no cell equations.
* Sec. 4.2: the pre-activation has a non-recurrent part (input times a weight
  matrix, computable for all frames of the minibatch at once) and a recurrent
  part (previous output times a recurrent matrix), followed by the gating
  step; the backward pass first runs back through time, then forms the
  gradients with respect to weights and inputs.
* Sec. 5: tensors are [time, batch, feature]; an index tensor says for each
  (time, batch) whether the frame belongs to the sequence, so that zero
  padding has no influence.
* Fig. 1: a layer has a ``direction`` (+1 / -1); a bidirectional layer is two
  such layers on the same input whose outputs are both fed (forward first) to
  the next layer.
* Sec. 4.3: gradients of a batch are plain sums (not scaled by batch size).

Reading used where the paper is silent (all listed in the design notes):
four gate blocks of width H in the column order i | f | o | g of the 4H-wide
pre-activation; no peepholes; logistic sigmoid on i, f, o; tanh on g and on
the cell for the output; a frame outside its sequence leaves the carried
(h, c) unchanged and emits y = 0; direction -1 scans the padded array from
t = T-1 down to 0 with the same mask.

Parity pins for every function here live in tests/test_oracle_*.py:
finite differences, closed forms for constant gates, torch.nn.LSTM (an
independent library implementation, packed variable-length, bidirectional,
stacked) for outputs and gradients, and the padding / direction invariants.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


def sigmoid(u: np.ndarray) -> np.ndarray:
    """Logistic function 1 / (1 + exp(-u))."""
    return 1.0 / (1.0 + np.exp(-u))


def _time_order(T: int, direction: int) -> range:
    """Order in which frames are processed (Fig. 1: direction +1 or -1)."""
    if direction == 1:
        return range(0, T)
    if direction == -1:
        return range(T - 1, -1, -1)
    raise ValueError("direction must be +1 or -1")


def lstm_forward(x, W, R, b, seq_lens, direction: int = 1, h0=None, c0=None) -> Dict[str, np.ndarray]:
    """One LSTM layer, one direction (Sec. 4.2 forward; Sec. 5 mask; Fig. 1 direction).

    x [T,B,D], W [D,4H], R [H,4H], b [4H], seq_lens [B] (frame t of sequence
    n is valid iff t < seq_lens[n]), h0/c0 [B,H] or None (= 0).

    Returns y [T,B,H] (0 at invalid frames), c [T,B,H] (carried cell state
    after frame t), hT/cT [B,H] (state after the last processed frame), and
    the per-frame quantities the backward pass needs.
    """
    x = np.asarray(x, F64)
    W = np.asarray(W, F64)
    R = np.asarray(R, F64)
    b = np.asarray(b, F64)
    T, B, D = x.shape
    H = R.shape[0]
    assert W.shape == (D, 4 * H) and R.shape == (H, 4 * H) and b.shape == (4 * H,)
    seq_lens = np.asarray(seq_lens).astype(np.int64)
    assert seq_lens.shape == (B,)
    h = np.zeros((B, H), F64) if h0 is None else np.array(h0, F64)
    c = np.zeros((B, H), F64) if c0 is None else np.array(c0, F64)

    y = np.zeros((T, B, H), F64)
    c_out = np.zeros((T, B, H), F64)
    gi = np.zeros((T, B, H), F64)
    gf = np.zeros((T, B, H), F64)
    go = np.zeros((T, B, H), F64)
    gg = np.zeros((T, B, H), F64)
    ct = np.zeros((T, B, H), F64)       # candidate cell c~ of frame t
    h_prev_all = np.zeros((T, B, H), F64)
    c_prev_all = np.zeros((T, B, H), F64)

    for t in _time_order(T, direction):
        h_prev_all[t] = h
        c_prev_all[t] = c
        a = b + x[t] @ W + h @ R                  # non-recurrent + recurrent part
        i = sigmoid(a[:, 0 * H:1 * H])
        f = sigmoid(a[:, 1 * H:2 * H])
        o = sigmoid(a[:, 2 * H:3 * H])
        g = np.tanh(a[:, 3 * H:4 * H])
        c_new = f * c + i * g
        h_new = o * np.tanh(c_new)
        m = (t < seq_lens)[:, None]               # index tensor of frame t
        c = np.where(m, c_new, c)
        h = np.where(m, h_new, h)
        y[t] = np.where(m, h_new, 0.0)
        c_out[t] = c
        gi[t], gf[t], go[t], gg[t], ct[t] = i, f, o, g, c_new

    return dict(y=y, c=c_out, hT=h, cT=c, i=gi, f=gf, o=go, g=gg, c_tilde=ct,
                h_prev=h_prev_all, c_prev=c_prev_all, x=x, W=W, R=R,
                seq_lens=seq_lens, direction=direction)


def lstm_backward(fwd: Dict[str, np.ndarray], dy, dhT=None, dcT=None) -> Dict[str, np.ndarray]:
    """Back-propagation through time for ``lstm_forward`` (Sec. 4.2 backward).

    dy [T,B,H] is the loss gradient w.r.t. y; dhT/dcT [B,H] (or None = 0)
    w.r.t. the final state.  Returns dx [T,B,D], dW, dR, db, dh0, dc0, and
    dz [T,B,4H] (gradient w.r.t. the pre-activation, exactly 0 at invalid
    frames).  Gradients are sums over frames and sequences (Sec. 4.3).
    """
    x, W, R = fwd["x"], fwd["W"], fwd["R"]
    seq_lens, direction = fwd["seq_lens"], fwd["direction"]
    T, B, D = x.shape
    H = R.shape[0]
    dy = np.asarray(dy, F64)
    assert dy.shape == (T, B, H)
    Dh = np.zeros((B, H), F64) if dhT is None else np.array(dhT, F64)
    Dc = np.zeros((B, H), F64) if dcT is None else np.array(dcT, F64)

    dz = np.zeros((T, B, 4 * H), F64)
    dW = np.zeros_like(W)
    dR = np.zeros_like(R)
    db = np.zeros((4 * H,), F64)
    dx = np.zeros_like(x)

    for t in reversed(_time_order(T, direction)):
        i, f, o, g = fwd["i"][t], fwd["f"][t], fwd["o"][t], fwd["g"][t]
        tc = np.tanh(fwd["c_tilde"][t])
        m = (t < seq_lens)[:, None].astype(F64)
        dh_new = m * (dy[t] + Dh)                       # y and the carried h both take h~ when valid
        d_o = dh_new * tc
        dc_new = m * Dc + dh_new * o * (1.0 - tc * tc)
        d_i = dc_new * g
        d_g = dc_new * i
        d_f = dc_new * fwd["c_prev"][t]
        da = np.concatenate([d_i * i * (1.0 - i),
                             d_f * f * (1.0 - f),
                             d_o * o * (1.0 - o),
                             d_g * (1.0 - g * g)], axis=1)
        dz[t] = da
        Dc = dc_new * f + (1.0 - m) * Dc
        Dh = da @ R.T + (1.0 - m) * Dh
        dW += x[t].T @ da
        dR += fwd["h_prev"][t].T @ da
        db += da.sum(axis=0)
        dx[t] = da @ W.T

    return dict(dx=dx, dW=dW, dR=dR, db=db, dh0=Dh, dc0=Dc, dz=dz)


Params = Sequence[Sequence[Tuple[np.ndarray, np.ndarray, np.ndarray]]]


def blstm_stack_forward(x, params: Params, seq_lens) -> Tuple[np.ndarray, List[List[dict]]]:
    """Deep (bi)directional LSTM (Fig. 1): params[l] holds one (W, R, b) per
    direction, forward first; layer l's output is the feature-axis
    concatenation [y_fw | y_bw] and is layer l+1's input.  Initial states 0."""
    inp = np.asarray(x, F64)
    caches: List[List[dict]] = []
    for layer in params:
        outs = []
        for d, (W, R, b) in enumerate(layer):
            outs.append(lstm_forward(inp, W, R, b, seq_lens, direction=(1 if d == 0 else -1)))
        caches.append(outs)
        inp = np.concatenate([o["y"] for o in outs], axis=2)
    return inp, caches


def blstm_stack_backward(caches: List[List[dict]], dy_top) -> Tuple[List[List[dict]], np.ndarray]:
    """Backward through the stack: dy splits on the feature axis between the
    directions, and the directions' input gradients add."""
    dy = np.asarray(dy_top, F64)
    grads: List[Optional[List[dict]]] = [None] * len(caches)
    for l in range(len(caches) - 1, -1, -1):
        outs = caches[l]
        H = outs[0]["R"].shape[0]
        gl = []
        dx = None
        for d, fwd in enumerate(outs):
            g = lstm_backward(fwd, dy[:, :, d * H:(d + 1) * H])
            gl.append(g)
            dx = g["dx"] if dx is None else dx + g["dx"]
        grads[l] = gl
        dy = dx
    return grads, dy


def blstm_stack_loss(x, params: Params, seq_lens, G) -> float:
    """The measurement loss: sum over all elements of y_top * G."""
    y, _ = blstm_stack_forward(x, params, seq_lens)
    return float(np.sum(y * np.asarray(G, F64)))
