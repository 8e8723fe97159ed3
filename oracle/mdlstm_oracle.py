"""CPU oracle for the two-dimensional (multidimensional) LSTM layer: forward
scan over the pixels of a batch of images, backward pass, one scan direction
and the four-directional layer.

THIS IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the HIP
library is checked against; nothing in the product path may import it.  It
shares no code with the HIP path and never falls back to it.

Everything is numpy float64.  Pixels are visited ONE AT A TIME (vectorised
only over the images of the batch, which do not interact); each visit
evaluates the cell definition below once, with ``@`` as the only
non-elementwise step.  ``order`` selects the visiting order — row by row,
column by column, or anti-diagonal by anti-diagonal — and must not change
any result: that is the observation the paper builds its GPU kernel on.

What the paper fixes (RETURNN, arXiv 1608.00895, Sec. 4.2)
----------------------------------------------------------
* The hidden state h(u, v) of position (u, v) is computed from the
  predecessor activations h(u-1, v) and h(u, v-1), so it can only be computed
  once both are known; all positions on a common anti-diagonal can be
  computed at the same time.
* A multi-directional layer runs four such scans (one per corner of the
  image) and processes several images at once.
* The cell itself is named by citation only (the multidimensional LSTM of
  Graves et al.); the paper prints no equations.  The "stable cell" it
  mentions as an option is not part of this oracle.

Reading used where the paper is silent (listed in the design notes): the
multidimensional LSTM cell with one forget gate per dimension, i.e. five
gate blocks of width H in the column order i | f_u | f_v | o | g of the
5H-wide pre-activation

    a(u,v)  = b + x(u,v) W + h(u',v) R_u + h(u,v') R_v
    c~      = f_u * c(u',v) + f_v * c(u,v') + i * g ,    h~ = o * tanh(c~)

with (u', v') the predecessor row / column in scan order, logistic sigmoid
on i, f_u, f_v, o and tanh on g; a predecessor outside the image contributes
zero state; images share the height and have their own widths, and a pixel
at or beyond its image's width is outside the image: h = c = y = 0 there, so
that every image is processed as if it were alone; the four directions are
(du, dv) in (+1,+1), (+1,-1), (-1,+1), (-1,-1) and the layer's output is
their concatenation [.., 4H] in that order; gradients are plain sums.

Pins: tests/test_mdlstm_oracle_pins.py (finite differences, autograd of an
independent torch formulation, reduction to the one-dimensional LSTM oracle
for images of height 1 or width 1, closed forms on the image border,
visiting-order, flip and batch-independence invariants).
"""
from __future__ import annotations

from typing import Dict, Iterator, List, Sequence, Tuple

import numpy as np

F64 = np.float64
DIRECTIONS: Tuple[Tuple[int, int], ...] = ((1, 1), (1, -1), (-1, 1), (-1, -1))


def _sigmoid(u: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-u))


def visiting_order(Hh: int, Ww: int, du: int, dv: int, order: str = "rows") -> List[Tuple[int, int]]:
    """Pixels in an order in which every pixel comes after both its predecessors (u-du, v) and (u, v-dv)."""
    us = list(range(Hh)) if du == 1 else list(range(Hh - 1, -1, -1))
    vs = list(range(Ww)) if dv == 1 else list(range(Ww - 1, -1, -1))
    if order == "rows":
        return [(u, v) for u in us for v in vs]
    if order == "columns":
        return [(u, v) for v in vs for u in us]
    if order == "diagonals":
        out = []
        for s in range(Hh + Ww - 1):
            for iu in range(Hh):
                iv = s - iu
                if 0 <= iv < Ww:
                    out.append((us[iu], vs[iv]))
        return out
    raise ValueError("order must be rows, columns or diagonals")


def mdlstm_forward(x, W, Ru, Rv, b, widths, du: int, dv: int, order: str = "rows", dtype=F64) -> Dict[str, np.ndarray]:
    """One scan direction.  x [Hh,Ww,B,D]; W [D,5H]; Ru, Rv [H,5H]; b [5H]; widths [B].
    Returns y, c [Hh,Ww,B,H], the activated gates [Hh,Ww,B,5H] and what the backward pass needs.
    dtype: float64 is the oracle; float32 evaluates the same definition in single precision, which
    tests use only to see how far rounding alone moves a result (to set tolerances)."""
    F64 = dtype
    x = np.asarray(x, F64)
    W, Ru, Rv, b = (np.asarray(a, F64) for a in (W, Ru, Rv, b))
    widths = np.asarray(widths).astype(np.int64)
    Hh, Ww, B, D = x.shape
    H = Ru.shape[0]
    assert W.shape == (D, 5 * H) and Ru.shape == (H, 5 * H) and Rv.shape == (H, 5 * H) and b.shape == (5 * H,)
    assert du in (1, -1) and dv in (1, -1) and widths.shape == (B,)
    h = np.zeros((Hh, Ww, B, H), F64)
    c = np.zeros((Hh, Ww, B, H), F64)
    gates = np.zeros((Hh, Ww, B, 5 * H), F64)
    zero = np.zeros((B, H), F64)
    for (u, v) in visiting_order(Hh, Ww, du, dv, order):
        pu, pv = u - du, v - dv
        h_up, c_up = (h[pu, v], c[pu, v]) if 0 <= pu < Hh else (zero, zero)
        h_left, c_left = (h[u, pv], c[u, pv]) if 0 <= pv < Ww else (zero, zero)
        a = b + x[u, v] @ W + h_up @ Ru + h_left @ Rv
        gi, gfu, gfv, go = (_sigmoid(a[:, k * H:(k + 1) * H]) for k in range(4))
        gg = np.tanh(a[:, 4 * H:])
        ct = gfu * c_up + gfv * c_left + gi * gg
        ht = go * np.tanh(ct)
        m = (v < widths).astype(F64)[:, None]
        h[u, v] = m * ht
        c[u, v] = m * ct
        gates[u, v] = np.concatenate([gi, gfu, gfv, go, gg], axis=1)
    return dict(y=h, c=c, gates=gates, x=x, W=W, Ru=Ru, Rv=Rv, widths=widths, du=du, dv=dv, dtype=dtype)


def mdlstm_backward(fwd: Dict[str, np.ndarray], dy, order: str = "rows") -> Dict[str, np.ndarray]:
    """Gradients of sum(y * dy) for one scan direction: dx, dW, dRu, dRv, db and dz (the gradient
    with respect to the pre-activation, zero outside the images)."""
    x, W, Ru, Rv, widths = fwd["x"], fwd["W"], fwd["Ru"], fwd["Rv"], fwd["widths"]
    du, dv = fwd["du"], fwd["dv"]
    h, c, gates = fwd["y"], fwd["c"], fwd["gates"]
    F64 = fwd["dtype"]
    dy = np.asarray(dy, F64)
    Hh, Ww, B, D = x.shape
    H = Ru.shape[0]
    Dh = np.zeros((Hh, Ww, B, H), F64)     # gradient arriving at h(u,v) from its successors
    Dc = np.zeros((Hh, Ww, B, H), F64)     # gradient arriving at c(u,v) from its successors
    dz_all = np.zeros((Hh, Ww, B, 5 * H), F64)
    dx = np.zeros_like(x)
    dW = np.zeros_like(W)
    dRu = np.zeros_like(Ru)
    dRv = np.zeros_like(Rv)
    db = np.zeros((5 * H,), F64)
    zero = np.zeros((B, H), F64)
    for (u, v) in reversed(visiting_order(Hh, Ww, du, dv, order)):
        pu, pv = u - du, v - dv
        has_up, has_left = 0 <= pu < Hh, 0 <= pv < Ww
        h_up, c_up = (h[pu, v], c[pu, v]) if has_up else (zero, zero)
        h_left, c_left = (h[u, pv], c[u, pv]) if has_left else (zero, zero)
        g = gates[u, v]
        gi, gfu, gfv, go, gg = (g[:, k * H:(k + 1) * H] for k in range(5))
        m = (v < widths).astype(F64)[:, None]
        # inside the image c[u,v] is the cell value c~; outside nothing depends on the pre-activation
        tc = np.tanh(c[u, v])
        dh = m * (dy[u, v] + Dh[u, v])
        d_o = dh * tc
        dct = m * Dc[u, v] + dh * go * (1.0 - tc * tc)
        dz = np.concatenate([dct * gg * gi * (1.0 - gi),
                             dct * c_up * gfu * (1.0 - gfu),
                             dct * c_left * gfv * (1.0 - gfv),
                             d_o * go * (1.0 - go),
                             dct * gi * (1.0 - gg * gg)], axis=1)
        dz_all[u, v] = dz
        if has_up:
            Dh[pu, v] += dz @ Ru.T
            Dc[pu, v] += dct * gfu
        if has_left:
            Dh[u, pv] += dz @ Rv.T
            Dc[u, pv] += dct * gfv
        dW += x[u, v].T @ dz
        dRu += h_up.T @ dz
        dRv += h_left.T @ dz
        db += dz.sum(axis=0)
        dx[u, v] = dz @ W.T
    return dict(dx=dx, dW=dW, dRu=dRu, dRv=dRv, db=db, dz=dz_all)


Params = Sequence[Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]]   # per direction (W, Ru, Rv, b)


def mdlstm4_forward(x, params: Params, widths, order: str = "rows", dtype=F64):
    """The four-directional layer: y [Hh,Ww,B,4H] = concatenation of the four scans, in the order of DIRECTIONS."""
    assert len(params) == 4
    fwds = [mdlstm_forward(x, *params[d], widths, *DIRECTIONS[d], order=order, dtype=dtype) for d in range(4)]
    return np.concatenate([f["y"] for f in fwds], axis=3), fwds


def mdlstm4_backward(fwds, dy, order: str = "rows"):
    """Gradients of sum(y * dy): per direction dict(dW, dRu, dRv, db), and dx summed over the directions."""
    H = fwds[0]["Ru"].shape[0]
    dy = np.asarray(dy, fwds[0]["dtype"])
    grads, dx = [], None
    for d in range(4):
        g = mdlstm_backward(fwds[d], dy[..., d * H:(d + 1) * H], order=order)
        dx = g["dx"] if dx is None else dx + g["dx"]
        grads.append(dict(dW=g["dW"], dRu=g["dRu"], dRv=g["dRv"], db=g["db"]))
    return grads, dx
