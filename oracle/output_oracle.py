"""CPU oracle for the frame-wise softmax / cross-entropy output layer and the parameter updates that
turn the stack's forward + backward pass into a training step.

THIS IS TEST INFRASTRUCTURE (see lstm_oracle.py); numpy float64, no code shared with the HIP path.

What the paper fixes (RETURNN, arXiv 1608.00895): Sec. 3.2 — output layers with the cross-entropy loss
exist; Sec. 6 — the experiments classify every frame into one of 1501 classes and report the share of
misclassified frames; Sec. 4.3 — updates by stochastic gradient descent with a classical momentum term or
with Adam (cited), gradients of a batch are sums (not scaled by the batch size); Sec. 5 — frames
outside their sequence must have no influence.
Readings where the paper is silent: the output layer is an affine map of the top layer's output followed
by a softmax over the classes; the loss is the sum over the valid frames of -log p(label); a frame counts
as misclassified when the largest logit is not the label's (first index wins a tie); a frame whose label is
not a class index (negative, or >= C) is left out like a frame outside its sequence; Adam as published by
Kingma & Ba (bias-corrected first and second moments); momentum as v <- mu v + g, theta <- theta - lr v.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def softmax_ce_forward(y, Wo, bo, labels, seq_lens):
    """y [T,B,F], Wo [F,C], bo [C], labels [T,B] int, seq_lens [B].
    Returns dict(loss = sum over valid frames of -log softmax(y Wo + bo)[label], errors = number of
    valid frames whose arg max is not the label, p [T,B,C] class posteriors (zero rows outside the
    sequences), and the inputs)."""
    y, Wo, bo = np.asarray(y, F64), np.asarray(Wo, F64), np.asarray(bo, F64)
    labels = np.asarray(labels).astype(np.int64)
    seq_lens = np.asarray(seq_lens).astype(np.int64)
    T, B, _ = y.shape
    C = Wo.shape[1]
    p = np.zeros((T, B, C), F64)
    loss, errors = 0.0, 0
    for t in range(T):
        z = y[t] @ Wo + bo                                  # [B, C]
        z = z - z.max(axis=1, keepdims=True)
        logp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
        for b in range(B):
            if t < seq_lens[b] and 0 <= labels[t, b] < C:
                p[t, b] = np.exp(logp[b])
                loss -= logp[b, labels[t, b]]
                errors += int(np.argmax(z[b]) != labels[t, b])
    return dict(loss=loss, errors=errors, p=p, y=y, Wo=Wo, labels=labels, seq_lens=seq_lens)


def softmax_ce_backward(fwd):
    """Gradients of the loss: dy [T,B,F], dWo [F,C], dbo [C]; d loss / d logits = p - onehot(label) on valid frames."""
    p, y, Wo, labels, seq_lens = fwd["p"], fwd["y"], fwd["Wo"], fwd["labels"], fwd["seq_lens"]
    T, B, C = p.shape
    dz = p.copy()
    for t in range(T):
        for b in range(B):
            if t < seq_lens[b] and 0 <= labels[t, b] < C:
                dz[t, b, labels[t, b]] -= 1.0
    dWo = np.zeros_like(Wo)
    dbo = np.zeros(C, F64)
    dy = np.zeros_like(y)
    for t in range(T):
        dWo += y[t].T @ dz[t]
        dbo += dz[t].sum(axis=0)
        dy[t] = dz[t] @ Wo.T
    return dict(dy=dy, dWo=dWo, dbo=dbo)


def sgd_momentum_step(param, grad, velocity, lr: float, momentum: float):
    """v <- momentum * v + grad ; param <- param - lr * v.  Returns (param, velocity)."""
    v = momentum * np.asarray(velocity, F64) + np.asarray(grad, F64)
    return np.asarray(param, F64) - lr * v, v


def adam_step(param, grad, m, v, lr: float, beta1: float, beta2: float, eps: float, step: int):
    """One Adam update with bias correction; step counts from 1.  Returns (param, m, v)."""
    g = np.asarray(grad, F64)
    m = beta1 * np.asarray(m, F64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, F64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return np.asarray(param, F64) - lr * mhat / (np.sqrt(vhat) + eps), m, v
