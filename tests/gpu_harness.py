"""Helpers for the GPU parity tests: move numpy inputs to the device, call the
C ABI through the binding, bring results back as numpy.  No LSTM arithmetic."""
from __future__ import annotations

import numpy as np
import torch

from paper_1608_00895_amd import binding as rl

DEV = "cuda:0"


def dev(a, dtype=torch.float32):
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(DEV)


def rel_err(got, ref) -> float:
    """max |got - ref| / max |ref| over the tensor (floored), the norm the tolerances are stated in."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def run_lstm_layer(x, W, R, b, seq_lens, direction, h0=None, c0=None, dy=None, dhT=None, dcT=None,
                   engine=rl.RLSTM_ENGINE_AUTO, ldx=0, ldy=0, want_dx=True, fill=float("nan"), operand_dtype=0, **tuning):
    """lstm_fwd then lstm_bwd on the GPU.  x/y/dy may use padded row strides ldx/ldy
    (padding is filled with `fill` to show that it is neither read into results nor written)."""
    T, B, D = x.shape
    H = R.shape[0]
    desc = rl.rlstm_desc(T=T, B=B, D=D, H=H, direction=direction, operand_dtype=operand_dtype, ldx=ldx, ldy=ldy,
                         engine=engine, **tuning)        # tuning: batch_groups, bwd_exchange, gemm_variant
    lx = ldx or D
    ly = ldy or H
    xd = torch.full((T, B, lx), fill, device=DEV)
    xd[:, :, :D] = dev(x)
    Wd, Rd, bd = dev(W), dev(R), dev(b)
    h0d, c0d = dev(h0), dev(c0)
    sl = dev(seq_lens, torch.int32)
    y = torch.full((T, B, ly), fill, device=DEV)
    c = torch.full((T, B, H), fill, device=DEV)
    hT = torch.full((B, H), fill, device=DEV)
    cT = torch.full((B, H), fill, device=DEV)
    reserve = torch.empty(rl.rlstm_reserve_bytes(desc), dtype=torch.uint8, device=DEV)
    ws = torch.empty(rl.rlstm_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    rl.lstm_fwd(desc, xd, Wd, Rd, bd, h0d, c0d, sl, y, c, hT, cT, reserve, ws)
    assert rl.rlstm_last_timeout(ws) == 0
    out = dict(y=y[:, :, :H].cpu().numpy(), c=c.cpu().numpy(), hT=hT.cpu().numpy(), cT=cT.cpu().numpy(),
               y_pad=y[:, :, H:].cpu().numpy())
    if dy is None:
        return out
    dyd = torch.full((T, B, ly), fill, device=DEV)
    dyd[:, :, :H] = dev(dy)
    dx = torch.full((T, B, lx), fill, device=DEV) if want_dx else None
    dW = torch.full((D, 4 * H), fill, device=DEV)
    dR = torch.full((H, 4 * H), fill, device=DEV)
    db = torch.full((4 * H,), fill, device=DEV)
    dh0 = torch.full((B, H), fill, device=DEV)
    dc0 = torch.full((B, H), fill, device=DEV)
    rl.lstm_bwd(desc, xd, Wd, Rd, sl, h0d, c0d, y, c, reserve, dyd, dev(dhT), dev(dcT), dx, dW, dR, db, dh0, dc0, ws)
    assert rl.rlstm_last_timeout(ws) == 0
    out.update(dW=dW.cpu().numpy(), dR=dR.cpu().numpy(), db=db.cpu().numpy(), dh0=dh0.cpu().numpy(),
               dc0=dc0.cpu().numpy())
    if want_dx:
        out["dx"] = dx[:, :, :D].cpu().numpy()
    return out


class StackRun:
    """Device buffers for blstm_stack_fwd_bwd on one workload."""

    def __init__(self, wl, engine=rl.RLSTM_ENGINE_AUTO, want_dx=True, two_streams=True, **tuning):
        """tuning: the descriptor's tuning fields (first_piece, batch_groups, overlap_mode, gemm_variant, bwd_exchange)."""
        assert wl.bidirectional
        self.wl = wl
        self.desc = rl.rblstm_desc(L=wl.L, T=wl.T, B=wl.B, D=wl.D, H=wl.H, operand_dtype=wl.operand_dtype,
                                   engine=engine, **tuning)
        self.x = dev(wl.x)
        self.seq_lens = dev(wl.seq_lens, torch.int32)
        self.params = [dev(a) for layer in wl.params for p in layer for a in p]
        self.grads = [torch.full_like(p, float("nan")) for p in self.params]
        self.G = dev(wl.G)
        self.y_top = torch.full((wl.T, wl.B, 2 * wl.H), float("nan"), device=DEV)
        self.dx = torch.full((wl.T, wl.B, wl.D), float("nan"), device=DEV) if want_dx else None
        self.reserve = torch.empty(rl.rblstm_reserve_bytes(self.desc), dtype=torch.uint8, device=DEV)
        self.ws = torch.empty(rl.rblstm_workspace_bytes(self.desc), dtype=torch.uint8, device=DEV)
        self.stream_b = torch.cuda.Stream() if two_streams else None

    def step(self):
        rl.blstm_stack_fwd_bwd(self.desc, self.x, self.params, self.seq_lens, self.G, self.y_top, self.grads,
                               self.dx, self.reserve, self.ws, None, self.stream_b)

    def forward_only(self):
        rl.blstm_stack_fwd(self.desc, self.x, self.params, self.seq_lens, self.y_top, self.reserve, self.ws, None)

    def results(self):
        torch.cuda.synchronize()
        assert rl.rlstm_last_timeout(self.ws) == 0
        out = dict(y=self.y_top.cpu().numpy(), grads=[g.cpu().numpy() for g in self.grads])
        if self.dx is not None:
            out["dx"] = self.dx.cpu().numpy()
        return out


def oracle_stack(wl):
    from oracle import blstm_stack_backward, blstm_stack_forward
    params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    y, caches = blstm_stack_forward(wl.x.astype(np.float64), params, wl.seq_lens)
    grads, dx = blstm_stack_backward(caches, wl.G.astype(np.float64))
    flat = []
    for l in range(wl.L):
        for d in range(2):
            flat += [grads[l][d]["dW"], grads[l][d]["dR"], grads[l][d]["db"]]
    return dict(y=y, dx=dx, grads=flat)


def paper_batch_from_corpus():
    """The paper-shaped minibatch (81 segments of 250 frames) cut from the synthetic corpus BY THE LIBRARY: segment
    table on the host (rlstm_chunk_plan), gather on the device (rlstm_chunk_gather).  Returns the Workload."""
    from paper_1608_00895_amd import synth
    cx, clens = synth.paper_corpus()
    size, nb = synth.PAPER_SEGMENT_FRAMES, synth.PAPER_BATCH_SEGMENTS
    seq, start, length = rl.rlstm_chunk_plan(clens, size, size)
    xc = torch.empty((size, nb, cx.shape[2]), device=DEV)
    rl.rlstm_chunk_gather(dev(cx), dev(seq[:nb], torch.int32), dev(start[:nb], torch.int32), dev(length[:nb], torch.int32),
                          size, xc)
    torch.cuda.synchronize()
    return synth.paper_workload(xc.cpu().numpy(), length[:nb])


def check_structured_samples(g, prefix, y, dx, grads, seq_lens, L, tol_y, tol_grad, what):
    """Compares the places a golden file stores beyond its random samples: whole frames of y_top / dx (`frames`,
    `y_slab`, `dx_slab`), every sequence's last valid and first padded frame (`y_end`, `dx_end`), the last rows and
    the last units' columns of every dW / dR, every db whole.  y, dx: device tensors [T,B,.]; grads: list of device
    tensors (dW, dR, db per layer and direction).  Errors are relative to the tensors' largest absolute values as
    stored with the random samples (`<name>_max`).  Returns the worst errors (forward, gradients)."""
    T, B = y.shape[0], y.shape[1]
    frames = [int(t) for t in g[prefix + "frames"]]
    worst_y = worst_g = 0.0

    def upd(got, ref, scale):
        return float(np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64)).max() / scale)

    ymax, dxmax = float(g[prefix + "y_max"]), float(g[prefix + "dx_max"])
    worst_y = max(worst_y, upd(y[frames].cpu().numpy(), g[prefix + "y_slab"], ymax))
    if dx is not None:
        worst_g = max(worst_g, upd(dx[frames].cpu().numpy(), g[prefix + "dx_slab"], dxmax))
    lens = np.asarray(seq_lens, np.int64)
    nidx = torch.arange(B, device=y.device)
    last = torch.from_numpy(lens - 1).to(y.device)
    worst_y = max(worst_y, upd(y[last, nidx].cpu().numpy(), g[prefix + "y_end"][:, 0], ymax))
    if dx is not None:
        worst_g = max(worst_g, upd(dx[last, nidx].cpu().numpy(), g[prefix + "dx_end"][:, 0], dxmax))
    short = np.nonzero(lens < T)[0]
    if len(short):
        first_pad = torch.from_numpy(lens[short]).to(y.device)
        sidx = torch.from_numpy(short).to(y.device)
        assert not bool(y[first_pad, sidx].any()), what + ": y is not zero at a sequence's first padded frame"
        assert not g[prefix + "y_end"][short, 1].any()
        if dx is not None:
            assert not bool(dx[first_pad, sidx].any()), what + ": dx is not zero at a sequence's first padded frame"
    cols = torch.from_numpy(np.asarray(g[prefix + "cols"], np.int64)).to(y.device)
    k = 0
    for l in range(L):
        for d in range(2):
            for nm in ("dW", "dR"):
                t = grads[k]
                scale = float(g[f"{prefix}{nm}_{l}_{d}_max"])
                worst_g = max(worst_g, upd(t[-4:, :].cpu().numpy(), g[f"{prefix}{nm}_{l}_{d}_lastrows"], scale))
                worst_g = max(worst_g, upd(t[:, cols].cpu().numpy(), g[f"{prefix}{nm}_{l}_{d}_lastcols"], scale))
                k += 1
            ref = g[f"{prefix}db_{l}_{d}_whole"] if f"{prefix}db_{l}_{d}_whole" in g.files else g[f"{prefix}db_{l}_{d}"]
            worst_g = max(worst_g, upd(grads[k].cpu().numpy(), ref, max(float(np.abs(ref).max()), 1e-30)))
            k += 1
    print(f"{what}: structured samples (frames {frames}, sequence ends, last rows / columns, bias gradients): "
          f"forward {worst_y:.2e}, gradients {worst_g:.2e}", flush=True)
    assert worst_y < tol_y, (what, "forward", worst_y)
    assert worst_g < tol_grad, (what, "gradients", worst_g)
    return worst_y, worst_g
