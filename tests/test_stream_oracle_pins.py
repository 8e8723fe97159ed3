"""Pins of the streaming oracle (segments chained by their final states, gradients truncated at the segment
boundaries) against things other than itself: invariance of the forward result under cutting, reduction to the
uncut layer for a single segment, and autograd of an independent torch formulation with detached states."""
import numpy as np
import torch

from oracle import lstm_backward, lstm_forward, lstm_stream_forward_backward, segment_lengths


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _case(seed, L=2, S=3, Tc=4, B=3, D=5, H=6, lens=(12, 7, 2)):
    rng = _rng(seed)
    T = S * Tc
    x = rng.standard_normal((T, B, D))
    params = []
    for l in range(L):
        din = D if l == 0 else H
        params.append((rng.uniform(-0.6, 0.6, (din, 4 * H)), rng.uniform(-0.6, 0.6, (H, 4 * H)), rng.uniform(-0.3, 0.3, 4 * H)))
    lens = np.array(lens)
    G = rng.standard_normal((T, B, H))
    state0 = [(rng.uniform(-0.5, 0.5, (B, H)), rng.uniform(-0.5, 0.5, (B, H))) for _ in range(L)]
    return x, params, lens, G, state0


def _uncut(x, params, lens, state0):
    inp, fwds = x, []
    for l, (W, R, b) in enumerate(params):
        f = lstm_forward(inp, W, R, b, lens, 1, state0[l][0], state0[l][1])
        fwds.append(f)
        inp = f["y"]
    return inp, fwds


def test_segment_lengths():
    assert list(segment_lengths([12, 7, 2, 0, 4], 0, 4)) == [4, 4, 2, 0, 4]
    assert list(segment_lengths([12, 7, 2, 0, 4], 1, 4)) == [4, 3, 0, 0, 0]
    assert list(segment_lengths([12, 7, 2, 0, 4], 2, 4)) == [4, 0, 0, 0, 0]


def test_forward_does_not_depend_on_where_the_sequences_are_cut():
    x, params, lens, G, state0 = _case(1)
    y_ref, fwds = _uncut(x, params, lens, state0)
    for Tc in (1, 2, 3, 4, 6, 12):
        y, _, _, state = lstm_stream_forward_backward(x, params, lens, G, Tc, state0)
        assert np.abs(y - y_ref).max() < 1e-14, Tc
        for l in range(len(params)):
            assert np.abs(state[l][0] - fwds[l]["hT"]).max() < 1e-14 and np.abs(state[l][1] - fwds[l]["cT"]).max() < 1e-14


def test_one_segment_is_the_uncut_layer_stack():
    x, params, lens, G, state0 = _case(2)
    y, grads, dx, _ = lstm_stream_forward_backward(x, params, lens, G, x.shape[0], state0)
    y_ref, fwds = _uncut(x, params, lens, state0)
    d = G
    for l in range(len(params) - 1, -1, -1):
        g = lstm_backward(fwds[l], d)
        for k in ("dW", "dR", "db"):
            assert np.abs(grads[l][k] - g[k]).max() < 1e-13
        d = g["dx"]
    assert np.abs(dx - d).max() < 1e-13


def _torch_truncated(x, params, lens, G, Tc, state0):
    """Independent formulation: frame-by-frame cell in torch, states detached at the segment boundaries, autograd."""
    T, B, _ = x.shape
    tp = [[torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in p] for p in params]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tl = torch.tensor(lens)
    state = [(torch.tensor(h), torch.tensor(c)) for h, c in state0]
    loss = torch.zeros((), dtype=torch.float64)
    ys = []
    for s0 in range(0, T, Tc):
        state = [(h.detach(), c.detach()) for h, c in state]
        inp = [tx[t] for t in range(s0, s0 + Tc)]
        for l, (W, R, b) in enumerate(tp):
            h, c = state[l]
            H = R.shape[0]
            out = []
            for k, t in enumerate(range(s0, s0 + Tc)):
                a = inp[k] @ W + h @ R + b
                i, f, o = (torch.sigmoid(a[:, j * H:(j + 1) * H]) for j in range(3))
                g = torch.tanh(a[:, 3 * H:])
                cn = f * c + i * g
                hn = o * torch.tanh(cn)
                m = (t < tl).to(torch.float64)[:, None]
                h = m * hn + (1 - m) * h
                c = m * cn + (1 - m) * c
                out.append(m * hn)
            state[l] = (h, c)
            inp = out
        for k, t in enumerate(range(s0, s0 + Tc)):
            loss = loss + (inp[k] * torch.tensor(G[t])).sum()
            ys.append(inp[k])
    loss.backward()
    return torch.stack(ys).detach().numpy(), tp, tx.grad.numpy()


def test_against_torch_autograd_with_detached_states():
    for seed, Tc in ((3, 4), (4, 3), (5, 1)):
        x, params, lens, G, state0 = _case(seed, S=12 // Tc, Tc=Tc)
        y, grads, dx, _ = lstm_stream_forward_backward(x, params, lens, G, Tc, state0)
        ty, tp, tdx = _torch_truncated(x, params, lens, G, Tc, state0)
        assert np.abs(y - ty).max() < 1e-13
        assert np.abs(dx - tdx).max() < 1e-12
        for l in range(len(params)):
            for k, a in zip(("dW", "dR", "db"), tp[l]):
                assert np.abs(grads[l][k] - a.grad.numpy()).max() < 1e-12, (seed, l, k)


def test_truncation_changes_the_gradient_and_only_through_the_recurrence():
    x, params, lens, G, state0 = _case(6)
    _, g_cut, dx_cut, _ = lstm_stream_forward_backward(x, params, lens, G, 4, state0)
    _, g_all, dx_all, _ = lstm_stream_forward_backward(x, params, lens, G, 12, state0)
    assert np.abs(g_cut[0]["dR"] - g_all[0]["dR"]).max() > 1e-3          # the truncated terms are not small here
    # the last segment of the longest sequence sees no truncation at all: its input gradient is the uncut one
    assert np.abs(dx_cut[8:, 0] - dx_all[8:, 0]).max() < 1e-13
    assert np.abs(dx_cut[:8, 0] - dx_all[:8, 0]).max() > 1e-4
