"""GPU parity of the streaming mode (segments chained by their final states, truncated back-propagation) and of
the final-state hand-off between two layers (encoder -> decoder, gradients handed back), through the C ABI,
against the CPU oracle.  Tolerances: 1e-5 forward, 1e-4 gradients (max abs difference over max abs oracle value)."""
import numpy as np
import pytest
import torch

from oracle import lstm_backward, lstm_forward, lstm_stream_forward_backward
from paper_1608_00895_amd import binding as rl

import gpu_harness as gh

pytestmark = pytest.mark.gpu

TOL_FWD = 1e-5
TOL_GRAD = 1e-4
ENGINES = [rl.RLSTM_ENGINE_PERSISTENT, rl.RLSTM_ENGINE_STEPWISE]


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _stream_case(seed, L, S, Tc, B, D, H, lens=None, wscale=0.3):
    rng = _rng(seed)
    T = S * Tc
    x = rng.standard_normal((T, B, D)).astype(np.float32)
    params = []
    for l in range(L):
        din = D if l == 0 else H
        params.append((rng.uniform(-wscale, wscale, (din, 4 * H)).astype(np.float32),
                       rng.uniform(-wscale, wscale, (H, 4 * H)).astype(np.float32),
                       rng.uniform(-0.2, 0.2, 4 * H).astype(np.float32)))
    lens = np.array(lens if lens is not None else rng.integers(0, T + 1, B), np.int32)
    G = rng.standard_normal((T, B, H)).astype(np.float32)
    state0 = rng.uniform(-0.5, 0.5, (L, 2, B, H)).astype(np.float32)
    return x, params, lens, G, state0


class StreamRun:
    def __init__(self, L, S, Tc, B, D, H, engine, want_dx=True, operand_dtype=0, two_streams=False):
        self.stream_b = torch.cuda.Stream() if two_streams else None      # takes the weight gradients
        self.desc = rl.rlstm_stream_desc(L=L, S=S, Tc=Tc, B=B, D=D, H=H, operand_dtype=operand_dtype, engine=engine)
        self.y = torch.full((S * Tc, B, H), float("nan"), device=gh.DEV)
        self.dx = torch.full((S * Tc, B, D), float("nan"), device=gh.DEV) if want_dx else None
        self.reserve = torch.empty(rl.rlstm_stream_reserve_bytes(self.desc), dtype=torch.uint8, device=gh.DEV)
        self.ws = torch.empty(rl.rlstm_stream_workspace_bytes(self.desc), dtype=torch.uint8, device=gh.DEV)

    def run(self, x, params, lens, G, state0):
        dp = [gh.dev(a) for p in params for a in p]
        grads = [torch.full_like(a, float("nan")) for a in dp]
        state = gh.dev(state0) if state0 is not None else None
        rl.lstm_stream_fwd_bwd(self.desc, gh.dev(x), dp, gh.dev(lens, torch.int32), gh.dev(G), self.y, grads, self.dx, state,
                               self.reserve, self.ws, stream_b=self.stream_b)
        torch.cuda.synchronize()
        assert rl.rlstm_last_timeout(self.ws) == 0
        return dict(y=self.y.cpu().numpy(), grads=[g.cpu().numpy() for g in grads],
                    dx=self.dx.cpu().numpy() if self.dx is not None else None,
                    state=state.cpu().numpy() if state is not None else None)


def _check_stream(got, x, params, lens, G, Tc, state0, tag):
    print(tag, flush=True)
    L = len(params)
    st0 = [(state0[l, 0], state0[l, 1]) for l in range(L)] if state0 is not None else None
    y, grads, dx, state = lstm_stream_forward_backward(x, params, lens, G, Tc, st0)
    assert gh.rel_err(got["y"], y) < TOL_FWD, (tag, "y", gh.rel_err(got["y"], y))
    for b, n in enumerate(lens):
        assert not got["y"][max(int(n), 0):, b].any(), (tag, "y not zero after the end of a sequence")
    if got["state"] is not None:
        for l in range(L):
            for k in range(2):
                assert gh.rel_err(got["state"][l, k], state[l][k]) < TOL_FWD, (tag, "state", l, k)
    for l in range(L):
        for j, k in enumerate(("dW", "dR", "db")):
            e = gh.rel_err(got["grads"][3 * l + j], grads[l][k])
            assert e < TOL_GRAD, (tag, l, k, e)
    if got["dx"] is not None:
        assert gh.rel_err(got["dx"], dx) < TOL_GRAD, (tag, "dx", gh.rel_err(got["dx"], dx))


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("shape", [
    # L, S, Tc, B, D, H, lens
    (1, 3, 5, 4, 6, 12, (15, 7, 2, 0)),          # sequences that end inside, at the edge of and before a segment
    (2, 4, 6, 5, 7, 20, None),                   # two layers, random lengths
    (3, 2, 9, 18, 10, 36, None),                 # three layers, B beyond one 16-row tile
    (2, 5, 1, 3, 4, 8, (5, 3, 1)),               # segments of one frame: every step is a hand-off
    (1, 1, 11, 2, 5, 130, (11, 4)),              # one segment: the plain layer with an initial state
])
def test_stream_against_oracle(engine, shape):
    L, S, Tc, B, D, H, lens = shape
    x, params, lens, G, state0 = _stream_case(9000 + L + S * 3 + Tc * 5 + B + H, L, S, Tc, B, D, H, lens)
    got = StreamRun(L, S, Tc, B, D, H, engine).run(x, params, lens, G, state0)
    _check_stream(got, x, params, lens, G, Tc, state0, f"stream shape={shape} engine={engine}")
    # the weight gradients on a second stream, beside the layers below and the next segment: the oracle's results
    # again, and the very same y, state and dx (the chain's kernels and their inputs do not change)
    two = StreamRun(L, S, Tc, B, D, H, engine, two_streams=True).run(x, params, lens, G, state0)
    _check_stream(two, x, params, lens, G, Tc, state0, f"stream shape={shape} engine={engine}, two streams")
    assert np.array_equal(two["y"], got["y"]) and np.array_equal(two["state"], got["state"])
    assert np.array_equal(two["dx"], got["dx"])


def test_stream_without_state_array_and_without_dx_starts_from_zero():
    L, S, Tc, B, D, H = 2, 3, 4, 6, 5, 16
    x, params, lens, G, _ = _stream_case(9100, L, S, Tc, B, D, H)
    got = StreamRun(L, S, Tc, B, D, H, rl.RLSTM_ENGINE_AUTO, want_dx=False).run(x, params, lens, G, None)
    _check_stream(got, x, params, lens, G, Tc, None, "stream, state = null, dx = null")


def test_stream_call_per_segment_equals_one_call_bit_for_bit():
    """S = 1 calls that pass the state array on give the result of the one call over all segments: same y, same
    final state (bit for bit: the same kernels on the same data), gradients that sum to the one call's."""
    L, S, Tc, B, D, H = 2, 4, 7, 9, 6, 24
    x, params, lens, G, state0 = _stream_case(9200, L, S, Tc, B, D, H)
    whole = StreamRun(L, S, Tc, B, D, H, rl.RLSTM_ENGINE_AUTO).run(x, params, lens, G, state0)
    one = StreamRun(L, 1, Tc, B, D, H, rl.RLSTM_ENGINE_AUTO)
    state = state0
    ys, gsum = [], None
    for s in range(S):
        seg_lens = np.clip(lens - s * Tc, 0, Tc).astype(np.int32)
        got = one.run(x[s * Tc:(s + 1) * Tc], params, seg_lens, G[s * Tc:(s + 1) * Tc], state)
        state = got["state"]
        ys.append(got["y"])
        gsum = got["grads"] if gsum is None else [a + b for a, b in zip(gsum, got["grads"])]
    assert np.array_equal(np.concatenate(ys), whole["y"]) and np.array_equal(state, whole["state"])
    for a, b in zip(gsum, whole["grads"]):
        assert gh.rel_err(a, b) < 1e-6


def test_stream_bad_arguments():
    L = rl.lib()
    import ctypes
    d = rl.rlstm_stream_desc(L=1, S=2, Tc=3, B=2, D=3, H=4, operand_dtype=0, engine=0)
    assert rl.rlstm_stream_reserve_bytes(d) > 0 and rl.rlstm_stream_workspace_bytes(d) > 0
    assert L.lstm_stream_fwd_bwd(ctypes.byref(d), *([None] * 12)) == -1
    bad = rl.rlstm_stream_desc(L=1, S=0, Tc=3, B=2, D=3, H=4, operand_dtype=0, engine=0)
    assert rl.rlstm_stream_reserve_bytes(bad) == 0 and L.lstm_stream_fwd_bwd(ctypes.byref(bad), *([None] * 12)) == -2
    bad = rl.rlstm_stream_desc(L=1, S=1, Tc=3, B=2, D=3, H=4, operand_dtype=3, engine=0)
    assert L.lstm_stream_fwd_bwd(ctypes.byref(bad), *([None] * 12)) == -3


@pytest.mark.parametrize("engine", ENGINES)
def test_encoder_decoder_hand_off(engine):
    """Two layers connected by the final state (Sec. 3.2): the decoder starts from the encoder's (hT, cT); in the
    backward pass the decoder's (dh0, dc0) arrive at the encoder as (dhT, dcT).  Existing entry points lstm_fwd /
    lstm_bwd; the oracle is the same composition of the layer oracle."""
    rng = _rng(9300)
    Te, Td, B, De, Dd, H = 9, 6, 5, 7, 4, 20
    xe = rng.standard_normal((Te, B, De)).astype(np.float32)
    xd = rng.standard_normal((Td, B, Dd)).astype(np.float32)
    le = np.array([9, 4, 1, 0, 7], np.int32)
    ld = np.array([6, 6, 3, 2, 0], np.int32)
    mk = lambda d: (rng.uniform(-0.4, 0.4, (d, 4 * H)).astype(np.float32), rng.uniform(-0.4, 0.4, (H, 4 * H)).astype(np.float32),
                    rng.uniform(-0.2, 0.2, 4 * H).astype(np.float32))
    (We, Re, be), (Wd, Rd, bd) = mk(De), mk(Dd)
    Gd = rng.standard_normal((Td, B, H)).astype(np.float32)
    Ge = rng.standard_normal((Te, B, H)).astype(np.float32)
    # oracle
    fe = lstm_forward(xe, We, Re, be, le, 1)
    fd = lstm_forward(xd, Wd, Rd, bd, ld, 1, fe["hT"], fe["cT"])
    gd = lstm_backward(fd, Gd)
    ge = lstm_backward(fe, Ge, gd["dh0"], gd["dc0"])
    # library
    enc = gh.run_lstm_layer(xe, We, Re, be, le, 1, engine=engine)
    dec = gh.run_lstm_layer(xd, Wd, Rd, bd, ld, 1, h0=enc["hT"], c0=enc["cT"], dy=Gd, engine=engine)
    enc = gh.run_lstm_layer(xe, We, Re, be, le, 1, dy=Ge, dhT=dec["dh0"], dcT=dec["dc0"], engine=engine)
    assert gh.rel_err(dec["y"], fd["y"]) < TOL_FWD and gh.rel_err(dec["hT"], fd["hT"]) < TOL_FWD
    for k in ("dx", "dW", "dR", "db", "dh0", "dc0"):
        assert gh.rel_err(dec[k], gd[k]) < TOL_GRAD, ("decoder", k, gh.rel_err(dec[k], gd[k]))
    for k in ("dx", "dW", "dR", "db"):
        assert gh.rel_err(enc[k], ge[k]) < TOL_GRAD, ("encoder", k, gh.rel_err(enc[k], ge[k]))
    # sequence 3 has no encoder frames: the decoder starts from zero there; sequence 4 has no decoder frames:
    # nothing but the hand-back of zero reaches the encoder from it
    assert not enc["hT"][3].any() and not dec["dh0"][4].any()


def test_paper_stream_full_size_against_oracle_samples():
    """The streaming workload at full size (64 sequences, 6 segments of 250 frames, 3 x 512 units), in the launch
    configuration bench.py times: sampled entries of every output against values the oracle wrote
    (tests/golden/make_paper_stream_golden.py)."""
    import os
    from paper_1608_00895_amd import synth
    g = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_stream_oracle_samples.npz"))
    wl = synth.paper_stream()
    assert np.array_equal(g["seq_lens"], wl.seq_lens)
    run = StreamRun(wl.L, wl.S, wl.Tc, wl.B, wl.D, wl.H, rl.RLSTM_ENGINE_PERSISTENT, two_streams=True)
    got = run.run(wl.x, wl.params, wl.seq_lens, wl.G, np.zeros((wl.L, 2, wl.B, wl.H), np.float32))

    def check(name, arr, tol):
        err = np.abs(arr.reshape(-1)[g[name + "_idx"]].astype(np.float64) - g[name + "_val"]).max() / float(g[name + "_max"])
        print(name, err, flush=True)
        assert err < tol, (name, err)

    check("y", got["y"], TOL_FWD)
    check("state", got["state"], TOL_FWD)
    check("dx", got["dx"], TOL_GRAD)
    for l in range(wl.L):
        for j, nm in enumerate(("dW", "dR", "db")):
            check(f"{nm}_{l}", got["grads"][3 * l + j], TOL_GRAD)
