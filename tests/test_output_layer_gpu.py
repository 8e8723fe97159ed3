"""GPU parity of the softmax / cross-entropy output layer, of the parameter updates and of a whole training
step (stack forward, output layer, stack backward, update), through the C ABI, against the CPU oracle.
Tolerances: loss 1e-5 relative, gradients 1e-4 (max abs difference over max abs oracle value); the error
count is an integer decided by comparisons of float32 logits, so it must equal the oracle's count once the
frames whose two largest oracle logits lie closer than float32 rounding can resolve are set aside."""
import numpy as np
import pytest
import torch

from oracle import (adam_step, blstm_stack_backward, blstm_stack_forward, sgd_momentum_step, softmax_ce_backward,
                    softmax_ce_forward)
from paper_1608_00895_amd import binding as rl
from paper_1608_00895_amd import synth

import gpu_harness as gh

pytestmark = pytest.mark.gpu

TOL_LOSS = 1e-5
TOL_GRAD = 1e-4


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


class CeRun:
    def __init__(self, T, B, F, C, operand_dtype=0):
        self.shape = (T, B, F, C)
        self.operand_dtype = operand_dtype
        self.loss = torch.full((1,), float("nan"), device=gh.DEV)
        self.errors = torch.full((1,), -1, dtype=torch.int32, device=gh.DEV)
        self.dy = torch.full((T, B, F), float("nan"), device=gh.DEV)
        self.dWo = torch.full((F, C), float("nan"), device=gh.DEV)
        self.dbo = torch.full((C,), float("nan"), device=gh.DEV)
        self.ws = torch.empty(rl.rlstm_ce_workspace_bytes(T, B, F, C), dtype=torch.uint8, device=gh.DEV)

    def run(self, y, Wo, bo, labels, lens):
        T, B, F, C = self.shape
        rl.softmax_ce_fwd_bwd(T, B, F, C, self.operand_dtype, y, Wo, bo, labels, lens, self.loss, self.errors, self.dy,
                              self.dWo, self.dbo, self.ws)
        torch.cuda.synchronize()
        return dict(loss=float(self.loss.item()), errors=int(self.errors.item()), dy=self.dy.cpu().numpy(),
                    dWo=self.dWo.cpu().numpy(), dbo=self.dbo.cpu().numpy())


def _ambiguous_frames(y, Wo, bo, labels, lens, eps=1e-5):
    """Valid frames whose decision (is the arg max the label?) float32 rounding of the logits could flip."""
    z = np.asarray(y, np.float64) @ np.asarray(Wo, np.float64) + np.asarray(bo, np.float64)
    T, B, C = z.shape
    n = 0
    for t in range(T):
        for b in range(B):
            if t < lens[b] and 0 <= labels[t, b] < C:
                zz = z[t, b]
                top = np.sort(zz)[-2:]
                if C > 1 and top[1] - top[0] < eps * max(1.0, np.abs(zz).max()):
                    n += 1
    return n


def _check(got, y, Wo, bo, labels, lens, tag, tol_loss=TOL_LOSS, tol_grad=TOL_GRAD):
    print(tag, flush=True)
    f = softmax_ce_forward(y, Wo, bo, labels, lens)
    g = softmax_ce_backward(f)
    assert abs(got["loss"] - f["loss"]) <= tol_loss * max(abs(f["loss"]), 1e-30), (tag, got["loss"], f["loss"])
    assert abs(got["errors"] - f["errors"]) <= _ambiguous_frames(y, Wo, bo, labels, lens), (tag, got["errors"], f["errors"])
    for k in ("dy", "dWo", "dbo"):
        assert gh.rel_err(got[k], g[k]) < tol_grad, (tag, k, gh.rel_err(got[k], g[k]))
    T, B = labels.shape
    for b in range(B):
        assert not got["dy"][max(int(lens[b]), 0):, b].any(), (tag, "dy not zero outside the sequence")
    return f, g


@pytest.mark.parametrize("shape", [
    # T, B, F, C, lens
    (7, 4, 5, 9, (7, 3, 0, 6)),                 # tiny, a sequence of length 0, C not a multiple of 4
    (37, 5, 24, 1501, None),                    # the paper's class count, several 256-column sweeps per row
    (19, 33, 130, 260, None),                   # F and C beyond one product tile, C a multiple of 4
    (1, 1, 3, 1, (1,)),                         # one class: loss 0, gradient 0
    (64, 40, 64, 517, None),                    # 2560 rows: several row chunks in the column sums
])
def test_softmax_ce_against_oracle(shape):
    T, B, F, C, lens = shape
    rng = _rng(7000 + T + B + F + C)
    y = rng.standard_normal((T, B, F)).astype(np.float32)
    Wo, bo, labels = synth.output_layer(T, B, F, C, seed=7100 + C, wscale=0.5)
    lens = np.array(lens if lens is not None else rng.integers(0, T + 1, B), np.int32)
    lens[0] = T
    run = CeRun(T, B, F, C)
    got = run.run(gh.dev(y), gh.dev(Wo), gh.dev(bo), gh.dev(labels, torch.int32), gh.dev(lens, torch.int32))
    f, _ = _check(got, y, Wo, bo, labels, lens, f"softmax_ce shape={shape}")
    if C == 1:
        assert got["loss"] == 0.0 and got["errors"] == 0 and not got["dy"].any()
    else:
        assert f["errors"] > 0            # random labels: the count is not trivially zero


def test_softmax_ce_learned_like_case_counts_errors_exactly():
    """Logits with a clear winner per frame (the label on most frames): the error count is exact."""
    T, B, F, C = 23, 6, 32, 300
    rng = _rng(7200)
    Wo, bo, labels = synth.output_layer(T, B, F, C, seed=7201, wscale=1.0)
    wrong = rng.random((T, B)) < 0.3
    target = np.where(wrong, (labels + 1 + rng.integers(0, C - 1, (T, B))) % C, labels)
    y = (Wo.T[target] * 0.5 + 0.05 * rng.standard_normal((T, B, F))).astype(np.float32)     # y points at the target class
    lens = np.array([23, 20, 11, 1, 0, 17], np.int32)
    got = CeRun(T, B, F, C).run(gh.dev(y), gh.dev(Wo), gh.dev(bo), gh.dev(labels, torch.int32), gh.dev(lens, torch.int32))
    f, _ = _check(got, y, Wo, bo, labels, lens, "softmax_ce clear winners")
    assert _ambiguous_frames(y, Wo, bo, labels, lens) == 0 and got["errors"] == f["errors"] and 0 < f["errors"] < lens.sum()


def test_softmax_ce_edge_cases():
    T, B, F, C = 9, 3, 8, 11
    rng = _rng(7300)
    y = rng.standard_normal((T, B, F)).astype(np.float32)
    Wo, bo, labels = synth.output_layer(T, B, F, C, seed=7301)
    run = CeRun(T, B, F, C)
    dv = lambda lens, lab: (gh.dev(y), gh.dev(Wo), gh.dev(bo), gh.dev(lab, torch.int32), gh.dev(lens, torch.int32))
    # every sequence empty: nothing contributes
    got = run.run(*dv(np.zeros(B, np.int32), labels))
    assert got["loss"] == 0.0 and got["errors"] == 0
    assert not got["dy"].any() and not got["dWo"].any() and not got["dbo"].any()
    # lengths outside [0, T] are clamped; labels that are no class index are left out like padding
    lab = labels.copy()
    lab[2, 0], lab[5, 1], lab[0, 2] = -1, C, -100
    lens = np.array([T + 5, -3, T], np.int32)
    got = run.run(*dv(lens, lab))
    _check(got, y, Wo, bo, lab, np.clip(lens, 0, T), "softmax_ce clamped lengths, invalid labels")
    assert not got["dy"][2, 0].any() and not got["dy"][0, 2].any()
    # a tie for the largest logit: the first index wins (the oracle's rule), so label 0 is right and label 1 is wrong
    Wz, bz = np.zeros((F, C), np.float32), np.zeros(C, np.float32)
    for lab_value, want in ((0, 0), (1, T * B)):
        lab = np.full((T, B), lab_value, np.int32)
        got = run.run(gh.dev(y), gh.dev(Wz), gh.dev(bz), gh.dev(lab, torch.int32), gh.dev(np.full(B, T, np.int32), torch.int32))
        assert got["errors"] == want and abs(got["loss"] - T * B * np.log(C)) < 1e-4 * T * B * np.log(C)
    # bad arguments are reported, nothing is launched
    L = rl.lib()
    assert L.softmax_ce_fwd_bwd(T, B, F, 0, 0, *([None] * 11), 0, None) == -2
    assert L.softmax_ce_fwd_bwd(T, B, F, C, 0, *([None] * 11), 0, None) == -1
    assert L.softmax_ce_fwd_bwd(T, B, F, C, 7, *([None] * 11), 0, None) == -3
    small = torch.empty(64, dtype=torch.uint8, device=gh.DEV)
    assert rl.softmax_ce_fwd_bwd(T, B, F, C, 0, *dv(np.full(B, T, np.int32), labels), run.loss, run.errors, run.dy, run.dWo,
                                 run.dbo, small, check=False) == -4


def test_softmax_ce_is_reproducible_bit_for_bit_and_bf16_variant():
    T, B, F, C = 50, 20, 96, 1501
    rng = _rng(7400)
    y = rng.standard_normal((T, B, F)).astype(np.float32)
    Wo, bo, labels = synth.output_layer(T, B, F, C, seed=7401, wscale=0.3)
    lens = rng.integers(1, T + 1, B).astype(np.int32)
    args = (gh.dev(y), gh.dev(Wo), gh.dev(bo), gh.dev(labels, torch.int32), gh.dev(lens, torch.int32))
    run = CeRun(T, B, F, C)
    a = run.run(*args)
    b = run.run(*args)
    assert a["loss"] == b["loss"] and a["errors"] == b["errors"]
    for k in ("dy", "dWo", "dbo"):
        assert np.array_equal(a[k], b[k]), k
    # operands of the three products rounded to bf16: the documented 2e-2 bar
    got = CeRun(T, B, F, C, operand_dtype=1).run(*args)
    f = softmax_ce_forward(y, Wo, bo, labels, lens)
    g = softmax_ce_backward(f)
    assert abs(got["loss"] - f["loss"]) < 2e-2 * f["loss"]
    for k in ("dy", "dWo", "dbo"):
        assert gh.rel_err(got[k], g[k]) < 2e-2, (k, gh.rel_err(got[k], g[k]))


def test_update_rules_against_oracle():
    rng = _rng(7500)
    for n in (1, 255, 4097, 300001):
        p = rng.standard_normal(n).astype(np.float32)
        # SGD with momentum, three steps
        dp, dvel = gh.dev(p), torch.zeros(n, device=gh.DEV)
        rp, rv = p.astype(np.float64), np.zeros(n)
        for k in range(3):
            g = rng.standard_normal(n).astype(np.float32)
            rl.rlstm_sgd_momentum_step(dp, gh.dev(g), dvel, 0.01, 0.9)
            rp, rv = sgd_momentum_step(rp, g, rv, 0.01, 0.9)
        assert gh.rel_err(dp.cpu().numpy(), rp) < 1e-6 and gh.rel_err(dvel.cpu().numpy(), rv) < 1e-6, n
        # Adam, four steps; the first step moves every parameter by about the learning rate
        dp, dm, dv2 = gh.dev(p), torch.zeros(n, device=gh.DEV), torch.zeros(n, device=gh.DEV)
        rp, rm, rv = p.astype(np.float64), np.zeros(n), np.zeros(n)
        for k in range(1, 5):
            g = rng.standard_normal(n).astype(np.float32)
            rl.rlstm_adam_step(dp, gh.dev(g), dm, dv2, 1e-3, 0.9, 0.999, 1e-8, k)
            rp, rm, rv = adam_step(rp, g, rm, rv, 1e-3, 0.9, 0.999, 1e-8, k)
            assert np.abs(dp.cpu().numpy() - rp).max() < 1e-6, (n, k)     # steps are ~1e-3: 1e-6 is 1e-3 of a step
        assert gh.rel_err(dm.cpu().numpy(), rm) < 1e-6 and gh.rel_err(dv2.cpu().numpy(), rv) < 1e-6, n
    L = rl.lib()
    t = torch.zeros(4, device=gh.DEV)
    assert rl.rlstm_adam_step(t, t, t, t, 1e-3, 0.9, 0.999, 1e-8, 0, check=False) == -2
    assert rl.rlstm_adam_step(t, t, t, t, 1e-3, 1.0, 0.999, 1e-8, 1, check=False) == -2
    assert L.rlstm_sgd_momentum_step(None, None, None, 4, 0.1, 0.9, None) == -1
    assert L.rlstm_sgd_momentum_step(None, None, None, 0, 0.1, 0.9, None) == 0


@pytest.mark.parametrize("rule", ["adam", "sgd"])
def test_training_step_against_oracle(rule):
    """Stack forward, output layer, stack backward, update of every parameter: two steps in a row, so that the second
    step runs on the parameters the first one wrote."""
    wl = synth.small_blstm(seed=77, L=2, B=7, D=10, H=24, len_lo=2, len_hi=15, T=17)
    C = 41
    T, B, H = wl.T, wl.B, wl.H
    Wo, bo, labels = synth.output_layer(T, B, 2 * H, C, seed=78, wscale=0.3)
    run = gh.StackRun(wl, want_dx=False)
    ce = CeRun(T, B, 2 * H, C)
    dWo_, dbo_ = gh.dev(Wo), gh.dev(bo)
    dlab = gh.dev(labels, torch.int32)
    dev_params = run.params + [dWo_, dbo_]
    dev_grads = run.grads + [ce.dWo, ce.dbo]
    state1 = [torch.zeros_like(p) for p in dev_params]
    state2 = [torch.zeros_like(p) for p in dev_params]

    ref_params = [[tuple(a.astype(np.float64) for a in p) for p in layer] for layer in wl.params]
    ref_flat = [a for layer in ref_params for p in layer for a in p] + [Wo.astype(np.float64), bo.astype(np.float64)]
    ref_s1 = [np.zeros_like(a) for a in ref_flat]
    ref_s2 = [np.zeros_like(a) for a in ref_flat]
    slack = [np.zeros_like(a) for a in ref_flat]
    for step in (1, 2):
        # library
        run.forward_only()
        rl.softmax_ce_fwd_bwd(T, B, 2 * H, C, 0, run.y_top, dWo_, dbo_, dlab, run.seq_lens, ce.loss, ce.errors, ce.dy,
                              ce.dWo, ce.dbo, ce.ws)
        rl.blstm_stack_bwd(run.desc, run.x, run.params, run.seq_lens, ce.dy, run.y_top, run.grads, None, run.reserve,
                           run.ws, None, run.stream_b)
        torch.cuda.synchronize()
        assert rl.rlstm_last_timeout(run.ws) == 0
        got_grads = [g.cpu().numpy() for g in dev_grads]
        got_loss, got_err = float(ce.loss.item()), int(ce.errors.item())
        for p, g, s1, s2 in zip(dev_params, dev_grads, state1, state2):
            if rule == "adam":
                rl.rlstm_adam_step(p, g, s1, s2, 1e-3, 0.9, 0.999, 1e-8, step)
            else:
                rl.rlstm_sgd_momentum_step(p, g, s1, 1e-3, 0.9)
        torch.cuda.synchronize()
        # oracle
        it = iter(ref_flat[:-2])
        params = [[(next(it), next(it), next(it)) for _ in range(2)] for _ in range(wl.L)]
        y, caches = blstm_stack_forward(wl.x.astype(np.float64), params, wl.seq_lens)
        f = softmax_ce_forward(y, ref_flat[-2], ref_flat[-1], labels, wl.seq_lens)
        g = softmax_ce_backward(f)
        grads, _ = blstm_stack_backward(caches, g["dy"])
        ref_grads = [grads[l][d][k] for l in range(wl.L) for d in range(2) for k in ("dW", "dR", "db")] + [g["dWo"], g["dbo"]]
        print(f"training step {step} ({rule}): loss {got_loss:.6f} / {f['loss']:.6f}, errors {got_err} / {f['errors']}", flush=True)
        assert abs(got_loss - f["loss"]) < TOL_LOSS * f["loss"]
        assert abs(got_err - f["errors"]) <= _ambiguous_frames(y, ref_flat[-2], ref_flat[-1], labels, wl.seq_lens)
        for i, (a, r) in enumerate(zip(got_grads, ref_grads)):
            assert gh.rel_err(a, r) < TOL_GRAD, (step, i, gh.rel_err(a, r))
        for i in range(len(ref_flat)):
            if rule == "adam":
                ref_flat[i], ref_s1[i], ref_s2[i] = adam_step(ref_flat[i], ref_grads[i], ref_s1[i], ref_s2[i], 1e-3, 0.9,
                                                              0.999, 1e-8, step)
            else:
                ref_flat[i], ref_s1[i] = sgd_momentum_step(ref_flat[i], ref_grads[i], ref_s1[i], 1e-3, 0.9)
        # The updated parameters.  A gradient within delta = TOL_GRAD * max|g| of the oracle's moves an SGD update by
        # at most lr * delta per step (the rule is linear).  Adam's step is lr * m^ / (sqrt(v^) + eps): m^ moves by at
        # most delta and sqrt(v^), a weighted 2-norm of the gradients with weights summing to one, by at most delta
        # too, and |m^| <= sqrt(v^), so the step moves by about 2 lr delta / (sqrt(v^) + eps) -- large where the
        # gradient itself is within rounding of zero, which is Adam's own conditioning and not the kernel's.
        for i, (p, r) in enumerate(zip(dev_params, ref_flat)):
            delta = TOL_GRAD * np.abs(ref_grads[i]).max()
            if rule == "adam":
                vhat = ref_s2[i] / (1.0 - 0.999 ** step)
                slack[i] = slack[i] + 3.0 * 1e-3 * delta / (np.sqrt(vhat) + 1e-8)
            else:
                slack[i] = slack[i] + 2.0 * 1e-3 * delta * step
            err = np.abs(p.cpu().numpy() - r)
            assert np.all(err <= 2e-7 + slack[i]), (step, i, float((err - slack[i]).max()))
            assert np.median(err) < 1e-6, (step, i, float(np.median(err)))       # and the typical entry is far inside


def test_paper_train_step_full_size_against_oracle_samples():
    """A whole training step at full size, in the launch configuration bench.py times (81 segments of 250 frames,
    3 x 512 BLSTM, 1501 classes, flat parameter / gradient / moment buffers, one Adam launch): loss, frame errors and
    sampled entries of every gradient and of the updated parameters against values the oracle wrote
    (tests/golden/make_paper_train_golden.py)."""
    import os
    g = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_train_oracle_samples.npz"))
    wl = gh.paper_batch_from_corpus()      # cut from the corpus by the library
    assert np.array_equal(g["seq_lens"], wl.seq_lens)
    C, lr = 1501, 1e-3
    T, B, F = wl.T, wl.B, 2 * wl.H
    Wo, bo, labels = synth.output_layer(T, B, F, C, seed=67, wscale=0.05)
    host = [a for layer in wl.params for p in layer for a in p] + [Wo, bo]
    n_all = sum(a.size for a in host)
    flat_p = torch.empty(n_all, device=gh.DEV)
    flat_g = torch.full((n_all,), float("nan"), device=gh.DEV)
    params, grads, o = [], [], 0
    for a in host:
        flat_p[o:o + a.size] = gh.dev(a).reshape(-1)
        params.append(flat_p[o:o + a.size].view(a.shape))
        grads.append(flat_g[o:o + a.size].view(a.shape))
        o += a.size
    desc = rl.rblstm_desc(L=wl.L, T=T, B=B, D=wl.D, H=wl.H, operand_dtype=0, engine=rl.RLSTM_ENGINE_PERSISTENT)
    x, sl, lab = gh.dev(wl.x), gh.dev(wl.seq_lens, torch.int32), gh.dev(labels, torch.int32)
    y_top = torch.empty((T, B, F), device=gh.DEV)
    dy = torch.empty((T, B, F), device=gh.DEV)
    reserve = torch.empty(rl.rblstm_reserve_bytes(desc), dtype=torch.uint8, device=gh.DEV)
    ws = torch.empty(rl.rblstm_workspace_bytes(desc), dtype=torch.uint8, device=gh.DEV)
    cews = torch.empty(rl.rlstm_ce_workspace_bytes(T, B, F, C), dtype=torch.uint8, device=gh.DEV)
    loss = torch.zeros(1, device=gh.DEV)
    errors = torch.zeros(1, dtype=torch.int32, device=gh.DEV)
    m, v = torch.zeros(n_all, device=gh.DEV), torch.zeros(n_all, device=gh.DEV)
    sb = torch.cuda.Stream()
    print("paper train step: forward", flush=True)
    rl.blstm_stack_fwd(desc, x, params[:-2], sl, y_top, reserve, ws)
    rl.softmax_ce_fwd_bwd(T, B, F, C, 0, y_top, params[-2], params[-1], lab, sl, loss, errors, dy, grads[-2], grads[-1], cews)
    print("paper train step: backward", flush=True)
    rl.blstm_stack_bwd(desc, x, params[:-2], sl, dy, y_top, grads[:-2], None, reserve, ws, None, sb)
    torch.cuda.synchronize()
    assert rl.rlstm_last_timeout(ws) == 0
    got_g = [a.cpu().numpy() for a in grads]
    rl.rlstm_adam_step(flat_p, flat_g, m, v, lr, 0.9, 0.999, 1e-8, 1)
    torch.cuda.synchronize()
    assert abs(float(loss.item()) - float(g["loss"])) < TOL_LOSS * float(g["loss"]), (float(loss.item()), float(g["loss"]))
    # the error count is an integer decided by float32 comparisons: exact unless a valid frame's two largest logits
    # are closer than float32 resolves (the oracle recorded how many such frames there are, and the smallest gap)
    assert abs(int(errors.item()) - int(g["errors"])) <= int(g["frames_with_gap_below_1e_5"]), (int(errors.item()), int(g["errors"]))
    err = np.abs(dy.cpu().numpy().reshape(-1)[g["dy_idx"]] - g["dy_val"]).max() / float(g["dy_max"])
    assert err < TOL_GRAD, ("dy", err)
    for i, (a, p) in enumerate(zip(got_g, params)):
        idx = g[f"grad_{i}_idx"]
        err = np.abs(a.reshape(-1)[idx] - g[f"grad_{i}_val"]).max() / float(g[f"grad_{i}_max"])
        print(f"tensor {i}: gradient error {err:.2e}", flush=True)
        assert err < TOL_GRAD, (i, err)
        # first Adam step: lr * g / (|g| + eps); a gradient within delta of the oracle's moves it by at most
        # about 2 lr delta / (|g| + eps) (see test_training_step_against_oracle)
        delta = TOL_GRAD * float(g[f"grad_{i}_max"])
        slack = 2e-7 + 3.0 * lr * delta / (np.abs(g[f"grad_{i}_val"]) + 1e-8)
        perr = np.abs(p.cpu().numpy().reshape(-1)[idx] - g[f"param_{i}_val"])
        assert np.all(perr <= slack), (i, float((perr - slack).max()))
        moved = np.abs(g[f"param_{i}_val"] - g[f"param_{i}_old"])
        assert np.median(perr) < 1e-3 * np.median(moved) + 1e-7, (i, float(np.median(perr)), float(np.median(moved)))
