"""Pins for oracle/output_oracle.py: finite differences, closed forms, and torch's cross_entropy / optimizers
(independent library implementations) on the CPU."""
import math

import numpy as np
import torch

from oracle import adam_step, sgd_momentum_step, softmax_ce_backward, softmax_ce_forward


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _case(seed, T=5, B=3, F=4, C=6, lens=(5, 2, 0)):
    rng = _rng(seed)
    return (rng.standard_normal((T, B, F)), rng.uniform(-0.5, 0.5, (F, C)), rng.uniform(-0.5, 0.5, C),
            rng.integers(0, C, (T, B)), np.array(lens))


def test_uniform_logits_closed_form():
    y, Wo, bo, labels, lens = _case(1)
    f = softmax_ce_forward(y, np.zeros_like(Wo), np.full_like(bo, 0.3), labels, lens)
    n = int(lens.sum())
    assert abs(f["loss"] - n * math.log(6)) < 1e-12
    assert np.allclose(f["p"][:5, 0], 1 / 6) and not f["p"][2:, 1].any() and not f["p"][:, 2].any()
    # all logits equal: the first class wins the tie
    assert f["errors"] == int(sum((labels[t, b] != 0) for b in range(3) for t in range(lens[b])))


def test_one_hot_certainty_and_error_count():
    T, B, F, C = 3, 2, 2, 4
    y = np.zeros((T, B, F)); y[..., 0] = 1.0
    Wo = np.zeros((F, C)); Wo[0, 2] = 50.0            # class 2 gets all the mass
    labels = np.array([[2, 1], [2, 2], [0, 2]])
    f = softmax_ce_forward(y, Wo, np.zeros(C), labels, np.array([3, 3]))
    assert f["errors"] == 2
    assert abs(f["loss"] - 2 * 50.0) < 1e-6           # the two wrong frames cost log(e^50 + 3) - 0 each


def test_central_finite_differences():
    y, Wo, bo, labels, lens = _case(2)
    f = softmax_ce_forward(y, Wo, bo, labels, lens)
    g = softmax_ce_backward(f)
    eps = 1e-6
    for name, arr, grad in (("y", y, g["dy"]), ("Wo", Wo, g["dWo"]), ("bo", bo, g["dbo"])):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + eps; lp = softmax_ce_forward(y, Wo, bo, labels, lens)["loss"]
            arr[i] = old - eps; lm = softmax_ce_forward(y, Wo, bo, labels, lens)["loss"]
            arr[i] = old
            num[i] = (lp - lm) / (2 * eps)
        assert np.abs(num - grad).max() < 1e-8, name
    # frames outside their sequence get no gradient and their values do not matter
    assert not g["dy"][2:, 1].any() and not g["dy"][:, 2].any()
    y2 = y.copy(); y2[2:, 1] = 77.0; y2[:, 2] = -5.0
    f2 = softmax_ce_forward(y2, Wo, bo, labels, lens)
    assert f2["loss"] == f["loss"] and np.array_equal(softmax_ce_backward(f2)["dWo"], g["dWo"])


def test_against_torch_cross_entropy():
    y, Wo, bo, labels, lens = _case(3, T=7, B=4, F=5, C=9, lens=(7, 3, 0, 6))
    f = softmax_ce_forward(y, Wo, bo, labels, lens)
    g = softmax_ce_backward(f)
    ty, tW, tb = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (y, Wo, bo))
    z = ty @ tW + tb
    mask = torch.tensor(np.arange(7)[:, None] < lens[None, :])
    loss = torch.nn.functional.cross_entropy(z[mask], torch.tensor(labels)[mask], reduction="sum")
    loss.backward()
    assert abs(loss.item() - f["loss"]) < 1e-10
    assert np.abs(ty.grad.numpy() - g["dy"]).max() < 1e-12
    assert np.abs(tW.grad.numpy() - g["dWo"]).max() < 1e-12 and np.abs(tb.grad.numpy() - g["dbo"]).max() < 1e-12
    wrong = (z.argmax(dim=2) != torch.tensor(labels)) & mask
    assert int(wrong.sum()) == f["errors"]


def test_labels_outside_the_classes_are_left_out_like_padding():
    y, Wo, bo, labels, lens = _case(5, T=6, B=3, F=4, C=7, lens=(6, 4, 5))
    labels = labels.copy()
    labels[1, 0], labels[3, 1], labels[0, 2] = -1, 7, -100
    f = softmax_ce_forward(y, Wo, bo, labels, lens)
    g = softmax_ce_backward(f)
    ty, tW, tb = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (y, Wo, bo))
    z = ty @ tW + tb
    mask = torch.tensor(np.arange(6)[:, None] < lens[None, :])
    tl = torch.tensor(np.where((labels < 0) | (labels >= 7), -100, labels))
    loss = torch.nn.functional.cross_entropy(z[mask], tl[mask], reduction="sum", ignore_index=-100)
    loss.backward()
    assert abs(loss.item() - f["loss"]) < 1e-10
    assert np.abs(ty.grad.numpy() - g["dy"]).max() < 1e-12 and np.abs(tW.grad.numpy() - g["dWo"]).max() < 1e-12
    assert not g["dy"][1, 0].any() and not f["p"][3, 1].any()
    wrong = (z.argmax(dim=2) != tl) & mask & (tl >= 0)
    assert int(wrong.sum()) == f["errors"]


def test_updates_against_torch_optimizers():
    rng = _rng(4)
    p0 = rng.standard_normal(50)
    grads = [rng.standard_normal(50) for _ in range(4)]
    for kind in ("sgd", "adam"):
        tp = torch.tensor(p0.copy(), dtype=torch.float64, requires_grad=True)
        opt = (torch.optim.SGD([tp], lr=0.05, momentum=0.9) if kind == "sgd"
               else torch.optim.Adam([tp], lr=0.01, betas=(0.9, 0.999), eps=1e-8))
        p, a, b = p0.copy(), np.zeros(50), np.zeros(50)
        for k, g in enumerate(grads):
            tp.grad = torch.tensor(g)
            opt.step()
            if kind == "sgd":
                p, a = sgd_momentum_step(p, g, a, 0.05, 0.9)
            else:
                p, a, b = adam_step(p, g, a, b, 0.01, 0.9, 0.999, 1e-8, k + 1)
            assert np.abs(tp.detach().numpy() - p).max() < 1e-12, (kind, k)
