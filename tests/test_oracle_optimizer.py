"""Pins of the update oracle: a library implementation of the same published algorithm, the
closed form of its first step, and the limits that fix each term's sign and place."""
import numpy as np
import torch

from oracle.optimizer import AdamW


def tensors(seed):
    rng = np.random.default_rng(seed)
    p = {"w": rng.standard_normal((5, 7)), "b": rng.standard_normal(7), "e": rng.standard_normal((3, 4))}
    gs = [{k: rng.standard_normal(v.shape) * 10.0 ** rng.integers(-3, 2) for k, v in p.items()} for _ in range(6)]
    return p, gs


def test_matches_library_adamw_over_several_steps():
    p, gs = tensors(1)
    hp = dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    opt = torch.optim.AdamW(
        [{"params": [tp["w"], tp["e"]], "weight_decay": hp["weight_decay"]}, {"params": [tp["b"]], "weight_decay": 0.0}],
        lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"])
    ours = AdamW(**hp)
    cur = p
    for g in gs:
        for k in tp:
            tp[k].grad = torch.tensor(g[k], dtype=torch.float64)
        opt.step()
        cur = ours.step(cur, g)
        for k in cur:
            np.testing.assert_allclose(cur[k], tp[k].detach().numpy(), rtol=1e-12, atol=1e-14)


def test_first_step_closed_form():
    # m = (1-b1) g, v = (1-b2) g^2, both bias corrections cancel: step = g / (|g| + eps)
    p, gs = tensors(2)
    o = AdamW(lr=0.01, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.05)
    new = o.step(p, gs[0])
    for k in p:
        wd = 0.05 if p[k].ndim >= 2 else 0.0
        want = p[k] - 0.01 * (gs[0][k] / (np.abs(gs[0][k]) + 1e-8) + wd * p[k])
        np.testing.assert_allclose(new[k], want, rtol=1e-12)


def test_limits():
    p, gs = tensors(3)
    zero = {k: np.zeros_like(v) for k, v in p.items()}
    # no gradient, no decay: nothing moves; no gradient with decay: matrices shrink by lr * wd, vectors stay
    np.testing.assert_array_equal(AdamW(weight_decay=0.0).step(p, zero)["w"], p["w"])
    d = AdamW(lr=0.1, weight_decay=0.5).step(p, zero)
    np.testing.assert_allclose(d["w"], p["w"] * (1 - 0.1 * 0.5), rtol=1e-15)
    np.testing.assert_array_equal(d["b"], p["b"])
    # constant gradient: the bias-corrected moments are exact, every step moves by lr * sign(g)
    o = AdamW(lr=0.01, eps=0.0, weight_decay=0.0)
    cur = p
    for t in range(1, 5):
        cur = o.step(cur, gs[0])
        np.testing.assert_allclose(cur["w"], p["w"] - 0.01 * t * np.sign(gs[0]["w"]), rtol=1e-12, atol=1e-14)
    # the update opposes the gradient
    assert np.all((AdamW(weight_decay=0.0).step(p, gs[1])["b"] - p["b"]) * gs[1]["b"] <= 0)
