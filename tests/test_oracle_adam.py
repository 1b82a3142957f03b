"""Pins for the fp64 Adam oracle (CPU only)."""
import numpy as np
import torch

from oracle.adam import adam_step
from oracle.step import train_step
from oracle import layer as L
from workloads.synthetic import ADAM, CONFIGS, PARAM_NAMES, make_layer_inputs


def test_first_step_closed_form():
    rng = np.random.default_rng(0)
    w, g = rng.standard_normal(100), rng.standard_normal(100) * 1024
    lr, eps = 1e-4, 1e-8
    w1, m1, v1 = adam_step(w, g, np.zeros(100), np.zeros(100), 1, lr, 0.9, 0.999, eps, 0.0, 1 / 1024)
    gu = g / 1024
    assert np.allclose(w1 - w, -lr * gu / (np.abs(gu) + eps), rtol=1e-9, atol=0)
    assert np.allclose(m1, 0.1 * gu) and np.allclose(v1, 0.001 * gu * gu)


def test_constant_gradient_closed_form_all_steps():
    g = np.array([0.3, -2.0, 1e-3])
    w = np.zeros(3)
    m = np.zeros(3)
    v = np.zeros(3)
    lr, eps = 1e-3, 1e-8
    for t in range(1, 8):
        w_new, m, v = adam_step(w, g, m, v, t, lr, 0.9, 0.999, eps)
        assert np.allclose(m, g * (1 - 0.9 ** t), rtol=1e-12)
        assert np.allclose(v, g * g * (1 - 0.999 ** t), rtol=1e-12)
        assert np.allclose(w_new - w, -lr * g / (np.abs(g) + eps), rtol=1e-10)
        w = w_new


def test_matches_torch_optim_adam():
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal((5, 7))
    for wd in (0.0, 0.01):
        tw = torch.tensor(w0, requires_grad=True)
        opt = torch.optim.Adam([tw], lr=1e-2, betas=(0.8, 0.95), eps=1e-6, weight_decay=wd)
        w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
        for t in range(1, 6):
            g = rng.standard_normal((5, 7))
            tw.grad = torch.tensor(g)
            opt.step()
            w, m, v = adam_step(w, g * 8.0, m, v, t, 1e-2, 0.8, 0.95, 1e-6, wd, 1 / 8.0)
            assert np.allclose(w, tw.detach().numpy(), rtol=1e-11, atol=1e-13)


def test_train_step_composition_on_tiny_config():
    cfg = CONFIGS["tiny"]
    inp = make_layer_inputs(cfg, seed=0)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    z = {k: np.zeros_like(v) for k, v in p.items()}
    hyper = dict(ADAM, loss_scale=4.0)
    out = train_step(cfg, p, z, z, inp["x"], inp["G"], inp["seq_lens"], 1, hyper)
    # loss is sum(y*G); grads are loss-scaled; the update undoes the scale
    assert np.isclose(out["loss"], (out["y"] * inp["G"].reshape(out["y"].shape)).sum())
    y, C = L.layer_forward(cfg, p, inp["x"], None, 1)
    _, g1 = L.layer_backward(cfg, C, inp["G"].reshape(y.shape))
    for k in PARAM_NAMES:
        assert np.allclose(out["grads"][k], 4.0 * g1[k], rtol=1e-12, atol=1e-300)
        gu = g1[k].reshape(p[k].shape)
        assert np.allclose(out["params"][k] - p[k], -ADAM["lr"] * gu / (np.abs(gu) + ADAM["eps"]),
                           rtol=1e-9, atol=1e-18)
