"""Pins of the dynamic loss-scaling oracle (CPU): the scale rule against torch's GradScaler (library routine),
closed forms, and the reduction to the statically scaled step."""
import numpy as np
import pytest
import torch

from oracle import scaler as SC
from oracle.step import train_step
from workloads.synthetic import ADAM, CONFIGS, PARAM_NAMES, make_layer_inputs

SCALER = dict(growth_factor=2.0, backoff_factor=0.5, growth_interval=3)


@pytest.mark.parametrize("pattern", ["0000000000", "0010000100", "1100010000", "0001110001"])
def test_scale_rule_matches_library_grad_scaler(pattern):
    """Same skip decisions and the same scale after every step as torch.amp.GradScaler on the CPU, driven by
    gradients that are made non-finite on the steps marked 1."""
    w = torch.nn.Parameter(torch.ones(4, dtype=torch.float32))
    opt = torch.optim.SGD([w], lr=0.125)
    gs = torch.amp.GradScaler("cpu", init_scale=1024.0, growth_factor=2.0, backoff_factor=0.5, growth_interval=3)
    state = SC.scaler_new(1024.0)
    taken = 0
    for ch in pattern:
        bad = ch == "1"
        loss = (w * 1.0).sum()
        gs.scale(loss).backward()
        if bad:
            w.grad[1] = float("inf")
        before = w.detach().clone()
        gs.step(opt)
        gs.update()
        opt.zero_grad()
        skipped = torch.equal(before, w.detach())
        state = SC.scaler_update(state, bad, **SCALER)
        taken += 0 if bad else 1
        assert skipped == bad
        assert state["scale"] == gs.get_scale()
        assert state["t"] == taken


def test_closed_forms():
    s = SC.scaler_new(8.0)
    for _ in range(3 * 4):
        s = SC.scaler_update(s, False, **SCALER)
    assert s == dict(scale=8.0 * 2 ** 4, good_steps=0, t=12)          # growth every 3 good steps
    s = SC.scaler_update(s, False, **SCALER)
    s = SC.scaler_update(s, True, **SCALER)                            # overflow: halve, restart the count
    assert s == dict(scale=64.0, good_steps=0, t=13)
    s = SC.scaler_update(SC.scaler_update(s, False, **SCALER), False, **SCALER)
    assert s == dict(scale=64.0, good_steps=2, t=15)
    assert SC.any_nonfinite({"a": np.ones(3), "b": np.array([1.0, np.nan])})
    assert SC.any_nonfinite({"a": np.array([-np.inf])})
    assert not SC.any_nonfinite({"a": np.ones(3), "b": np.zeros(2)})


def _state(inp):
    p = {k: np.asarray(inp["params"][k], dtype=np.float64) for k in PARAM_NAMES}
    z = {k: np.zeros_like(p[k]) for k in PARAM_NAMES}
    return p, dict(z), {k: np.zeros_like(p[k]) for k in PARAM_NAMES}


def test_good_steps_reduce_to_the_static_step():
    """Without overflow and before any growth the dynamic step is the statically scaled step (pinned elsewhere)."""
    cfg = dict(CONFIGS["tiny"], dropout_p=0.1)
    inp = make_layer_inputs(cfg, seed=3)
    p, m, v = _state(inp)
    st = SC.scaler_new(256.0)
    p2, m2, v2 = p, m, v
    for t in (1, 2):
        d = SC.train_step_dynamic(cfg, p, m, v, inp["x"], inp["G"], inp["seq_lens"], st, ADAM,
                                  dict(SCALER, growth_interval=1000), step=t)
        r = train_step(cfg, p2, m2, v2, inp["x"], inp["G"], inp["seq_lens"], t, dict(ADAM, loss_scale=256.0))
        assert not d["found_inf"]
        for k in PARAM_NAMES:
            assert np.array_equal(d["params"][k], r["params"][k]) and np.array_equal(d["grads"][k], r["grads"][k])
        p, m, v, st = d["params"], d["m"], d["v"], d["state"]
        p2, m2, v2 = r["params"], r["m"], r["v"]
    assert st == dict(scale=256.0, good_steps=2, t=2)


def test_poisoned_step_is_skipped_and_next_step_uses_the_old_count():
    cfg = dict(CONFIGS["tiny"], dropout_p=0.0)
    inp = make_layer_inputs(cfg, seed=4)
    p, m, v = _state(inp)
    st = SC.scaler_new(64.0)
    G_bad = np.array(inp["G"], dtype=np.float64)
    G_bad.reshape(-1)[5] = np.inf
    d = SC.train_step_dynamic(cfg, p, m, v, inp["x"], G_bad, inp["seq_lens"], st, ADAM, SCALER, step=1)
    assert d["found_inf"] and d["state"] == dict(scale=32.0, good_steps=0, t=0)
    for k in PARAM_NAMES:
        assert np.array_equal(d["params"][k], p[k]) and not d["m"][k].any() and not d["v"][k].any()
    # the retry runs Adam's first step (bias corrections of t = 1) at the halved scale
    d2 = SC.train_step_dynamic(cfg, d["params"], d["m"], d["v"], inp["x"], inp["G"], inp["seq_lens"], d["state"], ADAM,
                               SCALER, step=2)
    r = train_step(cfg, p, m, v, inp["x"], inp["G"], inp["seq_lens"], 1, dict(ADAM, loss_scale=32.0))
    assert not d2["found_inf"] and d2["state"] == dict(scale=32.0, good_steps=1, t=1)
    for k in PARAM_NAMES:
        assert np.allclose(d2["params"][k], r["params"][k], rtol=0, atol=0)
