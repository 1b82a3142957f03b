"""fp64 oracle of dynamic loss scaling with a non-finite skip.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper trains with float16 automatic mixed precision (Section 5.1) and has
the system, not the user, apply AMP (Section 3.1.2); it prints no rule for
the loss scale.  Reading taken here: the standard dynamic rule of mixed
precision training (Micikevicius et al., ICLR 2018) as the framework the
paper compares with applies it: the loss gradient is multiplied by the
current scale; if any gradient of the step is non-finite the optimizer step
is skipped (parameters, moments and the optimizer's step count stay as they
are) and the scale is multiplied by the backoff factor; otherwise the step is
taken with the gradients divided by the scale, and after `growth_interval`
consecutive good steps the scale is multiplied by the growth factor.
"""
import numpy as np

from .layer import PARAM_NAMES, layer_forward, layer_backward, loss_and_seed
from .adam import adam_step


def scaler_new(init_scale):
    """State: current scale, consecutive good steps, optimizer steps taken so far."""
    return dict(scale=float(init_scale), good_steps=0, t=0)


def any_nonfinite(grads):
    return any(not np.isfinite(np.asarray(g)).all() for g in grads.values())


def scaler_update(state, found_inf, growth_factor=2.0, backoff_factor=0.5, growth_interval=2000):
    """Returns the state after one step whose gradients were (found_inf) or were not non-finite."""
    s = dict(state)
    if found_inf:
        s["scale"] = state["scale"] * backoff_factor
        s["good_steps"] = 0
    else:
        s["t"] = state["t"] + 1
        s["good_steps"] = state["good_steps"] + 1
        if s["good_steps"] == growth_interval:
            s["scale"] = state["scale"] * growth_factor
            s["good_steps"] = 0
    return s


def train_step_dynamic(cfg, params, m, v, x, G, seq_lens, state, hyper, scaler, step):
    """One training step under the dynamic scaler.  `step` is the dropout step counter (it advances with every
    attempt); Adam's step count is state["t"] + 1 and advances only when the step is taken.  `scaler`: dict with
    growth_factor, backoff_factor, growth_interval.  Returns dict(y, loss, dx, grads (scaled), found_inf, params, m,
    v, state)."""
    ls = state["scale"]
    y, cache = layer_forward(cfg, params, x, seq_lens, step=step)
    loss, dy = loss_and_seed(y, G, ls)
    with np.errstate(invalid="ignore", over="ignore"):
        dx, grads = layer_backward(cfg, cache, dy)
    found = any_nonfinite(grads)
    new_p, new_m, new_v = {}, {}, {}
    for k in PARAM_NAMES:
        if found:
            new_p[k], new_m[k], new_v[k] = (np.array(params[k], dtype=np.float64), np.array(m[k], dtype=np.float64),
                                            np.array(v[k], dtype=np.float64))
        else:
            new_p[k], new_m[k], new_v[k] = adam_step(
                params[k], grads[k].reshape(np.shape(params[k])), m[k], v[k], state["t"] + 1,
                hyper["lr"], hyper["beta1"], hyper["beta2"], hyper["eps"], hyper.get("weight_decay", 0.0), 1.0 / ls)
    new_state = scaler_update(state, found, scaler["growth_factor"], scaler["backoff_factor"],
                              scaler["growth_interval"])
    return dict(y=y, loss=loss, dx=dx, grads=grads, found_inf=found, params=new_p, m=new_m, v=new_v, state=new_state)
