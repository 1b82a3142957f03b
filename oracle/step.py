"""One whole training step on the oracle: forward, loss seed, backward, Adam.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Composition as in the
paper's Section 2.1: forward graph, loss, backward graph, optimizer.
"""
import numpy as np

from .layer import PARAM_NAMES, layer_forward, layer_backward, loss_and_seed
from .adam import adam_step


def train_step(cfg, params, m, v, x, G, seq_lens, t, hyper):
    """params/m/v: dicts of fp64 arrays (not mutated).  t is 1-based and is also
    the dropout step counter.  Returns dict(y, loss, dx, grads (loss-scaled),
    params, m, v)."""
    ls = float(hyper.get("loss_scale", 1.0))
    y, cache = layer_forward(cfg, params, x, seq_lens, step=t)
    loss, dy = loss_and_seed(y, G, ls)
    dx, grads = layer_backward(cfg, cache, dy)
    new_p, new_m, new_v = {}, {}, {}
    for k in PARAM_NAMES:
        new_p[k], new_m[k], new_v[k] = adam_step(
            params[k], grads[k].reshape(np.shape(params[k])), m[k], v[k], t,
            hyper["lr"], hyper["beta1"], hyper["beta2"], hyper["eps"],
            hyper.get("weight_decay", 0.0), 1.0 / ls)
    return dict(y=y, loss=loss, dx=dx, grads=grads, params=new_p, m=new_m, v=new_v, cache=cache)
