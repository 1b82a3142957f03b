"""Smoke check: one tiny training step on cuda:0 through the C ABI, compared
with the CPU oracle (the only place outside tests/bench that touches it)."""
import os
import sys

import numpy as np


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (den if den > 0 else 1.0))


def smoke():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("smoke() needs a GPU")
    from workloads.synthetic import ADAM, CONFIGS, PARAM_NAMES, make_layer_inputs
    from oracle.step import train_step
    from .harness import DeviceLayer

    cfg = CONFIGS["tiny"]
    inp = make_layer_inputs(cfg, seed=0)
    lay = DeviceLayer(cfg, inp, ADAM)
    lay.train_step(1)
    torch.cuda.synchronize()
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    z = {k: np.zeros_like(v) for k, v in p.items()}
    ref = train_step(cfg, p, z, z, inp["x"], inp["G"], inp["seq_lens"], 1, dict(ADAM, loss_scale=cfg["loss_scale"]))
    errs = {"y": rel_fro(lay.host(lay.y), ref["y"]), "dx": rel_fro(lay.host(lay.dx), ref["dx"])}
    for k in PARAM_NAMES:
        g_ref = ref["grads"][k].reshape(inp["params"][k].shape)
        errs["g_" + k] = rel_fro(lay.host(lay.grads[k]), g_ref)
        # Adam's first step is sign-like: where the true gradient vanishes (the key bias) its sign is
        # rounding noise on either side, so updated weights are compared where |g| is not negligible
        cond = np.abs(g_ref) > 1e-4 * np.sqrt(np.mean(g_ref ** 2))
        errs["w_" + k] = rel_fro(lay.host(lay.master[k])[cond], ref["params"][k][cond])
    worst_fwd = errs["y"]
    worst_bwd = max(v for k, v in errs.items() if k != "y")
    print("smoke: fwd rel err %.3e, worst grad/weight rel err %.3e" % (worst_fwd, worst_bwd))
    if not (worst_fwd <= 1e-5 and worst_bwd <= 1e-4):
        raise AssertionError("smoke parity failed: %r" % errs)
