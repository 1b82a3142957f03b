"""Helpers for the GPU parity tests."""
import sys

import numpy as np
import torch

from oracle.adam import adam_step


def announce(*what):
    """Name the case before any GPU work, flushed, so a lost box still tells which case ran."""
    print("[gpu-case]", *what, flush=True)
    sys.stdout.flush()


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (den if den > 0 else 1.0))


BWD_TOL = {0: 1e-4, 1: 3e-2}      # relative Frobenius, gradients and updates: fp32 mode / bf16 AMP


def comparable(cfg, k, shape):
    """All elements except the key block of b_qkv.  The key-bias gradient vanishes identically (a constant added to
    every key of a row cancels in the softmax), so Adam's sign-like step there is decided by rounding noise on either
    side; it is the one place excluded from the updated-weight comparisons."""
    sel = np.ones(shape, dtype=bool)
    if k == "b_qkv":
        sel[cfg["hidden"]:2 * cfg["hidden"]] = False
    return sel


def check_update(cfg, k, t, prec, adam, before, dev, ref, min_conditioned=0.9):
    """One parameter tensor after one optimizer step.  before/dev: device values (w, m, v[, g]) before and after the
    step; ref: the oracle's free-running trajectory (w_before, w, m, v).  Returns the update's relative error."""
    tol = BWD_TOL[prec]
    ls = cfg["loss_scale"]
    # (1) the optimizer kernel itself, on every element of every tensor: the oracle's rule applied to the device's own
    # inputs.  The update is compared as w_after - w_before, element by element; the bound is fp32 rounding of the
    # master weight (an ulp of |w| against a step of about lr), the rounding of the derived constants, and 1e-4 of
    # lr for cancellation in the first moment (b1*m and (1-b1)*g of opposite sign).
    w1, m1, v1 = adam_step(before["w"], dev["g"], before["m"], before["v"], t, adam["lr"], adam["beta1"], adam["beta2"],
                           adam["eps"], adam.get("weight_decay", 0.0), 1.0 / ls)
    dw_k, dw_o = dev["w"] - before["w"], w1 - before["w"]
    bound = 2.0 ** -23 * np.maximum(np.abs(before["w"]), np.abs(dev["w"])) + 2e-5 * np.abs(dw_o) + 1e-4 * adam["lr"]
    assert (np.abs(dw_k - dw_o) <= bound).all(), ("adam kernel dw", k, t, float(np.abs(dw_k - dw_o).max()))
    assert rel_fro(dev["m"], m1) <= 1e-5 and rel_fro(dev["v"], v1) <= 1e-5, ("adam kernel m/v", k, t)
    # (2) against the oracle's trajectory.  Moments are smooth in g: whole tensors, at the stated tolerance.
    if np.linalg.norm(ref["m"]) > 1e-12:
        e_m, e_v = rel_fro(dev["m"], ref["m"]), rel_fro(dev["v"], ref["v"])
        assert e_m <= tol and e_v <= tol, ("m/v", k, t, e_m, e_v)
    sel = comparable(cfg, k, dev["w"].shape)
    # updated weights, whole tensor (key-bias block excepted) where |w| >> lr: matrices and LayerNorm gains
    if k.startswith("w_") or k.endswith("_g") or k in ("word", "pos", "head_w"):
        e_w = rel_fro(dev["w"][sel], ref["w"][sel])
        assert e_w <= tol, ("w", k, t, e_w)
    # the update itself.  Adam's step lr*m_hat/(sqrt(v_hat)+eps) is sign-like at small t: an element whose first
    # moment is below the rounding error of the gradient takes a step of either sign on either side.  Elements with
    # |m| above tol * rms(m) - at least 90 % of every tensor - must agree to the tolerance; all must respect the
    # step bound.  rms is taken where the rounding error of a gradient element scales: per row of a weight (one
    # output feature; table rows differ by orders of magnitude), per block of b_qkv (query/key gradients are much
    # smaller than value gradients).  Vectors that start at zero (biases, LayerNorm shifts) have w_after = update,
    # so this is their updated-weight check.
    m_full = ref["m"]

    def scale(a):      # rms of `a` per weight row / per b_qkv block / per vector
        if a.ndim == 2:
            return np.sqrt(np.mean(a ** 2, axis=1, keepdims=True))
        if k == "b_qkv":
            return np.repeat(np.sqrt(np.mean(a.reshape(3, -1) ** 2, axis=1)), a.size // 3)
        return np.sqrt(np.mean(a ** 2))
    # ... and never below four times the rounding error the first moment actually shows there (deep stacks bring it
    # close to the tolerance; the fraction floor below keeps that from excusing a wrong gradient)
    cond = (np.abs(m_full) > np.maximum(tol * scale(m_full), 4.0 * scale(dev["m"] - m_full)))[sel]
    m_ref = m_full[sel]
    cond |= (m_ref == 0) & (dev["m"][sel] == 0)          # rows no sample touched: no step on either side
    assert cond.mean() >= min_conditioned, ("conditioned fraction", k, t, cond.mean())
    dw_dev, dw_ref = (dev["w"] - before["w"])[sel], (ref["w"] - ref["w_before"])[sel]
    e_dw = rel_fro(dw_dev[cond], dw_ref[cond])
    assert e_dw <= (2e-2 if prec == 0 else tol), ("dw", k, t, e_dw)
    # |step| <= lr * max(1, (1-b1)/sqrt(1-b2)) / (1-b1^t) ... <= 3.2 lr for t <= 3 with these betas
    assert np.abs(dev["w"] - before["w"]).max() <= 4.0 * adam["lr"], ("step bound", k, t)
    return e_dw


def to_dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(dtype).contiguous()


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def cdtype(precision):
    return torch.bfloat16 if precision == 1 else torch.float32
