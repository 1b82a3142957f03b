"""Helpers for the GPU parity tests."""
import sys

import numpy as np
import torch


def announce(*what):
    """Name the case before any GPU work, flushed, so a lost box still tells which case ran."""
    print("[gpu-case]", *what, flush=True)
    sys.stdout.flush()


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (den if den > 0 else 1.0))


def to_dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(dtype).contiguous()


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def cdtype(precision):
    return torch.bfloat16 if precision == 1 else torch.float32
