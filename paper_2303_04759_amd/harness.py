"""Device-side plumbing for tests, the smoke check and the benchmark: owns the
torch buffers of one layer and calls the C ABI in step order.  No arithmetic
of the method happens here; torch is used for allocation, host<->device
copies and dtype conversion of inputs only."""
import numpy as np
import torch

from . import (PARAM_NAMES, RAF_BF16_AMP, RAF_LOSS_PARTIALS, make_adam_list, make_desc, make_tensors,
               raf_adam_step, raf_layer_bwd, raf_layer_fwd, raf_layer_workspace, raf_loss_seed)


class DeviceLayer:
    def __init__(self, cfg, inputs, adam, device="cuda:0", scratch=None):
        if not torch.cuda.is_available():
            raise RuntimeError("DeviceLayer needs a GPU; there is no CPU path")
        self.cfg = dict(cfg)
        self.adam = dict(adam)
        self.dev = torch.device(device)
        self.desc = make_desc(cfg)
        self.amp = cfg["precision"] == RAF_BF16_AMP
        self.cdtype = torch.bfloat16 if self.amp else torch.float32
        B, S, H = cfg["batch"], cfg["seq"], cfg["hidden"]
        self.T, self.H = B * S, H
        dev = self.dev
        self.x = torch.from_numpy(inputs["x"]).to(dev).reshape(self.T, H).to(self.cdtype).contiguous()
        self.G = torch.from_numpy(inputs["G"]).to(dev).reshape(self.T, H).to(self.cdtype).contiguous()
        self.seq_lens = None
        if inputs.get("seq_lens") is not None:
            self.seq_lens = torch.from_numpy(np.asarray(inputs["seq_lens"], dtype=np.int32)).to(dev)
        self.master = {k: torch.from_numpy(np.asarray(inputs["params"][k], dtype=np.float32)).to(dev).contiguous()
                       for k in PARAM_NAMES}
        self.lowp = {k: (self.master[k].to(torch.bfloat16) if (self.amp and k.startswith("w_")) else None)
                     for k in PARAM_NAMES}
        self.m = {k: torch.zeros_like(v) for k, v in self.master.items()}
        self.v = {k: torch.zeros_like(v) for k, v in self.master.items()}
        self.grads = {k: torch.empty_like(v) for k, v in self.master.items()}
        sv, sc = raf_layer_workspace(self.desc)
        self.saved = torch.empty(sv, dtype=torch.uint8, device=dev)
        self.scratch = scratch if scratch is not None else torch.empty(sc, dtype=torch.uint8, device=dev)
        assert self.scratch.numel() >= sc
        self.y = torch.empty(self.T, H, dtype=self.cdtype, device=dev)
        self.dy = torch.empty_like(self.y)
        self.dx = torch.empty_like(self.y)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.partial = torch.empty(RAF_LOSS_PARTIALS, dtype=torch.float32, device=dev)
        self.w_struct = make_tensors({k: (self.lowp[k] if self.lowp[k] is not None else self.master[k])
                                      for k in PARAM_NAMES})
        self.g_struct = make_tensors(self.grads)
        self.adam_list, self.adam_count = make_adam_list(
            (self.master[k], self.grads[k], self.m[k], self.v[k], self.lowp[k]) for k in PARAM_NAMES)

    # one call per C entry point, in step order
    def fwd(self, step, stream=None):
        raf_layer_fwd(self.desc, self.w_struct, self.x, self.seq_lens, self.y, self.saved, self.scratch, step, stream)

    def loss_seed(self, stream=None):
        raf_loss_seed(self.cfg["precision"], self.y, self.G, self.y.numel(), self.cfg["loss_scale"], self.loss,
                      self.dy, self.partial, stream)

    def bwd(self, step, stream=None):
        raf_layer_bwd(self.desc, self.w_struct, self.x, self.dy, self.seq_lens, self.saved, self.dx, self.g_struct,
                      self.scratch, step, stream)

    def adam_step(self, t, stream=None):
        a = self.adam
        raf_adam_step(self.adam_list, self.adam_count, a["lr"], a["beta1"], a["beta2"], a["eps"],
                      a.get("weight_decay", 0.0), t, 1.0 / self.cfg["loss_scale"], stream)

    def train_step(self, t, stream=None):
        """forward, loss seed, backward, Adam: one pass of the whole hot path."""
        self.fwd(t, stream)
        self.loss_seed(stream)
        self.bwd(t, stream)
        self.adam_step(t, stream)

    def host(self, t):
        return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)
