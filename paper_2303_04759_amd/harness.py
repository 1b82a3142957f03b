"""Device-side plumbing for tests, the smoke check and the benchmark: owns the
torch buffers of one layer and calls the C ABI in step order.  No arithmetic
of the method happens here; torch is used for allocation, host<->device
copies and dtype conversion of inputs only."""
import numpy as np
import torch

from . import (PARAM_NAMES, RAF_BF16_AMP, RAF_LOSS_PARTIALS, make_adam_list, make_desc, make_tensors,
               raf_adam_step, raf_adam_step_scaled, raf_grads_check, raf_layer_bwd, raf_layer_fwd,
               raf_layer_fwd_loss, raf_layer_workspace, raf_loss_seed, raf_loss_seed_scaled, raf_scaler_update)


class DeviceLayer:
    def __init__(self, cfg, inputs, adam, device="cuda:0", scratch=None, transposed_copies=True):
        """transposed_copies: keep [in,out] bf16 copies of the matrices (written by raf_adam_step) and hand them to
        raf_layer_bwd; False: the backward pass transposes the weights itself on every call."""
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
        # transposed bf16 copies of the four matrices for the input-gradient products, kept up to date by the optimizer
        self.lowp_t = {k: (self.lowp[k].t().contiguous() if (self.lowp[k] is not None and transposed_copies) else None)
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
        wd = {k: (self.lowp[k] if self.lowp[k] is not None else self.master[k]) for k in PARAM_NAMES}
        wd.update({"wt" + k[1:]: self.lowp_t[k] for k in PARAM_NAMES if self.lowp_t[k] is not None})
        self.w_struct = make_tensors(wd)
        self.g_struct = make_tensors(self.grads)
        self.adam_list, self.adam_count = make_adam_list(
            (self.master[k], self.grads[k], self.m[k], self.v[k], self.lowp[k], self.lowp_t[k]) for k in PARAM_NAMES)

    # one call per C entry point, in step order
    def fwd(self, step, stream=None):
        raf_layer_fwd(self.desc, self.w_struct, self.x, self.seq_lens, self.y, self.saved, self.scratch, step, stream)

    def fwd_loss(self, step, stream=None, state=None):
        """forward and loss seed in one call (the kernel that writes y forms dy and the loss partial sums)"""
        raf_layer_fwd_loss(self.desc, self.w_struct, self.x, self.seq_lens, self.y, self.G, self.cfg["loss_scale"], state,
                           self.loss, self.dy, self.saved, self.scratch, step, stream)

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

    def train_step_dynamic(self, step, state, scaler, stream=None, fused_loss=True, epilogue_check=True):
        """The same pass under the dynamic loss scaler: every decision (scale, skip, Adam's step count) is taken on
        the device from `state` (a device byte buffer initialised with raf_scaler_init).  `step` only numbers the
        dropout masks.  epilogue_check: the backward call raises state.found_inf itself (raf_layer_tensors.nonfinite)
        instead of a raf_grads_check pass over the gradients afterwards."""
        from . import ScalerState
        a = self.adam
        g_struct = self.g_struct
        if epilogue_check:
            g_struct = make_tensors(dict(self.grads, nonfinite=state.data_ptr() + ScalerState.found_inf.offset))
        if fused_loss:
            self.fwd_loss(step, stream, state)
        else:
            self.fwd(step, stream)
            raf_loss_seed_scaled(self.cfg["precision"], self.y, self.G, self.y.numel(), state, self.loss, self.dy,
                                 self.partial, stream)
        raf_layer_bwd(self.desc, self.w_struct, self.x, self.dy, self.seq_lens, self.saved, self.dx, g_struct,
                      self.scratch, step, stream)
        if not epilogue_check:
            raf_grads_check(self.adam_list, self.adam_count, state, stream)
        raf_adam_step_scaled(self.adam_list, self.adam_count, a["lr"], a["beta1"], a["beta2"], a["eps"],
                             a.get("weight_decay", 0.0), state, stream)
        raf_scaler_update(state, scaler["growth_factor"], scaler["backoff_factor"], scaler["growth_interval"], stream)

    def train_step(self, t, stream=None, fused_loss=True):
        """forward, loss seed, backward, Adam: one pass of the whole hot path.  fused_loss=False takes the loss seed
        with its own call (raf_loss_seed) instead of inside the forward call."""
        if fused_loss:
            self.fwd_loss(t, stream)
        else:
            self.fwd(t, stream)
            self.loss_seed(stream)
        self.bwd(t, stream)
        self.adam_step(t, stream)

    def host(self, t):
        return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


class DeviceModel:
    """Embedding + L layers + MLM head on the device: buffers and the step-ordered C-ABI calls."""

    EMBED = ("word", "pos", "emb_ln_g", "emb_ln_b")
    HEAD = ("head_w", "head_b", "head_ln_g", "head_ln_b", "dec_b")

    def __init__(self, cfg, inputs, adam, device="cuda:0", remat=None):
        """remat: per-layer raf_layer_desc.remat values (as raf_layer_stack_remat returns them), or None."""
        from . import (make_embed_desc, make_mlm_desc, make_mlm_tensors, raf_embed_workspace, raf_mlm_workspace)
        if not torch.cuda.is_available():
            raise RuntimeError("DeviceModel needs a GPU; there is no CPU path")
        self.cfg, self.adam = dict(cfg), dict(adam)
        dev = self.dev = torch.device(device)
        self.amp = cfg["precision"] == RAF_BF16_AMP
        cd = self.cdtype = torch.bfloat16 if self.amp else torch.float32
        B, S, H = cfg["batch"], cfg["seq"], cfg["hidden"]
        self.T, self.H, self.L = B * S, H, cfg["layers"]
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).contiguous()
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev).contiguous()
        self.ids, self.seq_lens = i32(inputs["ids"].reshape(-1)), i32(inputs["seq_lens"])
        self.sel, self.labels = i32(inputs["sel"]), i32(inputs["labels"])
        self.n_sel = int(self.sel.numel())
        # parameters: master (f32), optional bf16 copy for matrices/tables, Adam state, gradients
        self.master, self.lowp, self.lowp_t, self.m, self.v, self.grads = {}, {}, {}, {}, {}, {}
        matrices = {"word", "pos", "head_w"}
        for k in self.EMBED + self.HEAD:
            self._add_param(k, f32(inputs["P"][k]), k in matrices)
        self.layer_keys = []
        for l, lp in enumerate(inputs["layers"]):
            for k in PARAM_NAMES:
                self._add_param((l, k), f32(lp[k]), k.startswith("w_"))
            self.layer_keys.append([(l, k) for k in PARAM_NAMES])
        # descriptors and workspaces
        self.edesc = make_embed_desc(cfg)
        self.mdesc = make_mlm_desc(cfg, self.n_sel)
        self.ldesc = []
        for l in range(self.L):
            c = dict(cfg)
            c["layer_id"] = cfg["layer_id_base"] + l
            c["remat"] = int(remat[l]) if remat is not None else 0
            self.ldesc.append(make_desc(c))
        esv, esc = raf_embed_workspace(self.edesc)
        lws = [raf_layer_workspace(d) for d in self.ldesc]
        msc = raf_mlm_workspace(self.mdesc)
        u8 = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device=dev)
        self.esaved, self.scratch = u8(esv), u8(max([esc, msc] + [sc for _, sc in lws]))
        self.lsaved = [u8(sv) for sv, _ in lws]
        self.saved_bytes = sum(sv for sv, _ in lws)
        act = lambda: torch.empty(self.T, H, dtype=cd, device=dev)
        self.x = [act() for _ in range(self.L + 1)]       # x[0] = embedding output, x[l+1] = layer l output
        self.dx = [act(), act()]                          # ping-pong gradient buffers
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        w = lambda k: self.lowp[k] if self.lowp[k] is not None else self.master[k]
        self.lw = []
        for l in range(self.L):
            wd = {k: w((l, k)) for k in PARAM_NAMES}
            wd.update({"wt" + k[1:]: self.lowp_t[(l, k)] for k in PARAM_NAMES if self.lowp_t[(l, k)] is not None})
            self.lw.append(make_tensors(wd))
        self.lg = [make_tensors({k: self.grads[(l, k)] for k in PARAM_NAMES}) for l in range(self.L)]
        names = dict(head_w="head_w", head_b="head_b", ln_g="head_ln_g", ln_b="head_ln_b", word="word", dec_b="dec_b")
        self.mw = make_mlm_tensors({a: w(b) for a, b in names.items()})
        self.mg = make_mlm_tensors({a: self.grads[b] for a, b in names.items()})
        keys = list(self.master)
        self.adam_list, self.adam_count = make_adam_list(
            (self.master[k], self.grads[k], self.m[k], self.v[k], self.lowp[k], self.lowp_t[k]) for k in keys)
        # the optimizer's tensor table in device memory: all tensors of the model in one launch
        from . import raf_adam_table_bytes, raf_adam_table_fill
        self.adam_table = torch.empty(raf_adam_table_bytes(self.adam_list, self.adam_count), dtype=torch.uint8, device=dev)
        raf_adam_table_fill(self.adam_list, self.adam_count, self.adam_table)
        torch.cuda.synchronize()

    def _add_param(self, key, master, has_lowp):
        self.master[key] = master
        self.lowp[key] = master.to(torch.bfloat16) if (self.amp and has_lowp) else None
        # layer matrices also keep the transposed copy the input-gradient products read (written by the optimizer)
        layer_matrix = isinstance(key, tuple) and self.lowp[key] is not None
        self.lowp_t[key] = self.lowp[key].t().contiguous() if layer_matrix else None
        self.m[key] = torch.zeros_like(master)
        self.v[key] = torch.zeros_like(master)
        self.grads[key] = torch.zeros_like(master)

    def _w(self, k):
        return self.lowp[k] if self.lowp[k] is not None else self.master[k]

    def forward(self, step, stream=None):
        from . import raf_embed_fwd
        raf_embed_fwd(self.edesc, self.ids, self._w("word"), self._w("pos"), self.master["emb_ln_g"],
                      self.master["emb_ln_b"], self.x[0], self.esaved, step, stream)
        for l in range(self.L):
            raf_layer_fwd(self.ldesc[l], self.lw[l], self.x[l], self.seq_lens, self.x[l + 1], self.lsaved[l],
                          self.scratch, step, stream)

    def head_and_backward(self, step, stream=None):
        from . import raf_embed_bwd, raf_mlm_head_fwd_bwd
        cur = 0
        raf_mlm_head_fwd_bwd(self.mdesc, self.mw, self.x[self.L], self.sel, self.labels, self.cfg["loss_scale"],
                             self.loss, self.dx[cur], self.mg, self.scratch, stream)
        for l in reversed(range(self.L)):
            raf_layer_bwd(self.ldesc[l], self.lw[l], self.x[l], self.dx[cur], self.seq_lens, self.lsaved[l],
                          self.dx[cur ^ 1], self.lg[l], self.scratch, step, stream)
            cur ^= 1
        raf_embed_bwd(self.edesc, self.ids, self.dx[cur], self.esaved, self.master["emb_ln_g"], self.grads["word"],
                      self.grads["pos"], self.grads["emb_ln_g"], self.grads["emb_ln_b"], self.scratch, step, stream)

    def adam_step(self, t, stream=None, one_launch=True):
        from . import raf_adam_step_table
        a = self.adam
        if one_launch:
            raf_adam_step_table(self.adam_list, self.adam_count, self.adam_table, a["lr"], a["beta1"], a["beta2"],
                                a["eps"], a.get("weight_decay", 0.0), t, 1.0 / self.cfg["loss_scale"], None, stream)
        else:
            raf_adam_step(self.adam_list, self.adam_count, a["lr"], a["beta1"], a["beta2"], a["eps"],
                          a.get("weight_decay", 0.0), t, 1.0 / self.cfg["loss_scale"], stream)

    def train_step(self, t, stream=None):
        self.forward(t, stream)
        self.head_and_backward(t, stream)
        self.adam_step(t, stream)

    def host(self, t):
        return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)
