"""Thin ctypes binding of libraf_mi355.so (see include/raf_mi355.h).

Argument marshalling only: every function has the name and the argument order
of its C entry point, takes torch tensors (or None) where the C call takes
device pointers, and raises RafError on a non-zero status.  There is no CPU
fallback: without the built library, or without a GPU for the calls that
launch kernels, it fails loudly.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libraf_mi355.so")

RAF_F32, RAF_BF16_AMP = 0, 1
RAF_OK, RAF_EINVAL, RAF_ENOTSUP, RAF_EWORKSPACE, RAF_EHIP = 0, -1, -2, -3, -4
RAF_LOSS_PARTIALS = 1024
RAF_NOALLOC_LN_BWD_PARTIAL_FLOATS = 256 * 3 * 1024
RAF_REMAT_QKV, RAF_REMAT_CTX, RAF_REMAT_FFN1 = 1, 2, 4
EPI_NONE, EPI_BIAS, EPI_BIAS_GELU, EPI_MUL_GELU_GRAD, EPI_ADD_RES, EPI_BIAS_GELU_DERIV, EPI_MUL_AUX = range(7)

PARAM_NAMES = ("w_qkv", "b_qkv", "w_o", "b_o", "ln1_g", "ln1_b",
               "w_1", "b_1", "w_2", "b_2", "ln2_g", "ln2_b")


class RafError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = "%s failed: %s (%d)" % (where, status_string(status), status)
        if status == RAF_EHIP:
            msg += ": " + last_hip_error()
        super().__init__(msg)


class LayerDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32),
                ("ffn", C.c_int32), ("pre_ln", C.c_int32), ("causal", C.c_int32), ("gelu_tanh", C.c_int32),
                ("precision", C.c_int32), ("ln_eps", C.c_float), ("dropout_p", C.c_double),
                ("seed", C.c_uint64), ("layer_id", C.c_uint32), ("remat", C.c_uint32)]


WT_NAMES = ("wt_qkv", "wt_o", "wt_1", "wt_2")      # optional transposed bf16 copies of the four matrices


class LayerTensors(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES + WT_NAMES + ("nonfinite",)]


class EmbedDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq", C.c_int32), ("hidden", C.c_int32), ("vocab", C.c_int32),
                ("max_pos", C.c_int32), ("precision", C.c_int32), ("ln_eps", C.c_float), ("layer_id", C.c_uint32),
                ("dropout_p", C.c_double), ("seed", C.c_uint64)]


class MlmDesc(C.Structure):
    _fields_ = [("rows", C.c_int32), ("hidden", C.c_int32), ("vocab", C.c_int32), ("n_sel", C.c_int32),
                ("precision", C.c_int32), ("gelu_tanh", C.c_int32), ("ln_eps", C.c_float), ("reserved", C.c_int32)]


MLM_NAMES = ("head_w", "head_b", "ln_g", "ln_b", "word", "dec_b")


class MlmTensors(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in MLM_NAMES]


class AdamTensor(C.Structure):
    _fields_ = [("master", C.c_void_p), ("grad", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("lowp", C.c_void_p), ("n", C.c_int64), ("lowp_t", C.c_void_p), ("rows", C.c_int32),
                ("cols", C.c_int32)]


class ScalerState(C.Structure):
    """Device-resident state of the dynamic loss scaler (raf_scaler_state): 32 bytes."""
    _fields_ = [("scale", C.c_float), ("inv_scale", C.c_float), ("good_steps", C.c_int32), ("found_inf", C.c_int32),
                ("t", C.c_int64), ("lr_over_bc1", C.c_float), ("inv_bc2", C.c_float)]


class OpGraph(C.Structure):
    _fields_ = [("n_ops", C.c_int32), ("n_tensors", C.c_int32), ("in_begin", C.POINTER(C.c_int32)),
                ("in_ids", C.POINTER(C.c_int32)), ("out_begin", C.POINTER(C.c_int32)),
                ("out_ids", C.POINTER(C.c_int32)), ("latency", C.POINTER(C.c_double)),
                ("bytes", C.POINTER(C.c_int64)), ("flags", C.POINTER(C.c_uint8))]


class RematSummary(C.Structure):
    _fields_ = [("peak_before", C.c_int64), ("peak_after", C.c_int64), ("fits", C.c_int32), ("reserved", C.c_int32),
                ("extra_latency", C.c_double)]


_lib = None

_SIGNATURES = {
    "raf_layer_workspace": (C.c_int, [C.POINTER(LayerDesc), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "raf_layer_fwd": (C.c_int, [C.POINTER(LayerDesc), C.POINTER(LayerTensors), C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    "raf_layer_bwd": (C.c_int, [C.POINTER(LayerDesc), C.POINTER(LayerTensors), C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_void_p, C.POINTER(LayerTensors), C.c_void_p, C.c_uint64, C.c_void_p]),
    "raf_layer_fwd_loss": (C.c_int, [C.POINTER(LayerDesc), C.POINTER(LayerTensors), C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_uint64, C.c_void_p]),
    "raf_loss_seed": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_void_p]),
    "raf_adam_table_bytes": (C.c_size_t, [C.POINTER(AdamTensor), C.c_int32]),
    "raf_adam_table_fill": (C.c_int, [C.POINTER(AdamTensor), C.c_int32, C.c_void_p, C.c_void_p]),
    "raf_adam_step_table": (C.c_int, [C.POINTER(AdamTensor), C.c_int32, C.c_void_p, C.c_double, C.c_double, C.c_double,
                                      C.c_double, C.c_double, C.c_int64, C.c_double, C.c_void_p, C.c_void_p]),
    "raf_adam_step": (C.c_int, [C.POINTER(AdamTensor), C.c_int32, C.c_double, C.c_double, C.c_double, C.c_double,
                                C.c_double, C.c_int64, C.c_double, C.c_void_p]),
    "raf_scaler_init": (C.c_int, [C.c_void_p, C.c_float, C.c_void_p]),
    "raf_loss_seed_scaled": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p]),
    "raf_grads_check": (C.c_int, [C.POINTER(AdamTensor), C.c_int32, C.c_void_p, C.c_void_p]),
    "raf_adam_step_scaled": (C.c_int, [C.POINTER(AdamTensor), C.c_int32, C.c_double, C.c_double, C.c_double,
                                       C.c_double, C.c_double, C.c_void_p, C.c_void_p]),
    "raf_scaler_update": (C.c_int, [C.c_void_p, C.c_float, C.c_float, C.c_int32, C.c_void_p]),
    "raf_debug_dropout_mask": (C.c_int, [C.POINTER(LayerDesc), C.c_int32, C.c_uint64, C.c_void_p, C.c_int64,
                                         C.c_void_p]),
    "raf_embed_workspace": (C.c_int, [C.POINTER(EmbedDesc), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "raf_embed_fwd": (C.c_int, [C.POINTER(EmbedDesc)] + [C.c_void_p] * 7 + [C.c_uint64, C.c_void_p]),
    "raf_embed_bwd": (C.c_int, [C.POINTER(EmbedDesc)] + [C.c_void_p] * 9 + [C.c_uint64, C.c_void_p]),
    "raf_mlm_workspace": (C.c_int, [C.POINTER(MlmDesc), C.POINTER(C.c_size_t)]),
    "raf_mlm_head_fwd_bwd": (C.c_int, [C.POINTER(MlmDesc), C.POINTER(MlmTensors), C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_float, C.c_void_p, C.c_void_p, C.POINTER(MlmTensors), C.c_void_p,
                                       C.c_void_p]),
    "raf_op_gemm": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                              C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float,
                              C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "raf_op_softmax_fwd": (C.c_int, [C.POINTER(LayerDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_uint64, C.c_void_p]),
    "raf_op_softmax_bwd": (C.c_int, [C.POINTER(LayerDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_float, C.c_void_p]),
    "raf_op_attention_fwd": (C.c_int, [C.POINTER(LayerDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_uint64, C.c_void_p]),
    "raf_op_attention_keep_bytes": (C.c_size_t, [C.POINTER(LayerDesc)]),
    "raf_op_attention_bwd": (C.c_int, [C.POINTER(LayerDesc)] + [C.c_void_p] * 8 + [C.c_uint64, C.c_void_p]),
    "raf_op_dropout_residual_ln_fwd": (C.c_int, [C.POINTER(LayerDesc), C.c_int32, C.c_int64, C.c_void_p, C.c_void_p,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                 C.c_void_p, C.c_uint64, C.c_void_p]),
    "raf_op_ln_bwd_partial_floats": (C.c_size_t, [C.c_int32, C.c_int64]),
    "raf_op_dropout_residual_ln_bwd": (C.c_int, [C.POINTER(LayerDesc), C.c_int32, C.c_int64] + [C.c_void_p] * 13 +
                                       [C.c_uint64, C.c_void_p]),
    "raf_op_dropout_residual_ln_bwd_noalloc": (C.c_int, [C.POINTER(LayerDesc), C.c_int32, C.c_int64] +
                                               [C.c_void_p] * 12 + [C.c_uint64, C.c_void_p]),
    "raf_memory_profile": (C.c_int, [C.POINTER(OpGraph), C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int64)]),
    "raf_schedule_ops": (C.c_int, [C.POINTER(OpGraph), C.POINTER(C.c_int32)]),
    "raf_remat_plan": (C.c_int, [C.POINTER(OpGraph), C.c_int64, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32),
                                 C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32),
                                 C.POINTER(RematSummary)]),
    "raf_layer_stack_graph": (C.c_int, [C.POINTER(LayerDesc), C.c_int32, C.POINTER(C.c_double), C.POINTER(OpGraph),
                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                        C.POINTER(C.c_uint8), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "raf_layer_stack_remat": (C.c_int, [C.POINTER(LayerDesc), C.c_int32, C.c_int64, C.POINTER(C.c_double),
                                        C.POINTER(C.c_uint32), C.POINTER(RematSummary)]),
    "raf_status_string": (C.c_char_p, [C.c_int]),
    "raf_last_hip_error": (C.c_char_p, []),
    "raf_version": (C.c_char_p, []),
}
EXPORTS = tuple(_SIGNATURES)


def load_library():
    """Load the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: run `python __graft_entry__.py` (build()) first; "
                           "there is no fallback path" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def status_string(status):
    return load_library().raf_status_string(int(status)).decode()


def last_hip_error():
    return load_library().raf_last_hip_error().decode()


def version():
    return load_library().raf_version().decode()


def _check(status, where):
    if status != RAF_OK:
        raise RafError(status, where)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_desc(cfg):
    """LayerDesc from a config dict (keys as in workloads.synthetic.CONFIGS)."""
    return LayerDesc(batch=cfg["batch"], seq=cfg["seq"], hidden=cfg["hidden"], heads=cfg["heads"], ffn=cfg["ffn"],
                     pre_ln=cfg.get("pre_ln", 0), causal=cfg.get("causal", 0), gelu_tanh=cfg.get("gelu_tanh", 0),
                     precision=cfg["precision"], ln_eps=cfg["ln_eps"], dropout_p=cfg["dropout_p"],
                     seed=cfg["seed"], layer_id=cfg.get("layer_id", 0), remat=cfg.get("remat", 0))


def make_tensors(d):
    """LayerTensors from a dict name -> tensor (the wt_* entries are optional)."""
    t = LayerTensors()
    for n in PARAM_NAMES:
        setattr(t, n, _ptr(d[n]))
    for n in WT_NAMES:
        setattr(t, n, _ptr(d.get(n)))
    t.nonfinite = _ptr(d.get("nonfinite"))   # a device address (int), a tensor or None
    return t


def raf_layer_workspace(desc):
    sv, sc = C.c_size_t(0), C.c_size_t(0)
    _check(load_library().raf_layer_workspace(C.byref(desc), C.byref(sv), C.byref(sc)), "raf_layer_workspace")
    return sv.value, sc.value


def raf_layer_fwd(desc, w, x, seq_lens, y, saved, scratch, step, stream=None):
    _check(load_library().raf_layer_fwd(C.byref(desc), C.byref(w), _ptr(x), _ptr(seq_lens), _ptr(y), _ptr(saved),
                                        _ptr(scratch), int(step), _stream(stream)), "raf_layer_fwd")


def raf_layer_fwd_loss(desc, w, x, seq_lens, y, G, loss_scale, state, loss_out, dy, saved, scratch, step, stream=None):
    _check(load_library().raf_layer_fwd_loss(C.byref(desc), C.byref(w), _ptr(x), _ptr(seq_lens), _ptr(y), _ptr(G),
                                             float(loss_scale), _ptr(state), _ptr(loss_out), _ptr(dy), _ptr(saved),
                                             _ptr(scratch), int(step), _stream(stream)), "raf_layer_fwd_loss")


def raf_layer_bwd(desc, w, x, dy, seq_lens, saved, dx, grads, scratch, step, stream=None):
    _check(load_library().raf_layer_bwd(C.byref(desc), C.byref(w), _ptr(x), _ptr(dy), _ptr(seq_lens), _ptr(saved),
                                        _ptr(dx), C.byref(grads), _ptr(scratch), int(step), _stream(stream)),
           "raf_layer_bwd")


def raf_loss_seed(precision, y, G, n, loss_scale, loss_out, dy, partial, stream=None):
    _check(load_library().raf_loss_seed(int(precision), _ptr(y), _ptr(G), int(n), float(loss_scale), _ptr(loss_out),
                                        _ptr(dy), _ptr(partial), _stream(stream)), "raf_loss_seed")


def raf_scaler_init(state, init_scale, stream=None):
    """state: a device buffer of at least ctypes.sizeof(ScalerState) bytes."""
    _check(load_library().raf_scaler_init(_ptr(state), float(init_scale), _stream(stream)), "raf_scaler_init")


def raf_loss_seed_scaled(precision, y, G, n, state, loss_out, dy, partial, stream=None):
    _check(load_library().raf_loss_seed_scaled(int(precision), _ptr(y), _ptr(G), int(n), _ptr(state), _ptr(loss_out),
                                               _ptr(dy), _ptr(partial), _stream(stream)), "raf_loss_seed_scaled")


def raf_grads_check(adam_list, count, state, stream=None):
    _check(load_library().raf_grads_check(adam_list, int(count), _ptr(state), _stream(stream)), "raf_grads_check")


def raf_adam_step_scaled(adam_list, count, lr, beta1, beta2, eps, weight_decay, state, stream=None):
    _check(load_library().raf_adam_step_scaled(adam_list, int(count), float(lr), float(beta1), float(beta2),
                                               float(eps), float(weight_decay), _ptr(state), _stream(stream)),
           "raf_adam_step_scaled")


def raf_scaler_update(state, growth_factor, backoff_factor, growth_interval, stream=None):
    _check(load_library().raf_scaler_update(_ptr(state), float(growth_factor), float(backoff_factor),
                                            int(growth_interval), _stream(stream)), "raf_scaler_update")


def read_scaler_state(state):
    """Copies the device state to the host (synchronises) and returns it as a dict."""
    raw = bytes(state[:C.sizeof(ScalerState)].cpu().numpy().tobytes())
    st = ScalerState.from_buffer_copy(raw)
    return dict(scale=st.scale, inv_scale=st.inv_scale, good_steps=st.good_steps, found_inf=st.found_inf, t=st.t)


def make_adam_list(entries):
    """entries: iterable of (master, grad, m, v, lowp_or_None[, lowp_t_or_None]) tensors -> (ctypes array, count).
    With lowp_t the master must be a matrix; its [rows, cols] are passed along."""
    entries = list(entries)
    arr = (AdamTensor * max(1, len(entries)))()
    for i, e in enumerate(entries):
        w, g, m, v, lowp = e[:5]
        lowp_t = e[5] if len(e) > 5 else None
        rows, cols = (w.shape[0], w.shape[1]) if lowp_t is not None else (0, 0)
        arr[i] = AdamTensor(_ptr(w), _ptr(g), _ptr(m), _ptr(v), _ptr(lowp), w.numel(), _ptr(lowp_t), rows, cols)
    return arr, len(entries)


def raf_adam_step(adam_list, count, lr, beta1, beta2, eps, weight_decay, t, inv_loss_scale, stream=None):
    _check(load_library().raf_adam_step(adam_list, int(count), float(lr), float(beta1), float(beta2), float(eps),
                                        float(weight_decay), int(t), float(inv_loss_scale), _stream(stream)),
           "raf_adam_step")


def raf_adam_table_bytes(adam_list, count):
    return int(load_library().raf_adam_table_bytes(adam_list, int(count)))


def raf_adam_table_fill(adam_list, count, table, stream=None):
    _check(load_library().raf_adam_table_fill(adam_list, int(count), _ptr(table), _stream(stream)), "raf_adam_table_fill")


def raf_adam_step_table(adam_list, count, table, lr, beta1, beta2, eps, weight_decay, t, inv_loss_scale, state=None,
                        stream=None):
    _check(load_library().raf_adam_step_table(adam_list, int(count), _ptr(table), float(lr), float(beta1), float(beta2),
                                              float(eps), float(weight_decay), int(t), float(inv_loss_scale),
                                              _ptr(state), _stream(stream)), "raf_adam_step_table")


def raf_debug_dropout_mask(desc, site, step, mask_out, n, stream=None):
    _check(load_library().raf_debug_dropout_mask(C.byref(desc), int(site), int(step), _ptr(mask_out), int(n),
                                                 _stream(stream)), "raf_debug_dropout_mask")


def raf_op_gemm(precision, M, N, K, a, lda, a_kmajor, b, ldb, b_kmajor, c, ldc, out_f32=0, alpha=1.0,
                epilogue=EPI_NONE, bias=None, aux=None, gelu_tanh=0, stream=None):
    _check(load_library().raf_op_gemm(int(precision), M, N, K, _ptr(a), lda, int(a_kmajor), _ptr(b), ldb,
                                      int(b_kmajor), _ptr(c), ldc, int(out_f32), float(alpha), int(epilogue),
                                      _ptr(bias), _ptr(aux), int(gelu_tanh), _stream(stream)), "raf_op_gemm")


def raf_op_softmax_fwd(desc, s, seq_lens, prob, prob_d, step, stream=None):
    _check(load_library().raf_op_softmax_fwd(C.byref(desc), _ptr(s), _ptr(seq_lens), _ptr(prob), _ptr(prob_d),
                                             int(step), _stream(stream)), "raf_op_softmax_fwd")


def raf_op_softmax_bwd(desc, prob, prob_d, dprob_d, ds, scale_out, stream=None):
    _check(load_library().raf_op_softmax_bwd(C.byref(desc), _ptr(prob), _ptr(prob_d), _ptr(dprob_d), _ptr(ds),
                                             float(scale_out), _stream(stream)), "raf_op_softmax_bwd")


def raf_op_attention_fwd(desc, qkv, seq_lens, ctx, lse, step, stream=None, keep=None):
    _check(load_library().raf_op_attention_fwd(C.byref(desc), _ptr(qkv), _ptr(seq_lens), _ptr(ctx), _ptr(lse),
                                               _ptr(keep), int(step), _stream(stream)), "raf_op_attention_fwd")


def raf_op_attention_keep_bytes(desc):
    return load_library().raf_op_attention_keep_bytes(C.byref(desc))


def raf_op_attention_bwd(desc, dctx, qkv, ctx, lse, seq_lens, dqkv, dvec, step, stream=None, keep=None):
    _check(load_library().raf_op_attention_bwd(C.byref(desc), _ptr(dctx), _ptr(qkv), _ptr(ctx), _ptr(lse), _ptr(keep),
                                               _ptr(seq_lens), _ptr(dqkv), _ptr(dvec), int(step), _stream(stream)),
           "raf_op_attention_bwd")


def raf_op_dropout_residual_ln_fwd(desc, site, rows, a, res, gamma, beta, out, z_out, mu, rstd, step, stream=None):
    _check(load_library().raf_op_dropout_residual_ln_fwd(C.byref(desc), int(site), int(rows), _ptr(a), _ptr(res),
                                                         _ptr(gamma), _ptr(beta), _ptr(out), _ptr(z_out), _ptr(mu),
                                                         _ptr(rstd), int(step), _stream(stream)),
           "raf_op_dropout_residual_ln_fwd")


def raf_op_ln_bwd_partial_floats(hidden, rows):
    return load_library().raf_op_ln_bwd_partial_floats(int(hidden), int(rows))


def raf_op_dropout_residual_ln_bwd(desc, site, rows, dout, dout2, z, mu, rstd, gamma, dres, dz, da, dgamma, dbeta,
                                   dbias, partial, step, stream=None):
    _check(load_library().raf_op_dropout_residual_ln_bwd(
        C.byref(desc), int(site), int(rows), _ptr(dout), _ptr(dout2), _ptr(z), _ptr(mu), _ptr(rstd), _ptr(gamma),
        _ptr(dres), _ptr(dz), _ptr(da), _ptr(dgamma), _ptr(dbeta), _ptr(dbias), _ptr(partial), int(step),
        _stream(stream)), "raf_op_dropout_residual_ln_bwd")


def raf_op_dropout_residual_ln_bwd_noalloc(desc, site, rows, dout, dout2, z, mu, rstd, gamma, dres, dz, da, dgamma,
                                           dbeta, dbias, step, stream=None):
    _check(load_library().raf_op_dropout_residual_ln_bwd_noalloc(
        C.byref(desc), int(site), int(rows), _ptr(dout), _ptr(dout2), _ptr(z), _ptr(mu), _ptr(rstd), _ptr(gamma),
        _ptr(dres), _ptr(dz), _ptr(da), _ptr(dgamma), _ptr(dbeta), _ptr(dbias), int(step), _stream(stream)),
        "raf_op_dropout_residual_ln_bwd_noalloc")


def make_embed_desc(cfg):
    return EmbedDesc(batch=cfg["batch"], seq=cfg["seq"], hidden=cfg["hidden"], vocab=cfg["vocab"],
                     max_pos=cfg["max_pos"], precision=cfg["precision"], ln_eps=cfg["ln_eps"],
                     layer_id=cfg["embed_layer_id"], dropout_p=cfg["dropout_p"], seed=cfg["seed"])


def make_mlm_desc(cfg, n_sel):
    return MlmDesc(rows=cfg["batch"] * cfg["seq"], hidden=cfg["hidden"], vocab=cfg["vocab"], n_sel=int(n_sel),
                   precision=cfg["precision"], gelu_tanh=cfg.get("gelu_tanh", 0), ln_eps=cfg["ln_eps"], reserved=0)


def make_mlm_tensors(d):
    t = MlmTensors()
    for n in MLM_NAMES:
        setattr(t, n, _ptr(d[n]))
    return t


def raf_embed_workspace(desc):
    sv, sc = C.c_size_t(0), C.c_size_t(0)
    _check(load_library().raf_embed_workspace(C.byref(desc), C.byref(sv), C.byref(sc)), "raf_embed_workspace")
    return sv.value, sc.value


def raf_embed_fwd(desc, ids, word, pos, gamma, beta, x0, saved, step, stream=None):
    _check(load_library().raf_embed_fwd(C.byref(desc), _ptr(ids), _ptr(word), _ptr(pos), _ptr(gamma), _ptr(beta),
                                        _ptr(x0), _ptr(saved), int(step), _stream(stream)), "raf_embed_fwd")


def raf_embed_bwd(desc, ids, dx0, saved, gamma, dword, dpos, dgamma, dbeta, scratch, step, stream=None):
    _check(load_library().raf_embed_bwd(C.byref(desc), _ptr(ids), _ptr(dx0), _ptr(saved), _ptr(gamma), _ptr(dword),
                                        _ptr(dpos), _ptr(dgamma), _ptr(dbeta), _ptr(scratch), int(step),
                                        _stream(stream)), "raf_embed_bwd")


def raf_mlm_workspace(desc):
    sc = C.c_size_t(0)
    _check(load_library().raf_mlm_workspace(C.byref(desc), C.byref(sc)), "raf_mlm_workspace")
    return sc.value


def raf_mlm_head_fwd_bwd(desc, w, x, sel, labels, loss_scale, loss_out, dx, grads, scratch, stream=None):
    _check(load_library().raf_mlm_head_fwd_bwd(C.byref(desc), C.byref(w), _ptr(x), _ptr(sel), _ptr(labels),
                                               float(loss_scale), _ptr(loss_out), _ptr(dx), C.byref(grads),
                                               _ptr(scratch), _stream(stream)), "raf_mlm_head_fwd_bwd")


# ---- memory passes on an operator list (host only).  A graph is a dict(ops=[dict(inputs, outputs, latency)],
# tensors=[dict(bytes, remat_ok, persistent)]); the wrappers only lay it out in the C structure.
RAF_TENSOR_REMAT_OK, RAF_TENSOR_PERSISTENT = 1, 2


class _GraphArrays:
    def __init__(self, graph):
        ops, tensors = graph["ops"], graph["tensors"]
        in_begin, in_ids, out_begin, out_ids = [0], [], [0], []
        for op in ops:
            in_ids += list(op["inputs"])
            out_ids += list(op["outputs"])
            in_begin.append(len(in_ids))
            out_begin.append(len(out_ids))
        self.keep = [(C.c_int32 * len(in_begin))(*in_begin), (C.c_int32 * max(1, len(in_ids)))(*in_ids),
                     (C.c_int32 * len(out_begin))(*out_begin), (C.c_int32 * max(1, len(out_ids)))(*out_ids),
                     (C.c_double * max(1, len(ops)))(*[float(op["latency"]) for op in ops]),
                     (C.c_int64 * max(1, len(tensors)))(*[int(t["bytes"]) for t in tensors]),
                     (C.c_uint8 * max(1, len(tensors)))(*[(RAF_TENSOR_REMAT_OK if t["remat_ok"] else 0) |
                                                          (RAF_TENSOR_PERSISTENT if t["persistent"] else 0)
                                                          for t in tensors])]
        k = self.keep
        self.c = OpGraph(len(ops), len(tensors), k[0], k[1], k[2], k[3], k[4], k[5], k[6])


def raf_memory_profile(graph, sequence=None):
    g = _GraphArrays(graph)
    n = len(graph["ops"]) if sequence is None else len(sequence)
    out = (C.c_int64 * max(1, n))()
    seq = None if sequence is None else (C.c_int32 * max(1, n))(*sequence)
    _check(load_library().raf_memory_profile(C.byref(g.c), seq, n, out), "raf_memory_profile")
    return list(out[:n])


def raf_schedule_ops(graph):
    g = _GraphArrays(graph)
    n = len(graph["ops"])
    out = (C.c_int32 * max(1, n))()
    _check(load_library().raf_schedule_ops(C.byref(g.c), out), "raf_schedule_ops")
    return list(out[:n])


def raf_remat_plan(graph, budget):
    g = _GraphArrays(graph)
    cap = 9 * len(graph["ops"]) + 8
    seq, ev_t, ev_p = (C.c_int32 * cap)(), (C.c_int32 * cap)(), (C.c_int32 * cap)()
    n_seq, n_ev, summ = C.c_int32(), C.c_int32(), RematSummary()
    _check(load_library().raf_remat_plan(C.byref(g.c), int(budget), seq, cap, C.byref(n_seq), ev_t, ev_p, cap,
                                         C.byref(n_ev), C.byref(summ)), "raf_remat_plan")
    return dict(sequence=list(seq[:n_seq.value]), evicted=list(zip(ev_t[:n_ev.value], ev_p[:n_ev.value])),
                peak_before=summ.peak_before, peak_after=summ.peak_after, fits=bool(summ.fits),
                extra_latency=summ.extra_latency)


def raf_layer_stack_graph(desc, layers, replay_us=None):
    """The library's operator list of a layer stack as a graph dict, plus owner_layer / owner_bit per tensor."""
    lib = load_library()
    rep = None if replay_us is None else (C.c_double * 3)(*replay_us)
    sizes, n_in, n_out = OpGraph(), C.c_int32(), C.c_int32()
    null32 = C.POINTER(C.c_int32)()
    _check(lib.raf_layer_stack_graph(C.byref(desc), layers, rep, C.byref(sizes), null32, null32, null32, null32, None,
                                     None, None, null32, null32, C.byref(n_in), C.byref(n_out)),
           "raf_layer_stack_graph")
    no, nt = sizes.n_ops, sizes.n_tensors
    in_begin, in_ids = (C.c_int32 * (no + 1))(), (C.c_int32 * max(1, n_in.value))()
    out_begin, out_ids = (C.c_int32 * (no + 1))(), (C.c_int32 * max(1, n_out.value))()
    lat, byt, flg = (C.c_double * no)(), (C.c_int64 * nt)(), (C.c_uint8 * nt)()
    own_l, own_b = (C.c_int32 * nt)(), (C.c_int32 * nt)()
    _check(lib.raf_layer_stack_graph(C.byref(desc), layers, rep, C.byref(sizes), in_begin, in_ids, out_begin, out_ids,
                                     lat, byt, flg, own_l, own_b, C.byref(n_in), C.byref(n_out)),
           "raf_layer_stack_graph")
    ops = [dict(inputs=list(in_ids[in_begin[k]:in_begin[k + 1]]), outputs=list(out_ids[out_begin[k]:out_begin[k + 1]]),
                latency=lat[k]) for k in range(no)]
    tensors = [dict(bytes=byt[t], remat_ok=bool(flg[t] & RAF_TENSOR_REMAT_OK),
                    persistent=bool(flg[t] & RAF_TENSOR_PERSISTENT)) for t in range(nt)]
    return dict(ops=ops, tensors=tensors), list(own_l), list(own_b)


def raf_layer_stack_remat(desc, layers, budget, replay_us=None):
    rep = None if replay_us is None else (C.c_double * 3)(*replay_us)
    masks, summ = (C.c_uint32 * max(1, layers))(), RematSummary()
    _check(load_library().raf_layer_stack_remat(C.byref(desc), layers, int(budget), rep, masks, C.byref(summ)),
           "raf_layer_stack_remat")
    return list(masks[:layers]), dict(peak_before=summ.peak_before, peak_after=summ.peak_after, fits=bool(summ.fits),
                             extra_latency=summ.extra_latency)
