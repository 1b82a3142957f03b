"""Whole-model parity on the GPU through the C ABI: embedding, layer stack,
MLM head with tied decoder and summed cross-entropy, backward and Adam, against
the fp64 oracle on identical seeded inputs.  Tolerances as for the layer."""
import numpy as np
import pytest
import torch

import paper_2303_04759_amd as raf
from paper_2303_04759_amd.harness import DeviceModel
from oracle import model as M
from oracle.layer import PARAM_NAMES
from workloads.synthetic import ADAM, MODEL_CONFIGS, make_model_inputs

from gpu_util import announce, check_update, host, rel_fro

pytestmark = pytest.mark.gpu

FWD_TOL = {0: 1e-5, 1: 2e-2}
BWD_TOL = {0: 1e-4, 1: 3e-2}


def oracle_state(inp):
    P = {k: v.astype(np.float64) for k, v in inp["P"].items()}
    layers = [{k: v.astype(np.float64) for k, v in lp.items()} for lp in inp["layers"]]
    zP = {k: np.zeros_like(v) for k, v in P.items()}
    zL = [{k: np.zeros_like(v) for k, v in lp.items()} for lp in layers]
    return P, layers, zP, zL


def run_model(cfg, seed):
    inp = make_model_inputs(cfg, seed=seed)
    mod = DeviceModel(cfg, inp, ADAM)
    prec = cfg["precision"]
    P, layers, zP, zL = oracle_state(inp)
    hyper = dict(ADAM, loss_scale=cfg["loss_scale"])
    before = {k: dict(w=host(mod.master[k]), m=host(mod.m[k]), v=host(mod.v[k])) for k in mod.master}
    mod.train_step(1)
    torch.cuda.synchronize()
    ref = M.model_train_step(cfg, P, layers, zP, zP, zL, zL, inp["ids"], inp["seq_lens"], inp["sel"], inp["labels"], 1,
                             hyper)
    # forward: final hidden state and loss
    e_x = rel_fro(host(mod.x[mod.L]), ref["xL"])
    assert e_x <= FWD_TOL[prec], ("xL", e_x)
    loss = float(mod.loss.item())
    assert abs(loss - ref["loss"]) <= FWD_TOL[prec] * abs(ref["loss"]), (loss, ref["loss"])
    worst, worst_dw = 0.0, 0.0
    V = cfg["vocab"]

    def check(key, name, g_ref, w_old, w_ref, m_ref, v_ref):
        nonlocal worst, worst_dw
        g_dev = host(mod.grads[key])
        g_ref = g_ref.reshape(g_dev.shape)
        if name == "word":
            assert (g_dev[V:] == 0).all()          # padded table rows take no gradient
        e = rel_fro(g_dev, g_ref)
        assert e <= BWD_TOL[prec], ("grad", key, e)
        worst = max(worst, e)
        # gradients, both moments, the optimizer kernel on every element, updated weights and the update itself
        # (the rules are check_update's); the word table's gradient is dominated by the few hundred rows the batch
        # uses, so fewer of its elements lie above the rounding floor
        dev = dict(w=host(mod.master[key]), m=host(mod.m[key]), v=host(mod.v[key]), g=g_dev)
        shape = dev["w"].shape
        e_dw = check_update(cfg, name, 1, prec, ADAM, before[key], dev,
                            dict(w_before=w_old.reshape(shape), w=w_ref.reshape(shape), m=m_ref.reshape(shape),
                                 v=v_ref.reshape(shape)), min_conditioned=0.5 if name == "word" else 0.9)
        worst_dw = max(worst_dw, e_dw)
        if mod.lowp[key] is not None:
            assert torch.equal(mod.lowp[key], mod.master[key].to(torch.bfloat16)), key
        if mod.lowp_t[key] is not None:
            assert torch.equal(mod.lowp_t[key], mod.lowp[key].t()), key

    for k in M.EMBED_PARAMS + M.HEAD_PARAMS:
        check(k, k, ref["grads"][k], P[k], ref["P"][k], ref["mP"][k], ref["vP"][k])
    for l in range(cfg["layers"]):
        for k in PARAM_NAMES:
            check((l, k), k, ref["layer_grads"][l][k], layers[l][k], ref["layers"][l][k], ref["mL"][l][k], ref["vL"][l][k])
    print("model parity: xL %.2e loss dev %.6g ref %.6g worst grad %.2e worst update %.2e n_sel %d" % (
        e_x, loss, ref["loss"], worst, worst_dw, len(inp["sel"])), flush=True)


def test_tiny_model_fp32():
    announce("model tiny fp32")
    run_model(MODEL_CONFIGS["tiny_model"], seed=0)


def test_tiny_model_duplicate_ids_and_odd_vocab_fp32():
    announce("model tiny fp32 small vocab")
    cfg = dict(MODEL_CONFIGS["tiny_model"], vocab=37, batch=3)      # heavy id collisions, vocab not a multiple of 8
    run_model(cfg, seed=1)


def test_small_model_bf16_amp():
    announce("model small bf16")
    cfg = dict(MODEL_CONFIGS["bert_base_12l_mlm"], batch=4, layers=2, hidden=256, heads=4, ffn=1024, vocab=5003,
               len_lo=40, len_hi=128)
    run_model(cfg, seed=2)


def test_bert_base_model_reduced_depth_bf16_amp():
    announce("model bert-base shapes, 3 layers, batch 16")
    cfg = dict(MODEL_CONFIGS["bert_base_12l_mlm"], batch=16, layers=3)
    run_model(cfg, seed=3)


def test_full_bert_base_12_layer_model_bf16_amp():
    announce("model full size: 12 layers, batch 64, vocab 30522")
    run_model(MODEL_CONFIGS["bert_base_12l_mlm"], seed=0)


def test_model_is_deterministic():
    announce("model determinism")
    cfg = dict(MODEL_CONFIGS["bert_base_12l_mlm"], batch=8, layers=2, vocab=2000)   # many duplicate ids
    inp = make_model_inputs(cfg, seed=4)
    a, b = DeviceModel(cfg, inp, ADAM), DeviceModel(cfg, inp, ADAM)
    a.train_step(1)
    b.train_step(1)
    torch.cuda.synchronize()
    assert torch.equal(a.loss, b.loss)
    for k in a.master:
        assert torch.equal(a.grads[k], b.grads[k]), k
        assert torch.equal(a.master[k], b.master[k]), k
