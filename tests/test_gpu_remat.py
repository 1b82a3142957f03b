"""Rematerialised layer steps on the GPU: a tensor that the forward pass does
not keep is regenerated in the backward pass by replaying its operator, so
every output of the step must be bit-identical to the step that kept it, and
the saved buffer must shrink by exactly the tensor's size.  One case also runs
the usual whole-step parity against the fp64 oracle with every bit set."""
import numpy as np
import pytest
import torch

import paper_2303_04759_amd as raf
from paper_2303_04759_amd.harness import DeviceLayer, DeviceModel
from workloads.synthetic import ADAM, CONFIGS, MODEL_CONFIGS, PARAM_NAMES, make_layer_inputs, make_model_inputs

from gpu_util import announce
from test_gpu_layer import run_and_compare

pytestmark = pytest.mark.gpu

QKV, CTX, FFN1 = raf.RAF_REMAT_QKV, raf.RAF_REMAT_CTX, raf.RAF_REMAT_FFN1


def rounded(n):
    return (n + 255) // 256 * 256


def expected_saving(cfg, mask):
    e = 2 if cfg["precision"] == raf.RAF_BF16_AMP else 4
    T, H, F = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["ffn"]
    s = 0
    if mask & QKV:
        s += rounded(3 * T * H * e)
    if mask & CTX:
        s += rounded(T * H * e)
    if mask & FFN1:
        s += 2 * rounded(T * F * e)
    return s


CASES = [
    # bf16, one-block attention, the headline shape
    ("bert_base", {}, [QKV, CTX, FFN1, QKV | CTX | FFN1]),
    # bf16, blockwise attention (row statistics saved), pre-LN, causal, ragged tiles
    ("bert_base", dict(batch=3, seq=160, hidden=320, heads=5, ffn=1056, pre_ln=1, causal=1, ln_eps=1e-5),
     [CTX, QKV | CTX, QKV | CTX | FFN1]),
    # fp32
    ("tiny", dict(batch=3, seq=96, hidden=192, heads=3, ffn=320, ln_eps=1e-5, dropout_p=0.1), [QKV, FFN1, QKV | FFN1]),
]


@pytest.mark.parametrize("name,over,masks", CASES)
def test_rematerialised_step_is_bit_identical(name, over, masks):
    cfg0 = dict(CONFIGS[name], **over)
    announce("remat %s %s" % (name, over))
    inp = make_layer_inputs(cfg0, seed=11, random_affine=True)
    base = DeviceLayer(cfg0, inp, ADAM)
    sv0, _ = raf.raf_layer_workspace(base.desc)
    for t in (1, 2):
        base.train_step(t)
    torch.cuda.synchronize()
    for mask in masks:
        cfg = dict(cfg0, remat=mask)
        lay = DeviceLayer(cfg, inp, ADAM)
        sv, _ = raf.raf_layer_workspace(lay.desc)
        assert sv0 - sv == expected_saving(cfg0, mask), (mask, sv0, sv)
        for t in (1, 2):
            lay.train_step(t)
        torch.cuda.synchronize()
        assert torch.equal(lay.y, base.y) and torch.equal(lay.dx, base.dx), mask
        assert torch.equal(lay.loss, base.loss)
        for k in PARAM_NAMES:
            assert torch.equal(lay.grads[k], base.grads[k]), (mask, k)
            assert torch.equal(lay.master[k], base.master[k]), (mask, k)


def test_rematerialised_step_against_oracle():
    announce("remat oracle parity")
    cfg = dict(CONFIGS["bert_base"], batch=3, seq=160, hidden=320, heads=5, ffn=1056, remat=QKV | CTX | FFN1)
    run_and_compare(cfg, seed=5, steps=2, random_affine=True, lens_override=[160, 77, 5])


def test_rematerialisation_argument_checks():
    announce("remat arg checks")
    cfg = dict(CONFIGS["tiny"])
    with pytest.raises(raf.RafError):
        raf.raf_layer_workspace(raf.make_desc(dict(cfg, remat=8)))       # unknown bit
    with pytest.raises(raf.RafError):
        raf.raf_layer_workspace(raf.make_desc(dict(cfg, remat=CTX)))     # fp32: attention is not on chip


def test_planned_model_step_is_bit_identical():
    """Layer stack planned under half of its liveness estimate: same loss, gradients and weights as the model that
    keeps everything, with the saved buffers smaller by what the plan drops."""
    announce("remat planned model")
    cfg = dict(MODEL_CONFIGS["bert_base_12l_mlm"], batch=8, layers=4, vocab=2000)
    inp = make_model_inputs(cfg, seed=6)
    desc = raf.make_desc(dict(cfg, layer_id=0))
    graph, own_l, own_b = raf.raf_layer_stack_graph(desc, cfg["layers"])
    peak = max(raf.raf_memory_profile(graph))
    masks, summ = raf.raf_layer_stack_remat(desc, cfg["layers"], peak // 2)
    assert summ["fits"] and summ["peak_after"] <= peak // 2 and any(masks)
    base, plan = DeviceModel(cfg, inp, ADAM), DeviceModel(cfg, inp, ADAM, remat=masks)
    dropped = sum(graph["tensors"][t]["bytes"] for t in range(len(own_l)) if own_b[t] & masks[own_l[t]])
    assert base.saved_bytes - plan.saved_bytes == dropped > 0
    for t in (1, 2):
        base.train_step(t)
        plan.train_step(t)
    torch.cuda.synchronize()
    assert torch.equal(base.loss, plan.loss)
    for k in base.master:
        assert torch.equal(base.grads[k], plan.grads[k]), k
        assert torch.equal(base.master[k], plan.master[k]), k


def test_rematerialised_step_replays_in_a_graph():
    """The rematerialising step is launches only (no memset or copy nodes): captured once and replayed, with eager
    work and synchronisations between the replays, every replay must leave what the eager kept-activations step
    leaves (same dropout step, weights restored before each replay)."""
    announce("remat graph replay")
    cfg0 = dict(CONFIGS["bert_base"], batch=4)
    inp = make_layer_inputs(cfg0, seed=8, random_affine=True)
    base = DeviceLayer(cfg0, inp, ADAM)
    lay = DeviceLayer(dict(cfg0, remat=QKV | CTX | FFN1), inp, ADAM)
    state0 = {k: (lay.master[k].clone(), None if lay.lowp[k] is None else lay.lowp[k].clone()) for k in PARAM_NAMES}
    base.train_step(3)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        lay.train_step(1, stream)                     # warm-up outside the graph
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            lay.train_step(3, stream)
        for _ in range(3):
            for k in PARAM_NAMES:                     # eager work between replays: back to the initial state
                lay.master[k].copy_(state0[k][0])
                if lay.lowp[k] is not None:
                    lay.lowp[k].copy_(state0[k][1])
                    lay.lowp_t[k].copy_(state0[k][1].t())
                lay.m[k].zero_()
                lay.v[k].zero_()
            lay.y.zero_()
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            assert torch.equal(lay.y, base.y) and torch.equal(lay.dx, base.dx) and torch.equal(lay.loss, base.loss)
            for k in PARAM_NAMES:
                assert torch.equal(lay.grads[k], base.grads[k]), k
                assert torch.equal(lay.master[k], base.master[k]), k
