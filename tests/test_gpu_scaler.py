"""Dynamic loss scaling on the GPU through the C ABI against the oracle: the same sequence of steps, some with a
non-finite loss gradient, must give the same skip decisions, the same scale and step counters exactly, untouched
weights on skipped steps, and updated weights within the layer tolerances on the others."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2303_04759_amd as raf
from paper_2303_04759_amd.harness import DeviceLayer
from oracle import scaler as SC
from workloads.synthetic import ADAM, CONFIGS, PARAM_NAMES, make_layer_inputs

from gpu_util import announce, host, rel_fro

pytestmark = pytest.mark.gpu

SCALER = dict(growth_factor=2.0, backoff_factor=0.5, growth_interval=2)
BWD_TOL = {0: 1e-4, 1: 3e-2}


@pytest.mark.parametrize("precision,poison", [(0, "inf"), (1, "inf"), (1, "nan")])
def test_dynamic_scaler_sequence(precision, poison):
    announce("dynamic scaler", precision, poison)
    cfg = dict(CONFIGS["tiny"], precision=precision, dropout_p=0.1)
    inp = make_layer_inputs(cfg, seed=5)
    lay = DeviceLayer(cfg, inp, ADAM)
    state = torch.zeros(C.sizeof(raf.ScalerState), dtype=torch.uint8, device="cuda")
    raf.raf_scaler_init(state, 512.0)
    G_good = lay.G.clone()
    G_bad = lay.G.clone()
    G_bad.view(-1)[7] = float(poison)
    G_ref_bad = np.array(inp["G"], dtype=np.float64)
    G_ref_bad.reshape(-1)[7] = float(poison)

    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    m = {k: np.zeros_like(v) for k, v in p.items()}
    v = {k: np.zeros_like(v) for k, v in p.items()}
    st = SC.scaler_new(512.0)
    pattern = [0, 1, 0, 0, 1, 1, 0, 0]                      # growth after two good steps, two overflows in a row
    for step, bad in enumerate(pattern, start=1):
        lay.G.copy_(G_bad if bad else G_good)
        before = {k: host(lay.master[k]) for k in PARAM_NAMES}
        m_before = {k: host(lay.m[k]) for k in PARAM_NAMES}
        lay.train_step_dynamic(step, state, SCALER)
        torch.cuda.synchronize()
        ref = SC.train_step_dynamic(cfg, p, m, v, inp["x"], G_ref_bad if bad else inp["G"], inp["seq_lens"], st, ADAM,
                                    SCALER, step)
        got = raf.read_scaler_state(state)
        assert ref["found_inf"] == bool(bad)
        assert got["scale"] == ref["state"]["scale"] and got["good_steps"] == ref["state"]["good_steps"]
        assert got["t"] == ref["state"]["t"] and got["found_inf"] == 0
        assert got["inv_scale"] == 1.0 / got["scale"]
        for k in PARAM_NAMES:
            if bad:      # skipped: bit-identical state
                assert np.array_equal(host(lay.master[k]), before[k]), k
                assert np.array_equal(host(lay.m[k]), m_before[k]), k
            else:
                g_ref = ref["grads"][k].reshape(p[k].shape)
                assert rel_fro(host(lay.grads[k]), g_ref) <= BWD_TOL[precision], (k, step)
                # one Adam step moves a weight by at most about lr; both sides must have moved from the same start
                assert np.abs(host(lay.master[k]) - ref["params"][k]).max() <= 2.5 * ADAM["lr"] * (1 + step), (k, step)
        p, m, v, st = ref["params"], ref["m"], ref["v"], ref["state"]
    assert st["t"] == 5 and st["scale"] == 256.0


@pytest.mark.parametrize("name,epilogue_check", [("bert_base", True), ("bert_base", False), ("bert_large", True)])
def test_non_finite_test_in_the_backward_epilogues_at_full_size(name, epilogue_check):
    """Weight gradients and all reductions leave raf_layer_bwd in one launch, which also raises found_inf; the
    decisions must be those of the separate pass over the gradients (raf_grads_check).  BERT-base shape: fewer
    weight-gradient tiles than CUs; BERT-large shape: more, the reductions ride in the last round of tiles."""
    announce("dynamic scaler, non-finite test in the epilogues", name, epilogue_check)
    cfg = CONFIGS[name]
    inp = make_layer_inputs(cfg, seed=7)
    lay = DeviceLayer(cfg, inp, ADAM)
    state = torch.zeros(C.sizeof(raf.ScalerState), dtype=torch.uint8, device="cuda")
    raf.raf_scaler_init(state, 1024.0)
    G_good = lay.G.clone()
    expect = SC.scaler_new(1024.0)
    for step, bad in enumerate(("", "", "inf", "", "nan", ""), start=1):
        lay.G.copy_(G_good)
        if bad in ("inf", "nan"):
            lay.G.view(-1)[step * 1000 + 3] = float(bad)
        w0 = {k: lay.master[k].clone() for k in PARAM_NAMES}
        lay.train_step_dynamic(step, state, SCALER, epilogue_check=epilogue_check)
        torch.cuda.synchronize()
        overflow = not all(bool(torch.isfinite(lay.grads[k]).all()) for k in PARAM_NAMES)
        if bad in ("inf", "nan"):
            assert overflow
        expect = SC.scaler_update(expect, overflow, **SCALER)
        got = raf.read_scaler_state(state)
        assert (got["scale"], got["good_steps"], got["t"], got["found_inf"]) == (
            expect["scale"], expect["good_steps"], expect["t"], 0), (step, bad, got, expect)
        changed = any(not torch.equal(w0[k], lay.master[k]) for k in PARAM_NAMES)
        assert changed == (not overflow), (step, bad)


def test_dynamic_step_replays_in_a_graph():
    """The whole dynamically scaled step is captured once; replays take their decisions from the device state."""
    announce("dynamic scaler graph")
    cfg = dict(CONFIGS["tiny"], precision=1, dropout_p=0.1)
    inp = make_layer_inputs(cfg, seed=6)
    lay = DeviceLayer(cfg, inp, ADAM)
    state = torch.zeros(C.sizeof(raf.ScalerState), dtype=torch.uint8, device="cuda")
    raf.raf_scaler_init(state, 128.0)
    stream = torch.cuda.Stream()
    G_good = lay.G.clone()
    with torch.cuda.stream(stream):
        lay.train_step_dynamic(1, state, SCALER, stream)          # warm-up outside the graph
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            lay.train_step_dynamic(2, state, SCALER, stream)
        expect = SC.scaler_update(SC.scaler_new(128.0), False, **SCALER)
        for bad in (0, 1, 0, 0, 1):
            lay.G.copy_(G_good)
            if bad:
                lay.G.view(-1)[3] = float("inf")
            w0 = {k: lay.master[k].clone() for k in PARAM_NAMES}
            graph.replay()
            stream.synchronize()
            expect = SC.scaler_update(expect, bool(bad), **SCALER)
            got = raf.read_scaler_state(state)
            assert (got["scale"], got["good_steps"], got["t"]) == (expect["scale"], expect["good_steps"], expect["t"])
            changed = any(not torch.equal(w0[k], lay.master[k]) for k in PARAM_NAMES)
            assert changed == (not bad)
