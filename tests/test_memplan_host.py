"""The library's host-side memory passes (liveness estimate, p - c scheduling,
rematerialisation plan; Sections 3.1.4 and 3.1.5) against the oracle's, exact
on every output; and the layer-stack planner against the oracle run on the
operator list the library exports.  Host code only: runs without a GPU."""
import random

import pytest

import paper_2303_04759_amd as raf
from oracle import memplan
from workloads.synthetic import CONFIGS

from test_oracle_memplan import CHAIN, OP, T, random_graph


def same_plan(graph, budget):
    got = raf.raf_remat_plan(graph, budget)
    ref = memplan.remat_plan(graph, budget)
    for k in ("sequence", "evicted", "peak_before", "peak_after", "fits", "extra_latency"):
        assert got[k] == ref[k], (k, budget, got[k], ref[k])
    assert raf.raf_memory_profile(graph, got["sequence"]) == memplan.memory_profile(graph, ref["sequence"])
    return got


def test_chain():
    assert raf.raf_memory_profile(CHAIN) == [5, 11, 13, 15, 15, 9, 5]
    for budget in (15, 12, 10, 0):
        same_plan(CHAIN, budget)
    assert raf.raf_schedule_ops(CHAIN) == list(range(7))


@pytest.mark.parametrize("seed", range(40))
def test_random_graphs(seed):
    rng = random.Random(1000 + seed)
    g = random_graph(rng, rng.randint(1, 30), fanin=3)
    assert raf.raf_memory_profile(g) == memplan.memory_profile(g)
    assert raf.raf_schedule_ops(g) == memplan.schedule_ops(g)
    peak = memplan.peak_memory(g)
    for frac in (1.0, 0.9, 0.8, 0.65, 0.5, 0.3):
        same_plan(g, int(peak * frac))
    # the two passes in the paper's order: schedule first, then plan on the new order
    g2 = memplan.apply_order(g, memplan.schedule_ops(g))
    same_plan(g2, int(memplan.peak_memory(g2) * 0.7))


def test_empty_and_malformed_graphs():
    empty = dict(ops=[], tensors=[])
    assert raf.raf_memory_profile(empty) == [] and raf.raf_schedule_ops(empty) == []
    r = raf.raf_remat_plan(empty, 0)
    assert r["sequence"] == [] and r["fits"] and r["peak_before"] == 0
    two_producers = dict(tensors=[T(1, False), T(1)], ops=[OP([0], [1]), OP([0], [1])])
    read_before_write = dict(tensors=[T(1, False), T(1), T(1)], ops=[OP([2], [1]), OP([0], [2])])
    bad_id = dict(tensors=[T(1, False)], ops=[OP([0], [3])])
    negative = dict(tensors=[T(-1, False), T(1)], ops=[OP([0], [1])])
    for g in (two_producers, read_before_write, bad_id, negative):
        with pytest.raises(raf.RafError):
            raf.raf_remat_plan(g, 10)
    # the scheduler may repair an order (it only needs a DAG) but not a cycle
    assert raf.raf_schedule_ops(read_before_write) == memplan.schedule_ops(read_before_write) == [1, 0]
    cycle = dict(tensors=[T(1), T(1)], ops=[OP([1], [0]), OP([0], [1])])
    with pytest.raises(raf.RafError):
        raf.raf_schedule_ops(cycle)
    # sequences that read a tensor nobody has written yet, or name an item that does not exist
    for seq in ([1, 0], [0, -4], [0, 7], [0, -1], [0, -100]):
        with pytest.raises(raf.RafError):
            raf.raf_memory_profile(CHAIN, seq)


STACKS = [("bert_base", {}, 12), ("gpt2_medium", {}, 4), ("bert_large", {}, 3),
          ("tiny", {}, 5), ("bert_base", dict(pre_ln=1), 2)]


@pytest.mark.parametrize("name,over,layers", STACKS)
def test_layer_stack_plan(name, over, layers):
    cfg = dict(CONFIGS[name], **over)
    desc = raf.make_desc(cfg)
    replay = [17.0, 11.0, 25.0]
    graph, own_l, own_b = raf.raf_layer_stack_graph(desc, layers, replay)
    # the list is executable as given and the droppable tensors have the sizes by which the saved buffer shrinks
    profile = memplan.memory_profile(graph)
    assert raf.raf_memory_profile(graph) == profile
    sv0, _ = raf.raf_layer_workspace(desc)
    seen = set()
    for t, (l, b) in enumerate(zip(own_l, own_b)):
        if b:
            assert graph["tensors"][t]["remat_ok"] and 0 <= l < layers
            sv, _ = raf.raf_layer_workspace(raf.make_desc(dict(cfg, remat=b)))
            assert sv0 - sv == graph["tensors"][t]["bytes"], (t, b)
            assert graph["ops"][memplan.producers(graph)[t]]["latency"] == replay[{1: 0, 2: 1, 4: 2}[b]]
            seen.add((l, b))
        else:
            assert not graph["tensors"][t]["remat_ok"]
    bits = {1, 4} | ({2} if cfg["precision"] == raf.RAF_BF16_AMP else set())
    assert seen == {(l, b) for l in range(layers) for b in bits}
    peak = max(profile)
    for frac in (1.0, 0.85, 0.7, 0.55, 0.4, 0.2):
        budget = int(peak * frac)
        masks, summ = raf.raf_layer_stack_remat(desc, layers, budget, replay)
        ref = memplan.remat_plan(graph, budget)
        want = [0] * layers
        for t, _ in ref["evicted"]:
            want[own_l[t]] |= own_b[t]
        assert masks == want, (frac, masks, want)
        assert (summ["peak_before"], summ["peak_after"], summ["fits"], summ["extra_latency"]) == \
               (ref["peak_before"], ref["peak_after"], ref["fits"], ref["extra_latency"])
        if frac == 1.0:
            assert masks == [0] * layers and summ["fits"]
    # the estimate without measured latencies is positive and ordered like the work
    g2, _, _ = raf.raf_layer_stack_graph(desc, 1)
    lat = sorted(op["latency"] for op in g2["ops"] if op["latency"] > 0)
    assert len(lat) == 3 and lat[0] > 0


@pytest.mark.parametrize("name,layers", [("bert_base", 12), ("gpt2_medium", 4)])
def test_scheduling_rule_on_the_layer_stack(name, layers):
    """The p - c rule applied to the library's own launch order: same order from library and oracle, still
    executable, and no higher in peak (the peak sits at the turn from forward to backward, which no order moves)."""
    graph, _, _ = raf.raf_layer_stack_graph(raf.make_desc(CONFIGS[name]), layers)
    order = raf.raf_schedule_ops(graph)
    assert order == memplan.schedule_ops(graph) and sorted(order) == list(range(len(order)))
    moved = memplan.apply_order(graph, order)
    assert max(raf.raf_memory_profile(moved)) <= max(raf.raf_memory_profile(graph))
    # forward launches keep their places: nothing there releases memory early
    n_fwd = next(k for k, op in enumerate(graph["ops"]) if any(graph["tensors"][t]["persistent"] for t in op["outputs"]))
    first_moved = next((i for i, k in enumerate(order) if i != k), len(order))
    assert first_moved > n_fwd // 2


def test_plan_capacity_error_reports_needed_lengths():
    """Too small an output capacity: RAF_EWORKSPACE, with the needed lengths and the summary still written."""
    import ctypes as C
    lib = raf.load_library()
    g = raf._GraphArrays(CHAIN)
    seq, ev_t, ev_p = (C.c_int32 * 4)(), (C.c_int32 * 4)(), (C.c_int32 * 4)()
    n_seq, n_ev, summ = C.c_int32(), C.c_int32(), raf.RematSummary()
    rc = lib.raf_remat_plan(C.byref(g.c), 12, seq, 4, C.byref(n_seq), ev_t, ev_p, 4, C.byref(n_ev), C.byref(summ))
    assert rc == raf.RAF_EWORKSPACE
    assert (n_seq.value, n_ev.value, summ.peak_before, summ.peak_after, summ.fits) == (8, 1, 15, 11, 1)
    assert lib.raf_remat_plan(None, 12, seq, 4, C.byref(n_seq), ev_t, ev_p, 4, C.byref(n_ev), C.byref(summ)) == raf.RAF_EINVAL
    assert lib.raf_remat_plan(C.byref(g.c), 12, seq, 4, None, ev_t, ev_p, 4, C.byref(n_ev), C.byref(summ)) == raf.RAF_EINVAL


def test_layer_stack_argument_checks():
    desc = raf.make_desc(CONFIGS["tiny"])
    for layers in (0, -1, 513):
        with pytest.raises(raf.RafError):
            raf.raf_layer_stack_remat(desc, layers, 1 << 30)
        with pytest.raises(raf.RafError):
            raf.raf_layer_stack_graph(desc, layers)
    with pytest.raises(raf.RafError):
        raf.raf_layer_stack_remat(desc, 2, 1 << 30, [1.0, -1.0, 1.0])      # negative latency
