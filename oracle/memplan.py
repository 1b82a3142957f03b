"""Memory planning passes of the paper on an operator list: liveness-based
memory estimate, operator scheduling by the p - c rule (Section 3.1.4) and
rematerialisation under a byte budget (Section 3.1.5).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Pure Python, written for
small graphs; shares no code with the library's planner.

A graph is a dict
    ops:     list of dict(inputs=[tensor ids], outputs=[tensor ids], latency=float)
             in execution order; a tensor is the output of at most one op
    tensors: list of dict(bytes=int, remat_ok=bool, persistent=bool)
A tensor that no op produces is external (a parameter, an input): it is
resident all the time.  `persistent` marks results that must outlive the list
(gradients, the output).

An execution sequence is a list of items: k >= 0 runs op k; -1 - t replays the
producer of tensor t, regenerating t only.

Readings of the paper taken here (it states the ingredients, not the formulas):
  * memory at an execution point = bytes of every tensor alive while that
    item runs (its inputs and outputs included); a tensor is alive from the
    item that materialises it to the last item that this materialisation
    serves, i.e. the last use before the next materialisation of the same
    tensor;
  * the cost of regenerating a tensor is latency(producer) * (uses still to
    come) / bytes: cheap, rarely needed, large tensors go first.  Ties go to
    the larger tensor, then to the lower id;
  * the regenerating replay is placed directly before the tensor's next use,
    and replays exactly one operator: a tensor qualifies only if every input
    of its producer is still alive at that place (or external), so that no
    liveness is stretched back over points already planned; a tensor that the
    very next item reads is left alone;
  * p - c rule as list scheduling: among the operators whose inputs are
    computed, the one with the smallest p - c runs next (p = bytes it
    produces, c = bytes it lets go: inputs whose other consumers have all
    run), ties in the given order.
"""


def _item_io(graph, producer, item):
    if item >= 0:
        op = graph["ops"][item]
        return op["inputs"], op["outputs"]
    t = -1 - item
    return graph["ops"][producer[t]]["inputs"], [t]


def producers(graph):
    prod = [-1] * len(graph["tensors"])
    for k, op in enumerate(graph["ops"]):
        for t in op["outputs"]:
            assert prod[t] == -1, "tensor %d has two producers" % t
            prod[t] = k
    return prod


def intervals(graph, sequence=None):
    """For every tensor the list of (first, last) positions over which it is alive."""
    seq = list(range(len(graph["ops"]))) if sequence is None else list(sequence)
    prod = producers(graph)
    n_t = len(graph["tensors"])
    events = [[] for _ in range(n_t)]     # (position, kind): kind 0 = materialised, 1 = used
    for pos, item in enumerate(seq):
        ins, outs = _item_io(graph, prod, item)
        for t in set(ins):
            events[t].append((pos, 1))
        for t in set(outs):
            events[t].append((pos, 0))
    out = []
    last = len(seq) - 1
    for t in range(n_t):
        if prod[t] < 0:
            out.append([(0, last)] if last >= 0 else [])
            continue
        iv = []
        cur = None
        for pos, kind in sorted(events[t]):
            if kind == 0:
                if cur is not None:
                    iv.append(tuple(cur))
                cur = [pos, pos]
            else:
                assert cur is not None and cur[0] < pos, "tensor %d used at %d before it exists" % (t, pos)
                cur[1] = pos
        if cur is not None:
            if graph["tensors"][t]["persistent"]:
                cur[1] = last
            iv.append(tuple(cur))
        out.append(iv)
    return out


def memory_profile(graph, sequence=None):
    seq = list(range(len(graph["ops"]))) if sequence is None else list(sequence)
    mem = [0] * len(seq)
    for t, iv in enumerate(intervals(graph, seq)):
        b = graph["tensors"][t]["bytes"]
        for a, e in iv:
            for pos in range(a, e + 1):
                mem[pos] += b
    return mem


def peak_memory(graph, sequence=None):
    m = memory_profile(graph, sequence)
    return max(m) if m else 0


def sequence_latency(graph, sequence):
    prod = producers(graph)
    total = 0.0
    for item in sequence:
        total += graph["ops"][item if item >= 0 else prod[-1 - item]]["latency"]
    return total


def remat_plan(graph, budget):
    """Walks the execution order; wherever the estimate exceeds `budget`, evicts
    alive tensors in ascending cost until it fits (or nothing is left to evict)
    and inserts their replays.  Returns dict(sequence, evicted=[(tensor, position)],
    peak_before, peak_after, fits, extra_latency)."""
    prod = producers(graph)
    seq = list(range(len(graph["ops"])))
    peak_before = peak_memory(graph, seq)
    cap = 8 * len(seq) + 8            # replays never outnumber this in a sane graph; a hard stop all the same
    evicted = []
    fits = True
    i = 0
    while i < len(seq):
        while True:
            mem = memory_profile(graph, seq)
            if mem[i] <= budget:
                break
            if len(seq) >= cap:
                fits = False
                break
            iv = intervals(graph, seq)
            ins, outs = _item_io(graph, prod, seq[i])
            busy = set(ins) | set(outs)
            best = None
            for t, info in enumerate(graph["tensors"]):
                if not info["remat_ok"] or prod[t] < 0 or t in busy or info["bytes"] <= 0:
                    continue
                cover = [(a, e) for (a, e) in iv[t] if a < i <= e]
                if not cover:
                    continue
                # uses still to come that this materialisation serves
                uses = []
                for pos in range(i + 1, cover[0][1] + 1):
                    pin, _ = _item_io(graph, prod, seq[pos])
                    if t in pin:
                        uses.append(pos)
                if not uses:
                    continue           # alive only because it is persistent
                j = uses[0]            # the replay would go in front of the item now at j
                if j == i + 1:
                    continue           # read by the very next item: nothing to gain
                if not all(prod[s] < 0 or any(a < j <= e for (a, e) in iv[s]) for s in graph["ops"][prod[t]]["inputs"]):
                    continue
                trial = seq[:j] + [-1 - t] + seq[j:]
                cost = graph["ops"][prod[t]]["latency"] * len(uses) / info["bytes"]
                key = (cost, -info["bytes"], t)
                if best is None or key < best[0]:
                    best = (key, t, trial)
            if best is None:
                fits = False
                break
            evicted.append((best[1], i))
            seq = best[2]
        i += 1
    return dict(sequence=seq, evicted=evicted, peak_before=peak_before, peak_after=peak_memory(graph, seq),
                fits=fits, extra_latency=sequence_latency(graph, seq) - sequence_latency(graph, range(len(graph["ops"]))))


def schedule_ops(graph):
    """Execution order by the p - c rule."""
    ops, tensors = graph["ops"], graph["tensors"]
    prod = producers(graph)
    consumers_left = [0] * len(tensors)
    for op in ops:
        for t in set(op["inputs"]):
            consumers_left[t] += 1
    done = [False] * len(ops)
    computed = [prod[t] < 0 for t in range(len(tensors))]
    order = []
    for _ in range(len(ops)):
        best = None
        for k, op in enumerate(ops):
            if done[k] or not all(computed[t] for t in op["inputs"]):
                continue
            p = sum(tensors[t]["bytes"] for t in set(op["outputs"]))
            c = sum(tensors[t]["bytes"] for t in set(op["inputs"])
                    if prod[t] >= 0 and not tensors[t]["persistent"] and consumers_left[t] == 1)
            # an output that nothing reads and that need not outlive the list is let go at once
            c += sum(tensors[t]["bytes"] for t in set(op["outputs"])
                     if consumers_left[t] == 0 and not tensors[t]["persistent"])
            if best is None or p - c < best[0]:
                best = (p - c, k)
        assert best is not None, "cycle in the operator list"
        k = best[1]
        done[k] = True
        order.append(k)
        for t in set(ops[k]["inputs"]):
            consumers_left[t] -= 1
        for t in ops[k]["outputs"]:
            computed[t] = True
    return order


def apply_order(graph, order):
    """The same graph with its ops listed in `order` (tensor ids unchanged)."""
    return dict(ops=[graph["ops"][k] for k in order], tensors=graph["tensors"])
