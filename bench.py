#!/usr/bin/env python3
"""Benchmark of the layer training step on one MI355X.

One "step" is one pass of the whole hot path over one batch: forward, loss
seed, backward, fused Adam of a BERT-base-shaped layer in bf16 AMP (inputs
resident in HBM).  Prints ONE JSON line with the metric, a roofline object for
the dominant kernel and the CPU oracle timed on the host cores.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert_base] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")


def profiled_traffic(workload, kernel_key):
    """HBM bytes per launch of a kernel as measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs, each scaled
    by what the counter reads for a plain copy of known size): read from the machine-readable lines
    '# traffic_bytes_per_launch <kernel key> <bytes>' of profiles/bench_<workload>_hbm_traffic.txt, which the same
    counter runs wrote.  None when that workload or kernel has no counter profile."""
    try:
        for line in open(os.path.join(PROFILES, "bench_%s_hbm_traffic.txt" % workload)):
            f = line.split()
            if len(f) == 4 and f[0] == "#" and f[1] == "traffic_bytes_per_launch" and f[2] == kernel_key:
                return float(f[3])
    except OSError:
        pass
    return None


def gemm_launches(cfg):
    """The dense contractions of one step as (name, M, N, K, a_kmajor, b_kmajor, out_f32, epilogue, batch).

    In bf16 AMP the input-gradient products read K-major transposed weight copies, so they have the same
    layout as the forward products."""
    B, S, H, F, nh = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["ffn"], cfg["heads"]
    T = B * S
    z = B * nh
    return [
        ("qkv_fwd", T, 3 * H, H, 1, 1, 0, 1, 1), ("scores_fwd", S, S, 64, 1, 1, 0, 0, z),
        ("context_fwd", S, 64, S, 1, 0, 0, 0, z), ("out_fwd", T, H, H, 1, 1, 0, 1, 1),
        ("ffn1_fwd", T, F, H, 1, 1, 0, 2, 1), ("ffn2_fwd", T, H, F, 1, 1, 0, 1, 1),
        ("ffn2_wgrad", H, F, T, 0, 0, 1, 0, 1), ("ffn2_dgrad", T, F, H, 1, 1, 0, 3, 1),
        ("ffn1_wgrad", F, H, T, 0, 0, 1, 0, 1), ("ffn1_dgrad", T, H, F, 1, 1, 0, 0, 1),
        ("out_wgrad", H, H, T, 0, 0, 1, 0, 1), ("out_dgrad", T, H, H, 1, 1, 0, 0, 1),
        ("dprob", S, S, 64, 1, 1, 0, 0, z), ("dv", S, 64, S, 0, 0, 0, 0, z),
        ("dq", S, 64, S, 1, 0, 0, 0, z), ("dk", S, 64, S, 0, 0, 0, 0, z),
        ("qkv_wgrad", 3 * H, H, T, 0, 0, 1, 0, 1), ("qkv_dgrad", T, H, 3 * H, 1, 1, 0, 4, 1),
    ]


# ------------------------------------------------------------------ per-kernel report --
def launch_work(cfg, n_params_matrix, n_params_vector):
    """Algorithmic work of every launch class of one bf16 layer step, in launch order per class:
    class -> list of (operator label, bound, flops or bytes).  Bytes are the tensors an operator has to read and write
    once (what SURVEY-style accounting calls algorithmic), not what an implementation happens to move."""
    B, S, H, F = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["ffn"]
    T = B * S
    e = 2 if cfg["precision"] == 1 else 4
    TH, TF = T * H * e, T * F * e
    pre = bool(cfg["pre_ln"])
    fl = lambda M, N, K: 2.0 * M * N * K
    w = {}
    w["gemm"] = [("qkv_fwd", "mfma", fl(T, 3 * H, H)), ("out_fwd", "mfma", fl(T, H, H)),
                 ("ffn1_fwd+gelu", "mfma", fl(T, F, H)), ("ffn2_fwd", "mfma", fl(T, H, F)),
                 ("ffn2_dgrad*gelu'", "mfma", fl(T, F, H)), ("ffn1_dgrad", "mfma", fl(T, H, F)),
                 ("out_dgrad", "mfma", fl(T, H, H)), ("qkv_dgrad+res", "mfma", fl(T, H, 3 * H))]
    w["wgrad_group"] = [("4 weight gradients (+ bias/LayerNorm column sums on idle CUs)", "mfma",
                         fl(3 * H, H, T) + fl(H, H, T) + fl(F, H, T) + fl(H, F, T))]
    if pre:
        w["ln_fwd"] = [("ln1", "hbm", 2 * TH), ("dropout+residual+ln2", "hbm", 4 * TH),
                       ("dropout+residual + loss seed", "hbm", 5 * TH)]
        w["ln_bwd"] = [("dropout3 adjoint", "hbm", 2 * TH), ("ln2 adjoint+residual", "hbm", 5 * TH),
                       ("ln1 adjoint+residual", "hbm", 4 * TH)]
    else:
        # the last forward kernel also takes the loss seed (reads G, writes dy): raf_layer_fwd_loss
        w["ln_fwd"] = [("dropout+residual+ln1", "hbm", 4 * TH), ("dropout+residual+ln2 + loss seed", "hbm", 6 * TH)]
        w["ln_bwd"] = [("ln2 adjoint", "hbm", 4 * TH), ("ln1 adjoint (two incoming gradients)", "hbm", 5 * TH)]
    w["attn_fwd"] = [("scores+mask+softmax+dropout+context", "hbm", 4 * TH)]
    w["attn_bwd"] = [("attention adjoint (dQ,dK,dV)", "hbm", 7 * TH)]
    w["attn_bwd_dq"] = [("attention adjoint dQ", "hbm", 6 * TH)]
    w["attn_bwd_dkv"] = [("attention adjoint dK,dV", "hbm", 6 * TH)]
    w["transpose"] = [("4 weight transposes", "hbm", 2 * 2 * n_params_matrix)]
    w["loss_seed"] = [("loss seed", "hbm", 3 * TH)]      # only when the loss seed is taken by its own call
    w["loss_final"] = [("loss partial sums", "hbm", 4096)]
    # per matrix element: g 4 r; m, v, master 12 r + 12 w; bf16 copy 2 w; transposed bf16 copy 2 w
    w["adam"] = [("fused Adam, 12 tensors (+ transposed bf16 copies)", "hbm", 32 * n_params_matrix + 28 * n_params_vector)]
    w["colsum"] = [("bias-gradient column sums", "hbm", TF + 3 * TH)]
    w["reduce"] = [("second stage of column sums", "hbm", None)]
    return w


KERNEL_CLASSES = (("gemm_bf16_spec_kernel", "wgrad_group"), ("gemm_bf16_group_kernel", "wgrad_group"),
                  ("gemm_bf16_", "gemm"), ("gemm_f32", "gemm"), ("attn_fwd_fused", "attn_fwd"),
                  ("attn_flash_fwd", "attn_fwd"), ("attn_bwd_full", "attn_bwd"), ("attn_flash_dq", "attn_bwd_dq"),
                  ("attn_flash_dkv", "attn_bwd_dkv"), ("ln_fwd_kernel", "ln_fwd"), ("ln_bwd_", "ln_bwd"),
                  ("transpose_bf16", "transpose"), ("loss_seed", "loss_seed"), ("loss_final", "loss_final"),
                  ("adam_kernel", "adam"), ("colsum_kernel", "colsum"), ("reduce_partials", "reduce"))


def short_kernel_name(name):
    """Readable kernel name without the argument list.  rocprofv3 leaves names with a bf16 template argument mangled
    (_ZN3raf<len><name>I<args>E...): those are decoded here as far as this library's kernels need (integer, bool,
    bf16 and float template arguments)."""
    import re
    m = re.match(r"_ZN3raf(\d+)", name)
    if m:
        n = int(m.group(1))
        base, rest = name[m.end():m.end() + n], name[m.end() + n:]
        targs = []
        if rest.startswith("I"):
            rest = rest[1:]
            while rest and not rest.startswith("E"):
                lit = re.match(r"L([ibjlm])(n?\d+)E", rest)
                if lit:
                    v = lit.group(2).replace("n", "-")
                    targs.append({"0": "false", "1": "true"}[v] if lit.group(1) == "b" else v)
                    rest = rest[lit.end():]
                elif rest.startswith("DF16b"):
                    targs.append("bf16")
                    rest = rest[5:]
                elif rest[0] in "fdi":
                    targs.append({"f": "float", "d": "double", "i": "int"}[rest[0]])
                    rest = rest[1:]
                else:
                    targs.append("...")
                    break
        return base + ("<" + ",".join(targs) + ">" if targs else "")
    name = name.replace("void ", "").replace("raf::", "")
    depth = 0
    for i, ch in enumerate(name):      # cut at the argument list (the first '(' outside template brackets)
        depth += ch == "<"
        depth -= ch == ">"
        if ch == "(" and depth == 0:
            return name[:i]
    return name


def kernel_breakdown(args, cfg, n_params_matrix, n_params_vector, steps=10, warmup=3, graph=True):
    """Every kernel of the step with its time INSIDE the step and its roofline fraction.

    The step is run in a child process under `rocprofv3 --kernel-trace`, as replays of the captured HIP graph like the
    timed region (graph=True; the profiler records every kernel of a replay as one dispatch) or eagerly; the
    per-dispatch begin/end stamps of the last `steps` steps are averaged per launch position, each position is given
    its operator and algorithmic work (launch_work), and positions are summed per kernel instantiation.  Returns
    (dict, None) or (None, reason)."""
    import csv
    import glob
    import shutil
    import subprocess
    import tempfile
    if shutil.which("rocprofv3") is None:
        return None, "rocprofv3 not on PATH"
    out_dir = tempfile.mkdtemp(prefix="raf_bench_trace_", dir="/tmp")
    cmd = ["rocprofv3", "--kernel-trace", "--output-format", "csv", "-d", out_dir, "-o", "trace", "--",
           sys.executable, os.path.abspath(__file__), "--workload", args.workload, "--steps", str(steps), "--warmup",
           str(warmup), "--no-cpu", "--trace-child"] + ([] if graph else ["--no-graph"])
    try:
        r = subprocess.run(cmd, cwd="/tmp", env=dict(os.environ, TMPDIR="/tmp"), stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, text=True, timeout=400)
    except Exception as ex:      # a time-out included: the child is killed by run()
        shutil.rmtree(out_dir, ignore_errors=True)
        return None, "profiler run failed: %r" % (ex,)
    files = glob.glob(os.path.join(out_dir, "**", "*kernel_trace.csv"), recursive=True)
    if r.returncode != 0 or not files:
        shutil.rmtree(out_dir, ignore_errors=True)
        return None, "profiler run gave rc %d and %d trace files: %s" % (r.returncode, len(files), r.stdout[-300:])
    rows = [x for x in csv.DictReader(open(files[0])) if "raf" in x["Kernel_Name"]]
    shutil.rmtree(out_dir, ignore_errors=True)
    rows.sort(key=lambda x: int(x["Start_Timestamp"]))
    # the child runs max(warmup, 1) eager steps, then (graph mode) captures one step and replays it 3 + steps times
    total_steps = steps + max(warmup, 1) + (3 if graph else 0)
    if not rows or len(rows) % total_steps:
        return None, "%d library dispatches do not divide into %d steps" % (len(rows), total_steps)
    n = len(rows) // total_steps
    timed = rows[-steps * n:]
    names = [x["Kernel_Name"] for x in timed[:n]]
    for k in range(steps):
        if [x["Kernel_Name"] for x in timed[k * n:(k + 1) * n]] != names:
            return None, "launch order differs between steps"
    dur_us = [sum(int(timed[k * n + i]["End_Timestamp"]) - int(timed[k * n + i]["Start_Timestamp"])
                  for k in range(steps)) / steps / 1e3 for i in range(n)]
    span_us = sum(int(timed[k * n + n - 1]["End_Timestamp"]) - int(timed[k * n]["Start_Timestamp"])
                  for k in range(steps)) / steps / 1e3
    work = launch_work(cfg, n_params_matrix, n_params_vector)
    seen, agg, order = {}, {}, []
    for i, name in enumerate(names):
        cls = next((c for key, c in KERNEL_CLASSES if key in name), None)
        k = seen.get(cls, 0)
        seen[cls] = k + 1
        op, bound, amount = (work[cls][k] if cls in work and k < len(work[cls]) else ("?", None, None))
        if name not in agg:
            agg[name] = dict(kernel=short_kernel_name(name), ops=[], launches_per_step=0, us_per_step=0.0, bound=bound,
                             work_per_step=0.0 if amount is not None else None)
            order.append(name)
        a = agg[name]
        a["ops"].append("%s %.1f us" % (op, dur_us[i]))
        a["launches_per_step"] += 1
        a["us_per_step"] += dur_us[i]
        if amount is None or a["work_per_step"] is None or bound != a["bound"]:
            a["work_per_step"] = None
        else:
            a["work_per_step"] += amount
    out = []
    for name in sorted(order, key=lambda q: -agg[q]["us_per_step"]):
        a = agg[name]
        a["us_per_step"] = round(a["us_per_step"], 2)
        if a["work_per_step"] is not None and a["bound"] is not None:
            rate = a["work_per_step"] / (a["us_per_step"] * 1e-6)
            if a["bound"] == "mfma":
                a.update(achieved=round(rate / 1e12, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                         frac=round(rate / 1e12 / PEAK_BF16_TFLOPS, 4))
            else:
                a.update(achieved=round(rate / 1e9, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                         frac=round(rate / 1e9 / PEAK_HBM_GBS, 4))
        out.append(a)
    gemm_us = sum(a["us_per_step"] for a in out if a["bound"] == "mfma")
    gemm_fl = sum(a["work_per_step"] for a in out if a["bound"] == "mfma" and a["work_per_step"])
    summary = {"launches_per_step": n, "sum_of_kernels_us": round(sum(dur_us), 1), "first_start_to_last_end_us": round(span_us, 1),
               "all_gemms_us": round(gemm_us, 1),
               "all_gemms_frac_of_mfma_peak": round(gemm_fl / (gemm_us * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4) if gemm_us else None,
               "source": "rocprofv3 --kernel-trace of %d %s steps in a child process" % (
                   steps, "HIP-graph replays of the" if graph else "eager")}
    return {"summary": summary, "per_kernel": out}, None



def measure_replay_us(cfg):
    """Run times (us) of the three operators a rematerialising layer replays — the QKV product, the attention
    forward kernel, the first feed-forward product with its GeLU epilogue — timed back to back on synthetic
    operands of the workload's shape: the latencies the rematerialisation planner is given."""
    import torch
    import paper_2303_04759_amd as raf
    dev = torch.device("cuda:0")
    T, H, F = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["ffn"]
    prec = cfg["precision"]
    cd = torch.bfloat16 if prec == 1 else torch.float32
    g = torch.Generator(device="cpu").manual_seed(0)
    rnd = lambda *shape: (torch.randn(*shape, generator=g) * 0.05).to(dev).to(cd).contiguous()
    x, wqkv, w1 = rnd(T, H), rnd(3 * H, H), rnd(F, H)
    bqkv, b1 = torch.zeros(3 * H, device=dev), torch.zeros(F, device=dev)
    qkv, ctx = torch.empty(T, 3 * H, dtype=cd, device=dev), torch.empty(T, H, dtype=cd, device=dev)
    gact, aux = torch.empty(T, F, dtype=cd, device=dev), torch.empty(T, F, dtype=cd, device=dev)
    lse = torch.empty(cfg["batch"] * cfg["heads"] * cfg["seq"], dtype=torch.float32, device=dev)
    desc = raf.make_desc(dict(cfg, layer_id=0))
    stream = torch.cuda.Stream()
    epi = raf.EPI_BIAS_GELU_DERIV if prec == 1 else raf.EPI_BIAS_GELU
    ops = [lambda: raf.raf_op_gemm(prec, T, 3 * H, H, x, H, 1, wqkv, H, 1, qkv, 3 * H, epilogue=raf.EPI_BIAS,
                                   bias=bqkv, stream=stream),
           lambda: raf.raf_op_attention_fwd(desc, qkv, None, ctx, lse, 1, stream),
           lambda: raf.raf_op_gemm(prec, T, F, H, x, H, 1, w1, H, 1, gact, F, epilogue=epi, bias=b1, aux=aux,
                                   gelu_tanh=cfg["gelu_tanh"], stream=stream)]
    if prec != 1:
        ops[1] = None           # attention is not one operator there (and its context is not droppable)
    out = []
    with torch.cuda.stream(stream):
        for op in ops:
            if op is None:
                out.append(0.0)
                continue
            for _ in range(3):
                op()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(20):
                op()
            e1.record(stream)
            stream.synchronize()
            out.append(e0.elapsed_time(e1) * 1000.0 / 20)
    return out


def bench_model(args, cfg):
    """Whole 12-layer model step (embedding, layers, MLM head, backward, Adam over all tensors)."""
    import numpy as np
    import torch
    from paper_2303_04759_amd.harness import DeviceModel
    from workloads.synthetic import ADAM, make_model_inputs
    inp = make_model_inputs(cfg, seed=0)
    remat, remat_info = None, None
    if args.activation_budget_frac < 1.0:
        # rematerialisation under a budget given as a fraction of the liveness estimate of the layer stack
        import paper_2303_04759_amd as raf
        desc = raf.make_desc(dict(cfg, layer_id=0))
        replay_us = None if args.estimated_replay_latency else measure_replay_us(cfg)
        graph_l, _, _ = raf.raf_layer_stack_graph(desc, cfg["layers"], replay_us)
        peak = max(raf.raf_memory_profile(graph_l))
        budget = int(peak * args.activation_budget_frac)
        remat, summ = raf.raf_layer_stack_remat(desc, cfg["layers"], budget, replay_us)
        remat_info = {"budget_bytes": budget, "layer_bits": remat, "planned_peak_bytes": summ["peak_after"],
                      "replay_us": replay_us if replay_us is not None else "library estimate",
                      "unplanned_peak_bytes": summ["peak_before"], "fits": summ["fits"],
                      "planned_extra_us": summ["extra_latency"]}
    mod = DeviceModel(cfg, inp, ADAM, remat=remat)
    if remat_info is not None:
        remat_info["saved_bytes_allocated"] = int(mod.saved_bytes)
    stream = torch.cuda.Stream()
    K, W = args.steps, args.warmup
    with torch.cuda.stream(stream):
        t_step = 1
        for _ in range(max(W, 1)):
            mod.train_step(t_step, stream)
            t_step += 1
        stream.synchronize()
        graph = None
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                mod.train_step(t_step, stream)
            graph.replay()
            stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(K):
            if graph is not None:
                graph.replay()
            else:
                mod.train_step(t_step, stream)
                t_step += 1
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / K
    n_params = sum(v.numel() for v in mod.master.values())
    out = {"metric": "train samples/sec, 12-layer BERT-base + MLM head fwd+bwd+Adam (bf16 AMP, 1 GPU)",
           "value": cfg["batch"] / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if cfg["precision"] == 1 else "f32", "data": "synthetic",
           "config": {"workload": args.workload, "batch": cfg["batch"], "seq_len": cfg["seq"], "layers": cfg["layers"],
                      "hidden": cfg["hidden"], "vocab": cfg["vocab"], "selected_positions": int(len(inp["sel"])),
                      "parameters": int(n_params), "launch": "eager" if graph is None else "hip_graph",
                      "parallelism": "single GPU"},
           "tokens_per_s_padded": mod.T / (ms * 1e-3),
           "tokens_per_s_valid": int(np.sum(inp["seq_lens"])) / (ms * 1e-3)}
    if remat_info is not None:
        out["rematerialisation"] = remat_info
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="bert_base")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline leg")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--dynamic-loss-scale", action="store_true",
                    help="time the step under the device-resident dynamic loss scaler (layer workloads)")
    ap.add_argument("--steps-per-graph", type=int, default=1,
                    help="consecutive steps captured into one HIP graph (layer workloads); the timed region still "
                         "covers exactly --steps steps")
    ap.add_argument("--activation-budget-frac", type=float, default=1.0,
                    help="model workloads: plan rematerialisation for an activation budget of this fraction of the "
                         "layer stack's liveness estimate (1.0 = keep everything)")
    ap.add_argument("--estimated-replay-latency", action="store_true",
                    help="with --activation-budget-frac: plan with the library's operation-count estimate of the "
                         "replay latencies instead of timing the three replayed operators first")
    ap.add_argument("--no-kernels", action="store_true",
                    help="skip the per-kernel report (an eager run of the step in a child process under rocprofv3)")
    ap.add_argument("--trace-child", action="store_true",
                    help="(used by the per-kernel report) run the eager steps only: no roofline replay, no report")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (5x) so FETCH_SIZE/WRITE_SIZE counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (no collectives, no sharding); run with --gpus 1")

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU; there is no CPU path for the library")
    import paper_2303_04759_amd as raf
    from paper_2303_04759_amd.harness import DeviceLayer
    from workloads.synthetic import ADAM, CONFIGS, MODEL_CONFIGS, make_layer_inputs

    if args.workload in MODEL_CONFIGS:
        return bench_model(args, MODEL_CONFIGS[args.workload])
    cfg = CONFIGS[args.workload]
    inp = make_layer_inputs(cfg, seed=0)
    lay = DeviceLayer(cfg, inp, ADAM)
    stream = torch.cuda.Stream()          # default priority
    K, W = args.steps, args.warmup

    if args.dynamic_loss_scale:
        import ctypes
        scaler_state = torch.zeros(ctypes.sizeof(raf.ScalerState), dtype=torch.uint8, device="cuda")
        raf.raf_scaler_init(scaler_state, cfg["loss_scale"])
        torch.cuda.synchronize()
        scaler_cfg = dict(growth_factor=2.0, backoff_factor=0.5, growth_interval=2000)
        one_step = lambda t, st: lay.train_step_dynamic(t, scaler_state, scaler_cfg, st)
    else:
        one_step = lambda t, st: lay.train_step(t, st)

    with torch.cuda.stream(stream):
        graph = None
        multi = None
        t_step = 1
        for _ in range(max(W, 1)):
            one_step(t_step, stream)
            t_step += 1
        stream.synchronize()
        if not args.no_graph:
            # one HIP graph of the whole step; replays re-run the same kernels on the same buffers
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                one_step(t_step, stream)
            for _ in range(3):
                graph.replay()
            stream.synchronize()
            multi = None
            G = max(1, args.steps_per_graph)
            if G > 1:
                multi = torch.cuda.CUDAGraph()
                with torch.cuda.graph(multi, stream=stream):
                    for i in range(G):
                        one_step(t_step + 1 + i, stream)
                multi.replay()
                stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        if graph is not None and multi is not None:
            for _ in range(K // G):
                multi.replay()
            for _ in range(K % G):
                graph.replay()
        else:
            for _ in range(K):
                if graph is not None:
                    graph.replay()
                else:
                    one_step(t_step, stream)
                    t_step += 1
        e1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_per_step = e0.elapsed_time(e1) / K
        if args.trace_child:
            print(json.dumps({"ms_per_step": ms_per_step, "steps": K, "warmup": W}))
            return

        # ---- roofline of the dominant kernel, timed with events on the launch stream: the K-major bf16 MFMA GEMM
        # instantiation that takes the most time per step, i.e. the one behind the five products with N = hidden
        # (out / ffn2 forward, ffn1 / out / qkv input gradients; 128x96 tiles on the bert_base workload)
        dt = lay.cdtype
        T, H, F = lay.T, cfg["hidden"], cfg["ffn"]
        big = max(3 * H, F)
        a_buf = torch.randn(T, big, device="cuda").to(dt)
        w_buf = (0.02 * torch.randn(big, big, device="cuda")).to(dt)
        c_buf = torch.empty(T, big, dtype=dt, device="cuda")
        u_buf = torch.empty(T, big, dtype=dt, device="cuda")
        bias = torch.zeros(big, device="cuda")
        dom = [g for g in gemm_launches(cfg) if g[4] == 1 and g[5] == 1 and g[8] == 1 and g[2] == H]
        reps = max(10, min(K, 50))

        def run_dom():
            for (_, M, N, Kd, ak, bk, of32, epi, _) in dom:
                raf.raf_op_gemm(cfg["precision"], M, N, Kd, a_buf, Kd, 1, w_buf, Kd, 1, c_buf, N, epilogue=epi,
                                bias=bias, aux=u_buf if epi >= 2 else None, stream=stream)
        for _ in range(3):
            run_dom()
        stream.synchronize()
        e0.record(stream)
        for _ in range(reps):
            run_dom()
        e1.record(stream)
        stream.synchronize()
        dom_ms = e0.elapsed_time(e1) / (reps * len(dom))
        dom_flops = sum(2.0 * M * N * Kd for (_, M, N, Kd, *_r) in dom) / len(dom)
        achieved = dom_flops / (dom_ms * 1e-3) / 1e12
        dom_name = ("K-major bf16 MFMA GEMM instantiation behind the %d products with N = hidden (%s)"
                    % (len(dom), ", ".join(g[0] for g in dom)))

    if args.calibrate_copy:
        src = torch.zeros(128 * 1024 * 1024, dtype=torch.bfloat16, device="cuda")     # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    samples_per_s = cfg["batch"] / (ms_per_step * 1e-3)
    valid_tokens = int(np.sum(inp["seq_lens"])) if inp["seq_lens"] is not None else lay.T
    total_flops = sum(2.0 * M * N * Kd * b for (_, M, N, Kd, _a, _b, _f, _e, b) in gemm_launches(cfg))
    out = {
        "metric": "train samples/sec, %s layer fwd+bwd+Adam (%s, 1 GPU)" %
                  ({"bert_base": "BERT-base", "bert_large": "BERT-large", "gpt2_medium": "GPT-2-medium"}.get(
                      args.workload, args.workload), "bf16 AMP" if cfg["precision"] == 1 else "fp32"),
        "value": samples_per_s, "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["precision"] == 1 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": cfg["batch"], "seq_len": cfg["seq"], "hidden": cfg["hidden"],
                   "heads": cfg["heads"], "ffn": cfg["ffn"], "dropout_p": cfg["dropout_p"],
                   "launch": "eager" if graph is None else "hip_graph", "parallelism": "single GPU",
                   "loss_scale": "dynamic" if args.dynamic_loss_scale else "static",
                   "steps_per_graph": (max(1, args.steps_per_graph) if graph is not None else 0)},
        "tokens_per_s_padded": lay.T / (ms_per_step * 1e-3),
        "tokens_per_s_valid": valid_tokens / (ms_per_step * 1e-3),
        "step_gemm_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "wall_ms_per_step": wall * 1e3 / K,
        "roofline": {"bound": "mfma", "kernel": dom_name, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "avg_launch_us": dom_ms * 1e3,
                     "flops_per_launch": dom_flops,
                     "timing": "HIP events on the launch stream around %d back-to-back replays of the kernel's %d "
                               "launches per step (same shapes and epilogues)" % (reps, len(dom)),
                     "traffic": profiled_traffic(args.workload, "dominant"), "traffic_unit": "bytes/launch"},
    }
    if not args.no_kernels:
        n_mat = sum(int(np.prod(inp["params"][k].shape)) for k in inp["params"] if k.startswith("w_"))
        n_vec = sum(int(np.prod(inp["params"][k].shape)) for k in inp["params"] if not k.startswith("w_"))
        kernels, why = kernel_breakdown(args, cfg, n_mat, n_vec)
        out["kernels"] = kernels if kernels is not None else {"unavailable": why}
        if kernels is not None:
            # the dominant kernel's figures inside the step (cold operands, neighbours' tails), beside the replay above
            for a in kernels["per_kernel"]:
                if a["bound"] == "mfma" and a["launches_per_step"] == len(dom) and a.get("frac") is not None:
                    out["roofline"]["in_step_avg_launch_us"] = round(a["us_per_step"] / a["launches_per_step"], 2)
                    out["roofline"]["in_step_frac"] = a["frac"]
                    break
    if not args.no_cpu:
        from oracle.step import train_step
        p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
        z = {k: np.zeros_like(v) for k, v in p.items()}
        hyper = dict(ADAM, loss_scale=cfg["loss_scale"])
        # a bounded sample: consecutive full steps until about ten seconds have gone by (at most eight)
        m_cpu, v_cpu, n_cpu = z, z, 0
        t0 = time.perf_counter()
        while n_cpu < 8 and (n_cpu == 0 or time.perf_counter() - t0 < 10.0):
            n_cpu += 1
            ref = train_step(cfg, p, m_cpu, v_cpu, inp["x"], inp["G"], inp["seq_lens"], n_cpu, hyper)
            p, m_cpu, v_cpu = ref["params"], ref["m"], ref["v"]
        dt_cpu = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        out["cpu_baseline"] = {"value": n_cpu * cfg["batch"] / dt_cpu, "unit": "samples/s", "cores": threads,
                               "kind": "oracle", "sample": "%d consecutive full steps (batch %d each) of the same workload, "
                               "numpy fp64, %.1f s" % (n_cpu, cfg["batch"], dt_cpu)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
