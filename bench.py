#!/usr/bin/env python3
"""Benchmark of the routed sparse FFN layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
route -> permute -> grouped FFN fwd -> combine -> combine bwd -> grouped FFN bwd
-> permute bwd -> route bwd -> layer_load -> host Partition call.
Prints ONE JSON line: metric, value (routed tokens/s, inputs resident in HBM), ms_per_step,
roofline (the dominant kernel against its published peak, from event durations taken inside
the timed region), cpu_baseline (the oracle on a bounded sample), the per-kernel list and the
imbalance of the exported loads before and after the Partition balancer.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_FLOPS = 2.5e15   # MI355X dense bf16 MFMA
PEAK_FP32_FLOPS = 157.3e12  # vector fp32
PEAK_HBM_BPS = 8.0e12


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    # the clocks of an idle GPU take about eight passes of this workload (70 ms) to settle
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (default 2: Mixtral-shaped MoE)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--print-kernel-sources-hash", action="store_true",
                    help="print the hash of the kernel sources (recorded in the counter summaries under profiles/) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run one plain 1 GiB device copy (a known-size reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--folded-combine", action="store_true",
                    help="configurations with one slot per token (4, 5): fold the combine into the last product "
                         "(dynmo_grouped_ffn_fwd_combine) and the scatter back to token order into the dX product "
                         "(dynmo_grouped_ffn_bwd_scatter) instead of the separate dynmo_combine / dynmo_permute_bwd passes")
    ap.add_argument("--reroute", type=int, default=0, metavar="N",
                    help="instead of the headline line: N iterations with fresh router inputs each (the routing "
                         "decision changes every iteration), the exported loads rebalanced every iteration; prints "
                         "the imbalance before/after per iteration and the balancers' host time")
    ap.add_argument("--protocol-text", default="", help="with --protocol: also write the result as a text table here")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="tokens in the oracle's timed sample (0 = auto)")
    ap.add_argument("--protocol", action="store_true",
                    help="instead of the headline line: the full timing protocol (>= 10 warm-up and >= 50 timed "
                         "repetitions, median and min per kernel, HBM-bound calls alone warm and cold, forward and "
                         "forward+backward chains, uniform and adversarial routing, the box's own MFMA and copy "
                         "ceilings); prints one JSON line")
    return ap.parse_args()


def kernel_work(name, w, R_total, T):
    """Algorithmic work of one launch of a kernel role: (bound, amount) with
    flops for the GEMMs and bytes for the row movers.  R_total is the number
    of routed rows the launch processes."""
    H, F, k = w.H, w.F, w.k
    b = 2 if w.dtype == "bf16" else 4
    HF = float(H) * F
    res = w.mode != "moe"
    table = {
        "ffn_gateup": ("mfma", 4 * HF * R_total),
        "ffn_down": ("mfma", 2 * HF * R_total),
        "ffn_dA": ("mfma", 2 * HF * R_total),
        "ffn_dX": ("mfma", 4 * HF * R_total),
        "ffn_dWd": ("mfma", 2 * HF * R_total),
        "ffn_dWg": ("mfma", 2 * HF * R_total),
        "ffn_dWu": ("mfma", 2 * HF * R_total),
        # x read once + x_p written, plus the dst_pos read
        "permute_rows": ("hbm", (min(T, R_total) + R_total) * H * b + 4.0 * T * k),
        # y_p read + out written (+ base read), plus dst_pos and gate_w
        "combine": ("hbm", (R_total + T + (T if res else 0)) * H * b + 8.0 * T * k),
        # dout + y_p read, dy_p written, plus dst_pos / gate_w / dgate
        "combine_bwd": ("hbm", (min(T, R_total) + 2 * R_total) * H * b + 12.0 * T * k),
        # dx_p read + dx written (+ dbase read)
        "permute_bwd": ("hbm", (R_total + T + (T if res else 0)) * H * b + 4.0 * T * k),
    }
    return table.get(name)


def kernel_sources_hash():
    """A short hash of the kernel sources (csrc/*.hip, *.h) the library is built from: counter summaries
    under profiles/ record the hash they were taken on, and a figure is only quoted for the same code."""
    import glob
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2505_14864_amd", "csrc")
    for path in sorted(glob.glob(os.path.join(csrc, "*.hip")) + glob.glob(os.path.join(csrc, "*.h"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(config, kernel):
    """(bytes, stale): HBM bytes per launch of `kernel` from the committed counter summary of this
    configuration (a table whose rows are: kernel, read MB, written MB, total MB, ...; a header line
    `kernel sources: <hash>` names the code it was measured on).  bytes is None when no summary covers
    the kernel, and also when the summary was taken on other kernel sources than the ones in the tree
    (then stale is True): a counter figure is never quoted for code it was not measured on."""
    import glob
    current = kernel_sources_hash()
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "hbm_traffic_config%d_*.txt" % config))):
        recorded, value = None, None
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == "kernel" and f[1] == "sources:":
                recorded = f[2]
            if len(f) >= 4 and f[0] in (kernel, kernel + "_kernel"):
                try:
                    value = int(round(float(f[3]) * 1e6))
                except ValueError:
                    pass
        if value is not None:
            return (value, False) if recorded == current else (None, True)
    return None, False


def main():
    a = parse()
    if a.print_kernel_sources_hash:
        print(kernel_sources_hash())
        return
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); --gpus %d is not supported. "
              "value is the one GPU's throughput." % a.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2505_14864_amd import binding as B
    from paper_2505_14864_amd import workloads as wl
    from paper_2505_14864_amd.layer import RoutedFFNLayer, to_device

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.CONFIGS[a.config]
    t0 = time.time()
    inp = wl.make_inputs(w, threads=16)
    gen_s = time.time() - t0
    dev = {n: to_device(v) for n, v in inp.items()}
    L = w.layers
    layers = [RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, w.mode) for _ in range(L)]
    for l in layers:
        l.alloc_backward()
    if w.mode == "early_exit":
        Ws = [(dev["Wg"][i], dev["Wu"][i], dev["Wd"][i]) for i in range(L)]
    else:
        Ws = [(dev["Wg"], dev["Wu"], dev["Wd"])]
    stage_split = 2 if L > 1 else min(4, w.E)

    if a.folded_combine and w.k != 1:
        print("bench.py: --folded-combine needs a configuration with one slot per token (4 or 5)", file=sys.stderr)
        sys.exit(2)
    primed = []
    primed_bwd = []

    def step():
        """One pass of the hot path; returns (routed rows, loads for the balancer)."""
        x = dev["x"]
        for i, layer in enumerate(layers):
            if w.mode == "moe":
                layer.route_topk(dev["logits"])
            elif w.mode == "mod":
                layer.route_capacity(dev["scores"], w.cap)
            else:
                layer.route_active(dev["exit_layer"], i + 1)
            if a.folded_combine:
                # The residual stream's rows of unrouted tokens are not rewritten.  Every step sees the same
                # routing, so each layer's output buffer is given them once, in the first (warm-up) step.
                if len(primed) < L:
                    layer.out.copy_(x)
                    primed.append(i)
                x = layer.forward_folded(x, *Ws[i], out=layer.out)
            else:
                x = layer.forward(x, *Ws[i])
            # the rows are permuted: the load is known, and its copy to the host can run behind the forward pass
            layer.load_begin()
        g = dev["dout"]
        for i in range(L - 1, -1, -1):
            if a.folded_combine:
                # as in the forward pass: the gradient rows of unrouted tokens are not rewritten, and every
                # step sees the same routing and the same upstream gradient, so they are given once
                if len(primed_bwd) < L:
                    layers[i].dx.copy_(g)
                    primed_bwd.append(i)
                g = layers[i].backward_folded(g, *Ws[i], dx=layers[i].dx)
            else:
                g = layers[i].backward(g, *Ws[i])
            if w.mode == "moe":
                layers[i].route_bwd()
            elif w.mode == "mod":
                layers[i].route_bwd(dev["scores"])
        rows, loads = 0, []
        for layer in layers:
            counts, load = layer.load_end()  # waits for this layer's copy only, which finished long ago
            rows += sum(counts)
            loads.append(load if L > 1 else [c * 18.0 * w.H * w.F for c in counts])
        per_task = loads if L > 1 else loads[0]
        if len(per_task) >= stage_split and stage_split > 0:
            B.dynmo_partition(per_task, stage_split)
        return rows, per_task

    if a.reroute > 0 and w.mode == "mod":
        print(json.dumps(reroute_mod_stack(a, w, dev)))
        return
    if a.reroute > 0:
        print(json.dumps(reroute(a, w, dev, layers, Ws, step, stage_split)))
        return
    if a.protocol:
        res = protocol(a, w, inp, dev, layers, Ws, step)
        if a.protocol_text:
            with open(a.protocol_text, "w") as f:
                f.write(protocol_text(res, a))
        print(json.dumps(res))
        return

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    B.dynmo_profile_reset()
    B.dynmo_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    rows = 0
    for _ in range(a.steps):
        r, per_task = step()
        rows += r
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.dynmo_profile_enable(False)
    elapsed = t1 - t0
    ms_per_step = elapsed * 1e3 / a.steps
    R_step = rows / a.steps
    value = rows / elapsed

    # per-kernel durations measured live (hipEvent pairs recorded by the library
    # on the launch stream during the timed region)
    kernels = []
    for i in range(B.dynmo_profile_kernel_count()):
        ms, n = B.dynmo_profile_read(i)
        if n == 0:
            continue
        name = B.dynmo_profile_kernel_name(i)
        launches_per_step = n / a.steps
        avg_ms = ms / n
        ent = {"name": name, "launches": int(n), "avg_us": round(avg_ms * 1e3, 2), "total_ms": round(ms, 3)}
        work = kernel_work(name, w, R_step / launches_per_step, w.T)
        if work:
            bound, amount = work
            if bound == "mfma":
                peak = PEAK_BF16_FLOPS if w.dtype == "bf16" else PEAK_FP32_FLOPS
                ach = amount / (avg_ms * 1e-3)
                ent.update(bound="mfma" if w.dtype == "bf16" else "alu", achieved=round(ach / 1e12, 2),
                           peak=peak / 1e12, unit="TFLOP/s", frac=round(ach / peak, 4))
            else:
                ach = amount / (avg_ms * 1e-3)
                ent.update(bound="hbm", achieved=round(ach / 1e9, 1), peak=PEAK_HBM_BPS / 1e9, unit="GB/s",
                           frac=round(ach / PEAK_HBM_BPS, 4))
        kernels.append(ent)
    kernels.sort(key=lambda e: -e["total_ms"])
    dom = next((e for e in kernels if "bound" in e), None)
    traffic, traffic_stale = measured_traffic(a.config, dom["name"]) if dom else (None, False)
    roofline = None
    if dom:
        roofline = {"kernel": dom["name"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                    "unit": dom["unit"], "frac": dom["frac"], "avg_us": dom["avg_us"], "traffic": traffic}
        if traffic_stale:  # the committed counter summary was taken on other kernel sources
            roofline["traffic_stale"] = True

    # imbalance of the exported load vector: equal-count split vs Partition
    imb = None
    if len(per_task) >= 2:
        S = stage_split
        ub = B.dynmo_stage_loads(per_task, B.dynmo_uniform_bounds(len(per_task), S))
        pb_bounds, _ = B.dynmo_partition(per_task, S)
        pb = B.dynmo_stage_loads(per_task, pb_bounds)
        imb = {"stages": S, "tasks": "layers" if L > 1 else "experts", "uniform": round(B.dynmo_imbalance(ub), 4),
               "partition": round(B.dynmo_imbalance(pb), 4)}

    if a.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if not a.no_cpu_baseline:
        cpu = cpu_baseline(w, inp, a.cpu_sample_tokens)

    out = {
        "metric": "routed tokens/s fwd+bwd per sparse FFN layer",
        "value": round(value, 1),
        "unit": "routed tokens/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "config %d: %s (T=%d H=%d F=%d E=%d k=%d%s)" % (
            a.config, w.name, w.T, w.H, w.F, w.E, w.k, ", %d layers" % L if L > 1 else ""),
            "routed_rows_per_step": R_step, "tokens_per_s": round(w.T * a.steps / elapsed, 1),
            "folded_combine": bool(a.folded_combine)},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "imbalance": imb,
        "input_generation_s": round(gen_s, 1),
    }
    print(json.dumps(out))


def reroute_mod_stack(a, w, dev, n_layers=8, S=4):
    """Sec. 4 (Mixture of Depths): the routing wraps whole blocks, and a block that is skipped is
    treated as a shadow layer when the layers are redistributed.  A stack of Mixture-of-Depths
    blocks of this configuration's shape (all sharing one set of weights: only the cost matters
    here); every iteration each block draws new router scores and its capacity from
    {0, 0, 1/16, 1/8, 1/4} of the sequence, a capacity of zero being a skipped block.  The whole
    stack runs forward and backward, the per-block loads are exported, and the stages are split
    four ways: equal layer counts; Partition on the parameter loads (all blocks alike, so it
    cannot see a skipped block); the same loads with the skipped blocks flagged as shadow layers;
    Partition on the exported loads.  All four are judged by the exported (flop) loads."""
    import torch
    from paper_2505_14864_amd import binding as B
    from paper_2505_14864_amd.layer import RoutedFFNLayer

    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    layers = [RoutedFFNLayer(w.T, w.H, w.F, 1, 1, w.dtype, "mod") for _ in range(n_layers)]
    for l in layers:
        l.alloc_backward()
    Ws = (dev["Wg"], dev["Wu"], dev["Wd"])
    choices = [0, 0, w.S // 16, w.S // 8, w.S // 4]
    param_loads = [3.0 * w.H * w.F] * n_layers
    names = ("uniform", "partition_by_param", "partition_by_param_shadow", "partition_by_load")
    rec = {n: [] for n in names}
    most = {"partition_by_load": [], "partition_by_param_shadow": []}
    shadow_count, t_step = [], []
    for it in range(max(1, a.warmup) + a.reroute):
        pick = torch.randint(0, len(choices), (n_layers,), generator=gen, device="cuda").tolist()
        caps = [choices[i] for i in pick]
        scores = [torch.randn(w.B, w.S, generator=gen, device="cuda") for _ in range(n_layers)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        x = dev["x"]
        for l, layer in enumerate(layers):
            layer.route_capacity(scores[l], caps[l])
            x = layer.forward(x, *Ws)
        g = dev["dout"]
        for l in range(n_layers - 1, -1, -1):
            g = layers[l].backward(g, *Ws)
            layers[l].route_bwd(scores[l])
        loads = [layer.load()[1] for layer in layers]  # device -> host, synchronises
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if it < max(1, a.warmup) or sum(loads) <= 0:
            continue
        shadow = [1 if c == 0 else 0 for c in caps]
        splits = {
            "uniform": B.dynmo_uniform_bounds(n_layers, S),
            "partition_by_param": B.dynmo_partition(param_loads, S)[0],
            "partition_by_param_shadow": B.dynmo_partition_shadow(param_loads, shadow, S)[0],
            "partition_by_load": B.dynmo_partition(loads, S)[0],
        }
        for n, b in splits.items():
            rec[n].append(round(B.dynmo_imbalance(B.dynmo_stage_loads(loads, b)), 4))
        for n in most:
            most[n].append(max(splits[n][i + 1] - splits[n][i] for i in range(S)))
        shadow_count.append(sum(shadow))
        t_step.append(t1 - t0)
    mean = lambda xs: sum(xs) / max(1, len(xs))
    return {"workload": "config %d: %s, a stack of %d blocks" % (a.config, w.name, n_layers), "iterations": a.reroute,
            "stages": S, "tasks": "layers", "capacities": choices, "mean_shadow_layers": round(mean(shadow_count), 2),
            "imbalance": rec, "mean_imbalance": {k: round(mean(v), 4) for k, v in rec.items()},
            "mean_most_layers_on_a_stage": {k: round(mean(v), 2) for k, v in most.items()},
            "ms_per_iteration": round(1e3 * mean(t_step), 4)}


def reroute(a, w, dev, layers, Ws, step, S):
    """Sec. 3.3 / Sec. 4: for MoE and MoD the load changes with every routing decision, so
    the balancer runs every iteration.  Each iteration draws new router inputs on the
    device, runs the whole path, exports the loads and rebalances them on the host with
    both balancers; reports the imbalance of the static equal split, of Partition and of
    Diffusion (started from the previous iteration's split), and what the balancing costs."""
    import torch
    from paper_2505_14864_amd import binding as B
    from paper_2505_14864_amd import workloads as wl

    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    bias = torch.from_numpy(wl.expert_bias(w)).cuda() if w.mode == "moe" else None
    for _ in range(max(1, a.warmup)):
        step()
    torch.cuda.synchronize()
    rec = {"uniform": [], "partition": [], "diffusion": [], "diffusion_rounds": []}
    t_step, t_bal = [], []
    prev = None
    by_time = {"split_by_param": [], "split_by_time": []} if len(layers) > 1 else None
    for it in range(a.reroute):
        # the routing decision of this iteration (drifting preference: the bias rotates over the experts)
        if w.mode == "moe":
            dev["logits"] = torch.randn(w.T, w.E, generator=gen, device="cuda") + torch.roll(bias, it)[None, :]
        elif w.mode == "mod":
            dev["scores"] = torch.randn(w.B, w.S, generator=gen, device="cuda")
        else:
            dev["exit_layer"] = torch.empty(w.T, device="cuda").geometric_(w.exit_p, generator=gen).to(torch.int32)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, loads = step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if len(loads) < S or sum(loads) <= 0:
            continue
        ub = B.dynmo_uniform_bounds(len(loads), S)
        pb, _ = B.dynmo_partition(loads, S)
        db, rounds, _, _ = B.dynmo_diffusion(loads, prev if prev is not None else ub)
        t2 = time.perf_counter()
        prev = db
        rec["uniform"].append(round(B.dynmo_imbalance(B.dynmo_stage_loads(loads, ub)), 4))
        rec["partition"].append(round(B.dynmo_imbalance(B.dynmo_stage_loads(loads, pb)), 4))
        rec["diffusion"].append(round(B.dynmo_imbalance(B.dynmo_stage_loads(loads, db)), 4))
        rec["diffusion_rounds"].append(rounds)
        t_step.append(t1 - t0)
        t_bal.append(t2 - t1)
        if by_time is not None:
            # The profiling step (Sec. 3.1, Sec. 5 "by Time"): time each layer's forward and backward with
            # events, balance once on the parameter/flop loads and once on the measured times, and judge
            # both splits by the measured stage times.
            L = len(layers)
            ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(L)]
            x = dev["x"]
            for i, layer in enumerate(layers):
                layer.route_active(dev["exit_layer"], i + 1)
                ev[i][0].record()
                x = layer.forward(x, *Ws[i])
                ev[i][1].record()
            g = dev["dout"]
            for i in range(L - 1, -1, -1):
                ev[i][2].record()
                g = layers[i].backward(g, *Ws[i])
                ev[i][3].record()
            torch.cuda.synchronize()
            times = [ev[i][0].elapsed_time(ev[i][1]) + ev[i][2].elapsed_time(ev[i][3]) for i in range(L)]
            tb, _ = B.dynmo_partition(times, S)
            by_time["split_by_param"].append(round(B.dynmo_imbalance(B.dynmo_stage_loads(times, pb)), 4))
            by_time["split_by_time"].append(round(B.dynmo_imbalance(B.dynmo_stage_loads(times, tb)), 4))
    n = max(1, len(t_step))
    mean = lambda xs: sum(xs) / max(1, len(xs))
    return {"workload": "config %d: %s" % (a.config, w.name), "iterations": a.reroute, "stages": S,
            "tasks": "layers" if len(layers) > 1 else "experts",
            "imbalance": rec,
            "mean_imbalance": {k: round(mean(v), 4) for k, v in rec.items() if k != "diffusion_rounds"},
            "imbalance_of_measured_stage_times": by_time,
            "mean_imbalance_of_measured_stage_times": (
                {k: round(mean(v), 4) for k, v in by_time.items()} if by_time else None),
            "ms_per_iteration": round(1e3 * sum(t_step) / n, 4),
            "balancing_us_per_iteration": round(1e6 * sum(t_bal) / n, 1),
            "balancing_overhead": round(sum(t_bal) / max(1e-12, sum(t_step)), 5)}


def _stats(xs):
    xs = sorted(xs)
    return {"median_us": round(xs[len(xs) // 2] * 1e3, 2), "min_us": round(xs[0] * 1e3, 2), "reps": len(xs)}


def protocol(a, w, inp, dev, layers, Ws, step):
    """Timing protocol of the whole path and of each call (times in microseconds).
    Durations of single kernels are the library's hipEvent pairs; chains are
    bracketed by events on the same stream."""
    import numpy as np
    import torch
    from paper_2505_14864_amd import binding as B
    from paper_2505_14864_amd import workloads as wl
    from paper_2505_14864_amd.layer import to_device

    reps, warm = max(50, a.steps), max(10, a.warmup)
    names = [B.dynmo_profile_kernel_name(i) for i in range(B.dynmo_profile_kernel_count())]
    out = {"workload": "config %d: %s" % (a.config, w.name), "reps": reps, "warmup": warm}

    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1)

    # ---- what this machine reaches: MFMA issue with no memory traffic, streaming copy
    sink = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    operands = torch.randn(4096, dtype=torch.float32, device="cuda").to(torch.bfloat16)  # 8 KiB of N(0,1)
    flops = [0.0]

    def mfma(ops=None, iters=20000):
        flops[0] = B.dynmo_peak_mfma_bf16(iters, sink, ops)
    mfma()
    torch.cuda.synchronize()
    t_mfma = min(timed(mfma) for _ in range(5))
    # the same loop on random operands, long enough (about 0.3 s) for the clock to settle under the power it draws
    mfma(operands)
    t_rand = min(timed(lambda: mfma(operands, 600000)) for _ in range(2))
    rand_flops = flops[0] / (t_rand * 1e-3)
    mfma()
    evict = torch.empty(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB: four times the Infinity Cache
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    B.dynmo_peak_copy(evict, src)
    t_copy = min(timed(lambda: B.dynmo_peak_copy(evict, src)) for _ in range(5))
    small = 48 << 20  # bytes each way: the footprint of a config-2 row kernel
    s_src, s_dst = src.view(torch.uint8)[:small], evict.view(torch.uint8)[small:2 * small]
    t_small_warm = min(timed(lambda: B.dynmo_peak_copy(s_dst, s_src)) for _ in range(10))
    t_small_cold, t_small_swept = [], []
    spare = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    for _ in range(10):
        spare.fill_(1.0)  # leaves the caches full of dirty lines: the call after it also pays for their write-back
        t_small_cold.append(timed(lambda: B.dynmo_peak_copy(s_dst, s_src)))
    for _ in range(10):
        spare.sum()       # a read sweep evicts as well, and leaves clean lines
        t_small_swept.append(timed(lambda: B.dynmo_peak_copy(s_dst, s_src)))
    meas_flops = flops[0] / (t_mfma * 1e-3)
    meas_bw = 2.0 * src.numel() * 4 / (t_copy * 1e-3)
    out["measured_peaks"] = {
        "mfma_bf16_tflops": round(meas_flops / 1e12, 1), "mfma_vs_nominal": round(meas_flops / PEAK_BF16_FLOPS, 3),
        "mfma_bf16_random_operands_sustained_tflops": round(rand_flops / 1e12, 1),
        "mfma_random_vs_nominal": round(rand_flops / PEAK_BF16_FLOPS, 3),
        "copy_1GiB_GBps": round(meas_bw / 1e9, 1), "copy_vs_nominal": round(meas_bw / PEAK_HBM_BPS, 3),
        "copy_96MiB_warm_GBps": round(2.0 * small / (t_small_warm * 1e-3) / 1e9, 1),
        "copy_96MiB_cold_GBps": round(2.0 * small / (sorted(t_small_cold)[5] * 1e-3) / 1e9, 1),
        "copy_96MiB_swept_GBps": round(2.0 * small / (sorted(t_small_swept)[5] * 1e-3) / 1e9, 1)}
    del src

    def cold():
        spare.fill_(1.0)

    def swept():
        spare.sum()

    # ---- every kernel inside the forward+backward chain, one repetition at a time
    for _ in range(warm):
        step()
    torch.cuda.synchronize()
    per = {n: [] for n in names}
    chain, rows = [], 0
    B.dynmo_profile_enable(True)
    for _ in range(reps):
        B.dynmo_profile_reset()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rows, _ = step()
        e1.record()
        e1.synchronize()
        chain.append(e0.elapsed_time(e1))
        for i, n in enumerate(names):
            ms, cnt = B.dynmo_profile_read(i)
            if cnt:
                per[n].append(ms)  # all launches of the role in one pass (one per layer)
    B.dynmo_profile_enable(False)
    kern = {}
    L = len(layers)
    for n, xs in per.items():
        if not xs:
            continue
        st = _stats(xs)
        work = kernel_work(n, w, rows, w.T) if L == 1 else None
        if work:
            peak = {"mfma": PEAK_BF16_FLOPS if w.dtype == "bf16" else PEAK_FP32_FLOPS, "hbm": PEAK_HBM_BPS}[work[0]]
            meas = {"mfma": meas_flops, "hbm": meas_bw}[work[0]]
            rate = work[1] / (st["median_us"] * 1e-6)
            st.update(bound=work[0], frac_nominal=round(rate / peak, 4))
            if w.dtype == "bf16" or work[0] == "hbm":
                st["frac_measured"] = round(rate / meas, 4)
            if w.dtype == "bf16" and work[0] == "mfma":
                st["frac_measured_random_operands"] = round(rate / rand_flops, 4)
        kern[n] = st
    out["in_chain"] = kern
    fb = _stats(chain)
    fb["routed_rows_per_s"] = round(rows / (fb["median_us"] * 1e-6), 1)
    out["fwd_bwd_chain"] = fb

    # ---- the forward chain alone
    def fwd_only():
        x = dev["x"]
        for i, layer in enumerate(layers):
            if w.mode == "moe":
                layer.route_topk(dev["logits"])
            elif w.mode == "mod":
                layer.route_capacity(dev["scores"], w.cap)
            else:
                layer.route_active(dev["exit_layer"], i + 1)
            x = layer.forward(x, *Ws[i])
    for _ in range(3):
        fwd_only()
    out["fwd_chain"] = _stats([timed(fwd_only) for _ in range(reps)])

    # ---- the same forward+backward kernels replayed as one HIP graph (no launch gaps;
    # the load export and the host balancer are not part of it)
    def device_part():
        fwd_only()
        g = dev["dout"]
        for i in range(L - 1, -1, -1):
            if a.folded_combine:
                # as in the forward pass: the gradient rows of unrouted tokens are not rewritten, and every
                # step sees the same routing and the same upstream gradient, so they are given once
                if len(primed_bwd) < L:
                    layers[i].dx.copy_(g)
                    primed_bwd.append(i)
                g = layers[i].backward_folded(g, *Ws[i], dx=layers[i].dx)
            else:
                g = layers[i].backward(g, *Ws[i])
            if w.mode == "moe":
                layers[i].route_bwd()
            elif w.mode == "mod":
                layers[i].route_bwd(dev["scores"])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        device_part()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        device_part()
    for _ in range(3):
        graph.replay()
    out["fwd_bwd_graph_replay"] = _stats([timed(graph.replay) for _ in range(reps)])
    out["fwd_bwd_eager_device_part"] = _stats([timed(device_part) for _ in range(reps)])
    del graph

    # ---- the HBM-bound calls alone, warm (back to back) and cold (caches evicted first)
    if L == 1:
        l0 = layers[0]
        d = l0.d
        base = dev["x"] if l0.residual else None
        dbase = dev["dout"] if l0.residual else None
        calls = {
            "permute_rows": lambda: B.dynmo_permute(d, dev["x"], l0.expert_idx, l0.x_p, l0.seg_offsets, l0.src_slot,
                                                    l0.dst_pos, l0.ws_permute),
            "combine": lambda: B.dynmo_combine(d, l0.y_p, l0.dst_pos, l0.gate_w, base, l0.out),
            "combine_bwd": lambda: B.dynmo_combine_bwd(d, dev["dout"], l0.y_p, l0.dst_pos, l0.gate_w, l0.dy_p, l0.dgate),
            "permute_bwd": lambda: B.dynmo_permute_bwd(d, l0.dx_p, l0.dst_pos, dbase, l0.dx),
        }
        alone = {}
        B.dynmo_profile_enable(True)
        for n, fn in calls.items():
            idx = names.index(n)
            bytes_ = kernel_work(n, w, rows, w.T)[1]
            ent = {}
            for label, pre in (("warm", None), ("cold", cold), ("swept", swept)):
                xs = []
                for _ in range(reps):
                    if pre:
                        pre()
                    B.dynmo_profile_reset()
                    fn()
                    xs.append(B.dynmo_profile_read(idx)[0])
                st = _stats(xs)
                rate = bytes_ / (st["median_us"] * 1e-6)
                st.update(GBps=round(rate / 1e9, 1), frac_nominal=round(rate / PEAK_HBM_BPS, 4),
                          frac_measured_copy=round(rate / meas_bw, 4))
                ent[label] = st
            ent["algorithmic_bytes"] = bytes_
            alone[n] = ent
        B.dynmo_profile_enable(False)
        out["hbm_calls_alone"] = alone

    # ---- other routing histograms at the same shape (reported, not the headline)
    if w.mode == "moe":
        variants = {}
        base_logits = inp["logits"] - wl.expert_bias(w)[None, :]
        adv = inp["logits"].copy()
        adv[:, 0] += 6.0          # everybody's first choice: T rows, the most one expert can get
        adv[:, w.E - 1] -= 40.0   # nobody's choice: an empty expert
        keep = dev["logits"]
        for label, lg in (("uniform_routing", base_logits), ("adversarial_histogram", adv)):
            dev["logits"] = to_device(np.ascontiguousarray(lg.astype(np.float32)))
            for _ in range(3):
                step()
            xs = []
            for _ in range(max(10, reps // 5)):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                r, _ = step()
                e1.record()
                e1.synchronize()
                xs.append(e0.elapsed_time(e1))
            st = _stats(xs)
            counts, _ = layers[0].load()
            st.update(routed_rows_per_s=round(r / (st["median_us"] * 1e-6), 1), counts=[int(c) for c in counts])
            variants[label] = st
        dev["logits"] = keep
        out["routing_variants"] = variants
    return out


def protocol_text(d, a):
    """The --protocol result as a table for reading."""
    pct = lambda v: "%.1f%%" % (100 * v) if v is not None else "-"
    L = ["Timing protocol, %s, one MI355X" % d["workload"],
         "command: python bench.py --protocol --config %d --protocol-text <this file>" % a.config,
         "%d warm-up passes, %d timed repetitions; times in microseconds." % (d["warmup"], d["reps"]),
         "nominal = 2.5 PFLOP/s bf16 MFMA, 8 TB/s HBM; measured = this box's own ceilings from the library's two",
         "reference kernels (dynmo_peak_mfma_bf16, dynmo_peak_copy).", ""]
    m = d["measured_peaks"]
    L += ["Measured ceilings of this box",
          "  register-resident bf16 MFMA loop, fixed operands      : %8.1f TFLOP/s  (%s of nominal)" % (
              m["mfma_bf16_tflops"], pct(m["mfma_vs_nominal"])),
          "  the same loop on N(0,1) operands, 0.3 s sustained     : %8.1f TFLOP/s  (%s of nominal; the clock drops "
          "under the power real data draws)" % (m["mfma_bf16_random_operands_sustained_tflops"],
                                                 pct(m["mfma_random_vs_nominal"])),
          "  streaming copy, 1 GiB each way                        : %8.1f GB/s     (%s of nominal)" % (
              m["copy_1GiB_GBps"], pct(m["copy_vs_nominal"])),
          "  streaming copy, 48 MiB each way                       : %8.1f GB/s back to back, %.1f GB/s after a "
          "1 GiB cache-evicting fill, %.1f GB/s after a 1 GiB read sweep" % (
              m["copy_96MiB_warm_GBps"], m["copy_96MiB_cold_GBps"], m.get("copy_96MiB_swept_GBps", 0.0)), ""]
    L += ["Kernels inside the forward+backward chain (all launches of a role in one pass)",
          "  %-16s %10s %10s  %-5s %9s %9s %12s" % ("kernel", "median", "min", "bound", "nominal", "measured",
                                                   "random-data")]
    for n, s in sorted(d["in_chain"].items(), key=lambda kv: -kv[1]["median_us"]):
        L.append("  %-16s %10.2f %10.2f  %-5s %9s %9s %12s" % (
            n, s["median_us"], s["min_us"], s.get("bound", "-"), pct(s.get("frac_nominal")),
            pct(s.get("frac_measured")), pct(s.get("frac_measured_random_operands"))))
    f, b = d["fwd_chain"], d["fwd_bwd_chain"]
    L += ["", "Chains (route .. combine; route .. route_bwd + layer_load + host Partition)",
          "  forward          median %.1f  min %.1f" % (f["median_us"], f["min_us"]),
          "  forward+backward median %.1f  min %.1f   -> %.0f routed rows/s" % (
              b["median_us"], b["min_us"], b["routed_rows_per_s"])]
    if "fwd_bwd_graph_replay" in d:
        g_, e_ = d["fwd_bwd_graph_replay"], d["fwd_bwd_eager_device_part"]
        L.append("  its kernels alone (no load export, no host balancer): launched one by one median %.1f, replayed as "
                 "one HIP graph median %.1f" % (e_["median_us"], g_["median_us"]))
    if "hbm_calls_alone" in d:
        L += ["", "HBM-bound calls alone: warm = back to back; cold = after a 1 GiB fill, which evicts L2 and the "
                  "Infinity Cache and leaves",
              "them full of dirty lines whose write-back the call then shares the memory with; swept = after a 1 GiB "
              "read sweep (evicted, clean)",
              "  %-14s %12s | %8s %9s %8s %9s | %8s %9s %8s | %8s %9s %8s" % (
                  "call", "alg. bytes", "warm us", "GB/s", "nominal", "vs copy", "cold us", "GB/s", "nominal",
                  "swept us", "GB/s", "nominal")]
        for n, e in d["hbm_calls_alone"].items():
            w_, c_, s_ = e["warm"], e["cold"], e.get("swept", e["cold"])
            L.append("  %-14s %12d | %8.2f %9.1f %8s %9s | %8.2f %9.1f %8s | %8.2f %9.1f %8s" % (
                n, e["algorithmic_bytes"], w_["median_us"], w_["GBps"], pct(w_["frac_nominal"]),
                pct(w_["frac_measured_copy"]), c_["median_us"], c_["GBps"], pct(c_["frac_nominal"]),
                s_["median_us"], s_["GBps"], pct(s_["frac_nominal"])))
        L.append("  ('vs copy' is against the 1 GiB copy rate; a copy of the calls' own footprint is two lines up.)")
    if "routing_variants" in d:
        L += ["", "Other routing histograms, same shape (forward+backward chain)"]
        for n, e in d["routing_variants"].items():
            L.append("  %-22s median %.1f  min %.1f  -> %.0f routed rows/s   rows per expert %s" % (
                n, e["median_us"], e["min_us"], e["routed_rows_per_s"], e["counts"]))
    return "\n".join(L) + "\n"


def cpu_baseline(w, inp, sample_tokens):
    """Times the CPU oracle, as it stands, on a bounded token sample of the same
    workload (all experts / all layers, fewer tokens)."""
    import numpy as np
    from oracle import dynmo_oracle as orc
    from paper_2505_14864_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    flops_per_row = 18.0 * w.H * w.F
    if sample_tokens <= 0:
        # aim at roughly 1e13 flop of float64 work (10-30 s on the machine's host cores)
        rows_target = max(64.0, 1e13 / flops_per_row)
        frac_routed = {"moe": w.k, "mod": (w.cap / w.S) if w.S else 1.0, "early_exit": 2.5}[w.mode]
        sample_tokens = int(min(w.T, max(64, rows_target / frac_routed)))
        if w.mode == "mod":
            sample_tokens = max(w.S, sample_tokens // w.S * w.S)
    n = min(w.T, sample_tokens)
    f = {k: wl.as_f32(v) for k, v in inp.items()}
    t0 = time.perf_counter()
    if w.mode == "moe":
        r = orc.moe_layer(f["logits"][:n], f["x"][:n], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"][:n])
        rows = int(r["seg_offsets"][-1])
    elif w.mode == "mod":
        r = orc.mod_layer(f["scores"][: n // w.S], w.cap, f["x"][:n], f["Wg"], f["Wu"], f["Wd"], f["dout"][:n])
        rows = int(r["seg_offsets"][-1])
    else:
        weights = [(f["Wg"][l], f["Wu"][l], f["Wd"][l]) for l in range(w.layers)]
        r = orc.early_exit_stack(inp["exit_layer"][:n], f["x"][:n], weights, f["dout"][:n])
        rows = int(r["active"].sum())
    dt = time.perf_counter() - t0
    return {"value": round(rows / dt, 1), "unit": "routed tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "first %d of %d tokens (all experts/layers), %d routed rows, %.1f s of float64 numpy" % (
                n, w.T, rows, dt)}


if __name__ == "__main__":
    main()
