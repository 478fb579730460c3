#!/usr/bin/env python3
"""Benchmark of the routed sparse FFN layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
route -> permute -> grouped FFN fwd -> combine -> combine bwd -> grouped FFN bwd
-> permute bwd -> route bwd -> layer_load -> host Partition call.
Prints ONE JSON line (see README for the fields).
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
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (default 2: Mixtral-shaped MoE)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run one plain 1 GiB device copy (a known-size reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="tokens in the oracle's timed sample (0 = auto)")
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


def main():
    a = parse()
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
            x = layer.forward(x, *Ws[i])
        g = dev["dout"]
        for i in range(L - 1, -1, -1):
            g = layers[i].backward(g, *Ws[i])
            if w.mode == "moe":
                layers[i].route_bwd()
            elif w.mode == "mod":
                layers[i].route_bwd(dev["scores"])
        rows, loads = 0, []
        for layer in layers:
            counts, load = layer.load()  # device -> host, synchronises the stream
            rows += sum(counts)
            loads.append(load if L > 1 else [c * 18.0 * w.H * w.F for c in counts])
        per_task = loads if L > 1 else loads[0]
        if len(per_task) >= stage_split and stage_split > 0:
            B.dynmo_partition(per_task, stage_split)
        return rows, per_task

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
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if dom and os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("%s/%s" % (dom["name"], w.name))
    roofline = None
    if dom:
        roofline = {"kernel": dom["name"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                    "unit": dom["unit"], "frac": dom["frac"], "avg_us": dom["avg_us"], "traffic": traffic}

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
            "routed_rows_per_step": R_step, "tokens_per_s": round(w.T * a.steps / elapsed, 1)},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "imbalance": imb,
        "input_generation_s": round(gen_s, 1),
    }
    print(json.dumps(out))


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
        # aim at roughly 1.5e12 flop of float64 work (10-30 s on a host CPU)
        rows_target = max(64.0, 1.5e12 / flops_per_row)
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
