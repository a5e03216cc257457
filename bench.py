#!/usr/bin/env python3
"""Benchmark of the cnnk training step on one MI355X.

A step is one pass of the whole hot path (forward, loss, backward, SGD-momentum update) over one
batch of seeded synthetic CIFAR-100-shaped data, resident in HBM before the timed region starts.
Workload: ResNet-18 adapted to 32x32 inputs, 100 classes, bf16 storage / fp32 accumulate, batch 256
(--config 1..5 picks another of the convolutional networks, --config 6 the paper's second model
family: ViT-B/16 on 224x224 inputs at batch 64).  Prints ONE JSON line: metric / value (images/s) / ms_per_step,
`roofline` for the call class with the largest time per step (measured with HIP events recorded
on the launch stream around every entry-point call, in extra single-stream steps that two marker
launches bracket in a kernel trace), `cpu_baseline` (the fp64 oracle timed on a
bounded sample on the host cores) and `validation_pass` (the inference-mode forward).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch of the roofline class, from two `rocprofv3 --pmc` runs of this very script
# (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for the calibration copy
# below (a plain copy kernel of known size in the same run); commands, raw counter means and the
# scale factors are in profiles/.  None for a class that was not measured.
MEASURED_TRAFFIC_BYTES = {
    "conv3x3 s1 64->64 @32 fwd+dgrad (patch_kernel)": 86084197,   # profiles/bench_resnet18_b256_hbm_traffic.md
    "fc1.gemm_gelu": 276733000,                                    # profiles/bench_vit_b16_b64_hbm_traffic.md (--config 6)
}
# Launches that exist to be found in a profiler's kernel trace (all through cnnk_grad_route, a plain
# copy kernel of the library, whose grid is its element count / 2048): one copy of CAL_ELEMS bf16
# values before the warm-up (256 MiB read, 256 MiB written: the known size that calibrates the
# traffic counters), and two small copies that bracket the steps timed per call, so that a trace
# can be cut to exactly the launches that `roofline` is computed from.
CAL_ELEMS = 128 << 20
MARK_BEGIN_ELEMS, MARK_END_ELEMS = 2048 * 777 - 8, 2048 * 778 - 8
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def layer_key(L, phase):
    if L["op"] == "conv":
        # the forward and input-gradient calls of a 3x3 stride-1 convolution with Cin == Cout are
        # launches of one kernel on one grid (operands swapped): one class
        if phase in ("fwd", "dgrad") and L["R"] == 3 and L["stride"] == 1 and L["Cin"] == L["Cout"] and L["Cin"] % 64 == 0:
            phase = "fwd+dgrad (patch_kernel)"
        return "conv%dx%d s%d %d->%d @%d %s" % (L["R"], L["S"], L["stride"], L["Cin"], L["Cout"], L["H"], phase)
    if L["op"] == "bn":
        return "bn%s%s C%d @%d %s" % ("+res" if L["res"] >= 0 else "", "+relu" if L["relu"] else "", L["C"], L["H"], phase)
    if L["op"] == "pool":
        return "pool-%s C%d @%d %s" % (L["mode"], L["C"], L["H"], phase)
    if L["op"] == "add":
        return "add C%d @%d %s" % (L["C"], L["H"], phase)
    return "fc_loss %s" % phase


def layer_work(L, phase, esz):
    """(flops, algorithmic HBM bytes) of one call; conv flops at true K."""
    if L["op"] == "conv":
        Ho = (L["H"] + 2 * L["pad"] - L["R"]) // L["stride"] + 1
        Wo = (L["W"] + 2 * L["pad"] - L["S"]) // L["stride"] + 1
        fl = 2.0 * L["N"] * Ho * Wo * L["Cout"] * L["R"] * L["S"] * L["Cin"]
        xin = L["N"] * L["H"] * L["W"] * L["Cin"] * esz
        yout = L["N"] * Ho * Wo * L["Cout"] * esz
        wb = L["Cout"] * L["R"] * L["S"] * L["Cin"]
        if phase == "wgrad":
            return fl, xin + yout + 4 * wb
        return fl, xin + yout + esz * wb
    if L["op"] == "bn":
        T = L["N"] * L["H"] * L["W"] * L["C"] * esz
        res = 1 if L["res"] >= 0 else 0
        if phase == "fwd":
            # inside the step the statistics arrive from the convolution's epilogue: the call reads x
            # (and the residual) and writes y
            return 0.0, (2 + res) * T
        # dy and x twice, dx once; with a residual branch: dy, y, x in, masked gradient out (it is the
        # residual gradient), then that and x in, dx out
        return 0.0, (5 + 2 * res) * T
    if L["op"] == "pool":
        T = L["N"] * L["H"] * L["W"] * L["C"] * esz
        out = T // 4 if L["mode"] == "max2" else L["N"] * L["C"] * esz
        return 0.0, T + out + (out // esz if L["mode"] == "max2" else 0)
    if L["op"] == "add":
        T = L["N"] * L["H"] * L["W"] * L["C"] * esz
        return 0.0, 3 * T
    return 0.0, 0.0


def vit_call_work(net, name):
    """(kind, flops, bytes) of one call of the transformer step, by its name without the block prefix.
    Algorithmic work: matrix products at their true sizes (recomputation inside the attention backward
    is not counted), element-wise calls at the tensors they must read and write once."""
    B, T, d, m, h = net.batch, net.tokens, net.dim, net.mlp, net.heads
    rows, es = B * T, 2 if net.dtype == "bf16" else 4
    lin = {"qkv": (d, 3 * d), "proj": (d, d), "fc1": (d, m), "fc2": (m, d), "embed": (net.patch * net.patch * 3, d)}
    part = name.split(".")
    if part[0] in lin and part[1] in ("gemm", "gemm_gelu", "gemm_res", "dgrad", "wgrad"):
        K, N = lin[part[0]]
        r = B * (T - 1) if part[0] == "embed" else rows
        out_b = {"gemm": r * N * es, "gemm_gelu": 2 * r * N * es, "gemm_res": r * N * es, "dgrad": r * K * es, "wgrad": N * K * 4}[part[1]]
        in_b = {"gemm": r * K * es, "gemm_gelu": r * K * es, "gemm_res": r * (K + N) * es, "dgrad": r * N * es,
                "wgrad": r * (K + N) * es}[part[1]]
        return "mfma", 2.0 * r * K * N, in_b + out_b + (0 if part[1] == "wgrad" else N * K * es)
    if name == "attn":
        return "mfma", 4.0 * B * h * T * T * (d // h), rows * 4 * d * es
    if name == "attn.bwd":
        return "mfma", 10.0 * B * h * T * T * (d // h), rows * (3 * d + 2 * d + 3 * d) * es
    ew = {"ln1": 2 * d, "ln2": 2 * d, "ln1.bwd": 4 * d, "ln2.bwd": 4 * d,
          "fc1.gelu.bwd": 3 * m, "qkv.dbias": 3 * d, "proj.dbias": d, "fc2.dbias": d}
    if name in ew:
        return "hbm", 0.0, rows * ew[name] * es
    if name == "update":
        return "hbm", 0.0, net.n_params() * 22
    return "hbm", 0.0, 0


def bench_vit(args):
    """The same measurement for the paper's second model family: ViT-B/16 on 224 x 224 inputs."""
    import numpy as np
    import torch
    import workloads as WL
    from paper_2503_23186_amd import cnnk as _cnnk
    from paper_2503_23186_amd.vit import VitRunner
    net = WL.vit_b16(batch=args.batch or 64)
    inp = WL.make_vit_inputs(net, 6)
    run = VitRunner(net, keep_probs=False)
    run.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    lr, mu, wd = 0.01, 0.9, 0.0
    stream = torch.cuda.current_stream().cuda_stream
    cal = torch.zeros(2 * CAL_ELEMS, dtype=torch.bfloat16, device="cuda:0")
    _cnnk.cnnk_grad_route(CAL_ELEMS, _cnnk.BF16, cal, cal[CAL_ELEMS:], 0, stream)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        run.step(lr, mu, wd)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run.step(lr, mu, wd)
    torch.cuda.synchronize()
    ms_per_step = 1e3 * (time.perf_counter() - t0) / args.steps
    loss = run.loss.item()
    assert np.isfinite(loss), "loss is not finite"

    run.enable_timing(True)
    nt = max(args.timed_steps, 1)
    acc = {}
    per_call = np.zeros(run.n_calls)
    _cnnk.cnnk_grad_route(MARK_BEGIN_ELEMS, _cnnk.BF16, cal, cal[CAL_ELEMS:], 0, stream)
    for _ in range(nt):
        run.step(lr, mu, wd)
        torch.cuda.synchronize()
        times = run.call_times_ms()
        per_call += np.asarray(times) / nt
        for name, t in zip(run.call_names, times):
            key = name.split(".", 1)[1] if name.startswith("block") else name
            a = acc.setdefault(key, dict(ms=0.0, calls=0))
            a["ms"] += t
            a["calls"] += 1
    _cnnk.cnnk_grad_route(MARK_END_ELEMS, _cnnk.BF16, cal, cal[CAL_ELEMS:], 0, stream)
    torch.cuda.synchronize()
    run.enable_timing(False)
    del cal
    # what an event pair costs with one tiny launch inside: the smallest call of the step
    ev_overhead = min(a["ms"] / a["calls"] for a in acc.values()) * 0.5
    rows = []
    for key, a in acc.items():
        kind, fl, by = vit_call_work(net, key)
        avg = max(a["ms"] / a["calls"] - ev_overhead, 1e-6)
        rows.append(dict(key=key, kind=kind, calls_per_step=a["calls"] // nt, avg_ms=avg, ms_per_step=avg * a["calls"] / nt,
                         flops=fl, bytes=by))
    rows.sort(key=lambda r: -r["ms_per_step"])
    if args.layers:
        for r in rows:
            sys.stderr.write("%-20s x%-2d %8.3f ms/call %8.3f ms/step %8.1f TFLOP/s %8.1f GB/s\n"
                             % (r["key"], r["calls_per_step"], r["avg_ms"], r["ms_per_step"], r["flops"] / r["avg_ms"] / 1e9,
                                r["bytes"] / r["avg_ms"] / 1e6))
    dom = rows[0]
    if dom["kind"] == "mfma":
        ach = dom["flops"] / dom["avg_ms"] / 1e9
        roof = dict(bound="mfma", kernel=dom["key"], achieved=round(ach, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(ach / PEAK_BF16_TFLOPS, 4),
                    traffic=MEASURED_TRAFFIC_BYTES.get(dom["key"]) if not args.batch else None, avg_ms=round(dom["avg_ms"], 4),
                    calls_per_step=dom["calls_per_step"])
    else:
        ach = dom["bytes"] / dom["avg_ms"] / 1e6
        roof = dict(bound="hbm", kernel=dom["key"], achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(ach / PEAK_HBM_GBS, 4), traffic=None, avg_ms=round(dom["avg_ms"], 4),
                    calls_per_step=dom["calls_per_step"])
    mm = [r for r in rows if r["kind"] == "mfma"]
    ew = [r for r in rows if r["kind"] == "hbm" and r["bytes"]]
    mm_ms, ew_ms = sum(r["ms_per_step"] for r in mm), sum(r["ms_per_step"] for r in ew)
    mm_fl = sum(r["flops"] * r["calls_per_step"] for r in mm)
    ew_by = sum(r["bytes"] * r["calls_per_step"] for r in ew)
    roof["matmul_all"] = dict(tflops=round(mm_fl / mm_ms / 1e9, 2), frac_of_mfma_peak=round(mm_fl / mm_ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                              ms_per_step=round(mm_ms, 4))
    roof["elementwise_all"] = dict(gbs=round(ew_by / ew_ms / 1e6, 1), frac_of_hbm_peak=round(ew_by / ew_ms / 1e6 / PEAK_HBM_GBS, 4),
                                   ms_per_step=round(ew_ms, 4))

    # the scheduler's choice for 8 such devices: components = embedding, per block its attention half
    # and its MLP half, head; times from the calls above (Section III-B/III-C; a prediction)
    from paper_2503_23186_amd import asa
    comps = asa.components_from_vit(net, run.call_names, [max(t - ev_overhead, 0.0) for t in per_call])
    plan = asa.solve(comps, asa.Cluster(K=8, mem=288e9, bw=153e9, lat=5e-6, d=2))
    by_part = {}
    for c, s_ in zip(comps, plan.assignment):
        part = c.name.split(".")[-1]
        by_part.setdefault(part, {}).setdefault(s_[0], 0)
        by_part[part][s_[0]] += 1
    asa_out = dict(devices=8, components=len(comps), predicted_ms_per_step=round(plan.time * 1e3, 4),
                   single_device_ms=round(sum(c.t for c in comps) * 1e3, 4), strategies=by_part,
                   basis="cost model of the paper's scheduler over this run's measured per-call times; prediction only")

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import vit as OV
        sample_batch = 2
        small = WL.vit_b16(batch=sample_batch)
        sinp = WL.make_vit_inputs(small, 6)
        t0 = time.perf_counter()
        OV.train_step(small.cfg(), sinp["x"], sinp["labels"], sinp["params"], sinp["mom"], lr, mu, wd)
        cdt = time.perf_counter() - t0
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
        cpu = dict(value=round(sample_batch / cdt, 3), unit="images/s", cores=cores, kind="oracle",
                   sample="one fp64 oracle step of the same network at batch %d (%.1f s)" % (sample_batch, cdt))
    out = {
        "metric": "train images/sec on 1 GPU (ViT-B/16 224x224 bf16 b%d); matmul MFMA %% of peak" % net.batch,
        "value": round(net.batch / (ms_per_step * 1e-3), 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": net.dtype, "data": "synthetic",
        "config": {"workload": "ViT-B/16 224x224x3 100-class (197 tokens, width 768, 12 blocks, 85.9 M parameters), batch %d, "
                               "%s storage / fp32 accumulate, SGD momentum" % (net.batch, net.dtype),
                   "config_id": 6, "global_batch": net.batch, "loss": round(loss, 5),
                   "tflops_per_step": round(net.flops() / 1e12, 3)},
        "roofline": roof, "cpu_baseline": cpu, "asa_plan": asa_out,
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--batch", type=int, default=0, help="override the config's batch (not a bench line)")
    ap.add_argument("--timed-steps", type=int, default=5, help="extra steps with per-call HIP events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", action="store_true", help="print the per-call table to stderr")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="kernel-selection override passed to cnnk_tune (experiments; not a bench line)")
    ap.add_argument("--one-stream", action="store_true",
                    help="keep the weight gradients on the main stream (default: a second stream)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)\n")
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as WL
    from paper_2503_23186_amd import StepRunner

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py needs a GPU (there is no CPU fallback)\n")
        sys.exit(2)
    for kv in args.tune:
        from paper_2503_23186_amd import cnnk
        k, v = kv.split("=")
        cnnk.cnnk_tune(int(k), int(v))
    if args.config == 6:
        return bench_vit(args)
    kw = {"batch": args.batch} if args.batch else {}
    net = WL.build_config(args.config, **kw)
    inp = WL.make_inputs(net, args.config)
    run = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype, keep_probs=False,
                     two_streams=not args.one_stream)
    run.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    lr, mu, wd = 0.1, 0.9, 0.0
    stream = torch.cuda.current_stream().cuda_stream

    from paper_2503_23186_amd import cnnk as _cnnk
    cal = torch.zeros(2 * CAL_ELEMS, dtype=torch.bfloat16, device="cuda:0")
    _cnnk.cnnk_grad_route(CAL_ELEMS, _cnnk.BF16, cal, cal[CAL_ELEMS:], 0, stream)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        run.step(lr, mu, wd, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run.step(lr, mu, wd, stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    loss = run.loss.item()
    assert np.isfinite(loss), "loss is not finite"

    # ---- per-call timing with HIP events recorded by the library on the same stream -----------
    esz = 2 if net.dtype == "bf16" else 4
    run.enable_timing(True)
    acc = {}
    empty = []
    nt = max(args.timed_steps, 1)
    mean_times = None
    _cnnk.cnnk_grad_route(MARK_BEGIN_ELEMS, _cnnk.BF16, cal, cal[CAL_ELEMS:], 0, stream)
    for _ in range(nt):
        run.step(lr, mu, wd, stream)
        torch.cuda.synchronize()
        times = run.group_times_ms()
        mean_times = times if mean_times is None else [a + b for a, b in zip(mean_times, times)]
        for g, li, phase in run.group_table():
            if phase == "none":
                # an empty event pair (a layer without a second backward call): what two event
                # records cost with nothing between them
                empty.append(times[g])
                continue
            if li < 0:
                continue
            L = net.layers[li]
            if L["op"] == "conv" and phase == "dgrad" and L["x"] == 0:
                continue
            key = layer_key(L, phase)
            fl, by = layer_work(L, phase, esz)
            a = acc.setdefault(key, dict(ms=0.0, calls=0, flops=fl, bytes=by, op=L["op"]))
            a["ms"] += times[g]
            a["calls"] += 1
    torch.cuda.synchronize()
    run.enable_timing(False)
    # Every timed call sits between two event records of its own; the pair costs a few microseconds
    # even when empty.  That overhead, measured on the empty pairs of the same steps, is taken off
    # each call so that the durations are the kernels' (they then agree with a kernel trace).
    ev_overhead = float(np.median(empty)) if empty else 0.0
    mean_times = [t / nt for t in mean_times]
    rows = []
    for key, a in acc.items():
        avg = max(a["ms"] / a["calls"] - ev_overhead, 1e-6)
        a["ms"] = avg * a["calls"]
        rows.append(dict(key=key, op=a["op"], calls_per_step=a["calls"] // nt, avg_ms=avg,
                         ms_per_step=a["ms"] / nt, flops=a["flops"], bytes=a["bytes"]))
    rows.sort(key=lambda r: -r["ms_per_step"])
    conv_ms = sum(r["ms_per_step"] for r in rows if r["op"] == "conv")
    conv_flops = sum(r["flops"] * r["calls_per_step"] for r in rows if r["op"] == "conv")
    ew_ms = sum(r["ms_per_step"] for r in rows if r["op"] in ("bn", "pool", "add"))
    ew_bytes = sum(r["bytes"] * r["calls_per_step"] for r in rows if r["op"] in ("bn", "pool", "add"))
    if args.layers:
        for r in rows:
            tf = r["flops"] / r["avg_ms"] / 1e9 if r["flops"] else 0.0
            gb = r["bytes"] / r["avg_ms"] / 1e6
            sys.stderr.write("%-34s x%-2d %8.3f ms/call %8.3f ms/step %8.1f TFLOP/s %8.1f GB/s\n"
                             % (r["key"], r["calls_per_step"], r["avg_ms"], r["ms_per_step"], tf, gb))
        sys.stderr.write("event-pair overhead taken off every call: %.4f ms\n" % ev_overhead)
        sys.stderr.write("timed-step total %.3f ms; conv %.3f ms (%.1f TFLOP/s); bn/pool/add %.3f ms (%.0f GB/s)\n"
                         % (sum(r["ms_per_step"] for r in rows), conv_ms, conv_flops / conv_ms / 1e9 if conv_ms else 0,
                            ew_ms, ew_bytes / ew_ms / 1e6 if ew_ms else 0))
    dom = rows[0]
    _cnnk.cnnk_grad_route(MARK_END_ELEMS, _cnnk.BF16, cal, cal[CAL_ELEMS:], 0, stream)
    torch.cuda.synchronize()
    del cal
    if dom["op"] == "conv":
        ach = dom["flops"] / dom["avg_ms"] / 1e9
        roof = dict(bound="mfma", kernel=dom["key"], achieved=round(ach, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(ach / PEAK_BF16_TFLOPS, 4),
                    traffic=MEASURED_TRAFFIC_BYTES.get(dom["key"]) if args.config == 3 and not args.batch else None,
                    avg_ms=round(dom["avg_ms"], 4),
                    timing="HIP events on the launch stream around each of the class's %d calls in %d single-stream "
                           "steps, less the cost of an empty event pair (%.4f ms)" % (dom["calls_per_step"] * nt, nt, ev_overhead),
                    calls_per_step=dom["calls_per_step"])
    else:
        ach = dom["bytes"] / dom["avg_ms"] / 1e6
        roof = dict(bound="hbm", kernel=dom["key"], achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(ach / PEAK_HBM_GBS, 4), traffic=None, avg_ms=round(dom["avg_ms"], 4),
                    calls_per_step=dom["calls_per_step"])
    roof["conv_all"] = dict(tflops=round(conv_flops / conv_ms / 1e9, 2) if conv_ms else None,
                            frac_of_mfma_peak=round(conv_flops / conv_ms / 1e9 / PEAK_BF16_TFLOPS, 4) if conv_ms else None,
                            ms_per_step=round(conv_ms, 4))
    roof["elementwise_all"] = dict(gbs=round(ew_bytes / ew_ms / 1e6, 1) if ew_ms else None,
                                   frac_of_hbm_peak=round(ew_bytes / ew_ms / 1e6 / PEAK_HBM_GBS, 4) if ew_ms else None,
                                   ms_per_step=round(ew_ms, 4))

    # ---- what the paper's scheduler would choose for 8 such devices, from the measured times ----
    # (Section III-B/III-C on the host: t_comp = the per-call times above, t_comm from byte counts;
    # a model's prediction, not a measurement: nothing here runs on more than one GPU)
    from paper_2503_23186_amd import asa
    prof_rows = []
    for g, li, phase in run.group_table():
        if phase != "none":
            prof_rows.append((li, phase, max(mean_times[g] - ev_overhead, 0.0)))
    comps = asa.components_from_tape(net.layers, prof_rows, net.dtype)
    cluster = asa.Cluster(K=8, mem=288e9, bw=153e9, lat=5e-6, d=2)   # xGMI: a ring is bound by one 153 GB/s link
    plan = asa.solve(comps, cluster)
    kinds = [s[0] for s in plan.assignment]
    asa_out = dict(devices=8, components=len(comps), predicted_ms_per_step=round(plan.time * 1e3, 4),
                   single_device_ms=round(sum(c.t for c in comps) * 1e3, 4),
                   strategies={k: kinds.count(k) for k in ("DP", "HP", "MP")},
                   basis="cost model of the paper's scheduler over this run's measured per-call times; prediction only")

    # ---- the validation pass of the epoch loop (inference-mode forward), reported beside the step ----
    for _ in range(3):
        _cnnk.cnnk_eval_step(run.c_layers, len(net.layers), run.buffers, run.labels, run.loss, run.pred, None, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_eval = 20
    for _ in range(n_eval):
        _cnnk.cnnk_eval_step(run.c_layers, len(net.layers), run.buffers, run.labels, run.loss, run.pred, None, stream)
    torch.cuda.synchronize()
    eval_ms = 1e3 * (time.perf_counter() - t0) / n_eval

    # ---- the oracle on the host cores, on a bounded sample of the same workload ---------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sample_batch = 64
        small = WL.build_config(args.config, batch=sample_batch)
        sinp = WL.make_inputs(small, args.config)
        t0 = time.perf_counter()
        oracle.train_step(small, sinp["x"], sinp["labels"], sinp["params"], sinp["mom"], lr, mu, wd)
        cdt = time.perf_counter() - t0
        cpu = dict(value=round(sample_batch / cdt, 3), unit="images/s", cores=oracle.ops.num_threads(), kind="oracle",
                   sample="one fp64 oracle step of the same network at batch %d (%.1f s)" % (sample_batch, cdt))

    out = {
        "metric": "train images/sec on 1 GPU (ResNet-18 32x32 bf16 b256); conv MFMA % of peak",
        "value": round(net.batch / (ms_per_step * 1e-3), 1),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": net.dtype,
        "data": "synthetic",
        "config": {"workload": "%s 32x32x3 100-class, batch %d, %s storage / fp32 accumulate, SGD momentum"
                               % (net.name, net.batch, net.dtype),
                   "config_id": args.config, "global_batch": net.batch, "loss": round(loss, 5)},
        "roofline": roof,
        "cpu_baseline": cpu,
        "asa_plan": asa_out,
        "validation_pass": {"ms_per_batch": round(eval_ms, 4), "images_per_s": round(net.batch / (eval_ms * 1e-3), 1)},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
