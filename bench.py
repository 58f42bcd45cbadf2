#!/usr/bin/env python3
"""Benchmark of the SACP gradient-synchronisation path on one MI355X.

One step = one whole iteration of the 8-layer CNN workload (config 5): route selection
for every layer, then top-down (Algorithm 2 order) on one stream per layer: the three FC
layers pack their P*B sufficient factors, rebuild dW on the MFMA pipe and apply
momentum-SGD in the epilogue; the five conv layers sum their P dense gradient copies per
key-range shard and update.  Inputs are synthetic, seeded, and resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--fc-dtype bf16|f32]
                    [--no-cpu-baseline] [--extras PATH]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "SFB reconstruct+update TFLOP/s (MFMA util %); dense shard-sum GB/s; ms/iter"
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by a copy kernel of known size); filled in from the committed
# profile summaries, None where not measured.
MEASURED_TRAFFIC_BYTES = {"bf16": 922_900_000, "f32": None}   # fc6 launch; profiles/bench_config5_bf16_hbm_traffic.txt


class HipEvents:
    """Raw HIP events (the library records them on each layer's own stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.all = []

    def new(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        self.all.append(ev)
        return ev.value

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return ms.value

    def close(self):
        for ev in self.all:
            self.hip.hipEventDestroy(ev)
        self.all = []


def build_device_sets(layers, fc_dtype, n_sets, psd, torch, dev, one_stream=False):
    """Uploads `n_sets` independent copies of every layer's buffers (rotated between steps so
    that a step never finds its operands in the 256 MB last-level cache from the step before)."""
    sets = []
    for _ in range(n_sets):
        streams = [torch.cuda.Stream(device=dev) for _ in layers]
        if one_stream:
            streams = [streams[0]] * len(layers)
        tasks = []
        for L, st in zip(layers, streams):
            if L["kind"] == "conv":
                plan = psd.plan_layer(psd.LAYER_CONV, L["n"], 1, L["B"], L["P"])
                tasks.append(dict(name=L["name"], kind="conv", plan=plan, S=L["S"],
                                  G=[torch.from_numpy(g).to(dev) for g in L["G"]],
                                  W=torch.from_numpy(L["W"]).to(dev), Mom=torch.from_numpy(L["Mom"]).to(dev),
                                  stream=st))
            else:
                plan = psd.plan_layer(psd.LAYER_FC, L["M"], L["N"], L["B"], L["P"])
                U, ldu, V, ldv = psd.alloc_factors(plan, fc_dtype, dev)
                tasks.append(dict(name=L["name"], kind="fc", plan=plan, factor_dtype=fc_dtype,
                                  delta=[torch.from_numpy(x).to(dev) for x in L["delta"]],
                                  act=[torch.from_numpy(x).to(dev) for x in L["act"]],
                                  U=U, ldu=ldu, V=V, ldv=ldv,
                                  W=torch.from_numpy(L["W"]).to(dev), Mom=torch.from_numpy(L["Mom"]).to(dev),
                                  stream=st))
        sets.append(tasks)
    return sets


def layer_work(L, fc_dtype_name):
    """Algorithmic flops and HBM bytes of one layer's sync kernel (and of its pack)."""
    if L["kind"] == "conv":
        n, P = L["n"], L["P"]
        return dict(flops=n * (P + 3), bytes=n * (4 * P + 16), pack_bytes=0)
    N, M, K = L["N"], L["M"], L["P"] * L["B"]
    es = 2 if fc_dtype_name == "bf16" else 4
    return dict(flops=2 * N * M * K, bytes=16 * N * M + K * (M + N) * es,
                pack_bytes=K * (M + N) * (4 + es))


def cpu_baseline(layers, fc_dtype_name, lr, mu):
    """The oracle, as it stands, on one pass of the same iteration (host cores of this machine)."""
    from oracle import psd_oracle as orc
    orc.lib()
    t0 = time.perf_counter()
    for L in reversed(layers):
        if L["kind"] == "conv":
            orc.sync_dense_ps(L["G"], L["W"], L["Mom"], lr, mu, L["S"])
        else:
            U, V = orc.pack_factors(L["delta"], L["act"], fc_dtype_name)
            orc.sync_fc_sfb(U, V, L["W"], L["Mom"], lr, mu)
    return time.perf_counter() - t0, orc.num_threads()


def cpu_baseline_configs(inputs):
    """The oracle on the single-layer FC configurations: reconstruct + update, all host threads, and
    one thread for the two small ones (part of the cpu_baseline leg; only run with --extras)."""
    from oracle import psd_oracle as orc
    orc.lib()
    all_threads = orc.num_threads()
    out = []
    for cfg in (1, 2, 3, 4):
        d = inputs.fc_config(cfg)
        name = d["factor_dtype"]
        U, V = orc.pack_factors(d["delta"], d["act"], name)
        flops = 2.0 * d["N"] * d["M"] * d["P"] * d["B"]
        for threads in ([all_threads, 1] if cfg <= 2 else [all_threads]):
            orc.set_num_threads(threads)
            t0 = time.perf_counter()
            orc.sync_fc_sfb(U, V, d["W"], d["Mom"], inputs.LR, inputs.MU)
            dt = time.perf_counter() - t0
            out.append({"config": cfg, "factor_dtype": name, "threads": threads, "ms": round(dt * 1e3, 2),
                        "GFLOPs": round(flops / dt / 1e9, 2)})
        orc.set_num_threads(all_threads)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--fc-dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--sets", type=int, default=2, help="rotating buffer sets")
    ap.add_argument("--rule", choices=["alg3", "vs_dense"], default="alg3")
    ap.add_argument("--one-stream", action="store_true",
                    help="put every layer on the same stream (comparison only; the path uses one stream per layer)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", default=None, help="also time configs 1-4 and a dense size sweep; write JSON here")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="only run a plain device-to-device copy of this many MiB, 10 times (calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters: the copy reads and writes exactly that many bytes)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (peers' factors and gradients are seeded buffers in "
              "device memory); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_1512_06216_amd import binding as psd
    from paper_1512_06216_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    psd.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_probe:
        n = args.copy_probe * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_MiB": args.copy_probe, "copies": 10}))
        return 0
    lr, mu = inputs.LR, inputs.MU
    fc_dtype = psd.BF16 if args.fc_dtype == "bf16" else psd.F32
    rule = psd.RULE_ALG3 if args.rule == "alg3" else psd.RULE_SFB_VS_DENSE

    layers = inputs.cnn_iteration()
    for L in layers:
        L["S"] = inputs.CNN_S
        L.setdefault("B", inputs.CNN_B)
    sets = build_device_sets(layers, fc_dtype, args.sets, psd, torch, dev, args.one_stream)
    work = [layer_work(L, args.fc_dtype) for L in layers]
    torch.cuda.synchronize()

    ev = HipEvents()
    total = args.warmup + args.steps
    iters, marks = [], []
    for i in range(total):
        tasks = [dict(t) for t in sets[i % args.sets]]
        m = []
        for t in tasks:
            t["ev_begin"], t["ev_end"] = ev.new(), ev.new()
            m.append((t["ev_begin"], t["ev_end"]))
        iters.append(psd.Iteration(tasks))
        marks.append(m)

    kinds = [psd.LAYER_CONV if L["kind"] == "conv" else psd.LAYER_FC for L in layers]
    dims = [(L["n"], 1) if L["kind"] == "conv" else (L["M"], L["N"]) for L in layers]

    def step(i):
        it = iters[i]
        # route selection for every layer (Algorithm 3), then the top-down issue
        for j, (kind, (M, N)) in enumerate(zip(kinds, dims)):
            it.tasks[j].plan = psd.plan_layer(kind, M, N, layers[j]["B"], layers[j]["P"])
        it.run(lr, mu, rule)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, total):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # per-kernel durations from the events recorded inside the timed steps
    dur = np.zeros((args.steps, len(layers)))
    for s in range(args.steps):
        for j, (a, b) in enumerate(marks[args.warmup + s]):
            dur[s, j] = ev.elapsed_ms(a, b)
    ev.close()
    mean_ms = dur.mean(axis=0)
    per_layer = {}
    for j, L in enumerate(layers):
        w = work[j]
        per_layer[L["name"]] = dict(ms=round(float(mean_ms[j]), 5), min_ms=round(float(dur[:, j].min()), 5),
                                    GBps=round(w["bytes"] / mean_ms[j] / 1e6, 1),
                                    TFLOPs=round(w["flops"] / mean_ms[j] / 1e9, 2))

    fc_idx = [j for j, L in enumerate(layers) if L["kind"] == "fc"]
    conv_idx = [j for j, L in enumerate(layers) if L["kind"] == "conv"]
    fc_flops = sum(work[j]["flops"] for j in fc_idx)
    value = fc_flops / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the bf16/fp32 reconstruct+update kernel of the largest layer (fc6); it has a
    # kernel instantiation of its own, so a per-kernel profile reports exactly these launches
    dom = [j for j in fc_idx if layers[j]["name"] == "fc6"]
    dom_bytes = float(np.mean([work[j]["bytes"] for j in dom]))
    dom_flops = float(np.mean([work[j]["flops"] for j in dom]))
    dom_ms = float(np.mean([mean_ms[j] for j in dom]))
    hbm_gbs = dom_bytes / dom_ms / 1e6
    mfma_tf = dom_flops / dom_ms / 1e9
    peak_tf = PEAK_MFMA_TFLOPS[args.fc_dtype]
    if args.fc_dtype == "bf16":
        # bf16 factors: 16 B of W/Mom traffic per 2K flops puts the kernel on the HBM side of the ridge
        roofline = dict(bound="hbm", achieved=round(hbm_gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(hbm_gbs / PEAK_HBM_GBS, 4), traffic=MEASURED_TRAFFIC_BYTES["bf16"])
    else:
        roofline = dict(bound="mfma", achieved=round(mfma_tf, 2), peak=peak_tf, unit="TFLOP/s",
                        frac=round(mfma_tf / peak_tf, 4), traffic=MEASURED_TRAFFIC_BYTES["f32"])
    roofline.update(kernel="sfb_%s_kernel, fc6 launches (9216 -> 4096, K = 2048)" % args.fc_dtype,
                    avg_launch_ms=round(dom_ms, 5), algorithmic_bytes_per_launch=int(dom_bytes),
                    flops_per_launch=int(dom_flops), mfma_tflops=round(mfma_tf, 2),
                    mfma_frac=round(mfma_tf / peak_tf, 4), hbm_gbps=round(hbm_gbs, 1),
                    hbm_frac=round(hbm_gbs / PEAK_HBM_GBS, 4))

    conv_bytes = sum(work[j]["bytes"] for j in conv_idx)
    conv_ms = float(sum(mean_ms[j] for j in conv_idx))
    out = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if args.fc_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "config5_full_8layer_cnn_iteration", "fc_factor_dtype": args.fc_dtype,
                   "accumulate": "f32", "B": inputs.CNN_B, "P": inputs.CNN_P, "S": inputs.CNN_S,
                   "conv_keys": inputs.conv_sizes(), "fc_shapes_MxN": inputs.FC_SHAPES,
                   "rule": args.rule, "rotating_sets": args.sets, "streams": 1 if args.one_stream else len(layers),
                   "fc_flops_per_step": fc_flops},
        "roofline": roofline,
        "dense_shard_sum": {"GBps_sum_of_kernels": round(conv_bytes / conv_ms / 1e6, 1),
                            "frac_hbm": round(conv_bytes / conv_ms / 1e6 / PEAK_HBM_GBS, 4),
                            "bytes_per_step": conv_bytes, "note": "five conv layers, 2.3M keys in all"},
        "per_layer": per_layer,
        "routes": {L["name"]: psd.ROUTE_NAMES[sets[0][j]["plan"].route_alg3 if rule == psd.RULE_ALG3
                                              else sets[0][j]["plan"].route_vs_dense]
                   for j, L in enumerate(layers)},
    }

    if args.extras:
        from paper_1512_06216_amd import bench_extras
        extras = bench_extras.run(psd, inputs, torch, dev)
        if not args.no_cpu_baseline:
            extras["cpu_baseline_configs"] = cpu_baseline_configs(inputs)
        with open(args.extras, "w") as f:
            json.dump(extras, f, indent=1)
        out["extras_file"] = args.extras

    if not args.no_cpu_baseline:
        del sets, iters
        torch.cuda.empty_cache()
        secs, threads = cpu_baseline(layers, args.fc_dtype, lr, mu)
        out["cpu_baseline"] = {"value": round(fc_flops / secs / 1e12, 5), "unit": "TFLOP/s", "cores": threads,
                               "kind": "oracle", "ms_per_step": round(secs * 1e3, 1),
                               "sample": "one full pass of the same config-5 iteration (all 8 layers, float64 oracle)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
