#!/usr/bin/env python3
"""Benchmark of the SACP gradient-synchronisation path on one MI355X.

One step = one whole iteration of the 8-layer CNN workload (config 5): route selection
for every layer, then top-down (Algorithm 2 order) on one stream per layer: the three FC
layers pack their P*B sufficient factors, rebuild dW on the MFMA pipe and apply
momentum-SGD in the epilogue; the five conv layers sum their P dense gradient copies per
key-range shard and update (one launch for the five).  Inputs are synthetic, seeded, and
resident in HBM before the timed region.  Prints ONE JSON line.

Timed region: K steps issued back to back; every layer keeps its own stream, so a layer's
synchronisation in step i+1 follows its synchronisation in step i (the data dependency
between iterations), while different layers of neighbouring steps may overlap, as they do
under wait-free backpropagation.  The same K steps with a full join between steps (every
stream waits until the step before has finished everywhere), on one stream, and with fp32
factors are timed as well and reported beside the headline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--fc-dtype bf16|f32]
                    [--no-cpu-baseline] [--no-side-legs] [--extras PATH]
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
PREWARM_MS = 150.0      # untimed work before the W warm-up steps: the clocks of an idle GPU take ~0.1 s to settle

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by a copy kernel of known size); filled in from the committed
# profile summaries, None where not measured.
MEASURED_TRAFFIC_BYTES = {"bf16": 938_400_000, "f32": None}   # fc6 launch; profiles/bench_config5_bf16_hbm_traffic.txt


class HipEvents:
    """Raw HIP events (the library records them on each layer's own stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipStreamWaitEvent.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint]
        self.all = []

    def new(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        self.all.append(ev)
        return ev.value

    def record(self, event, stream_handle):
        if self.hip.hipEventRecord(event, stream_handle) != 0:
            raise RuntimeError("hipEventRecord failed")

    def wait(self, stream_handle, event):
        if self.hip.hipStreamWaitEvent(stream_handle, event, 0) != 0:
            raise RuntimeError("hipStreamWaitEvent failed")

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


def build_device_sets(layers, fc_dtype, n_sets, psd, torch, dev, one_stream=False, bf16_blocks=False):
    """Uploads `n_sets` independent copies of every layer's buffers (rotated between steps so
    that a step never finds its operands in the 256 MB last-level cache from the step before)."""
    sets = []
    # one stream per layer, the same for every buffer set: a layer's synchronisations of consecutive steps
    # follow each other in stream order (step i+1 updates the weights step i wrote)
    streams = [torch.cuda.Stream(device=dev) for _ in layers]
    if one_stream:
        streams = [streams[0]] * len(layers)
    for _ in range(n_sets):
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
                t = dict(name=L["name"], kind="fc", plan=plan, factor_dtype=fc_dtype,
                         delta=[torch.from_numpy(x).to(dev) for x in L["delta"]],
                         act=[torch.from_numpy(x).to(dev) for x in L["act"]],
                         U=U, ldu=ldu, V=V, ldv=ldv, workspace=psd.alloc_workspace(plan, fc_dtype, dev),
                         W=torch.from_numpy(L["W"]).to(dev), Mom=torch.from_numpy(L["Mom"]).to(dev), stream=st)
                if bf16_blocks and fc_dtype == psd.BF16:
                    # the factors as P senders that round before sending would deliver them: one bf16 block per worker
                    one = psd.plan_layer(psd.LAYER_FC, L["M"], L["N"], L["B"], 1)
                    t["one"], t["U_blocks"], t["V_blocks"] = one, [], []
                    for p in range(L["P"]):
                        Ub, _, Vb, _ = psd.alloc_factors(one, psd.BF16, dev)
                        psd.pack_factors(one, [t["delta"][p]], [t["act"][p]], psd.BF16, Ub, ldu, Vb, ldv)
                        t["U_blocks"].append(Ub)
                        t["V_blocks"].append(Vb)
                tasks.append(t)
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


class Leg:
    """One timed configuration of the whole iteration (factor dtype, streams, step dependency)."""

    def __init__(self, layers, fc_dtype_name, psd, inputs, torch, dev, n_sets, rule, one_stream=False, bf16_blocks=False):
        self.layers, self.psd, self.inputs, self.torch = layers, psd, inputs, torch
        self.name = fc_dtype_name
        self.rule = rule
        fc_dtype = psd.BF16 if fc_dtype_name == "bf16" else psd.F32
        self.sets = build_device_sets(layers, fc_dtype, n_sets, psd, torch, dev, one_stream, bf16_blocks)
        self.n_sets = n_sets
        # FC layers handed over without stacked buffers (no pack launch): fp32 blocks as they are, or (sets built
        # with bf16_blocks) bf16 blocks as senders that round before sending deliver them
        self.blocks_in_place = False
        self.work = [layer_work(L, fc_dtype_name) for L in layers]
        self.kinds = [psd.LAYER_CONV if L["kind"] == "conv" else psd.LAYER_FC for L in layers]
        self.dims = [(L["n"], 1) if L["kind"] == "conv" else (L["M"], L["N"]) for L in layers]
        self.main = torch.cuda.current_stream().cuda_stream
        self.sync = HipEvents()                       # events of the step-to-step dependency
        self.ev_step_done = self.sync.new()
        self.ev_stream = {}
        for i in range(n_sets):
            for s in self.streams_of(i):
                self.ev_stream[s.cuda_stream] = self.sync.new()
        torch.cuda.synchronize()

    def streams_of(self, i):
        seen, out = set(), []
        for t in self.sets[i % self.n_sets]:
            if id(t["stream"]) not in seen:
                seen.add(id(t["stream"]))
                out.append(t["stream"])
        return out

    def run(self, steps, warmup, dependent, ev=None):
        """Returns (ms per step, per-step per-layer event pairs or None)."""
        psd, torch = self.psd, self.torch
        total = warmup + steps
        iters, marks = [], []
        for i in range(total):
            tasks = [dict(t) for t in self.sets[i % self.n_sets]]
            if self.blocks_in_place:
                for t in tasks:
                    if t["kind"] != "fc":
                        continue
                    if t["factor_dtype"] == psd.F32 and psd.sfb_blocks_supported(t["plan"]):
                        t.update(U=None, V=None, ldu=0, ldv=0)
                    elif "U_blocks" in t and psd.sfb_blocks_supported(t["plan"], psd.BF16, t["ldu"], t["ldv"]):
                        t.update(U=None, V=None, delta_f32=t["delta"], act_f32=t["act"], delta=t["U_blocks"], act=t["V_blocks"])
            if dependent:
                for t in tasks:
                    t["ev_ready"] = self.ev_step_done   # "the iteration before has finished on every stream"
            m = []
            if ev is not None and i >= warmup:
                for t in tasks:
                    t["ev_begin"], t["ev_end"] = ev.new(), ev.new()
                    m.append((t["ev_begin"], t["ev_end"]))
            iters.append(psd.Iteration(tasks))
            marks.append(m)

        own = [[t for t in self.sets[i % self.n_sets] if "U_blocks" in t] if self.blocks_in_place else []
               for i in range(total)]

        def step(i):
            it = iters[i]
            # bf16 blocks read in place: this worker still rounds its OWN block (1/P of the stacking pass)
            for t in own[i]:
                psd.pack_factors(t["one"], [t["delta"][0]], [t["act"][0]], psd.BF16, t["U_blocks"][0], t["ldu"],
                                 t["V_blocks"][0], t["ldv"], stream=t["stream"])
            # route selection for every layer (Algorithm 3), then the top-down issue; with `dependent` every
            # layer's stream first waits for ev_step_done of the step before
            for j, (kind, (M, N)) in enumerate(zip(self.kinds, self.dims)):
                it.tasks[j].plan = psd.plan_layer(kind, M, N, self.layers[j]["B"], self.layers[j]["P"])
            it.run(self.inputs.LR, self.inputs.MU, self.rule)
            if dependent:
                # join: the main stream waits for every layer's stream, then marks the step done
                for s in self.streams_of(i):
                    e = self.ev_stream[s.cuda_stream]
                    self.sync.record(e, s.cuda_stream)
                    self.sync.wait(self.main, e)
                self.sync.record(self.ev_step_done, self.main)

        if dependent:
            self.sync.record(self.ev_step_done, self.main)

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(warmup, total):
            step(i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        return ms, (marks[warmup:] if ev is not None else None)

    def prewarm(self):
        t0 = time.perf_counter()
        i = 0
        while (time.perf_counter() - t0) * 1e3 < PREWARM_MS:
            self.psd.Iteration(self.sets[i % self.n_sets]).run(self.inputs.LR, self.inputs.MU, self.rule)
            i += 1
            if i % 8 == 0:
                self.torch.cuda.synchronize()
        self.torch.cuda.synchronize()
        return i

    def layer_alone_ms(self, j, iters=40):
        """Median duration of layer j's sync kernel launched back to back with nothing else on the GPU."""
        psd, torch = self.psd, self.torch
        ts = []
        for rep in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for i in range(iters):
                t = self.sets[i % self.n_sets][j]
                psd.sync_fc_sfb(t["plan"], t["factor_dtype"], t["U"], t["ldu"], t["V"], t["ldv"], t["W"], t["Mom"],
                                self.inputs.LR, self.inputs.MU, workspace=t["workspace"])
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) / iters)
        return float(np.median(ts))

    def conv_alone_ms(self, iters=40):
        psd, torch = self.psd, self.torch
        conv = [j for j, L in enumerate(self.layers) if L["kind"] == "conv"]
        multi = [psd.DenseMulti([(tasks[j]["G"], tasks[j]["W"], tasks[j]["Mom"], tasks[j]["S"]) for j in conv])
                 for tasks in self.sets]
        ts = []
        for rep in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for i in range(iters):
                multi[i % self.n_sets].run(self.inputs.LR, self.inputs.MU)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) / iters)
        return float(np.median(ts))


def durations(ev, marks, n_layers):
    dur = np.zeros((len(marks), n_layers))
    for s, m in enumerate(marks):
        for j, (a, b) in enumerate(m):
            dur[s, j] = ev.elapsed_ms(a, b)
    return dur


def roofline_of(leg, dur, layers, name, alone=True):
    """Roofline object of the dominant kernel: the reconstruct+update kernel of fc6 (it has a kernel
    instantiation of its own, so a per-kernel profile reports exactly these launches)."""
    j = [i for i, L in enumerate(layers) if L["name"] == "fc6"][0]
    w = leg.work[j]
    avg_ms = float(dur[:, j].mean())
    med_ms = float(np.median(dur[:, j]))
    alone_ms = leg.layer_alone_ms(j) if alone else avg_ms
    peak_tf = PEAK_MFMA_TFLOPS[name]

    def fr(ms):
        return dict(avg_launch_ms=round(ms, 5), hbm_gbps=round(w["bytes"] / ms / 1e6, 1),
                    hbm_frac=round(w["bytes"] / ms / 1e6 / PEAK_HBM_GBS, 4), mfma_tflops=round(w["flops"] / ms / 1e9, 2),
                    mfma_frac=round(w["flops"] / ms / 1e9 / peak_tf, 4))
    inside, alone_fr = fr(avg_ms), (fr(alone_ms) if alone else None)
    if name == "bf16":
        # bf16 factors: 16 B of W/Mom traffic per 2K flops puts the kernel on the HBM side of the ridge
        r = dict(bound="hbm", achieved=inside["hbm_gbps"], peak=PEAK_HBM_GBS, unit="GB/s", frac=inside["hbm_frac"],
                 traffic=MEASURED_TRAFFIC_BYTES["bf16"])
    else:
        r = dict(bound="mfma", achieved=inside["mfma_tflops"], peak=peak_tf, unit="TFLOP/s", frac=inside["mfma_frac"],
                 traffic=MEASURED_TRAFFIC_BYTES["f32"])
    r.update(kernel="sfb_%s_kernel, fc6 launches (9216 -> 4096, K = 2048)" % name,
             algorithmic_bytes_per_launch=int(w["bytes"]), flops_per_launch=int(w["flops"]),
             note="achieved / frac: mean launch duration inside the timed iterations (other layers' kernels run "
                  "beside it on their own streams); 'alone': the same launch back to back with an idle GPU",
             in_iteration=dict(inside, median_launch_ms=round(med_ms, 5)), alone=alone_fr)
    return r


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
    ap.add_argument("--no-side-legs", action="store_true",
                    help="skip the legs reported beside the headline (overlapping steps, one stream, the other factor dtype, "
                         "dense sweep)")
    ap.add_argument("--no-alone", action="store_true",
                    help="skip the back-to-back launches of single kernels (so that a kernel trace of the run holds "
                         "nothing but whole iterations)")
    ap.add_argument("--extras", default=None, help="also time configs 1-4 and more; write JSON here")
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
    rule = psd.RULE_ALG3 if args.rule == "alg3" else psd.RULE_SFB_VS_DENSE

    layers = inputs.cnn_iteration()
    for L in layers:
        L["S"] = inputs.CNN_S
        L.setdefault("B", inputs.CNN_B)
    fc_idx = [j for j, L in enumerate(layers) if L["kind"] == "fc"]
    conv_idx = [j for j, L in enumerate(layers) if L["kind"] == "conv"]

    # ---------------- headline leg
    leg = Leg(layers, args.fc_dtype, psd, inputs, torch, dev, args.sets, rule, args.one_stream)
    prewarm_steps = leg.prewarm()
    ev = HipEvents()
    ms_per_step, marks = leg.run(args.steps, args.warmup, dependent=False, ev=ev)
    dur = durations(ev, marks, len(layers))
    ev.close()
    work = leg.work
    fc_flops = sum(work[j]["flops"] for j in fc_idx)
    value = fc_flops / (ms_per_step * 1e-3) / 1e12
    per_layer = {}
    for j, L in enumerate(layers):
        w, med = work[j], float(np.median(dur[:, j]))
        per_layer[L["name"]] = dict(median_ms=round(med, 5), mean_ms=round(float(dur[:, j].mean()), 5),
                                    min_ms=round(float(dur[:, j].min()), 5), GBps=round(w["bytes"] / med / 1e6, 1),
                                    TFLOPs=round(w["flops"] / med / 1e9, 2))
    roofline = roofline_of(leg, dur, layers, args.fc_dtype, alone=not args.no_alone)

    # the five conv layers are one launch: every conv layer's event pair brackets that launch
    conv_bytes = sum(work[j]["bytes"] for j in conv_idx)
    conv_ms = float(np.median(dur[:, conv_idx[0]]))
    conv_alone = leg.conv_alone_ms() if not args.no_alone else conv_ms
    dense = {"launch": "the five conv layers in one psd_sync_dense_ps_multi launch (2.3M keys, P = 8, S = 8)",
             "bytes_per_step": conv_bytes,
             "in_iteration": {"median_ms": round(conv_ms, 5), "GBps": round(conv_bytes / conv_ms / 1e6, 1),
                              "frac_hbm": round(conv_bytes / conv_ms / 1e6 / PEAK_HBM_GBS, 4)},
             "alone": {"median_ms": round(conv_alone, 5), "GBps": round(conv_bytes / conv_alone / 1e6, 1),
                       "frac_hbm": round(conv_bytes / conv_alone / 1e6 / PEAK_HBM_GBS, 4)}}

    out = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if args.fc_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "config5_full_8layer_cnn_iteration", "fc_factor_dtype": args.fc_dtype,
                   "accumulate": "f32", "B": inputs.CNN_B, "P": inputs.CNN_P, "S": inputs.CNN_S,
                   "conv_keys": inputs.conv_sizes(), "fc_shapes_MxN": inputs.FC_SHAPES,
                   "rule": args.rule, "rotating_sets": args.sets, "streams": 1 if args.one_stream else len(layers),
                   "fc_flops_per_step": fc_flops,
                   "step_dependency": "per layer, by stream order (no join between steps)",
                   "prewarm_steps_untimed": prewarm_steps},
        "roofline": roofline,
        "dense_shard_sum": dense,
        "per_layer": per_layer,
        "routes": {L["name"]: psd.ROUTE_NAMES[leg.sets[0][j]["plan"].route_alg3 if rule == psd.RULE_ALG3
                                              else leg.sets[0][j]["plan"].route_vs_dense]
                   for j, L in enumerate(layers)},
    }

    if not args.no_side_legs:
        side = {}
        ms_join, _ = leg.run(args.steps, args.warmup, dependent=True)
        side["joined_steps_ms_per_step"] = round(ms_join, 4)      # every stream waits for the whole step before
        del leg
        torch.cuda.empty_cache()
        one = Leg(layers, args.fc_dtype, psd, inputs, torch, dev, args.sets, rule, one_stream=not args.one_stream)
        ms_one, _ = one.run(args.steps, args.warmup, dependent=False)
        side["%s_ms_per_step" % ("eight_streams" if args.one_stream else "one_stream")] = round(ms_one, 4)
        del one
        torch.cuda.empty_cache()
        if args.fc_dtype == "bf16":
            # the same step when the peers' factors arrive as bf16 blocks (rounded by their senders) and are read in
            # place: no stacking pass, only this worker's own block is rounded (psd_sync_fc_sfb_blocks)
            inp = Leg(layers, "bf16", psd, inputs, torch, dev, args.sets, rule, args.one_stream, bf16_blocks=True)
            inp.blocks_in_place = True
            ms_inp, _ = inp.run(args.steps, args.warmup, dependent=False)
            side["bf16_blocks_read_in_place_ms_per_step"] = round(ms_inp, 4)
            del inp
            torch.cuda.empty_cache()
        other = "f32" if args.fc_dtype == "bf16" else "bf16"
        leg2 = Leg(layers, other, psd, inputs, torch, dev, args.sets, rule, args.one_stream)
        ev2 = HipEvents()
        ms2, marks2 = leg2.run(args.steps, args.warmup, dependent=False, ev=ev2)
        dur2 = durations(ev2, marks2, len(layers))
        ev2.close()
        side[other] = {"ms_per_step": round(ms2, 4), "value_TFLOPs": round(fc_flops / (ms2 * 1e-3) / 1e12, 3),
                       "roofline": roofline_of(leg2, dur2, layers, other),
                       "per_layer_median_ms": {L["name"]: round(float(np.median(dur2[:, j])), 5)
                                               for j, L in enumerate(layers)}}
        if other == "f32":
            # the same step with the fp32 factor blocks read where they lie (psd_sync_fc_sfb_blocks): no pack launches
            leg2.blocks_in_place = True
            ms3, _ = leg2.run(args.steps, args.warmup, dependent=False)
            side[other]["ms_per_step_blocks_read_in_place"] = round(ms3, 4)
        del leg2
        torch.cuda.empty_cache()
        import bench_extras
        side["dense_sweep_alone"] = bench_extras.dense_sweep(psd, inputs, torch, dev)
        out["beside_the_headline"] = side
    else:
        del leg
        torch.cuda.empty_cache()

    if args.extras:
        import bench_extras
        extras = bench_extras.run(psd, inputs, torch, dev)
        if not args.no_cpu_baseline:
            extras["cpu_baseline_configs"] = cpu_baseline_configs(inputs)
        with open(args.extras, "w") as f:
            json.dump(extras, f, indent=1)
        out["extras_file"] = args.extras

    if not args.no_cpu_baseline:
        secs, threads = cpu_baseline(layers, args.fc_dtype, lr, mu)
        out["cpu_baseline"] = {"value": round(fc_flops / secs / 1e12, 5), "unit": "TFLOP/s", "cores": threads,
                               "kind": "oracle", "ms_per_step": round(secs * 1e3, 1),
                               "sample": "one full pass of the same config-5 iteration (all 8 layers, float64 oracle)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
