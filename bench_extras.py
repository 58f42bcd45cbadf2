"""Optional per-configuration timings for bench.py --extras: the four single-layer FC
configurations (pack and reconstruct+update timed separately), the second-workload and VGG-16-sized
shapes, a sweep of the contraction length on the fc6 shape, a size sweep of the dense parameter-server
kernel and the wait-free issue measurement.  Timing only: no arithmetic of the method lives here.

Run alone it launches ONE kernel family back to back, for rocprofv3 (kernel stats or counters of exactly
that kernel):
    python3 bench_extras.py --layer fc6 --dtype bf16 [--iters 40]      # reconstruct + update only
    python3 bench_extras.py --dense 37748736 [--iters 40]              # parameter-server sum + update only
and two studies of how the MFMA loop and the W / Mom traffic share the chip (text on stdout):
    python3 bench_extras.py --study skew         # odd XCDs start late: does putting the phases out of step pay?
    python3 bench_extras.py --study partition    # reconstruction and a dense stream on disjoint sets of CUs
    python3 bench_extras.py --study ksweep       # time over the contraction length on the fc6 and fc8 shapes
"""
from __future__ import annotations

import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

PEAK_HBM_GBS = 8000.0
PEAK_TF = {"bf16": 2500.0, "f32": 157.3}


def _time_ms(torch, fn, n_sets, iters=20, warmup_ms=100.0, batches=5):
    """Median over `batches` of the mean milliseconds per call of fn(set_index), rotating over n_sets
    buffer sets, after at least warmup_ms of the same calls (an idle GPU's clocks take ~0.1 s to settle)."""
    import time
    t0 = time.perf_counter()
    i = 0
    while (time.perf_counter() - t0) * 1e3 < warmup_ms:
        fn(i % n_sets)
        i += 1
        if i % 16 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    ts = []
    for _ in range(batches):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(iters):
            fn(i % n_sets)
        b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b) / iters)
    return float(np.median(ts))


# FC shapes beyond the four configurations: the ImageNet-22K network's FC stack (Section 5.1.3), GoogLeNet's
# single FC layer at batch 32 per node (Section 5.1.2) and a VGG-16-sized FC stack (Table 3) at batch 256 per node
EXTRA_SHAPES = {"in22k_fc": (3000, 3000, 256, 8), "in22k_cls": (3000, 21841, 256, 8), "googlenet_fc": (1024, 1000, 32, 8),
                "vgg_fc6": (25088, 4096, 256, 8), "vgg_fc7": (4096, 4096, 256, 8), "vgg_fc8": (4096, 1000, 256, 8)}
NAMED_LAYERS = {"cfg1": 1, "cfg2": 2, "fc8": 2, "fc6": 3, "cfg3": 3, "cls22k": 4, "cfg4": 4}


def fc_config(psd, inputs, torch, dev, cfg_id, dtype_name=None, working_set_mb=600, shape=None, only_sfb_iters=0):
    """cfg_id 1..4, or shape=(name, M, N, B, P) for any other layer."""
    if shape is None:
        c = inputs.FC_CONFIGS[cfg_id]
        dtype_name = dtype_name or c["factor_dtype"]
        d = inputs.fc_config(cfg_id)
    else:
        c = dict(name=shape[0])
        d = inputs.fc_layer(shape[1], shape[2], shape[3], shape[4], seed=sum(shape[1:]),
                            delta_kind="softmax" if shape[2] == 21841 else "gauss")
    dtype = psd.BF16 if dtype_name == "bf16" else psd.F32
    M, N, B, P = d["M"], d["N"], d["B"], d["P"]
    K = P * B
    es = 2 if dtype_name == "bf16" else 4
    plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
    per_set = 8 * N * M + K * (M + N) * (4 + es)
    n_sets = int(min(16, max(2, np.ceil(working_set_mb * 1e6 / per_set))))
    sets = []
    for _ in range(n_sets):
        U, ldu, V, ldv = psd.alloc_factors(plan, dtype, dev)
        sets.append(dict(delta=[torch.from_numpy(x).to(dev) for x in d["delta"]],
                         act=[torch.from_numpy(x).to(dev) for x in d["act"]], U=U, ldu=ldu, V=V, ldv=ldv,
                         W=torch.from_numpy(d["W"]).to(dev), Mom=torch.from_numpy(d["Mom"]).to(dev)))

    def pack(i):
        s = sets[i]
        psd.pack_factors(plan, s["delta"], s["act"], dtype, s["U"], s["ldu"], s["V"], s["ldv"])

    ws = psd.alloc_workspace(plan, dtype, dev)

    def sfb(i):
        s = sets[i]
        psd.sync_fc_sfb(plan, dtype, s["U"], s["ldu"], s["V"], s["ldv"], s["W"], s["Mom"], inputs.LR, inputs.MU,
                        workspace=ws)

    def both(i):
        pack(i)
        sfb(i)

    bias_sets = [(torch.zeros(N, device=dev), torch.zeros(N, device=dev)) for _ in range(n_sets)]

    def bias(i):
        s = sets[i]
        psd.sync_fc_bias(plan, dtype, s["U"], s["ldu"], bias_sets[i][0], bias_sets[i][1], inputs.LR, inputs.MU)

    for i in range(n_sets):
        pack(i)
    if only_sfb_iters:                       # profiling mode: nothing but this kernel, back to back
        torch.cuda.synchronize()
        for i in range(only_sfb_iters):
            sfb(i % n_sets)
        torch.cuda.synchronize()
        return None
    t_pack = _time_ms(torch, pack, n_sets)
    t_sfb = _time_ms(torch, sfb, n_sets)
    t_both = _time_ms(torch, both, n_sets)
    t_bias = _time_ms(torch, bias, n_sets)
    # the same reconstruction from the per-worker blocks read in place (no stacked copy): fp32 blocks as they are,
    # bf16 blocks as senders that round before sending would deliver them (made here, outside the timing)
    t_blocks = None
    if dtype == psd.F32 and psd.sfb_blocks_supported(plan, dtype):
        def blocks(i):
            s = sets[i]
            psd.sync_fc_sfb_blocks(plan, dtype, s["delta"], 0, s["act"], 0, s["W"], s["Mom"], inputs.LR, inputs.MU)
        t_blocks = _time_ms(torch, blocks, n_sets)
    elif dtype == psd.BF16 and psd.sfb_blocks_supported(plan, dtype, sets[0]["ldu"], sets[0]["ldv"]):
        one = psd.plan_layer(psd.LAYER_FC, M, N, B, 1)
        for s in sets:
            s["Ub"], s["Vb"] = [], []
            for p in range(P):
                Ub, _, Vb, _ = psd.alloc_factors(one, dtype, dev)
                psd.pack_factors(one, [s["delta"][p]], [s["act"][p]], dtype, Ub, s["ldu"], Vb, s["ldv"])
                s["Ub"].append(Ub)
                s["Vb"].append(Vb)

        def blocks(i):
            s = sets[i]
            psd.sync_fc_sfb_blocks(plan, dtype, s["Ub"], s["ldu"], s["Vb"], s["ldv"], s["W"], s["Mom"], inputs.LR, inputs.MU)
        t_blocks = _time_ms(torch, blocks, n_sets)
    flops = 2 * N * M * K
    bytes_sfb = 16 * N * M + K * (M + N) * es
    bytes_pack = K * (M + N) * (4 + es)
    return dict(config=cfg_id, name=c["name"], M=M, N=N, B=B, P=P, K=K, factor_dtype=dtype_name, rotating_sets=n_sets,
                route_alg3=psd.ROUTE_NAMES[plan.route_alg3], route_vs_dense=psd.ROUTE_NAMES[plan.route_vs_dense],
                sfb_ms=round(t_sfb, 5), sfb_TFLOPs=round(flops / t_sfb / 1e9, 2),
                sfb_frac_mfma=round(flops / t_sfb / 1e9 / PEAK_TF[dtype_name], 4),
                sfb_GBps=round(bytes_sfb / t_sfb / 1e6, 1), sfb_frac_hbm=round(bytes_sfb / t_sfb / 1e6 / PEAK_HBM_GBS, 4),
                pack_ms=round(t_pack, 5), pack_GBps=round(bytes_pack / t_pack / 1e6, 1),
                pack_plus_sfb_ms=round(t_both, 5), pack_plus_sfb_TFLOPs=round(flops / t_both / 1e9, 2),
                sfb_blocks_in_place_ms=None if t_blocks is None else round(t_blocks, 5),
                bias_ms=round(t_bias, 5), bias_GBps=round((K * N * es + 16 * N) / t_bias / 1e6, 1))


def sfb_k_sweep(psd, inputs, torch, dev, M=9216, N=4096, P=8, batches=(4, 64, 128, 256, 512), dtype_name="bf16"):
    """Reconstruct + update on the fc6 shape at different contraction lengths K = P*B: the time is close
    to a + b*K; a is what the update of W and Mom costs (K = 32 is nothing else), b*K the k loop."""
    dtype = psd.BF16 if dtype_name == "bf16" else psd.F32
    td = torch.bfloat16 if dtype_name == "bf16" else torch.float32
    n_sets = int(min(16, max(2, np.ceil(600e6 / (8.0 * N * M)))))      # W and Mom rotate over > 600 MB: past the last-level cache
    W = [torch.randn(N, M, device=dev) * 1e-2 for _ in range(n_sets)]
    Mom = [torch.zeros(N, M, device=dev) for _ in range(n_sets)]
    out = []
    for B in batches:
        K = P * B
        plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
        ldu, ldv = psd.factor_ld(N, dtype), psd.factor_ld(M, dtype)
        U = [(torch.randn(K, ldu, device=dev) * 1e-3).to(td) for _ in range(n_sets)]
        V = [torch.relu(torch.randn(K, ldv, device=dev)).to(td) for _ in range(n_sets)]

        def run(i):
            psd.sync_fc_sfb(plan, dtype, U[i], ldu, V[i], ldv, W[i], Mom[i], inputs.LR, inputs.MU)
        t = _time_ms(torch, run, n_sets)
        out.append(dict(K=K, ms=round(t, 5), TFLOPs=round(2.0 * N * M * K / t / 1e9, 1),
                        GBps=round((16.0 * N * M + K * (M + N) * (2 if dtype_name == "bf16" else 4)) / t / 1e6, 1)))
    a = np.polyfit([o["K"] for o in out], [o["ms"] for o in out], 1)
    return dict(shape="%d -> %d" % (M, N), factor_dtype=dtype_name, points=out,
                fit_us_per_1024_k=round(float(a[0]) * 1024 * 1e3, 2), fit_intercept_us=round(float(a[1]) * 1e3, 2))


def _bf16_layer(psd, torch, dev, M, N, B, P=8, n_sets=2):
    plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
    K = B * P
    ldu, ldv = psd.factor_ld(N, psd.BF16), psd.factor_ld(M, psd.BF16)
    sets = []
    for _ in range(n_sets):
        U = (torch.randn(K, ldu, device=dev) * 1e-3).to(torch.bfloat16)
        V = torch.relu(torch.randn(K, ldv, device=dev)).to(torch.bfloat16)
        sets.append((U, V, torch.randn(N, M, device=dev) * 1e-2, torch.zeros(N, M, device=dev)))

    def run(i, stream=None):
        U, V, W, Mom = sets[i % n_sets]
        psd.sync_fc_sfb(plan, psd.BF16, U, ldu, V, ldv, W, Mom, 0.01, 0.9, stream=stream)
    return run


def phase_skew_study(psd, torch, dev, skews=(0, 10, 20, 30, 40, 60)):
    """bf16 reconstruct + update with the first workgroups of the odd XCDs started `skew` microseconds late
    (PSD_TUNE_SFB_BF16_SKEW_US).  If an XCD's MFMA loop ran faster while the other half of the chip is in its
    update phase, or its update faster while the other half computes, a skew of about half a round would pay
    back more than it costs, the more so the more rounds a launch has (fc6: 3, the 22K layer: 9)."""
    print("# time per launch (us, median of 5 x 20) over the start delay of the odd XCDs")
    for name, (M, N) in (("fc6 9216 -> 4096", (9216, 4096)), ("22K classifier 4096 -> 21841", (4096, 21841))):
        run = _bf16_layer(psd, torch, dev, M, N, 256)
        row = []
        for us in skews:
            psd.tune_set(psd.TUNE_SFB_BF16_SKEW_US, us)
            row.append("%d us: %.1f" % (us, _time_ms(torch, run, 2) * 1e3))
        psd.tune_set(psd.TUNE_SFB_BF16_SKEW_US, -1)
        print("%-30s %s" % (name, "   ".join(row)), flush=True)
        del run
        torch.cuda.empty_cache()


def cu_partition_study(psd, torch, dev, n=37748736, P=8):
    """A reconstruction that is nearly all MFMA loop (4096 -> 4096 at K = 16384) and the dense parameter-server
    stream, each alone on a subset of the CUs (streams created with a CU mask), then both at once on disjoint
    subsets, next to the two run one after the other on the whole chip."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32,
                                                 ctypes.POINTER(ctypes.c_uint32)]

    def masked_stream(lo, hi):
        bits = (ctypes.c_uint32 * 8)()
        for b in range(lo, hi):
            bits[b // 32] |= 1 << (b % 32)
        st = ctypes.c_void_p()
        if hip.hipExtStreamCreateWithCUMask(ctypes.byref(st), 8, bits) != 0:
            raise RuntimeError("hipExtStreamCreateWithCUMask failed")
        return st.value

    sfb = _bf16_layer(psd, torch, dev, 4096, 4096, 2048)
    G = [torch.randn(n, device=dev) * 1e-3 for _ in range(P)]
    dW, dMom = torch.randn(n, device=dev) * 1e-2, torch.zeros(n, device=dev)

    def dense(i, stream=None):
        psd.sync_dense_ps(G, dW, dMom, 0.01, 0.9, 8, stream=stream)

    def timed(fa, sa, fb, sb, reps=9):
        res = []
        for r in range(reps + 3):
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            if fa:
                xa = torch.cuda.ExternalStream(sa)
                ev[0].record(xa); fa(r, sa); fa(r + 1, sa); ev[1].record(xa)
            if fb:
                xb = torch.cuda.ExternalStream(sb)
                ev[2].record(xb); fb(r, sb); fb(r + 1, sb); ev[3].record(xb)
            torch.cuda.synchronize()
            res.append((ev[0].elapsed_time(ev[1]) * 1e3 if fa else 0.0, ev[2].elapsed_time(ev[3]) * 1e3 if fb else 0.0))
        return np.median(np.array(res[3:]), axis=0)

    _time_ms(torch, lambda i: sfb(i), 2, iters=4, batches=1)          # settle the clocks
    print("# A = two launches of the bf16 reconstruction 4096 -> 4096, K = 16384;  B = two launches of the dense sum + update,")
    print("# %d keys, P = %d;  microseconds, medians of 9" % (n, P))
    for a in (256, 192, 128, 224):
        sa = masked_stream(0, a)
        sb = masked_stream(a, 256) if a < 256 else masked_stream(0, 256)
        ta = timed(sfb, sa, None, None)[0]
        tb = timed(None, None, dense, sb)[1]
        both = timed(sfb, sa, dense, sb)
        tag = "disjoint" if a < 256 else "the same"
        print("A on %3d CUs alone %7.1f | B on %3d CUs alone %7.1f | at once on %s CUs: A %7.1f  B %7.1f" %
              (a, ta, 256 - a if a < 256 else 256, tb, tag, both[0], both[1]), flush=True)


def k_sweep_study(psd, inputs, torch, dev):
    for M, N in ((9216, 4096), (4096, 1000)):
        for dt, batches in (("bf16", (4, 64, 128, 256, 512)), ("f32", (4, 64, 128, 256))):
            r = sfb_k_sweep(psd, inputs, torch, dev, M=M, N=N, batches=batches, dtype_name=dt)
            print("%s %s: %s | fit %.1f us + %.1f us per 1024 k" % (
                r["shape"], dt, "  ".join("K=%d: %.1f us" % (p["K"], p["ms"] * 1e3) for p in r["points"]),
                r["fit_intercept_us"], r["fit_us_per_1024_k"]), flush=True)
            torch.cuda.empty_cache()


def dense_only(psd, inputs, torch, dev, n, iters, P=8, S=8):
    sets = [([torch.randn(n, device=dev) * 1e-3 for _ in range(P)], torch.randn(n, device=dev) * 1e-2,
             torch.zeros(n, device=dev)) for _ in range(2)]
    torch.cuda.synchronize()
    for i in range(iters):
        G, W, Mom = sets[i % 2]
        psd.sync_dense_ps(G, W, Mom, inputs.LR, inputs.MU, S)
    torch.cuda.synchronize()


def dense_sweep(psd, inputs, torch, dev, sizes=(2332704, 16777216, 37748736, 89460736), P=8, S=8):
    out = []
    for n in sizes:
        per_set = n * (4 * P + 8)
        n_sets = int(min(8, max(2, np.ceil(1.2e9 / per_set))))
        sets = []
        for _ in range(n_sets):
            G = [torch.randn(n, device=dev) * 1e-3 for _ in range(P)]
            sets.append((G, torch.randn(n, device=dev) * 1e-2, torch.zeros(n, device=dev)))

        def run(i):
            G, W, Mom = sets[i]
            psd.sync_dense_ps(G, W, Mom, inputs.LR, inputs.MU, S)

        t = _time_ms(torch, run, n_sets)
        b = n * (4 * P + 16)
        out.append(dict(n=n, P=P, S=S, rotating_sets=n_sets, ms=round(t, 5), GBps=round(b / t / 1e6, 1),
                        frac_hbm=round(b / t / 1e6 / PEAK_HBM_GBS, 4)))
        del sets
        torch.cuda.empty_cache()
    return out


# Forward multiply-adds per image of the 8 AlexNet layers (conv1..conv5, fc6..fc8); their sum matches the
# 1 352 M conv / 117 M FC FLOPs per image of the paper's Table 3 to within the rounding of that table when a
# multiply-add counts as one FLOP.
ALEXNET_MFLOP = [105.4, 223.9, 149.5, 112.1, 74.8, 37.7, 16.8, 4.1]


def dwbp_overlap(psd, inputs, torch, dev, iters=10):
    """Iteration time when the synchronisation of a layer starts as soon as its gradient exists
    (Algorithm 2) against starting all synchronisation after the whole backward pass.

    Backpropagation itself is outside this build, so each layer's backward work is a stand-in: a bf16
    matmul on a 'backward' stream sized to twice the layer's forward FLOPs at batch 256 (data and weight
    gradients).  Only the schedule is the subject here; the stand-in computes nothing that is used."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    layers = inputs.cnn_iteration()
    streams = [torch.cuda.Stream(device=dev) for _ in layers]
    backward = torch.cuda.Stream(device=dev)
    tasks, standins = [], []
    for L, st, mflop in zip(layers, streams, ALEXNET_MFLOP):
        ev = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(ev)) == 0
        if L["kind"] == "conv":
            plan = psd.plan_layer(psd.LAYER_CONV, L["n"], 1, inputs.CNN_B, L["P"])
            t = dict(plan=plan, G=[torch.from_numpy(g).to(dev) for g in L["G"]], S=inputs.CNN_S,
                     W=torch.from_numpy(L["W"]).to(dev), Mom=torch.from_numpy(L["Mom"]).to(dev), stream=st)
        else:
            plan = psd.plan_layer(psd.LAYER_FC, L["M"], L["N"], L["B"], L["P"])
            U, ldu, V, ldv = psd.alloc_factors(plan, psd.BF16, dev)
            t = dict(plan=plan, factor_dtype=psd.BF16, delta=[torch.from_numpy(x).to(dev) for x in L["delta"]],
                     act=[torch.from_numpy(x).to(dev) for x in L["act"]], U=U, ldu=ldu, V=V, ldv=ldv,
                     W=torch.from_numpy(L["W"]).to(dev), Mom=torch.from_numpy(L["Mom"]).to(dev), stream=st)
        t["_ev"] = ev.value
        tasks.append(t)
        # 2 * forward FLOPs * 256 images as one square-ish matmul: 2*n^3 = 2 * 2 * mflop*1e6 * 256
        n = int(round((2.0 * mflop * 1e6 * 256) ** (1.0 / 3.0) / 64.0)) * 64
        standins.append((torch.randn(n, n, device=dev, dtype=torch.bfloat16) * 0.01,
                         torch.randn(n, n, device=dev, dtype=torch.bfloat16) * 0.01))

    def backward_pass(record):
        with torch.cuda.stream(backward):
            for j in range(len(layers) - 1, -1, -1):          # top layer first
                a, b = standins[j]
                torch.matmul(a, b)
                if record:
                    assert hip.hipEventRecord(tasks[j]["_ev"], ctypes.c_void_p(backward.cuda_stream)) == 0

    it_plain = psd.Iteration(tasks)
    it_events = psd.Iteration([dict(t, ev_ready=t["_ev"]) for t in tasks])

    def one(mode):
        if mode == "backward_only":
            backward_pass(False)
        elif mode == "sync_only":
            it_plain.run(inputs.LR, inputs.MU)
        elif mode == "sync_after_backward":
            backward_pass(False)
            torch.cuda.synchronize()                           # all gradients exist, then synchronise
            it_plain.run(inputs.LR, inputs.MU)
        else:                                                  # wait-free: per-layer events
            backward_pass(True)
            it_events.run(inputs.LR, inputs.MU)

    import time
    out = {}
    for mode in ("backward_only", "sync_only", "sync_after_backward", "wait_free"):
        for _ in range(3):
            one(mode)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            one(mode)
            torch.cuda.synchronize()                           # one iteration at a time: no cross-iteration overlap
        out[mode + "_ms"] = round((time.perf_counter() - t0) / iters * 1e3, 4)
    out["note"] = ("backward = bf16 matmul stand-ins of 2x the AlexNet forward FLOPs per layer at batch 256; "
                   "sync = the 8-layer config-5 synchronisation, bf16 factors")
    return out


def run(psd, inputs, torch, dev):
    res = {"fc": [], "dense_sweep": None}
    for cfg, dt in [(1, "f32"), (2, "f32"), (2, "bf16"), (3, "bf16"), (3, "f32"), (4, "bf16")]:
        res["fc"].append(fc_config(psd, inputs, torch, dev, cfg, dt))
        torch.cuda.empty_cache()
    res["fc_other_shapes"] = []
    for name, (M, N, B, P) in EXTRA_SHAPES.items():
        for dt in ("bf16", "f32"):
            res["fc_other_shapes"].append(fc_config(psd, inputs, torch, dev, None, dt, shape=(name, M, N, B, P)))
            torch.cuda.empty_cache()
    res["fc6_k_sweep"] = [sfb_k_sweep(psd, inputs, torch, dev, dtype_name="bf16"),
                          sfb_k_sweep(psd, inputs, torch, dev, dtype_name="f32", batches=(4, 64, 128, 256))]
    torch.cuda.empty_cache()
    res["dense_sweep"] = dense_sweep(psd, inputs, torch, dev)
    res["dwbp_overlap"] = dwbp_overlap(psd, inputs, torch, dev)
    return res


def main():
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--layer", default=None, help="cfg1..cfg4, fc6, fc8, cls22k or one of %s" % ", ".join(EXTRA_SHAPES))
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--dense", type=int, default=0, metavar="KEYS")
    ap.add_argument("--iters", type=int, default=40)
    ap.add_argument("--study", choices=["skew", "partition", "ksweep"], default=None)
    args = ap.parse_args()
    import torch
    from paper_1512_06216_amd import binding as psd
    from paper_1512_06216_amd import inputs
    psd.lib()
    dev = "cuda:0"
    if args.study == "skew":
        phase_skew_study(psd, torch, dev)
    elif args.study == "partition":
        cu_partition_study(psd, torch, dev)
    elif args.study == "ksweep":
        k_sweep_study(psd, inputs, torch, dev)
    elif args.dense:
        dense_only(psd, inputs, torch, dev, args.dense, args.iters)
    elif args.layer in NAMED_LAYERS:
        fc_config(psd, inputs, torch, dev, NAMED_LAYERS[args.layer], args.dtype, only_sfb_iters=args.iters)
    elif args.layer in EXTRA_SHAPES:
        fc_config(psd, inputs, torch, dev, None, args.dtype, shape=(args.layer,) + EXTRA_SHAPES[args.layer],
                  only_sfb_iters=args.iters)
    else:
        ap.error("give --layer or --dense")
    print("done")


if __name__ == "__main__":
    main()
