#!/usr/bin/env python3
"""Benchmark of the early-exit serving hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic requests: admission, the
backbone segments on the matrix cores, the exit heads, compaction and slot refill, driven by the
exit-aware host scheduler on the wall clock.  The default workload is the ResNet-50-style
int8 stream: 10,000 requests, Poisson arrivals at 1.2x the static-batch throughput measured in
the same run, 64 batch slots refilled at the exit boundaries.  The timed policy is the stage-pool
refill (survivors of an exit wait in front of the next segment, segments run on full batches);
the same trace under Algorithm 1 of the paper and under static batching is printed beside it.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: this path is built
and measured on one GPU only.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"i8": 5000.0, "bf16": 2500.0}          # dense MFMA peak of MI355X, TOP/s resp. TFLOP/s
HBM_PEAK = 8000.0                               # GB/s


CONV_SOURCES = ("kernels_igemm.hip", "kernels_slab.hip", "kernels_pair.hip", "kernels_bneck.hip", "kernels_ir.hip", "igemm_device.hpp", "igemm_epilogue.hpp", "ir_device.hpp")


def conv_sources_digest():
    """sha256 over the sources of the matrix-core convolution kernels, in the order of CONV_SOURCES"""
    import hashlib
    h = hashlib.sha256()
    for name in CONV_SOURCES:
        with open(os.path.join(ROOT, "paper_2209_13443_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed counter runs (profiles/traffic.json), or
    None when there is no record for this workload or the kernel sources have changed since it was taken."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            rec = json.load(f).get(workload)
        digest = conv_sources_digest()
    except OSError:
        return None
    if not rec or rec.get("kernel_sha256") != digest:
        return None
    return rec["hbm_bytes_per_launch"]


WORKLOADS = {
    "resnet50_i8_stream": dict(net="resnet50_i8", n=10000, b_max=64, refill=2, load=1.2, spikes=False),
    "resnet50_eq_i8_stream": dict(net="resnet50_eq_i8", n=10000, b_max=64, refill=2, load=1.2, spikes=False),
    "inception_i8_stream": dict(net="inception_i8", n=6000, b_max=64, refill=2, load=1.2, spikes=False),
    "resnet50_bf16_stream": dict(net="resnet50_bf16", n=20000, b_max=256, refill=2, load=0.8, spikes=True),
    "mobilenetv2_i8_refill": dict(net="mobilenetv2_i8", n=4096, b_max=64, refill=2, load=None, spikes=False),
    "resnet18_i8_static": dict(net="resnet18_i8", n=1024, b_max=32, refill=0, load=None, spikes=False),
    "tiny_i8": dict(net="tiny_i8", n=64, b_max=8, refill=1, load=None, spikes=False),
}


def layer_table(args, ee, W, blob, dtype):
    """Isolated layers: each layer of the network alone on B samples with its tuned configuration, `reps` launches back
    to back between two HIP events.  One text line per layer on stderr, one JSON line on stdout."""
    B = args.layers
    eng = ee.Engine(blob, B)
    if args.load_tables:
        with open(args.load_tables) as f:
            eng.load_tables(json.load(f))
    elif not (args.layer >= 0 and args.cfg):
        eng.autotune(reps=5)
    if args.save_tables:
        with open(args.save_tables, "w") as f:
            json.dump(eng.tables(), f)
    rows = []
    for i, op in enumerate(blob.ops):
        if args.layer >= 0 and i != args.layer:
            continue
        r = eng.time_layer(i, B, args.cfg if args.layer >= 0 else 0, reps=30)
        if r is None:
            print(f"layer {i}: configuration {args.cfg:#x} does not exist for it", file=sys.stderr)
            continue
        us, ops, byt = r
        cfgs = eng.config_table(i)
        k = int(op["kh"]) * int(op["kw"]) * int(op["c_in"])
        row = dict(layer=i, kind=int(op["kind"]), h=int(op["h_in"]), w=int(op["w_in"]), ci=int(op["c_in"]), co=int(op["c_out"]), kh=int(op["kh"]),
                   kw=int(op["kw"]), stride=int(op["stride"]), res=bool(int(op["res"]) >= 0), M=B * int(op["h_out"]) * int(op["w_out"]), K=k,
                   us=round(us, 2), tops=round(ops / us / 1e6, 1), gbps=round(byt / us / 1e3, 1),
                   roof_us=round(max(ops / (PEAK[dtype] * 1e6), byt / (HBM_PEAK * 1e3)), 2),
                   cfg=cfgs[min(len(cfgs) - 1, max(0, (B - 1).bit_length()))] if cfgs else 0)
        rows.append(row)
        print("op%3d k%d %3dx%-3d ci%5d co%5d %dx%d s%d res%d M=%7d K=%5d: %8.2f us %8.1f T/s %7.1f GB/s  roof %6.2f us (%4.1f%%) cfg 0x%x" % (
            i, row["kind"], row["h"], row["w"], row["ci"], row["co"], row["kh"], row["kw"], row["stride"], row["res"], row["M"], row["K"],
            row["us"], row["tops"], row["gbps"], row["roof_us"], 100 * row["roof_us"] / row["us"], row["cfg"]), file=sys.stderr, flush=True)
    blocks = []
    if args.layer < 0 and eng.ir_count() > 0:                     # inverted-residual blocks: the fused launch beside its three layers
        for i in range(len(blob.ops) - 1):
            try:
                r = eng.time_layer(i, B, 0x20000, reps=30)
            except ee.EEError:
                continue                                          # the layer heads no block
            if r is None:
                continue
            span = eng.ir_layers(i)                                # 2: depthwise + projection; 4: with the convolution on the shortcut in front
            sep = sum(x["us"] for x in rows if i <= x["layer"] < i + span)
            tab = eng.ir_table(i)
            blocks.append(dict(head=i, layers=span, fused_us=round(r[0], 2), separate_us=round(sep, 2), gbps=round(r[2] / r[0] / 1e3, 1), tops=round(r[1] / r[0] / 1e6, 1),
                               table=tab[min(len(tab) - 1, max(0, (B - 1).bit_length()))] if tab else None))
            print("block at op%3d: fused %8.2f us (%6.1f T/s %7.1f GB/s), its %d layers %8.2f us, table says %s" % (
                i, r[0], blocks[-1]["tops"], blocks[-1]["gbps"], span, sep, blocks[-1]["table"]), file=sys.stderr, flush=True)
    conv = [r for r in rows if r["kind"] == W.OP_CONV]
    tot_us = sum(r["us"] for r in rows)
    conv_us = sum(r["us"] for r in conv)
    conv_ops = sum(r["tops"] * r["us"] for r in conv)             # T/s * us = Mop
    out = dict(mode="layers", workload=args.workload, net=WORKLOADS[args.workload]["net"], batch=B, dtype=dtype, total_us=round(tot_us, 1), conv_us=round(conv_us, 1),
               conv_tops=round(conv_ops / max(conv_us, 1e-9), 1), conv_frac_of_peak=round(conv_ops / max(conv_us, 1e-9) / PEAK[dtype], 4),
               roofline_us=round(sum(r["roof_us"] for r in rows), 1), layers=rows, ir_blocks=blocks)
    print(json.dumps(out))
    eng.close()


def policy_sweep(args, ee, W):
    """The serving policies of the evaluation (Sec. V-A "Baselines", Sec. V-B) on one workload, wall clock: SERIAL, adaptive
    batching <B_max, T_timeout> with windows of 5 / 45 / 95 % of the SLO (AdaptB-S/M/L), model-level batching without a
    window, Algorithm 1 as printed and with min_incr = B_max / 2, and the stage pools on one and on two lanes; over arrival
    rates (multiples of the static-batch throughput) at an SLO of twice the full-batch latency, then over SLOs at 0.8 x.
    One JSON line: rows of policy, load, slo_ms, samples/s, mean / p99 latency, violation rate, mean batch per segment."""
    import torch
    wl = WORKLOADS[args.workload]
    n = args.requests or min(wl["n"], 4000)
    b_max = wl["b_max"]
    blob = W.load_net(wl["net"])
    eng = ee.Engine(blob, b_max)
    eng.set_lanes(2)
    pool = torch.cat([torch.from_numpy((lambda p: p.view(np.int16) if p.dtype == np.uint16 else p)(W.input_pool(blob, min(1000, n - f), first=f))).cuda()
                      for f in range(0, n, 1000)])
    if args.load_tables:
        with open(args.load_tables) as f:
            eng.load_tables(json.load(f))
    else:
        eng.autotune(reps=3)
    lut = eng.measure_lut(reps=3)
    zeros = np.zeros(n, np.int64)
    eng.serve_stream(zeros, pool, lut, clock=0, refill=0)
    t0 = time.perf_counter()
    eng.serve_stream(zeros, pool, lut, clock=0, refill=0)
    static_rate = n / (time.perf_counter() - t0)
    full_ns = int(lut[:, b_max - 1].sum())                 # latency of a full batch through every segment
    lut1 = np.ascontiguousarray(lut[:, :1])
    rows = []

    def run(policy, load, slo_ns):
        arr = W.poisson_trace(n, load * static_rate)
        kw = dict(clock=0, t_slo_ns=slo_ns)
        if policy == "serial":
            res, st, _ = eng.serve_stream(arr, pool, lut1, b_max=1, refill=0, **kw)
        elif policy.startswith("adaptb"):
            frac = {"S": 0.05, "M": 0.45, "L": 0.95}[policy[-1]]
            res, st, _ = eng.serve_stream(arr, pool, lut, refill=0, t_timeout_ns=max(1, int(frac * slo_ns)), **kw)
        elif policy == "model_level":
            res, st, _ = eng.serve_stream(arr, pool, lut, refill=0, **kw)
        elif policy == "algorithm1_as_printed":
            res, st, _ = eng.serve_stream(arr, pool, lut, refill=1, min_incr=1, **kw)
        elif policy == "algorithm1_min_incr":
            res, st, _ = eng.serve_stream(arr, pool, lut, refill=1, min_incr=max(1, b_max // 2), **kw)
        else:
            res, st, _ = eng.serve_stream(arr, pool, lut, refill=2, lanes=int(policy[-1]), **kw)
        lat = res["latency_ns"].astype(np.float64)
        span = float(arr[-1] - arr[0] + lat[-1]) if n else 1.0
        done = (arr + res["latency_ns"]).max() - arr[0]
        rows.append(dict(policy=policy, load=load, slo_ms=round(slo_ns / 1e6, 3), samples_per_s=round(n / (done * 1e-9), 1),
                         latency_ms_mean=round(lat.mean() / 1e6, 3), latency_ms_p99=round(float(np.percentile(lat, 99)) / 1e6, 3),
                         slo_violation_rate=round(float(np.mean(lat > slo_ns)), 4), preemptions=st["preemptions"],
                         mean_batch_per_segment=[round(a / max(b, 1), 2) for a, b in zip(st["seg_samples"], st["seg_runs"])]))
        print(json.dumps(rows[-1]), file=sys.stderr, flush=True)

    policies = ["serial", "adaptb_S", "adaptb_M", "adaptb_L", "model_level", "algorithm1_as_printed", "algorithm1_min_incr", "stage_pools_1", "stage_pools_2"]
    for load in (0.25, 0.5, 0.8, 1.0, 1.2):
        for pol in policies:
            if pol == "serial" and load > 0.5:
                continue                                   # far beyond what one request at a time sustains: the queue only grows
            run(pol, load, 2 * full_ns)
    for mult in (1.0, 1.5, 3.0, 4.0):
        for pol in policies[1:]:
            run(pol, 0.8, int(mult * full_ns))
    print(json.dumps(dict(mode="policies", workload=args.workload, requests=n, b_max=b_max, static_batch_samples_per_s=round(static_rate, 1),
                          full_batch_latency_ms=round(full_ns / 1e6, 3), rows=rows)))
    eng.close()


def run_stream(args, name, steps, warmup, full=True):
    """One workload: tunes, measures the static-batch rate that sets the arrival rate, times `steps` steps of the stream
    under the workload's policy, then (full) the same trace under the other policies, the saturated capacity, the per-kernel
    timing of one more step and the CPU oracle.  Returns the JSON object."""
    import torch
    import paper_2209_13443_amd as ee
    import workloads as W

    wl = WORKLOADS[name]
    n = args.requests or wl["n"]
    b_max = wl["b_max"]
    blob = W.load_net(wl["net"])
    dtype = "i8" if blob.dtype == W.DT_I8 else "bf16"
    eng = ee.Engine(blob, b_max)

    # synthetic request pool, resident in HBM before any timed region
    chunks = []
    for first in range(0, n, 1000):
        part = W.input_pool(blob, min(1000, n - first), first=first)
        chunks.append(torch.from_numpy(part.view(np.int16) if part.dtype == np.uint16 else part).cuda())
    pool = torch.cat(chunks)
    del chunks
    torch.cuda.synchronize()

    if args.load_tables and full:                      # design-time per-(layer, batch) kernel configuration table
        with open(args.load_tables) as f:
            eng.load_tables(json.load(f))
    else:
        eng.autotune(reps=5 if full else 3)
    if args.save_tables and full:
        with open(args.save_tables, "w") as f:
            json.dump(eng.tables(), f)
    lut = eng.measure_lut(reps=3)                      # design-time exit-level latency table
    min_incr = args.min_incr or max(1, b_max // 2)

    # survivors of an exit stay where they are (zero-copy compaction) wherever the network allows it, under every policy
    zero_copy = int(eng.zero_copy_supported() and args.zero_copy != 0)

    # static-batch throughput (model-level batching, everything queued at t = 0) sets the arrival rate
    zeros = np.zeros(n, np.int64)
    eng.serve_stream(zeros, pool, lut, clock=0, refill=0, zero_copy=zero_copy)
    t0 = time.perf_counter()
    res_static, st_static, _ = eng.serve_stream(zeros, pool, lut, clock=0, refill=0, zero_copy=zero_copy)
    static_rate = n / (time.perf_counter() - t0)
    load = (args.load if full else 0.0) or wl["load"]
    if load is None:
        arrivals = zeros
    elif wl["spikes"]:
        arrivals = W.spiky_trace(n, load * static_rate)
    else:
        arrivals = W.poisson_trace(n, load * static_rate)
    t_slo_ns = int(args.t_slo_ms * 1e6) if args.t_slo_ms >= 0 and full else -1

    refill = wl["refill"] if args.refill < 0 or not full else args.refill
    lanes = ((args.lanes if full else 0) or wl.get("lanes", 2)) if refill == 2 else 1
    eng.set_lanes(lanes)

    zero_copy = int(zero_copy and lanes <= 2)          # its slots cover two steps in flight

    def step(policy=refill, arr=None, min_incr_=None, lanes_=None, zc=None):
        return eng.serve_stream(arrivals if arr is None else arr, pool, lut, clock=0, refill=policy, min_incr=min_incr_ or min_incr, t_slo_ns=t_slo_ns,
                                lanes=(lanes_ or lanes) if policy == 2 else 1, zero_copy=zero_copy if zc is None else zc)

    def timed_steps(k, **kw):
        step(**kw)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            r, s_, _ = step(**kw)
        torch.cuda.synchronize()
        return k * n / (time.perf_counter() - t0), r, s_

    def summary(rate, r, s_):
        lat_ = r["latency_ns"].astype(np.float64)
        return dict(samples_per_s=round(rate, 1), mean_batch_per_segment=[round(a / max(b, 1), 2) for a, b in zip(s_["seg_samples"], s_["seg_runs"])],
                    latency_ms_mean=round(lat_.mean() / 1e6, 3), latency_ms_p99=round(float(np.percentile(lat_, 99)) / 1e6, 3),
                    slo_violation_rate=round(float(np.mean(lat_ > t_slo_ns)), 4) if t_slo_ns >= 0 else None, preemptions=s_["preemptions"])

    for _ in range(warmup):
        step()
    marker = torch.zeros(64, device="cuda")
    torch.cuda.synchronize()
    marker.cos_()                                      # a kernel trace shows the timed region between a cos and a sin kernel
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        res, st, _ = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    marker.sin_()
    value = steps * n / elapsed

    # Outside the timed region: the same trace under the other refill policy (Algorithm 1 of the paper when the stage pools
    # were timed, and the other way round), Algorithm 1 exactly as printed (min_incr = 1), and the capacity of the timed
    # policy: every request queued at t = 0, so that the figure is bounded by the path and not by the arrival rate.
    other = printed = capacity = None
    k_side = max(1, min(steps, 2))
    if refill in (1, 2) and full:
        rate_o, res_o, st_o = timed_steps(k_side, policy=3 - refill)
        other = summary(rate_o, res_o, st_o)
        other["same_exits"] = bool(np.array_equal(res_o["exit_idx"], res["exit_idx"]))
        rate_p, res_p, st_p = timed_steps(1, policy=1, min_incr_=1)
        printed = summary(rate_p, res_p, st_p)
    if load is not None and full:
        rate_c, res_c, st_c = timed_steps(k_side, arr=zeros)
        capacity = summary(rate_c, res_c, st_c)
        if refill == 2 and lanes > 1:
            capacity["one_lane_samples_per_s"] = round(timed_steps(1, arr=zeros, lanes_=1)[0], 1)
        if zero_copy:
            capacity["copying_compaction_samples_per_s"] = round(timed_steps(k_side, arr=zeros, zc=0)[0], 1)

    # Per-kernel durations: HIP events on the library's streams around every launch of one more step of the same
    # workload on one lane (kernels of concurrent steps share the chip, so their durations would say nothing about a
    # kernel).  Bracketing each launch costs the stream its back-to-back dispatch, so it is kept out of the timed steps.
    kstats = {k: dict(launches=0, ms=0.0, ops=0.0, bytes=0.0) for k in ee.K_NAMES}
    layer_stats = []
    at_capacity = None
    if not args.no_kernel_timing:
        eng.profile(True)
        step(lanes_=1)
        kstats, layer_stats = eng.profile_read(len(blob.ops))
        if zero_copy:                                  # the compaction kernel only runs in the copying mode: one more step for its line
            step(lanes_=1, zc=0)
            kstats["compact"] = eng.profile_read(len(blob.ops))[0]["compact"]
        if kstats["gap"]["launches"] == 0 and full:    # the serving path pools inside the segment's last layer: the stand-alone
            for s_ in range(blob.n_stages):            # pooling kernel of ee_exit_head is timed on b_max resident samples per exit
                ex = blob.exits[s_]
                act = torch.randint(-100, 100, (b_max, int(ex["h"]), int(ex["w"]), int(ex["c"]) * (1 if dtype == "i8" else 2)), dtype=torch.int8, device="cuda")
                for _ in range(3):
                    eng.exit_head(s_, act, 2.0)
            kstats["gap"] = eng.profile_read(len(blob.ops))[0]["gap"]
        eng.profile(False)
        if "capacity" in (args.roofline_at or "") and load is not None and full:
            eng.profile(True)                          # the same per-launch timing with every batch full (all requests at t = 0)
            step(arr=zeros, lanes_=1)
            conv_c = eng.profile_read(len(blob.ops))[0]["conv_mfma"]
            eng.profile(False)
            at_capacity = dict(achieved=round(conv_c["ops"] / (conv_c["ms"] * 1e-3) / 1e12, 2), launches=conv_c["launches"],
                               avg_launch_us=round(conv_c["ms"] * 1e3 / conv_c["launches"], 2))
            at_capacity["frac"] = round(at_capacity["achieved"] / PEAK[dtype], 4)

    # dominant kernel: the MFMA implicit-GEMM convolution
    conv = kstats["conv_mfma"]
    roofline = None
    if conv["launches"]:
        achieved = conv["ops"] / (conv["ms"] * 1e-3) / 1e12
        roofline = dict(bound="mfma", kernel="conv_igemm_kernel, conv_slab_kernel, conv_pair_kernel, bneck_block_i8_kernel, ir_block_i8_kernel", achieved=round(achieved, 2), peak=PEAK[dtype],
                        unit="TOP/s" if dtype == "i8" else "TFLOP/s", frac=round(achieved / PEAK[dtype], 4), traffic=None,
                        launches=conv["launches"], avg_launch_us=round(conv["ms"] * 1e3 / conv["launches"], 2),
                        algorithmic_gops_per_launch=round(conv["ops"] / conv["launches"] / 1e9, 3),
                        algorithmic_mb_per_launch=round(conv["bytes"] / conv["launches"] / 1e6, 3),
                        algorithmic_tops_per_step=round(conv["ops"] / 1e12, 3), algorithmic_gb_per_step=round(conv["bytes"] / 1e9, 3),
                        kernel_ms_per_step=round(conv["ms"], 3),
                        hbm_gbps_algorithmic=round(conv["bytes"] / (conv["ms"] * 1e-3) / 1e9, 1))
        roofline["traffic"] = measured_traffic(name)
        if at_capacity:
            roofline["with_every_batch_full"] = at_capacity
        # Layer by layer the convolutions are also capped by their algorithmic bytes: the time the launches of
        # a layer need at best is max(ops / MFMA peak, bytes / HBM peak); the sum over the layers gives the
        # rate the stack could reach if every launch sat on its own roofline (ops and bytes of a layer are
        # proportional to the batch, so the per-layer totals decide the max).
        conv_layers = [l for op, l in zip(blob.ops, layer_stats) if int(op["kind"]) == W.OP_CONV and l["launches"] and l["ops"] > 0]
        best_s = sum(max(l["ops"] / (PEAK[dtype] * 1e12), l["bytes"] / (HBM_PEAK * 1e9)) for l in conv_layers)
        if best_s > 0:
            capped = sum(l["ops"] for l in conv_layers) / best_s / 1e12
            roofline["layerwise_cap"] = round(capped, 1)              # same unit as `peak`
            layers_s = sum(l["ms"] for l in conv_layers) * 1e-3
            roofline["frac_of_layerwise_cap"] = round(best_s / layers_s, 4)
    kernels = {k: dict(launches=v["launches"], ms=round(v["ms"], 3),
                       gbps=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else 0.0,
                       hbm_frac=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / HBM_PEAK, 4) if v["ms"] > 0 else 0.0,
                       tops=round(v["ops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["ms"] > 0 else 0.0)
               for k, v in kstats.items() if v["launches"]}

    # the CPU oracle on a bounded sample of the same requests, each sample alone until it exits: all cores, then one
    cpu = None
    if args.cpu_samples >= 0 and full:
        import oracle
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        per = {"resnet50_i8": 16 * cores, "resnet50_eq_i8": 16 * cores, "inception_i8": 8 * cores, "resnet50_bf16": 2 * cores, "resnet18_i8": 32 * cores,
               "mobilenetv2_i8": 128 * cores}.get(wl["net"], 64)
        ns = min(n, args.cpu_samples or per)
        sample = W.input_pool(blob, ns)
        t0 = time.perf_counter()
        ref = oracle.forward_alone(blob, sample)
        dt = time.perf_counter() - t0
        agree = bool(np.array_equal(ref["exit_idx"], res["exit_idx"][:ns])) if dtype == "i8" else None
        n1 = max(1, min(ns, int(round(ns / dt / cores * 10))))              # about 10 s on one core
        t0 = time.perf_counter()
        oracle.forward_alone(blob, sample[:n1], threads=1)
        dt1 = time.perf_counter() - t0
        cpu = dict(value=round(ns / dt, 3), unit="samples/s", cores=cores, kind="oracle",
                   sample=f"first {ns} requests of the same pool, each alone through the segments until it exits, OpenMP over samples",
                   seconds=round(dt, 2), exits_agree_with_gpu=agree,
                   one_core=dict(value=round(n1 / dt1, 3), unit="samples/s", cores=1, sample=f"first {n1} of them", seconds=round(dt1, 2)))

    lat = res["latency_ns"].astype(np.float64)
    out = {
        "metric": "samples/sec early-exit CNN stream (1 GPU)", "value": round(value, 1), "unit": "samples/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": name, "requests": n, "b_max": b_max, "refill": refill,
                   "policy": ["static batches", "Algorithm 1", "stage pools"][refill], "lanes": lanes if refill == 2 else None,
                   "compaction": "zero-copy (slot tables)" if zero_copy else "copy",
                   "min_incr": min_incr if refill == 1 else None,
                   "arrival": "poisson" if load else "all_at_t0", "arrival_rate_per_s": round(load * static_rate, 1) if load else None,
                   "clock": "wall", "t_slo_ms": args.t_slo_ms if t_slo_ns >= 0 else None},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "static_batch_samples_per_s": round(static_rate, 1),
        "capacity": capacity,
        ("algorithm1" if refill == 2 else "stage_pools"): other,
        "algorithm1_min_incr": min_incr if refill == 2 else None,
        "algorithm1_as_printed": printed,
        "exit_counts": np.bincount(res["exit_idx"], minlength=eng.n_stages).tolist(),
        "mean_batch_per_segment": [round(a / max(b, 1), 2) for a, b in zip(st["seg_samples"], st["seg_runs"])],
        "mean_batch_per_segment_static": [round(a / max(b, 1), 2) for a, b in zip(st_static["seg_samples"], st_static["seg_runs"])],
        "slo_violation_rate": round(float(np.mean(lat > t_slo_ns)), 4) if t_slo_ns >= 0 else None,
        "preemptions": st["preemptions"], "latency_ms_mean": round(lat.mean() / 1e6, 3), "latency_ms_p99": round(float(np.percentile(lat, 99)) / 1e6, 3),
        "kernels": kernels,
    }
    eng.close()
    del pool
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="resnet50_i8_stream", choices=sorted(WORKLOADS))
    ap.add_argument("--requests", type=int, default=0, help="override the number of requests (0 = the workload's)")
    ap.add_argument("--min-incr", type=int, default=0, help="smallest catch-up batch (0 = b_max / 2; 1 = Algorithm 1 as printed)")
    ap.add_argument("--t-slo-ms", type=float, default=-1.0, help="latency SLO of Eq. 3 in ms (negative = none: throughput run)")
    ap.add_argument("--refill", type=int, default=-1, choices=[-1, 0, 1, 2],
                    help="serving policy of the timed steps: 0 model-level batching, 1 Algorithm 1, 2 stage pools (-1 = the workload's)")
    ap.add_argument("--lanes", type=int, default=0, help="stage pools: steps in flight at once (0 = the workload's)")
    ap.add_argument("--roofline-at", default="capacity", help="'capacity': also time the convolution launches of a step whose batches are all full")
    ap.add_argument("--zero-copy", type=int, default=-1, choices=[-1, 0, 1], help="0: always the copying compaction kernel; else zero-copy compaction where the network allows it")
    ap.add_argument("--load", type=float, default=0.0, help="arrival rate as a multiple of the static-batch throughput (0 = the workload's)")
    ap.add_argument("--cpu-samples", type=int, default=0, help="samples timed on the CPU oracle (0 = automatic, -1 = skip)")
    ap.add_argument("--save-tables", default="", help="write the tuned kernel-configuration tables to this JSON file")
    ap.add_argument("--load-tables", default="", help="load the kernel-configuration tables from this JSON file instead of tuning")
    ap.add_argument("--no-kernel-timing", action="store_true", help="skip the extra step that brackets every kernel launch with HIP events")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short runs of the other stream configurations")
    ap.add_argument("--layers", type=int, default=0, metavar="B",
                    help="instead of the stream: every layer of the workload's network alone on B samples, tuned, launches back to back")
    ap.add_argument("--layer", type=int, default=-1, help="with --layers: only this layer (an index into the network's layer list)")
    ap.add_argument("--cfg", type=lambda v: int(v, 0), default=0, help="with --layer: a forced kernel configuration word (0 = the tuned one)")
    ap.add_argument("--policies", action="store_true",
                    help="instead of the one stream: the serving policies of the evaluation over arrival rates and SLOs (see policy_sweep)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this program measures the path on ONE GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2209_13443_amd as ee
    import workloads as W
    torch.cuda.set_device(0)
    if args.layers:
        blob = W.load_net(WORKLOADS[args.workload]["net"])
        return layer_table(args, ee, W, blob, "i8" if blob.dtype == W.DT_I8 else "bf16")
    if args.policies:
        return policy_sweep(args, ee, W)
    out = run_stream(args, args.workload, args.steps, args.warmup)
    if args.workload == "resnet50_i8_stream" and not args.no_other_configs and not args.requests:
        # the other stream configurations, briefly: one timed step each, their dominant kernel class against its roofline
        others = {}
        for name in ("mobilenetv2_i8_refill", "resnet50_bf16_stream"):
            o = run_stream(args, name, 1, 1, full=False)
            k = o["kernels"]
            entry = dict(samples_per_s=o["value"], ms_per_step=o["ms_per_step"], static_batch_samples_per_s=o["static_batch_samples_per_s"],
                         dtype=o["dtype"], config=o["config"], mean_batch_per_segment=o["mean_batch_per_segment"])
            if o["roofline"]:
                entry["conv_mfma"] = {f: o["roofline"][f] for f in ("achieved", "peak", "unit", "frac", "launches", "avg_launch_us")}
            if "depthwise" in k:
                entry["depthwise"] = dict(bound="hbm", achieved=k["depthwise"]["gbps"], peak=HBM_PEAK, unit="GB/s", frac=k["depthwise"]["hbm_frac"], launches=k["depthwise"]["launches"])
            others[name] = entry
        out["other_configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
