"""Freeze the data-dependent constants of a synthetic network with the CPU oracle.

Random weights have no trained scales or exit policy, so the per-layer requantisation
shifts, the logit scaling and the exit thresholds are measured on a seeded calibration
batch -- by the oracle alone -- and stored as a small JSON record under
workloads/calib/.  The thresholds are confidence quantiles chosen to give the exit split
the configuration asks for (the paper tunes a threshold on its validation set instead,
Sec. IV "Benchmarks").

Rules (all data-driven, applied layer by layer on the calibration batch):
  shift      smallest s such that at most 0.1 % of |t| exceed 127 * 2^s, t = value to requantise
  res_shift  the shift the convolution alone (without residual) would get
  frac_bits  f with std(logits) * 2^-f closest to 2   (int8 nets)
  logit_scale  2 / std(raw logits)                   (bf16 nets)
  thr        between the k-th and (k+1)-th most confident sample reaching the exit,
             k = round(quantile * reaching)

Usage:  python -m oracle.calibrate NAME [N_CAL]      (run from the repository root)
"""
import json
import math
import os
import sys
import time

import numpy as np

import oracle as O
import workloads as W
from workloads.blob import OP_CONV, OP_DWCONV, OP_MAXPOOL, OP_AVGPOOL, DT_I8

CALIB_DIR = os.path.join(os.path.dirname(os.path.abspath(W.__file__)), "calib")

# exit split per configuration: fraction of ALL samples leaving at each exit
SPLITS = {
    "tiny_i8": (0.4, 0.3, 0.3), "tiny_bf16": (0.4, 0.3, 0.3),
    "resnet18_i8": (0.3, 0.3, 0.2, 0.2), "resnet18_small_i8": (0.3, 0.3, 0.2, 0.2),
    "mobilenetv2_i8": (0.25, 0.25, 0.5), "mobilenetv2_small_i8": (0.25, 0.25, 0.5),
    "resnet50_i8": (0.2, 0.2, 0.3, 0.3), "resnet50_small_i8": (0.2, 0.2, 0.3, 0.3),
    "resnet50_bf16": (0.2, 0.2, 0.3, 0.3), "resnet50_small_bf16": (0.2, 0.2, 0.3, 0.3),
    "resnet50_eq_i8": (0.2, 0.2, 0.3, 0.3),
    "inception_i8": (0.2, 0.2, 0.3, 0.3), "inception_small_i8": (0.2, 0.2, 0.3, 0.3), "inception_small_bf16": (0.2, 0.2, 0.3, 0.3),
    "zoo_i8": (0.35, 0.35, 0.3), "zoo_bf16": (0.35, 0.35, 0.3),
}
DEFAULT_N_CAL = {"tiny_i8": 64, "tiny_bf16": 64, "resnet18_i8": 96, "mobilenetv2_i8": 128, "resnet50_i8": 96,
                 "resnet50_bf16": 64, "resnet50_eq_i8": 96, "inception_i8": 96}
CAL_SEED_OFF = 7     # calibration inputs come from their own pool, not from the served one
N_SHIFT = 16         # samples used for the shift statistics


def _pick_shift(t):
    a = np.abs(t.astype(np.int64)).ravel()
    allowed = int(math.floor(0.001 * a.size))
    for s in range(0, 31):
        if int(np.count_nonzero(a > (127 << s))) <= allowed:
            return s
    return 30


def _threshold_from_scores(scores, k):
    """float32 thr such that the k most confident (smallest score) samples satisfy S <= floor(2^30/thr)."""
    n = scores.size
    if k <= 0:
        return 2.0
    srt = np.sort(scores)
    lo = int(srt[k - 1])
    hi = int(srt[k]) if k < n else lo + max(1, lo // 64)
    mid = (lo + hi) // 2
    thr = np.float32((1 << 30) / mid)
    for cand in (thr, np.nextafter(thr, np.float32(0)), np.nextafter(thr, np.float32(2))):
        if O.score_threshold(float(cand)) >= lo and (k == n or O.score_threshold(float(cand)) < hi):
            return float(cand)
    return float(thr)


def _threshold_from_conf(conf, k):
    """bf16 nets: midpoint of the widest gap between adjacent confidences within +-0.5 % rank of the quantile."""
    n = conf.size
    if k <= 0:
        return 2.0
    srt = np.sort(conf.astype(np.float64))[::-1]      # most confident first
    if k >= n:
        return float(np.float32(srt[-1] * 0.5))
    span = max(1, int(round(0.005 * n)))
    best, best_gap = k, -1.0
    for j in range(max(1, k - span), min(n - 1, k + span) + 1):
        gap = srt[j - 1] - srt[j]
        if gap > best_gap:
            best, best_gap = j, gap
    return float(np.float32(0.5 * (srt[best - 1] + srt[best])))


def calibrate(name, n_cal=None, log=print):
    blob = W.build_net(name)
    split = SPLITS[name]
    n_cal = n_cal or DEFAULT_N_CAL.get(name, 64)
    x = W.input_pool(blob, n_cal, seed_off=CAL_SEED_OFF)
    is_i8 = blob.dtype == DT_I8
    rec = dict(name=name, n_cal=n_cal, split=list(split), ops=[], exits=[])
    reaching = 1.0
    t0 = time.time()
    for s in range(blob.n_stages):
        tens = {0: x}
        for op in blob.stage_ops(s):
            kind, src = int(op["kind"]), tens[int(op["src"])]
            res = tens[int(op["res"])] if int(op["res"]) >= 0 else None
            stride, pad, pad_w = int(op["stride"]), int(op["pad"]), int(op["pad_w"])
            co, kh, kw, ci = int(op["c_out"]), int(op["kh"]), int(op["kw"]), int(op["c_in"])
            wt, bias = blob.op_weights(op)
            entry = dict(shift=0, res_shift=0)
            if kind == OP_MAXPOOL:
                y = O.maxpool_i8(src, kh, stride, pad) if is_i8 else O.maxpool_bf16(src, kh, stride, pad)
            elif kind == OP_AVGPOOL:
                y = O.avgpool_i8(src, kh, stride, pad) if is_i8 else O.avgpool_bf16(src, kh, stride, pad)
            elif is_i8:
                if kind == OP_CONV:
                    acc = O.conv_acc_i8(src, wt.reshape(co, kh, kw, ci), bias, stride, pad, pad_w=pad_w)
                else:
                    acc = O.dwconv_acc_i8(src, wt.reshape(co, kh, kw), bias, stride, pad)
                ns = min(N_SHIFT, acc.shape[0])
                shift = _pick_shift(acc[:ns])
                res_shift = 0
                if res is not None:
                    res_shift = min(shift, 23)
                    t = acc[:ns].astype(np.int64) + (res[:ns].astype(np.int64) << res_shift)
                    shift = _pick_shift(t)
                entry = dict(shift=shift, res_shift=res_shift)
                op["shift"], op["res_shift"] = shift, res_shift
                y = O.requant_i8(acc, res, shift, res_shift, int(op["lo"]), int(op["hi"]))
                del acc
            else:
                f_lo, f_hi = float(op["f_lo"]), float(op["f_hi"])
                if kind == OP_CONV:
                    y = O.conv_bf16(src, wt.reshape(co, kh, kw, ci), bias, stride, pad, res, f_lo, f_hi, pad_w=pad_w)
                else:
                    y = O.dwconv_bf16(src, wt.reshape(co, kh, kw), bias, stride, pad, f_lo, f_hi)
            dst, c_off, c_tot = int(op["dst"]), int(op["c_off"]), int(op["c_tot"])
            if c_tot == co:
                tens[dst] = y
            else:                                        # a channel slice of a concatenation tensor
                if dst not in tens:
                    tens[dst] = np.zeros(y.shape[:3] + (c_tot,), y.dtype)
                tens[dst][..., c_off:c_off + co] = y
            rec["ops"].append(entry)
        out = tens[int(blob.stages[s]["out_tensor"])]
        e = blob.exits[s]
        wfc, bfc = blob.exit_weights(s)
        n_cls, c = int(e["n_cls"]), int(e["c"])
        last = s == blob.n_stages - 1
        frac = min(1.0, split[s] / reaching) if not last else 1.0
        k = int(round(frac * out.shape[0]))
        if is_i8:
            _, g = O.gap_i8(out, int(e["gap_shift"]))
            a = O.fc_i8(g, wfc.reshape(n_cls, c), bfc)
            std = float(np.std(a.astype(np.float64), axis=1).mean())
            f = int(max(0, min(24, round(math.log2(max(std, 1.0) / 2.0)))))
            e["frac_bits"] = f
            _, score = O.softmax_top1_i8(a, f)
            thr = 2.0 if last else _threshold_from_scores(score, k)
            keep = ~(score <= O.score_threshold(thr)) if not last else np.zeros(out.shape[0], bool)
            ex = dict(gap_shift=int(e["gap_shift"]), frac_bits=f, logit_scale_bits=int(np.float32(1.0).view(np.uint32)))
        else:
            raw, _, _ = O.head_bf16(out, wfc.reshape(n_cls, c), bfc, 1.0)
            std = float(np.std(raw.astype(np.float64), axis=1).mean())
            scale = np.float32(2.0 / max(std, 1e-12))
            e["logit_scale"] = scale
            _, _, conf = O.head_bf16(out, wfc.reshape(n_cls, c), bfc, float(scale))
            thr = 2.0 if last else _threshold_from_conf(conf, k)
            keep = ~(conf >= np.float32(thr)) if not last else np.zeros(out.shape[0], bool)
            ex = dict(gap_shift=0, frac_bits=0, logit_scale_bits=int(scale.view(np.uint32)))
        e["thr"] = np.float32(thr)
        ex["thr_bits"] = int(np.float32(thr).view(np.uint32))
        ex["thr"] = float(np.float32(thr))
        ex["reached"], ex["exited"] = int(out.shape[0]), int(out.shape[0] - keep.sum())
        rec["exits"].append(ex)
        log(f"[{name}] stage {s}: reached {ex['reached']} exited {ex['exited']} thr {thr:.6f} ({time.time() - t0:.1f}s)")
        reaching -= split[s]
        x = np.ascontiguousarray(out[keep])
        if x.shape[0] == 0:
            for s2 in range(s + 1, blob.n_stages):
                raise RuntimeError("calibration batch ran dry before the last exit; use more samples")
    return rec, blob


def calib_path(name):
    return os.path.join(CALIB_DIR, f"{name}.json")


def main(argv):
    name = argv[1]
    n_cal = int(argv[2]) if len(argv) > 2 else None
    rec, _ = calibrate(name, n_cal)
    os.makedirs(CALIB_DIR, exist_ok=True)
    with open(calib_path(name), "w") as f:
        json.dump(rec, f, indent=1)
    print("wrote", calib_path(name))


if __name__ == "__main__":
    main(sys.argv)
