#!/usr/bin/env python3
"""Writes tests/golden/full_size_<net>.txt: exit index, label and score (int8 networks: the integer softmax
denominator S; bf16 networks: confidence) of the first N requests of each full-size benchmark network.
Calls the CPU oracle only (every request alone through the segments until it exits); the GPU tests compare
what the library serves, under every policy, with these lines.

    python tests/golden/make_full_size_golden.py [net ...]
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import workloads as W  # noqa: E402

NETS = {"resnet18_i8": 512, "resnet50_i8": 512, "mobilenetv2_i8": 512, "resnet50_eq_i8": 256, "inception_i8": 256, "resnet50_bf16": 64}


def main():
    for name in (sys.argv[1:] or NETS):
        n = NETS[name]
        blob = W.load_net(name)
        pool = W.input_pool(blob, n)
        t0 = time.time()
        res = oracle.forward_alone(blob, pool)
        with open(os.path.join(HERE, f"full_size_{name}.txt"), "w") as f:
            f.write(f"# {name}: oracle.forward_alone on requests 0..{n - 1} of workloads.input_pool (each alone, thresholds of the blob)\n")
            f.write("# columns: request exit label score conf\n")
            for k in range(n):
                f.write(f"{k} {int(res['exit_idx'][k])} {int(res['label'][k])} {int(res['score'][k])} {float(res['conf'][k])!r}\n")
        print(f"{name}: {n} requests in {time.time() - t0:.1f} s, exits {np.bincount(res['exit_idx'], minlength=blob.n_stages).tolist()}", flush=True)


if __name__ == "__main__":
    main()
