#!/usr/bin/env python3
"""Writes tests/golden/fullsize_<workload>.json: the CPU oracle's results at the full sizes of the workloads.

At 1M and 8M configurations the oracle needs minutes to hours for what the GPU sweeps in milliseconds, so its
results for the full-size parity tests are computed once, here, and stored: per k the loss (hex float), a
SHA-256 of the fp32 centroid array and one of the int32 label array, and the seeding chain; next to them a
SHA-256 of the input matrix, so that a test can tell whether it is looking at the same input.

This script calls the oracle and the input generator only - never the GPU library.
Usage: python tests/golden/make_fullsize_golden.py whole_layer|large|batched [--out DIR]
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_1905_12799_amd import synth  # noqa: E402

# which runs are stored: every k of whole_layer; on large the k up to past the knee of the loss curve plus a
# middle and the largest k; on batched eight of the 64 spaces, every k
PLAN = {
    "whole_layer": {"spaces": [0], "ks": list(range(1, 65))},
    "large": {"spaces": [0], "ks": list(range(1, 13)) + [37, 128]},
    "batched": {"spaces": [0, 7, 19, 30, 41, 52, 58, 63], "ks": list(range(1, 33))},
}


def sha(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", choices=sorted(PLAN))
    ap.add_argument("--out", default=HERE)
    args = ap.parse_args()
    w = synth.WORKLOADS[args.workload]
    plan = PLAN[args.workload]
    t0 = time.time()
    if w.batch > 1:
        shapes = synth.batched_conv_shapes(w.batch, w.seed)
    out = {"workload": w.name, "N": w.N, "d": w.d, "iters": w.iters, "k_min": w.k_min, "k_max": w.k_max,
           "oracle_threads": oracle.threads(), "spaces": {}}
    path = os.path.join(args.out, f"fullsize_{w.name}.json")
    for b in plan["spaces"]:
        seed = w.seed + b
        p = synth.make_problem(w, conv=shapes[b], seed=seed) if w.batch > 1 else synth.make_problem(w)
        print(f"[{time.time() - t0:7.1f}s] space {b}: X {p.X.shape}", flush=True)
        chain = oracle.kmeanspp_chain(p.X, w.k_max, seed)
        space = {"seed": seed, "x_sha256": sha(p.X), "chain": chain.tolist(), "runs": {}}
        for k in plan["ks"]:
            labels, C, J, _ = oracle.lloyd(p.X, k, w.iters, chain)
            space["runs"][str(k)] = {"inertia": float(J).hex(), "centroids_sha256": sha(C),
                                     "labels_sha256": sha(labels)}
            print(f"[{time.time() - t0:7.1f}s] space {b} k={k} J={J:.9g}", flush=True)
            out["spaces"][str(b)] = space
            with open(path + ".tmp", "w") as fh:
                json.dump(out, fh)
        out["spaces"][str(b)] = space
    with open(path, "w") as fh:
        json.dump(out, fh, indent=0)
    if os.path.exists(path + ".tmp"):
        os.remove(path + ".tmp")
    print(f"wrote {path} in {time.time() - t0:.0f} s")
    return 0


if __name__ == "__main__":
    sys.exit(main())
