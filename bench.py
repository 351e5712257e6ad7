#!/usr/bin/env python3
"""Benchmark of the adaptive-sampling hot path on one MI355X.

One step = one pass of the whole path over one synthetic trajectory already resident in HBM:
tree-ensemble scoring of every configuration, the k-means++ chain, the Lloyd sweep over all k
(assign + update rounds and the final assignment with labels and inertia), the knee pick on the host,
the snap of the chosen centroids, the per-dimension mode of the trajectory and the replacement of samples
that were visited before.  The headline value is config-iterations per second:
N x (number of k) x (Lloyd rounds) per step divided by the step time.

Prints ONE JSON line.  `roofline` describes the dominant kernel (the fused assign + update Lloyd step),
timed with HIP events recorded by the library on the launch stream during the timed steps;
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.  Outside the timed steps the
line also carries `early_exit` (the sweep that stops at the knee) and `lloyd_step_per_k` (the Lloyd step of a
sweep over one k at a time: launch time, points per second, fractions of the HBM and fp16 matrix peaks).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3   # dense fp32 matrix (for scale: the fp32 contraction runs as fp16 pieces)
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 matrix: the pipeline the distance tiles run on

# HBM bytes of one lloyd_step_kernel launch from rocprofv3 counters (profiles/lloyd_step_whole_layer_hbm_counters.md):
# FETCH_SIZE / WRITE_SIZE in KiB per dispatch and the factors a plain 1 GiB copy gives for each counter.  Valid
# only for the library version the counters were taken with; any other version reports traffic = null.
HBM_COUNTERS = {
    "whole_layer": {"version": 110, "fetch_kib": 169259.2, "write_kib": 59620.2, "fetch_scale": 2.0, "write_scale": 1.0},
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="whole_layer", choices=["tiny", "mid", "whole_layer", "large", "batched"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-labels", action="store_true", help="do not write the per-k label arrays")
    ap.add_argument("--serial-score", action="store_true",
                    help="score on the main stream before the sweep instead of beside it on a second stream")
    ap.add_argument("--no-early-exit", action="store_true", help="skip the extra timing of the sweep with early exit at the knee")
    ap.add_argument("--no-per-k", action="store_true", help="skip the extra timing of the Lloyd step for single values of k")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of 1 GiB (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1905_12799_amd import binding as rls
    from paper_1905_12799_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    rls.lib()   # fails loudly when the HIP library is not built

    w = synth.WORKLOADS[args.workload]
    batched = w.batch > 1
    if batched:
        probs = synth.make_batched_problems(w)
        X_host = np.stack([p.X for p in probs])
    else:
        probs = [synth.make_problem(w)]
        X_host = probs[0].X
    X = torch.as_tensor(X_host).cuda()
    forests = [rls.DeviceForest.from_host(p.forest) for p in probs]
    domains = [rls.DeviceDomains(p.dom_offsets, p.dom_values) for p in probs]
    n_visited = 65536
    visited = [torch.as_tensor(synth.visited_configs(p, n_visited, w.seed + 1000 + b)).cuda() for b, p in enumerate(probs)]
    B = w.batch
    n_k = w.k_max - w.k_min + 1
    ws_bytes = rls.kmeans_sweep_workspace_bytes(w.N, w.d, w.k_min, w.k_max, B)
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    scores = torch.empty((B, w.N) if batched else (w.N,), dtype=torch.float32, device="cuda")
    seeds = [w.seed + b for b in range(B)]
    knee_const = 1.05
    hists = [torch.empty(dm.n_values, dtype=torch.int32, device="cuda") for dm in domains]
    want_labels = not args.no_labels

    ev = {name: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for name in ("score", "sweep", "snap", "modes_visited")}
    stage_ms = {name: 0.0 for name in ev}

    # Tree scoring and clustering both only read the trajectory: the scores are computed on a second stream (default
    # priority) beside the sweep, whose seeding chain is a string of short bandwidth-bound launches.
    main_stream = torch.cuda.current_stream()
    side_stream = None if args.serial_score else torch.cuda.Stream()

    def step(record: bool):
        score_stream = main_stream if side_stream is None else side_stream
        if side_stream is not None:
            side_stream.wait_stream(main_stream)
        with torch.cuda.stream(score_stream):
            ev["score"][0].record()
            if batched:
                rls.gbt_score_batched(forests, X, out=scores)
            else:
                rls.gbt_score(forests[0], X, out=scores)
            ev["score"][1].record()
        ev["sweep"][0].record()
        if batched:
            res = rls.kmeans_sweep_batched(X, w.k_min, w.k_max, w.iters, seeds=seeds, want_labels=want_labels,
                                           workspace=ws, check_status=False)
        else:
            res = rls.kmeans_sweep(X, w.k_min, w.k_max, w.iters, seed=seeds[0], want_labels=want_labels,
                                   workspace=ws, check_status=False)
        ev["sweep"][1].record()
        inertia = res.inertia.cpu()            # the knee pick is a host step: one small copy, one sync
        status = res.status.cpu()
        if bool((status != 0).any()):
            raise RuntimeError(f"sweep status {status.tolist()}")
        ev["snap"][0].record()
        chosen, cfgs = [], []
        if batched:
            # one k per space; snap each space's chosen centroids (same k needed for a batched call, so loop)
            for b in range(B):
                k = rls.pick_knee(inertia[b].tolist(), w.k_min, w.k_max, knee_const)
                chosen.append(k)
                cfgs.append(rls.snap_to_valid(res.centroids_of(k, b), domains[b]))
        else:
            k = rls.pick_knee(inertia.tolist(), w.k_min, w.k_max, knee_const)
            chosen.append(k)
            cfgs.append(rls.snap_to_valid(res.centroids_of(k), domains[0]))
        ev["snap"][1].record()
        ev["modes_visited"][0].record()
        for b in range(B):
            mode, _ = rls.knob_modes(X[b] if batched else X, domains[b], hist=hists[b])
            rls.replace_visited(cfgs[b], visited[b], mode)
        ev["modes_visited"][1].record()
        if side_stream is not None:
            main_stream.wait_stream(side_stream)
        if record:
            torch.cuda.synchronize()
            for name in ev:
                stage_ms[name] += ev[name][0].elapsed_time(ev[name][1])
        return chosen

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    rls.profile_enable(True)
    rls.profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        chosen = step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    n_launch, kernel_ms_total = rls.profile_read()
    rls.profile_enable(False)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    point_iters = float(w.N) * B * n_k * w.iters
    value = point_iters / (ms_per_step * 1e-3)
    sweep_ms = stage_ms["sweep"] / args.steps
    score_ms = stage_ms["score"] / args.steps

    # dominant kernel: the Lloyd step (assign + update for every k in one launch)
    kernel_ms = kernel_ms_total / max(n_launch, 1)
    sum_k = sum(range(w.k_min, w.k_max + 1))
    alg_bytes = 4.0 * w.d * w.N * B * n_k                 # 4*d bytes per point and (k, round)
    alg_flops = 2.0 * w.d * sum_k * w.N * B               # 2*d*k flops per point and (k, round)
    gbs = alg_bytes / (kernel_ms * 1e-3) / 1e9
    tflops = alg_flops / (kernel_ms * 1e-3) / 1e12
    # The contraction is carried out on the fp16 matrix pipeline: per distance three products of fp16 pieces over the
    # padded features plus one bias step of 16.  Which roofline is the higher floor for the algorithmic work?
    d_pad = 8 if w.d <= 8 else (16 if w.d <= 16 else 32)
    mfma_flops = 2.0 * (3.0 * max(d_pad, 16) + 16.0) * sum_k * w.N * B
    mfma_tflops = mfma_flops / (kernel_ms * 1e-3) / 1e12
    hbm_time, mfma_time = alg_bytes / (HBM_PEAK_GBS * 1e9), mfma_flops / (MFMA_F16_PEAK_TFLOPS * 1e12)
    if hbm_time >= mfma_time:
        roofline = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                    "traffic": None}
    else:
        roofline = {"bound": "mfma", "achieved": mfma_tflops, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": mfma_tflops / MFMA_F16_PEAK_TFLOPS, "traffic": None}
    hc = HBM_COUNTERS.get(w.name)
    if hc is not None and hc["version"] == rls.version() and want_labels:
        hbm_bytes = (hc["fetch_kib"] * hc["fetch_scale"] + hc["write_kib"] * hc["write_scale"]) * 1024.0
        # same unit as `achieved` when the bound is HBM; the ratio to the algorithmic bytes is what matters
        roofline["traffic"] = hbm_bytes / (kernel_ms * 1e-3) / 1e9
        roofline["traffic_bytes_per_launch"] = hbm_bytes
    roofline["algorithmic_bytes_per_launch"] = alg_bytes
    roofline.update({"kernel": "lloyd_step_kernel", "launches_timed": n_launch, "avg_launch_ms": kernel_ms,
                     "algorithmic_GBps": gbs, "hbm_frac": gbs / HBM_PEAK_GBS,
                     "algorithmic_TFLOPs": tflops, "fp32_mfma_equivalent_frac": tflops / MFMA_F32_PEAK_TFLOPS,
                     "mfma_f16_TFLOPs": mfma_tflops, "mfma_f16_frac": mfma_tflops / MFMA_F16_PEAK_TFLOPS})

    out = {
        "metric": "config_iter_per_s", "value": value, "unit": "config*iter/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: N={w.N} d={w.d} batch={B} k={w.k_min}..{w.k_max} iters={w.iters} "
                               f"forest={w.n_trees}x{w.depth}", "labels_written": want_labels,
                   "knee_const": knee_const, "chosen_k": chosen[:4],
                   "score_stream": "main" if side_stream is None else "second stream beside the sweep"},
        "configs_scored_per_s": float(w.N) * B / (score_ms * 1e-3),
        "sweep_config_iter_per_s": point_iters / (sweep_ms * 1e-3),
        "stage_ms": {"gbt_score": score_ms, "kmeans_sweep": sweep_ms, "snap": stage_ms["snap"] / args.steps,
                     "modes_visited": stage_ms["modes_visited"] / args.steps},
        "roofline": roofline,
        # tree scoring: bound by LDS gathers and vector issue (T*D node visits per 4d+4 bytes), shown against HBM for scale
        "gbt_score": {"ms": score_ms, "node_visits_per_s": float(w.N) * B * w.n_trees * w.depth / (score_ms * 1e-3),
                      "algorithmic_GBps": (4.0 * w.d + 4.0) * w.N * B / (score_ms * 1e-3) / 1e9,
                      "hbm_frac": (4.0 * w.d + 4.0) * w.N * B / (score_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      # the walk is bound by LDS: 12 bytes per lane and visit (node 8, feature value 4) against
                      # 128 B/clk on each of 256 CUs at 2.4 GHz
                      "lds_GBps": 12.0 * float(w.N) * B * w.n_trees * w.depth / (score_ms * 1e-3) / 1e9,
                      "lds_frac": 12.0 * float(w.N) * B * w.n_trees * w.depth / (score_ms * 1e-3) / (256 * 128 * 2.4e9)},
    }

    if not batched and not args.no_early_exit:
        # Algorithm 1 with its early exit at the knee (k in waves of 8), outside the timed steps: same chosen k,
        # only the waves up to the knee are computed
        k_e, n_done, _ = rls.kmeans_sweep_until_knee(X, w.k_min, w.k_max, 8, w.iters, knee_const, seed=seeds[0],
                                                     want_labels=want_labels)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(3):
            k_e, n_done, _ = rls.kmeans_sweep_until_knee(X, w.k_min, w.k_max, 8, w.iters, knee_const, seed=seeds[0],
                                                         want_labels=want_labels)
        torch.cuda.synchronize()
        out["early_exit"] = {"ms": (time.perf_counter() - t2) * 1e3 / 3, "chosen_k": k_e, "k_computed": n_done, "k_wave": 8}

    if not batched and not args.no_per_k:
        # The Lloyd step for one k at a time (outside the timed steps): where the launch time leaves the floor set by
        # reading the trajectory and starts to follow the distance work.  Same kernel, a plan with a single run.
        per_k = []
        for k in [k for k in (1, 2, 4, 8, 16, 32, 64, 128) if w.k_min <= k <= w.k_max]:
            rls.kmeans_sweep(X, k, k, w.iters, seed=seeds[0], want_labels=False)
            torch.cuda.synchronize()
            rls.profile_enable(True)
            rls.profile_read()
            rls.kmeans_sweep(X, k, k, w.iters, seed=seeds[0], want_labels=False)
            n_l, ms_l = rls.profile_read()
            rls.profile_enable(False)
            t_l = ms_l / max(n_l, 1) * 1e-3
            flops_k = 2.0 * (3.0 * max(d_pad, 16) + 16.0) * max(k, 32) * w.N       # issued: tiles of 32 centroids
            per_k.append({"k": k, "launch_ms": t_l * 1e3, "config_iter_per_s": w.N / t_l,
                          "hbm_frac": 4.0 * w.d * w.N / t_l / 1e9 / HBM_PEAK_GBS,
                          "algorithmic_TFLOPs": 2.0 * w.d * k * w.N / t_l / 1e12,
                          "mfma_f16_frac": flops_k / t_l / 1e12 / MFMA_F16_PEAK_TFLOPS})
        out["lloyd_step_per_k"] = per_k

    if not args.no_cpu_baseline:
        import oracle
        p0 = probs[0]
        ks = [k for k in (8, 32, 64, 128) if w.k_min <= k <= w.k_max] or [w.k_max]
        iters_s = 20
        chain = oracle.kmeanspp_chain(p0.X, max(ks), w.seed)
        t = time.perf_counter()
        for k in ks:
            oracle.lloyd(p0.X, k, iters_s, chain)
        dt = time.perf_counter() - t
        n_s = min(w.N, 65536)
        t = time.perf_counter()
        oracle.gbt_score(p0.forest, p0.X[:n_s])
        dt_s = time.perf_counter() - t
        out["cpu_baseline"] = {
            "value": float(w.N) * len(ks) * iters_s / dt, "unit": "config*iter/s", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"Lloyd on the full N={w.N} of one space for k in {ks}, {iters_s} rounds each plus the final "
                      f"assignment ({dt:.1f} s); tree scoring of the first {n_s} configurations on 1 thread ({dt_s:.1f} s)",
            "configs_scored_per_s": n_s / dt_s,
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
