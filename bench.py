#!/usr/bin/env python3
"""Benchmark of the adaptive-sampling hot path on one MI355X.

One step = one pass of the whole path over one synthetic trajectory already resident in HBM:
tree-ensemble scoring of every configuration, the k-means++ chain, the Lloyd sweep over all k
(assign + update rounds and the final assignment with labels and inertia), the knee pick on the host,
the snap of the chosen centroids, the per-dimension mode of the trajectory and the replacement of samples
that were visited before.  The headline value is config-iterations per second:
N x (number of k) x (Lloyd rounds) per step divided by the step time.

Prints ONE JSON line.  The top-level fields describe the headline workload (default: `large`, the 8M x 32
configuration, the largest one a single GPU is asked to run), timed for exactly --steps steps after --warmup;
`workloads` holds the same block for every workload of the run (default: the 1M x 16 `whole_layer` and the 64 batched
spaces of 262,144 x 16 as well, with their own step counts stated inside).  Each block carries
  roofline      the dominant kernel (the fused assign + update Lloyd step), timed with HIP events recorded by the
                library on the launch stream during the timed steps.  Its contraction runs on the fp16 matrix
                pipeline, so `frac` is the method's distance arithmetic (2 d k flop per point and (k, round)) over
                the launch time over the dense fp16 MFMA peak; beside it the fraction of HBM peak the same launch
                would need if every k read the trajectory on its own (`hbm_equivalent_ratio`, can exceed 1: one read
                serves up to eight k), the matrix work actually issued, and - from rocprofv3 counters of this
                library version, else null - the HBM bytes really moved and the vector-issue utilisation
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload, with the scaling to the sweep's mix of k
  lloyd_step_per_k / early_exit / graph_replay   extra timings outside the timed steps (graph_replay: a short sweep
                recorded into a HIP graph once and replayed, against the same sweep launched kernel by kernel)
and the line ends with `hbm_copy_measured`: what a plain 1 GiB device-to-device copy moves per second on the same chip
(bytes read + written), the attainable figure next to the 8 TB/s that the HBM fractions are quoted against.
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
VALU_ISSUE_PEAK = 256 * 4 * 2.4e9 / 4.0   # wave64 vector instructions per second: 256 CUs x 4 SIMDs, one every 4 clocks

# rocprofv3 counters of one lloyd_step_kernel launch (mean over the rounds of a sweep), from the summaries under
# profiles/ (lloyd_step_<workload>_hbm_counters.md: FETCH_SIZE / WRITE_SIZE in KiB per dispatch with the factors a
# plain 1 GiB copy gives for each counter; lloyd_step_<workload>_sq_counters.md: SQ_INSTS_VALU).  Valid only for the
# library version they were taken with; any other version reports null.
COUNTERS = {
    # mean over the 30 rounds of a sweep (first round included, like the launches the events time)
    "whole_layer": {"version": 133, "fetch_kib": 190758.0, "write_kib": 44509.0, "fetch_scale": 2.0, "write_scale": 1.0,
                    "valu_insts": 1.482e8},
    "large": {"version": 133, "fetch_kib": 7479002.0, "write_kib": 912506.0, "fetch_scale": 2.0, "write_scale": 1.0,
              "valu_insts": 4.776e9},
}
DEFAULT_STEPS = {"tiny": (50, 5), "mid": (20, 5), "whole_layer": (10, 3), "large": (5, 2), "batched": (5, 2)}


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def run_workload(name, steps, warmup, args):
    """Times `steps` steps of workload `name` after `warmup`; returns its block of the JSON line."""
    import numpy as np
    import torch

    from paper_1905_12799_amd import binding as rls
    from paper_1905_12799_amd import synth

    w = synth.WORKLOADS[name]
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

    ev = {n: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for n in ("score", "sweep", "snap", "modes_visited")}
    stage_ms = {n: 0.0 for n in ev}

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
            for n in ev:
                stage_ms[n] += ev[n][0].elapsed_time(ev[n][1])
        return chosen

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    rls.profile_enable(True)
    rls.profile_read()
    t0 = time.perf_counter()
    for _ in range(steps):
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
        del src, dst

    ms_per_step = (t1 - t0) * 1e3 / steps
    point_iters = float(w.N) * B * n_k * w.iters
    value = point_iters / (ms_per_step * 1e-3)
    sweep_ms = stage_ms["sweep"] / steps
    score_ms = stage_ms["score"] / steps

    # ---- dominant kernel: the Lloyd step (assign + update for every k in one launch) -------------------------
    kernel_s = kernel_ms_total / max(n_launch, 1) * 1e-3
    sum_k = sum(range(w.k_min, w.k_max + 1))
    alg_bytes = 4.0 * w.d * w.N * B * n_k                 # 4 d bytes per point and (k, round): every k reads the row
    alg_flops = 2.0 * w.d * sum_k * w.N * B               # 2 d k flop per point and (k, round)
    # matrix work as issued: per distance three products of fp16 pieces over the padded features plus one bias step of 16
    d_pad = 8 if w.d <= 8 else (16 if w.d <= 16 else 32)
    issued_flops = 2.0 * (3.0 * max(d_pad, 16) + 16.0) * sum_k * w.N * B
    tflops = alg_flops / kernel_s / 1e12
    roofline = {
        # The launch is bound by vector-instruction issue beside the matrix pipeline (the fold of the distance tiles
        # into the two smallest keys per point), not by HBM: one read of a row serves up to eight k.  The fraction
        # reported is that of the contraction's own peak, the dense fp16 MFMA rate.
        "bound": "mfma", "dtype": "f16", "achieved": tflops, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": tflops / MFMA_F16_PEAK_TFLOPS, "traffic": None,
        "kernel": "lloyd_step_kernel", "launches_timed": n_launch, "avg_launch_ms": kernel_s * 1e3,
        "algorithmic_flops_per_launch": alg_flops, "algorithmic_bytes_per_launch": alg_bytes,
        "mfma_issued_frac": issued_flops / kernel_s / 1e12 / MFMA_F16_PEAK_TFLOPS,
        "fp32_mfma_equivalent_ratio": tflops / MFMA_F32_PEAK_TFLOPS,   # against the fp32 matrix peak an fp32 contraction would have had
        "hbm_equivalent_GBps": alg_bytes / kernel_s / 1e9,
        "hbm_equivalent_ratio": alg_bytes / kernel_s / 1e9 / HBM_PEAK_GBS,   # can pass 1: one read of a row serves up to eight k
        "hbm_traffic_frac": None, "valu_issue_frac": None,
        "limiting_resource": "vector instruction issue (an MFMA of this shape also holds the issue port for about 12 clocks), at "
                             "the clock the chip holds under this load (valu_issue_frac counts the vector instructions alone, at "
                             "the nominal 2.4 GHz; profiles/lloyd_step_*_sq_counters.md)",
    }
    hc = COUNTERS.get(w.name)
    if hc is not None and hc["version"] == rls.version() and want_labels:
        hbm_bytes = (hc["fetch_kib"] * hc["fetch_scale"] + hc["write_kib"] * hc["write_scale"]) * 1024.0
        roofline["traffic"] = hbm_bytes                  # HBM bytes really moved per launch (rocprofv3 FETCH_SIZE, WRITE_SIZE)
        roofline["hbm_traffic_frac"] = hbm_bytes / kernel_s / 1e9 / HBM_PEAK_GBS
        roofline["valu_issue_frac"] = hc["valu_insts"] / kernel_s / VALU_ISSUE_PEAK

    visits = float(w.N) * B * w.n_trees * w.depth
    out = {
        "value": value, "ms_per_step": ms_per_step, "steps": steps, "warmup": warmup,
        "config": {"workload": f"{w.name}: N={w.N} d={w.d} batch={B} k={w.k_min}..{w.k_max} iters={w.iters} "
                               f"forest={w.n_trees}x{w.depth}", "labels_written": want_labels,
                   "knee_const": knee_const, "chosen_k": chosen[:4],
                   "score_stream": "main" if side_stream is None else "second stream beside the sweep"},
        "configs_scored_per_s": float(w.N) * B / (score_ms * 1e-3),
        "sweep_config_iter_per_s": point_iters / (sweep_ms * 1e-3),
        "stage_ms": {"gbt_score": score_ms, "kmeans_sweep": sweep_ms, "snap": stage_ms["snap"] / steps,
                     "modes_visited": stage_ms["modes_visited"] / steps},
        "roofline": roofline,
        # tree scoring: bound by LDS gathers and vector issue (T*D node visits per 4d+4 bytes), shown against HBM for scale
        "gbt_score": {"ms": score_ms, "node_visits_per_s": visits / (score_ms * 1e-3),
                      "algorithmic_GBps": (4.0 * w.d + 4.0) * w.N * B / (score_ms * 1e-3) / 1e9,
                      "hbm_frac": (4.0 * w.d + 4.0) * w.N * B / (score_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      # the walk is bound by LDS: 12 bytes per lane and visit (node 8, feature value 4) against
                      # 128 B/clk on each of 256 CUs at 2.4 GHz
                      "lds_GBps": 12.0 * visits / (score_ms * 1e-3) / 1e9,
                      "lds_frac": 12.0 * visits / (score_ms * 1e-3) / (256 * 128 * 2.4e9)},
    }

    if not batched and not args.no_early_exit:
        # Algorithm 1 with its early exit at the knee (k in waves of 16: the groups of a wave share the reads of the points), outside the timed steps: same chosen k,
        # only the waves up to the knee are computed
        k_e, n_done, _ = rls.kmeans_sweep_until_knee(X, w.k_min, w.k_max, 16, w.iters, knee_const, seed=seeds[0],
                                                     want_labels=want_labels)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(3):
            k_e, n_done, _ = rls.kmeans_sweep_until_knee(X, w.k_min, w.k_max, 16, w.iters, knee_const, seed=seeds[0],
                                                         want_labels=want_labels)
        torch.cuda.synchronize()
        out["early_exit"] = {"ms": (time.perf_counter() - t2) * 1e3 / 3, "chosen_k": k_e, "k_computed": n_done, "k_wave": 16}

    if not batched and not args.no_graph and not (args.no_per_k and args.no_early_exit) and sweep_ms < 25.0:
        # A sweep enqueues kernels only, so a caller can record it into a HIP graph once and replay it on new rows of the
        # same shape.  Outside the timed steps: the recorded sweep replayed, against the same sweep launched kernel by
        # kernel (short sweeps are bound by their launches: about 2 (k_max - 1) + 2 rounds + 8 of them).
        side = torch.cuda.Stream()
        side.wait_stream(main_stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            rls.kmeans_sweep(X, w.k_min, w.k_max, w.iters, seed=seeds[0], want_labels=want_labels, workspace=ws, check_status=False)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                g_res = rls.kmeans_sweep(X, w.k_min, w.k_max, w.iters, seed=seeds[0], want_labels=want_labels, workspace=ws,
                                         check_status=False)
        main_stream.wait_stream(side)
        eager = rls.kmeans_sweep(X, w.k_min, w.k_max, w.iters, seed=seeds[0], want_labels=want_labels, workspace=ws, check_status=False)
        torch.cuda.synchronize()
        want_inertia = eager.inertia.clone()
        reps = 20
        graph.replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(reps):
            rls.kmeans_sweep(X, w.k_min, w.k_max, w.iters, seed=seeds[0], want_labels=want_labels, workspace=ws, check_status=False)
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        out["graph_replay"] = {"sweep_ms_replayed": (t3 - t2) * 1e3 / reps, "sweep_ms_launched": (t4 - t3) * 1e3 / reps,
                               "same_result": bool(torch.equal(g_res.inertia, want_inertia))}
        del graph, g_res, eager

    if not batched and not args.no_per_k:
        # The Lloyd step for one k at a time (outside the timed steps): where the launch time leaves the floor set by
        # reading the trajectory and starts to follow the distance work.  Same kernel, a plan with a single run; here
        # every launch reads the trajectory once for its one k, so the HBM fraction is a fraction.
        per_k = []
        for k in [k for k in (1, 2, 4, 8, 16, 32, 64, 128) if w.k_min <= k <= w.k_max]:
            rls.kmeans_sweep(X, k, k, w.iters, seed=seeds[0], want_labels=False, workspace=ws)
            torch.cuda.synchronize()
            rls.profile_enable(True)
            rls.profile_read()
            rls.kmeans_sweep(X, k, k, w.iters, seed=seeds[0], want_labels=False, workspace=ws)
            n_l, ms_l = rls.profile_read()
            rls.profile_enable(False)
            t_l = ms_l / max(n_l, 1) * 1e-3
            flops_k = 2.0 * (3.0 * max(d_pad, 16) + 16.0) * max(k, 32) * w.N       # issued: tiles of 32 centroids
            per_k.append({"k": k, "launch_ms": t_l * 1e3, "config_iter_per_s": w.N / t_l,
                          "hbm_frac": 4.0 * w.d * w.N / t_l / 1e9 / HBM_PEAK_GBS,
                          "mfma_f16_frac": 2.0 * w.d * k * w.N / t_l / 1e12 / MFMA_F16_PEAK_TFLOPS,
                          "mfma_issued_frac": flops_k / t_l / 1e12 / MFMA_F16_PEAK_TFLOPS})
        out["lloyd_step_per_k"] = per_k

    del X, ws, scores, visited, forests
    torch.cuda.empty_cache()

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, probs[0], value)
    return out


def cpu_baseline(w, p0, gpu_value):
    """The oracle as it stands on the host cores, on a bounded sample of the workload: full N of one space, a few k,
    a few Lloyd rounds (the cost of a round does not depend on which round it is: no early stop).  A round costs
    a + b k per point (the exact update, one thread; the assignment, all threads), so the sample's rate is also
    scaled to the sweep's own mix of k."""
    import numpy as np

    import oracle

    ks = [k for k in (8, 32, 64, 128) if w.k_min <= k <= w.k_max] or [w.k_max]
    if w.N * w.d > (1 << 27):
        ks = [k for k in ks if k in (8, 64)] or ks[:1]          # 8M x 32: two k, a few rounds each
    rounds = 4 if w.N * w.d > (1 << 27) else (16 if w.N >= (1 << 20) else 20)
    rounds = min(rounds, max(w.iters, 1))
    rng = np.random.default_rng(w.seed + 77)
    init = rng.choice(w.N, size=max(ks), replace=False).astype(np.int64)      # seeded rows as initial centres
    times = []
    for k in ks:
        t = time.perf_counter()
        oracle.lloyd(p0.X, k, rounds, init)
        times.append(time.perf_counter() - t)
    dt = sum(times)
    # time of one run ~ (rounds + 1) assignments + rounds updates; per round and point: a + b k (least squares over the sample)
    per_round = np.array(times) / (rounds + 0.5)
    if len(ks) >= 2:
        b_, a_ = np.polyfit(np.array(ks, dtype=np.float64), per_round, 1)
    else:
        b_, a_ = per_round[0] / ks[0], 0.0
    a_, b_ = max(a_, 0.0), max(b_, 0.0)
    n_k = w.k_max - w.k_min + 1
    sweep_est = w.batch * sum((a_ + b_ * k) * (w.iters + 0.5) for k in range(w.k_min, w.k_max + 1))
    est_value = float(w.N) * w.batch * n_k * w.iters / sweep_est if sweep_est > 0 else None
    n_s = min(w.N, 65536)
    t = time.perf_counter()
    oracle.gbt_score(p0.forest, p0.X[:n_s])
    dt_s = time.perf_counter() - t
    return {
        "value": float(w.N) * len(ks) * rounds / dt, "unit": "config*iter/s", "cores": oracle.threads(),
        "cpu_model": cpu_model(), "kind": "oracle",
        "sample": f"Lloyd on the full N={w.N} of one space for k in {ks}, {rounds} round(s) each plus the final "
                  f"assignment ({dt:.1f} s), from seeded random rows as initial centres; tree scoring of the first "
                  f"{n_s} configurations on 1 thread ({dt_s:.1f} s)",
        "scaled_to_sweep": {"config_iter_per_s": est_value, "sweep_seconds_estimate": sweep_est,
                            "model": "seconds per Lloyd round of one k = a + b*k, fitted to the sample; sweep = "
                                     "(rounds + 1/2) * sum over k of (a + b*k) * spaces",
                            "a": a_, "b": b_, "gpu_over_cpu": (gpu_value / est_value) if est_value else None},
        "configs_scored_per_s": n_s / dt_s,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps of the headline workload (default 5 for large)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="large", choices=["tiny", "mid", "whole_layer", "large", "batched"],
                    help="headline workload: its figures are the top-level fields of the line")
    ap.add_argument("--also", default=None,
                    help="comma-separated further workloads for the `workloads` block (default: whole_layer and batched "
                         "next to large, large next to whole_layer; 'none' for the headline alone)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="leave out the graph-replay timing of short sweeps")
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

    import torch

    from paper_1905_12799_amd import binding as rls

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    rls.lib()   # fails loudly when the HIP library is not built

    head = args.workload
    if args.also is None:
        also = {"large": ["whole_layer", "batched"], "whole_layer": ["large"]}.get(head, [])
    else:
        also = [n for n in args.also.split(",") if n and n != "none" and n != head]
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[head][0]
    warmup = args.warmup if args.warmup is not None else DEFAULT_STEPS[head][1]

    blocks = {}
    for name in also:      # the other workloads first, with their own (default) step counts
        s, wu = DEFAULT_STEPS[name]
        blocks[name] = run_workload(name, s, wu, args)
    blocks[head] = run_workload(head, steps, warmup, args)
    h = blocks[head]

    out = {
        "metric": "config_iter_per_s", "value": h["value"], "unit": "config*iter/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": h["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": h["config"], "roofline": h["roofline"],
    }
    if "cpu_baseline" in h:
        out["cpu_baseline"] = h["cpu_baseline"]
    for key in ("configs_scored_per_s", "sweep_config_iter_per_s", "stage_ms", "gbt_score", "early_exit", "graph_replay", "lloyd_step_per_k"):
        if key in h:
            out[key] = h[key]
    out["library_version"] = rls.version()
    out["workloads"] = {n: {k: v for k, v in b.items() if n != head or k in ("value", "ms_per_step", "steps", "warmup", "config", "roofline", "cpu_baseline")}
                        for n, b in blocks.items()}
    # what a plain device-to-device copy reaches on this chip, next to the 8 TB/s the fractions are quoted against
    # (an extra like the two above: left out when both are, so that a profiled run holds the path's own kernels only)
    if args.no_per_k and args.no_early_exit:
        print(json.dumps(out))
        return 0
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_s = e0.elapsed_time(e1) * 1e-3 / 5
    out["hbm_copy_measured"] = {"GBps": 2.0 * src.numel() * 4 / copy_s / 1e9, "frac_of_peak": 2.0 * src.numel() * 4 / copy_s / 1e9 / HBM_PEAK_GBS,
                                "what": "bytes read + written by a 1 GiB device-to-device copy over its time (mean of 5)"}
    del src, dst
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
