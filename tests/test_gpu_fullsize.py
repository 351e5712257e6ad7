"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py times.

The oracle cannot sweep every k at these sizes in test time, so each test runs the full sweep on the GPU and
compares (a) complete oracle runs for a few k, bit for bit as in test_gpu_parity.py, and (b) for every k,
sampled points: the label the GPU wrote must be the oracle's argmin against the centroids the GPU returned
(the final assignment is defined against the returned centroids), plus properties that hold at any size.
"""
import sys
import time

import numpy as np
import pytest
import torch

from paper_1905_12799_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rls():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_12799_amd import binding
    binding.lib()
    return binding


_T0 = time.time()


def progress(msg):
    """A line that shows even when pytest captures output: long runs must not look hung."""
    sys.__stderr__.write(f"[fullsize +{time.time() - _T0:6.1f}s] {msg}\n")
    sys.__stderr__.flush()


def check_run_against_oracle(orc, X, chain, k, iters, labels_g, C_g, J_g):
    progress(f"oracle Lloyd N={X.shape[0]} k={k} rounds={iters}")
    labels_o, C_o, J_o, _ = orc.lloyd(X, k, iters, chain)
    bad = np.flatnonzero(labels_g != labels_o)
    for i in bad[:50]:
        d1, d2, _ = orc.two_nearest(X[i], C_o)
        assert (d2 - d1) <= 1e-6 * d2, f"k={k} point {i}: {labels_g[i]} vs {labels_o[i]}"
    scale = np.abs(X).max(axis=0).astype(np.float64)
    scale[scale == 0] = 1.0
    err = np.abs(C_g.astype(np.float64) - C_o.astype(np.float64))
    assert np.all(err <= 1e-5 * np.maximum(np.abs(C_o.astype(np.float64)), scale[None, :])), f"k={k} centroids"
    assert abs(J_g - J_o) <= 1e-5 * max(J_o, 1e-300), f"k={k} inertia"
    if len(bad) == 0:
        np.testing.assert_array_equal(C_g, C_o, err_msg=f"k={k}: centroids not bit-identical")
    return len(bad)


def check_sampled_points(orc, X, res, k_min, k_max, rng, per_k=64, b=None):
    """Every k: sampled labels equal the oracle's argmin against the returned centroids; labels in range."""
    N = X.shape[0]
    idx = np.sort(rng.choice(N, size=per_k, replace=False))
    idx_dev = torch.as_tensor(idx).cuda()
    lab = res.labels if b is None else res.labels[b]
    sampled = lab[:, idx_dev].cpu().numpy()
    for k in range(k_min, k_max + 1):
        C = res.centroids_of(k, b).cpu().numpy()
        for t, i in enumerate(idx):
            d1, d2, arg = orc.two_nearest(X[i], C)
            got = int(sampled[k - res.k_min, t])
            assert 0 <= got < k
            assert got == arg or (d2 - d1) <= 1e-6 * d2, f"k={k} point {i}: label {got}, oracle {arg}"


@pytest.mark.timeout(400)
def test_whole_layer_full(rls, orc):
    w = synth.WORKLOADS["whole_layer"]
    p = synth.make_problem(w)
    X = torch.as_tensor(p.X).cuda()
    progress("whole_layer: GPU sweep")
    res = rls.kmeans_sweep(X, w.k_min, w.k_max, w.iters, seed=w.seed)
    torch.cuda.synchronize()
    progress("whole_layer: oracle chain")
    chain = orc.kmeanspp_chain(p.X, w.k_max, w.seed)
    np.testing.assert_array_equal(rls.kmeanspp_chain(X, w.k_max, w.seed).cpu().numpy(), chain)
    J = res.inertia.cpu().numpy()
    exempt = 0
    for k in (1, 7, 24, 33, 64):
        exempt += check_run_against_oracle(orc, p.X, chain, k, w.iters, res.labels[k - w.k_min].cpu().numpy(),
                                           res.centroids_of(k).cpu().numpy(), J[k - w.k_min])
    assert exempt == 0
    check_sampled_points(orc, p.X, res, w.k_min, w.k_max, np.random.default_rng(1))
    # tree scores of the same trajectory, sampled rows against the oracle
    scores = rls.gbt_score(rls.DeviceForest.from_host(p.forest), X).cpu().numpy()
    rows = np.random.default_rng(2).choice(w.N, size=4096, replace=False)
    np.testing.assert_array_equal(scores[rows], orc.gbt_score(p.forest, p.X[rows])[0])
    # chosen k and snapped configurations follow from the compared quantities
    k_star = rls.pick_knee(J.tolist(), w.k_min, w.k_max, 1.05)
    cfg = rls.snap_to_valid(res.centroids_of(k_star), rls.DeviceDomains(p.dom_offsets, p.dom_values)).cpu().numpy()
    np.testing.assert_array_equal(cfg, orc.snap_to_valid(res.centroids_of(k_star).cpu().numpy(), p.dom_offsets, p.dom_values))
    # per-dimension mode of the whole trajectory and the replacement of visited samples
    progress("whole_layer: modes and visited filter")
    dom = rls.DeviceDomains(p.dom_offsets, p.dom_values)
    mode, hist = rls.knob_modes(X, dom)
    mode_o, hist_o = orc.knob_modes(p.X, p.dom_offsets, p.dom_values)
    np.testing.assert_array_equal(hist.cpu().numpy().astype(np.int64), hist_o)
    np.testing.assert_array_equal(mode.cpu().numpy(), mode_o)
    visited = synth.visited_configs(p, 65536, w.seed + 1000)
    visited[:3] = cfg[:3]
    cfg_dev = torch.as_tensor(cfg).cuda()
    flags = rls.replace_visited(cfg_dev, torch.as_tensor(visited).cuda(), mode).cpu().numpy()
    want_cfg, want_flags = orc.replace_visited(cfg, visited, mode_o)
    assert want_flags[:3].tolist() == [1, 1, 1]
    np.testing.assert_array_equal(flags, want_flags)
    np.testing.assert_array_equal(cfg_dev.cpu().numpy(), want_cfg)


@pytest.mark.timeout(900)
def test_large_full(rls, orc):
    w = synth.WORKLOADS["large"]
    progress("large: generating 8M x 32")
    p = synth.make_problem(w)
    X = torch.as_tensor(p.X).cuda()
    progress("large: chains")
    chain_dev = rls.kmeanspp_chain(X, w.k_max, w.seed)
    head = orc.kmeanspp_chain(p.X, 12, w.seed)            # the oracle's chain is sequential: first 12 draws
    chain = chain_dev.cpu().numpy()
    np.testing.assert_array_equal(chain[:12], head)
    # (a) two Lloyd rounds, every k on the GPU, complete oracle runs for a small and a middle k
    progress("large: GPU sweep, 2 rounds")
    res = rls.kmeans_sweep(X, w.k_min, w.k_max, 2, init_idx=chain_dev)
    torch.cuda.synchronize()
    J = res.inertia.cpu().numpy()
    for k in (2, 37):
        check_run_against_oracle(orc, p.X, chain, k, 2, res.labels[k - w.k_min].cpu().numpy(),
                                 res.centroids_of(k).cpu().numpy(), J[k - w.k_min])
    check_sampled_points(orc, p.X, res, 120, 128, np.random.default_rng(5), per_k=24)
    del res
    # (b) the benchmark configuration: all rounds, every k; properties and sampled points
    progress("large: GPU sweep, all rounds, with trace")
    res = rls.kmeans_sweep(X, w.k_min, w.k_max, w.iters, init_idx=chain_dev, want_trace=True)
    torch.cuda.synchronize()
    progress("large: properties")
    t = res.trace.cpu().numpy()
    assert np.all(t[:, 1:] <= t[:, :-1] * (1 + 1e-6))
    np.testing.assert_array_equal(t[:, -1], res.inertia.cpu().numpy())
    check_sampled_points(orc, p.X, res, w.k_min, w.k_max, np.random.default_rng(3), per_k=24)
    # k = 1: the centroid is the exact column mean
    mean = (p.X.astype(np.float64).sum(axis=0) / w.N).astype(np.float32)
    np.testing.assert_allclose(res.centroids_of(1).cpu().numpy()[0], mean, rtol=1e-6, atol=1e-6)
    # every cluster's centroid of a sampled k is the mean of its members (the update step), to fp32 accuracy:
    # one more assignment of the GPU's own labels reproduces the loss it reported
    k = 128
    lab = res.labels[k - w.k_min].long()
    C = res.centroids_of(k).double()
    loss = ((X.double() - C[lab]) ** 2).sum().item()
    assert abs(loss - float(res.inertia[k - w.k_min])) <= 1e-9 * loss


@pytest.mark.timeout(600)
def test_batched_full(rls, orc):
    w = synth.WORKLOADS["batched"]
    probs = synth.make_batched_problems(w)
    X = torch.as_tensor(np.stack([p.X for p in probs])).cuda()
    seeds = [w.seed + b for b in range(w.batch)]
    progress("batched: GPU sweep of 64 spaces")
    res = rls.kmeans_sweep_batched(X, w.k_min, w.k_max, w.iters, seeds=seeds)
    torch.cuda.synchronize()
    J = res.inertia.cpu().numpy()
    for b in (0, 41, 63):
        p = probs[b]
        chain = orc.kmeanspp_chain(p.X, w.k_max, seeds[b])
        for k in (5, 32):
            check_run_against_oracle(orc, p.X, chain, k, w.iters, res.labels[b, k - w.k_min].cpu().numpy(),
                                     res.centroids_of(k, b).cpu().numpy(), J[b, k - w.k_min])
    for b in (7, 30):
        check_sampled_points(orc, probs[b].X, res, w.k_min, w.k_max, np.random.default_rng(b), per_k=16, b=b)
    forests = [rls.DeviceForest.from_host(p.forest) for p in probs]
    scores = rls.gbt_score_batched(forests, X).cpu().numpy()
    for b in (0, 63):
        rows = np.random.default_rng(b).choice(w.N, size=2048, replace=False)
        np.testing.assert_array_equal(scores[b, rows], orc.gbt_score(probs[b].forest, probs[b].X[rows])[0])
