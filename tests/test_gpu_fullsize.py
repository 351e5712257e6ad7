"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py times.

The oracle cannot sweep every k at these sizes in test time, so each test runs the full sweep on the GPU and
compares (a) the oracle's complete runs stored under tests/golden/ by make_fullsize_golden.py (which calls the oracle
only): labels and centroids bit for bit through SHA-256 hashes, the loss within 1e-5, the seeding chain, and the k
that the knee test of Algorithm 1 picks on both loss curves - every k of the 1M workload, the k up to past the knee
plus a middle and the largest k at 8M, every k of eight of the 64 batched spaces; (b) complete runs by the oracle as
built on this machine for a few k, bit for bit as in test_gpu_parity.py (more of them when the stored runs were made
for an input this machine's generator does not reproduce); and (c) for every k, sampled points: the label the GPU
wrote must be the oracle's argmin against the centroids the GPU returned (the final assignment is defined against
the returned centroids), plus properties that hold at any size.
"""
import hashlib
import json
import os
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


def check_run_against_oracle(orc, X, chain, k, iters, labels_g, C_g, J_g, J_out=None):
    progress(f"oracle Lloyd N={X.shape[0]} k={k} rounds={iters}")
    labels_o, C_o, J_o, _ = orc.lloyd(X, k, iters, chain)
    if J_out is not None:
        J_out[k] = J_o
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


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
KNEE_CONSTANTS = (1.01, 1.05, 1.1, 1.5, 2.0)


def sha(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def stored_oracle_runs(name, b, X):
    """The oracle's full-size results written by tests/golden/make_fullsize_golden.py for space b of a workload, or
    None when the file is missing or was made for another input (the generator's output differs on this machine)."""
    path = os.path.join(GOLDEN, f"fullsize_{name}.json")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        g = json.load(fh)
    space = g["spaces"].get(str(b))
    if space is None or space["x_sha256"] != sha(X):
        return None
    return space


def check_against_stored_oracle(rls, orc, space, res, k_min, k_max, b=None):
    """Every stored run: labels and centroids bit for bit (by hash), loss within 1e-5 relative; then the knee of
    Algorithm 1 on both loss curves.  Returns the list of k compared."""
    lab = res.labels if b is None else res.labels[b]
    J_g = (res.inertia if b is None else res.inertia[b]).cpu().numpy()
    ks = sorted(int(k) for k in space["runs"])
    for k in ks:
        run = space["runs"][str(k)]
        J_o = float.fromhex(run["inertia"])
        assert sha(lab[k - k_min].cpu().numpy()) == run["labels_sha256"], f"k={k}: labels differ from the oracle's"
        assert sha(res.centroids_of(k, b).cpu().numpy()) == run["centroids_sha256"], f"k={k}: centroids differ"
        assert abs(J_g[k - k_min] - J_o) <= 1e-5 * max(J_o, 1e-300), f"k={k}: inertia {J_g[k - k_min]} vs {J_o}"
    # chosen k: the oracle's curve is known on the leading range k_min .. k_top; Algorithm 1 stops at the first k
    # whose test fires, so a knee below k_top is the knee of the whole curve
    k_top = k_min
    while k_top + 1 in ks and k_top in ks:
        k_top += 1
    if k_min in ks and k_top > k_min:
        J_o = [float.fromhex(space["runs"][str(k)]["inertia"]) for k in range(k_min, k_top + 1)]
        decided = 0
        for const in KNEE_CONSTANTS:
            k_o = orc.pick_knee(J_o, k_min, k_top, const)
            assert rls.pick_knee(J_g[:k_top - k_min + 1].tolist(), k_min, k_top, const) == k_o
            if k_o < k_top or k_top == k_max:
                assert rls.pick_knee(J_g.tolist(), k_min, k_max, const) == k_o, f"chosen k, constant {const}"
                decided += 1
        assert decided >= 2, "the stored range must reach past the knee for some constants"
    return ks


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
    space = stored_oracle_runs("whole_layer", 0, p.X)
    if space is not None:
        progress("whole_layer: every k against the stored oracle runs")
        np.testing.assert_array_equal(chain, np.array(space["chain"], dtype=np.int64))
        assert check_against_stored_oracle(rls, orc, space, res, w.k_min, w.k_max) == list(range(w.k_min, w.k_max + 1))
        live = (7,)                                # one run by the oracle as it is built here, as a cross-check of the file
    else:
        progress("whole_layer: no stored oracle runs for this input: oracle runs for the k up to the knee and three more")
        live = tuple(range(1, 13)) + (24, 33, 64)
    exempt = 0
    J_o = {}
    for k in live:
        exempt += check_run_against_oracle(orc, p.X, chain, k, w.iters, res.labels[k - w.k_min].cpu().numpy(),
                                           res.centroids_of(k).cpu().numpy(), J[k - w.k_min], J_out=J_o)
    assert exempt == 0
    if space is None:
        decided = 0
        for const in KNEE_CONSTANTS:
            k_o = orc.pick_knee([J_o[k] for k in range(1, 13)], 1, 12, const)
            if k_o < 12:        # the test fired inside the range the oracle ran: that is the knee of the whole curve
                assert rls.pick_knee(J.tolist(), w.k_min, w.k_max, const) == k_o
                decided += 1
        assert decided >= 2
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
    space = stored_oracle_runs("large", 0, p.X)
    if space is not None:
        progress("large: all rounds against the stored oracle runs (k up to past the knee, a middle and the largest k)")
        np.testing.assert_array_equal(chain, np.array(space["chain"], dtype=np.int64))
        ks = check_against_stored_oracle(rls, orc, space, res, w.k_min, w.k_max)
        assert len(ks) >= 12
    else:
        progress("large: no stored oracle runs for this input: one complete oracle run of all rounds")
        check_run_against_oracle(orc, p.X, chain, 3, w.iters, res.labels[3 - w.k_min].cpu().numpy(),
                                 res.centroids_of(3).cpu().numpy(), float(res.inertia[3 - w.k_min]))
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
    n_stored = 0
    for b in range(w.batch):
        space = stored_oracle_runs("batched", b, probs[b].X)
        if space is not None:
            progress(f"batched: space {b}, every k against the stored oracle runs")
            check_against_stored_oracle(rls, orc, space, res, w.k_min, w.k_max, b=b)
            n_stored += 1
    for b in ((41,) if n_stored else (0, 41, 63)):
        p = probs[b]
        chain = orc.kmeanspp_chain(p.X, w.k_max, seeds[b])
        J_o = {}
        for k in ((5, 32) if n_stored else tuple(range(1, 13)) + (32,)):
            check_run_against_oracle(orc, p.X, chain, k, w.iters, res.labels[b, k - w.k_min].cpu().numpy(),
                                     res.centroids_of(k, b).cpu().numpy(), J[b, k - w.k_min], J_out=J_o)
        if not n_stored:
            decided = 0
            for const in KNEE_CONSTANTS:
                k_o = orc.pick_knee([J_o[k] for k in range(1, 13)], 1, 12, const)
                if k_o < 12:
                    assert rls.pick_knee(J[b].tolist(), w.k_min, w.k_max, const) == k_o
                    decided += 1
            assert decided >= 2
    for b in (7, 30):
        check_sampled_points(orc, probs[b].X, res, w.k_min, w.k_max, np.random.default_rng(b), per_k=16, b=b)
    forests = [rls.DeviceForest.from_host(p.forest) for p in probs]
    scores = rls.gbt_score_batched(forests, X).cpu().numpy()
    for b in (0, 63):
        rows = np.random.default_rng(b).choice(w.N, size=2048, replace=False)
        np.testing.assert_array_equal(scores[b, rows], orc.gbt_score(probs[b].forest, probs[b].X[rows])[0])


@pytest.mark.timeout(900)
def test_maximum_number_of_points(rls, orc):
    """N = RLS_MAX_N = 2^26 rows of 32 features (8 GiB of rows: element offsets reach 2^31, byte offsets 2^33), every
    kernel that walks the rows: complete oracle runs of Lloyd (one k that takes the prepared-copy path from the second
    round on, two small k side by side), the head of the seeding chain, sampled tree scores including the last
    row, histograms and modes over all rows.  The rows are 16 copies of a 4M-row draw of the 8M workload's
    generator, copy c shifted by c / 4 in the last column so that no two copies coincide."""
    w = synth.WORKLOADS["large"]
    M, copies = 1 << 22, 16
    N = M * copies
    assert N == 1 << 26
    progress("max N: generating 2^26 x 32")
    p = synth.make_problem(w, N=M)
    X = np.empty((N, w.d), dtype=np.float32)
    for c in range(copies):
        X[c * M:(c + 1) * M] = p.X
        X[c * M:(c + 1) * M, w.d - 1] += np.float32(0.25 * c)
    Xd = torch.from_numpy(X).cuda()
    # tree scores
    progress("max N: tree scores")
    scores = rls.gbt_score(rls.DeviceForest.from_host(p.forest), Xd)
    rows = np.unique(np.concatenate([[0, M - 1, M, N - 2, N - 1], np.random.default_rng(26).choice(N, size=4096, replace=False)]))
    got = scores[torch.as_tensor(rows).cuda()].cpu().numpy()
    np.testing.assert_array_equal(got, orc.gbt_score(p.forest, X[rows])[0])
    del scores
    # seeding chain: the first draws (the oracle's chain is sequential)
    progress("max N: seeding chain")
    chain = orc.kmeanspp_chain(X, 3, w.seed)
    np.testing.assert_array_equal(rls.kmeanspp_chain(Xd, 3, w.seed).cpu().numpy(), chain)
    # one k above a tile of centroids: two rounds, the second on the prepared copy; initial centres spread over all
    # rows, the last row among them
    k = 33
    init = np.linspace(0, N - 1, k).astype(np.int64)
    assert init[-1] == N - 1
    progress(f"max N: GPU sweep k={k}, 2 rounds")
    res = rls.kmeans_sweep(Xd, k, k, 2, init_idx=torch.as_tensor(init).cuda())
    torch.cuda.synchronize()
    assert check_run_against_oracle(orc, X, init, k, 2, res.labels[0].cpu().numpy(), res.centroids_of(k).cpu().numpy(),
                                    float(res.inertia[0])) == 0
    del res
    # two small k side by side from the seeded chain, one round
    progress("max N: GPU sweep k=2..3, 1 round")
    res = rls.kmeans_sweep(Xd, 2, 3, 1, seed=w.seed)
    torch.cuda.synchronize()
    for kk in (2, 3):
        assert check_run_against_oracle(orc, X, chain, kk, 1, res.labels[kk - 2].cpu().numpy(), res.centroids_of(kk).cpu().numpy(),
                                        float(res.inertia[kk - 2])) == 0
    del res
    progress("max N: modes")
    mode, hist = rls.knob_modes(Xd, rls.DeviceDomains(p.dom_offsets, p.dom_values))
    mode_o, hist_o = orc.knob_modes(X, p.dom_offsets, p.dom_values)
    np.testing.assert_array_equal(hist.cpu().numpy().astype(np.int64), hist_o)
    np.testing.assert_array_equal(mode.cpu().numpy(), mode_o)
    progress("max N: done")
