"""Pins for the oracle's counter-based draws and the k-means++ seeding chain."""
import os

import numpy as np

from paper_1905_12799_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_published_vectors(orc):
    with open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt")) as fh:
        want = [int(line) for line in fh if line.strip() and not line.startswith("#")]
    got = [orc.splitmix64(1234567, j) for j in range(len(want))]
    assert got == want


def test_uniform_is_top_53_bits(orc):
    for j in range(20):
        z = orc.splitmix64(99, j)
        assert orc.uniform(99, j) == (z >> 11) / float(1 << 53)
        assert 0.0 <= orc.uniform(99, j) < 1.0


def test_first_centre_and_prefix_property(orc):
    p = synth.make_problem(synth.WORKLOADS["tiny"], N=400)
    seed = 4242
    full = orc.kmeanspp_chain(p.X, 12, seed)
    assert full[0] == int(orc.uniform(seed, 0) * 400)
    for k in (1, 2, 5, 11):
        np.testing.assert_array_equal(orc.kmeanspp_chain(p.X, k, seed), full[:k])
    assert len(set(full.tolist())) == 12


def test_second_centre_follows_d2_law(orc):
    # N = 6 points on a line; the second centre must be drawn with probability D_i / S given the first
    X = np.array([[0.0], [1.0], [3.0], [3.0], [7.0], [10.0]], dtype=np.float32)
    n_seeds = 60000
    counts = np.zeros((6, 6))
    for s in range(n_seeds):
        a, b = orc.kmeanspp_chain(X, 2, 1000 + s)
        counts[a, b] += 1
    firsts = counts.sum(axis=1)
    # the first centre is uniform
    assert np.all(np.abs(firsts / n_seeds - 1 / 6) < 4 * np.sqrt((1 / 6) * (5 / 6) / n_seeds))
    for a in range(6):
        D = (X[:, 0].astype(np.float64) - float(X[a, 0])) ** 2
        prob = D / D.sum()
        n = firsts[a]
        sd = np.sqrt(np.maximum(prob * (1 - prob), 1e-12) / n)
        assert np.all(np.abs(counts[a] / n - prob) <= 4 * sd + 1e-12), (a, counts[a] / n, prob)
        assert counts[a, a] == 0          # a chosen point has D = 0 and is never drawn again


def test_brute_force_chain_matches_numpy(orc):
    # independent re-statement with NumPy cumulative sums on a small case (sequential cumsum = same order)
    rng = np.random.default_rng(5)
    X = rng.integers(0, 9, size=(40, 3)).astype(np.float32)
    seed = 77
    got = orc.kmeanspp_chain(X, 6, seed)
    Xd = X.astype(np.float64)
    idx = [int(orc.uniform(seed, 0) * 40)]
    D = None
    for j in range(1, 6):
        dist = ((Xd - Xd[idx[-1]]) ** 2).sum(axis=1)     # integer data: exact in any order
        D = dist if D is None else np.minimum(D, dist)
        pre = np.cumsum(D)
        r = orc.uniform(seed, j) * pre[-1]
        idx.append(int(np.argmax(pre > r)))
    assert got.tolist() == idx


def test_all_points_coincide_fallback(orc):
    X = np.ones((5, 2), dtype=np.float32)
    seed = 3
    got = orc.kmeanspp_chain(X, 4, seed)
    first = int(orc.uniform(seed, 0) * 5)
    rest = [i for i in range(5) if i != first][:3]
    assert got.tolist() == [first] + rest


def test_draw_index_against_cumsum_and_boundary_branch(orc):
    """The draw on its own: first prefix above r; r equal to (or above) the total takes the last positive entry."""
    rng = np.random.default_rng(8)
    for _ in range(200):
        n = int(rng.integers(1, 40))
        D = rng.integers(0, 5, size=n).astype(np.float64)          # integers: every prefix is exact
        D[rng.random(n) < 0.3] = 0.0
        total = D.sum()
        if total == 0:
            assert orc.draw_index(D, 0.0) == -1
            continue
        pre = np.cumsum(D)
        for r in (0.0, 0.5, float(rng.uniform(0, total)), total - 0.5):
            assert orc.draw_index(D, r) == int(np.argmax(pre > r))
        last_pos = int(np.flatnonzero(D > 0)[-1])
        assert orc.draw_index(D, total) == last_pos               # r rounded up to the total
        assert orc.draw_index(D, total + 1.0) == last_pos
    # an entry with D = 0 is never drawn: its prefix equals the one before it
    D = np.array([0.0, 2.0, 0.0, 0.0, 3.0, 0.0])
    assert [orc.draw_index(D, r) for r in (0.0, 1.9, 2.0, 4.9, 5.0)] == [1, 1, 4, 4, 4]
