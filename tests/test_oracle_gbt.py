"""Pins for the oracle's tree-ensemble scoring (cost-model query, Sec. 4.1)."""
import numpy as np

from paper_1905_12799_amd import synth


def numpy_walk(forest, X):
    """Independent re-walk: level by level over all rows at once, fp64 sum."""
    N = X.shape[0]
    n_int = (1 << forest.depth) - 1
    total = np.full(N, float(forest.base), dtype=np.float64)
    per_tree = []
    for t in range(forest.n_trees):
        node = np.zeros(N, dtype=np.int64)
        for _ in range(forest.depth):
            f = forest.feat[t, node]
            go_right = ~(X[np.arange(N), f] < forest.thr[t, node])
            node = 2 * node + 1 + go_right.astype(np.int64)
        v = forest.leaf[t, node - n_int]
        per_tree.append(v)
        total += v.astype(np.float64)
    return total, np.stack(per_tree, axis=1)


def test_brute_force_walk(orc):
    p = synth.make_problem(synth.WORKLOADS["tiny"], N=100)
    s32, s64 = orc.gbt_score(p.forest, p.X)
    ref, per_tree = numpy_walk(p.forest, p.X)
    np.testing.assert_array_equal(s64, ref)
    # fp32 sum in tree order, reproduced with explicit fp32 adds
    acc = np.full(100, np.float32(p.forest.base))
    for t in range(p.forest.n_trees):
        acc = (acc + per_tree[:, t]).astype(np.float32)
    np.testing.assert_array_equal(s32, acc)


def test_fp32_sum_within_sequential_bound(orc):
    p = synth.make_problem(synth.WORKLOADS["tiny"], N=500)
    s32, s64 = orc.gbt_score(p.forest, p.X)
    _, per_tree = numpy_walk(p.forest, p.X)
    bound = p.forest.n_trees * 2.0 ** -24 * np.abs(per_tree).sum(axis=1)
    assert np.all(np.abs(s32.astype(np.float64) - s64) <= bound)


def _stump(feature, thr, l0, l1, d, base=0.0):
    return synth.Forest(1, 1, d, base, np.array([[feature]], np.int32), np.array([[thr]], np.float32),
                        np.array([[l0, l1]], np.float32))


def test_stump_closed_form_and_equality_goes_right(orc):
    X = np.array([[0.0, 1.0], [0.0, 2.0], [0.0, 3.0], [5.0, np.float32(2.0)]], dtype=np.float32)
    f = _stump(1, 2.0, -1.5, 4.25, 2, base=0.5)
    s32, _ = orc.gbt_score(f, X)
    # x < thr -> left leaf; x == thr and x > thr -> right leaf
    np.testing.assert_array_equal(s32, np.array([0.5 - 1.5, 0.5 + 4.25, 0.5 + 4.25, 0.5 + 4.25], np.float32))


def test_infinite_thresholds(orc):
    rng = np.random.default_rng(3)
    X = rng.standard_normal((50, 5)).astype(np.float32)
    f = synth.random_forest(X, 7, 4, 0, rng)
    f.thr[:] = np.inf      # always left -> leaf 0 of every tree
    s32, s64 = orc.gbt_score(f, X)
    np.testing.assert_allclose(s64, f.leaf[:, 0].astype(np.float64).sum(), rtol=0, atol=1e-12)
    f.thr[:] = -np.inf     # always right -> last leaf
    s32, s64 = orc.gbt_score(f, X)
    np.testing.assert_allclose(s64, f.leaf[:, -1].astype(np.float64).sum(), rtol=0, atol=1e-12)


def test_row_permutation_permutes_scores(orc):
    p = synth.make_problem(synth.WORKLOADS["tiny"], N=300)
    perm = np.random.default_rng(0).permutation(300)
    a, _ = orc.gbt_score(p.forest, p.X)
    b, _ = orc.gbt_score(p.forest, p.X[perm])
    np.testing.assert_array_equal(a[perm], b)


def test_single_path_tree(orc):
    # depth 3, one feature, thresholds chosen so that x = 2.5 walks right, left, right -> leaf index 0b101 = 5
    feat = np.zeros((1, 7), np.int32)
    thr = np.array([[2.0, 0.0, 3.0, 0.0, 0.0, 2.25, 0.0]], np.float32)
    leaf = np.arange(8, dtype=np.float32).reshape(1, 8) * 10
    f = synth.Forest(1, 3, 1, 0.0, feat, thr, leaf)
    s32, _ = orc.gbt_score(f, np.array([[2.5]], np.float32))
    assert s32[0] == 50.0
