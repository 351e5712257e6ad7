"""Pins for the last loop of Algorithm 1: mode(s_Theta) per dimension and the replacement of visited samples."""
import numpy as np

from paper_1905_12799_amd import synth


def integer_domains(sizes):
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    values = np.concatenate([np.arange(s, dtype=np.float32) for s in sizes])
    return offsets, values


def test_modes_equal_bincount_on_index_columns(orc):
    # knob columns that hold domain indices: the mode is the most frequent integer, lowest on ties
    rng = np.random.default_rng(7)
    sizes = [5, 3, 9, 2]
    offsets, values = integer_domains(sizes)
    X = np.stack([rng.integers(0, s, size=4000) for s in sizes] + [rng.normal(size=4000)], axis=1).astype(np.float32)
    mode, hist = orc.knob_modes(X, offsets, values)
    for j, s in enumerate(sizes):
        counts = np.bincount(X[:, j].astype(np.int64), minlength=s)
        np.testing.assert_array_equal(hist[offsets[j]:offsets[j + 1]], counts)
        assert mode[j] == int(np.argmax(counts))          # argmax returns the first maximum
    assert hist.sum() == 4000 * len(sizes)


def test_modes_tie_goes_to_lower_index(orc):
    offsets, values = integer_domains([4])
    X = np.array([[2], [1], [2], [1], [3]], dtype=np.float32)   # 1 and 2 both twice
    mode, hist = orc.knob_modes(X, offsets, values)
    assert mode.tolist() == [1]
    assert hist.tolist() == [0, 2, 2, 1]


def test_modes_snap_values_between_domain_entries(orc):
    # non-integer domain, coordinates between entries: nearest entry counts, half-way goes to the lower one
    offsets = np.array([0, 3], dtype=np.int32)
    values = np.array([0.0, 1.0, 4.0], dtype=np.float32)
    X = np.array([[0.4], [0.5], [0.6], [2.5], [2.6], [100.0], [-7.0]], dtype=np.float32)
    mode, hist = orc.knob_modes(X, offsets, values)
    #            0.4->0, 0.5->0 (tie), 0.6->1, 2.5->1 (tie), 2.6->2, 100->2, -7->0
    assert hist.tolist() == [3, 2, 2]
    assert mode.tolist() == [0]


def test_modes_match_snap_of_every_point(orc):
    # the value a point takes in a knob is what snapping the point itself gives: brute force through the snap oracle
    w = synth.WORKLOADS["tiny"]
    p = synth.make_problem(w)
    mode, hist = orc.knob_modes(p.X, p.dom_offsets, p.dom_values)
    cfg = orc.snap_to_valid(p.X, p.dom_offsets, p.dom_values)            # rows of X as "centroids"
    n_knobs = len(p.dom_offsets) - 1
    for j in range(n_knobs):
        counts = np.bincount(cfg[:, j], minlength=p.dom_offsets[j + 1] - p.dom_offsets[j])
        np.testing.assert_array_equal(hist[p.dom_offsets[j]:p.dom_offsets[j + 1]], counts)
        assert mode[j] == int(np.argmax(counts))


def test_modes_permutation_invariant(orc):
    rng = np.random.default_rng(3)
    offsets, values = integer_domains([6, 4])
    X = np.stack([rng.integers(0, 6, 999), rng.integers(0, 4, 999)], axis=1).astype(np.float32)
    m0, h0 = orc.knob_modes(X, offsets, values)
    m1, h1 = orc.knob_modes(X[rng.permutation(999)], offsets, values)
    np.testing.assert_array_equal(m0, m1)
    np.testing.assert_array_equal(h0, h1)


def test_replace_visited_matches_set_membership(orc):
    rng = np.random.default_rng(11)
    n_knobs = 5
    visited = rng.integers(0, 3, size=(200, n_knobs)).astype(np.int32)
    cfg = rng.integers(0, 3, size=(60, n_knobs)).astype(np.int32)
    mode = np.array([9, 8, 7, 6, 5], dtype=np.int32)
    seen = {tuple(r) for r in visited.tolist()}
    out, replaced = orc.replace_visited(cfg, visited, mode)
    want_flags = np.array([tuple(r) in seen for r in cfg.tolist()], dtype=np.int32)
    assert 0 < want_flags.sum() < 60                          # the case exercises both branches
    np.testing.assert_array_equal(replaced, want_flags)
    for i in range(60):
        np.testing.assert_array_equal(out[i], mode if want_flags[i] else cfg[i])


def test_replace_visited_edge_cases(orc):
    mode = np.array([1, 1], dtype=np.int32)
    cfg = np.array([[0, 0], [2, 3]], dtype=np.int32)
    out, replaced = orc.replace_visited(cfg, np.zeros((0, 2), dtype=np.int32), mode)     # nothing visited yet
    np.testing.assert_array_equal(out, cfg)
    assert replaced.tolist() == [0, 0]
    # a row must match in every knob, not in some
    out, replaced = orc.replace_visited(cfg, np.array([[0, 3], [2, 0]], dtype=np.int32), mode)
    assert replaced.tolist() == [0, 0]
    # the mode itself being visited still replaces (Algorithm 1 does not re-check the replacement)
    out, replaced = orc.replace_visited(cfg, np.array([[0, 0], [1, 1]], dtype=np.int32), mode)
    assert replaced.tolist() == [1, 0]
    np.testing.assert_array_equal(out, [[1, 1], [2, 3]])
