"""Pins for the knee rule of Algorithm 1 and for snapping centroids to valid configurations."""
import os

import numpy as np

from paper_1905_12799_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_knee_cases():
    cases = []
    with open(os.path.join(GOLDEN, "knee_cases.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k_min, const, losses, want = [s.strip() for s in line.split(";")]
            cases.append((int(k_min), float(const), [float(v) for v in losses.split()], int(want)))
    return cases


def test_knee_golden_cases(orc):
    cases = read_knee_cases()
    assert len(cases) >= 8
    for k_min, const, losses, want in cases:
        assert orc.pick_knee(np.array(losses), k_min, k_min + len(losses) - 1, const) == want


def test_knee_geometric_closed_form(orc):
    # J_k = J_1 * rho^(k-1): the test fires at the second k iff const * rho > 1, otherwise never
    for rho in (0.3, 0.6, 0.9):
        J = 100.0 * rho ** np.arange(10)
        for const in (1.01, 1.2, 1.5, 2.0, 4.0):
            want = 2 if const * rho > 1.0 else 10
            assert orc.pick_knee(J, 1, 10, const) == want


def test_knee_equals_literal_early_break(orc):
    # the sweep computes every k; the early break of the pseudocode must land on the same k
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(1, 20))
        J = np.sort(rng.uniform(1, 100, size=n))[::-1].copy()
        if rng.uniform() < 0.3 and n > 2:
            J[rng.integers(1, n)] *= 1.5
        const = float(rng.choice([1.01, 1.05, 1.1, 1.5, 2.0]))
        previous, chosen = np.inf, None
        for k in range(8, 8 + n):
            loss = J[k - 8]
            chosen = k
            if const * loss > previous:
                break
            previous = loss
        assert orc.pick_knee(J, 8, 8 + n - 1, const) == chosen


def brute_snap(C, offsets, values):
    k = C.shape[0]
    n_knobs = len(offsets) - 1
    out = np.zeros((k, n_knobs), dtype=np.int32)
    for i in range(k):
        for j in range(n_knobs):
            dom = values[offsets[j]:offsets[j + 1]].astype(np.float64)
            gaps = np.abs(dom - float(C[i, j]))
            out[i, j] = int(np.flatnonzero(gaps == gaps.min())[0])
    return out


def test_snap_brute_force_on_irregular_domains(orc):
    rng = np.random.default_rng(2)
    sizes = [5, 1, 9, 3]
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    values = np.concatenate([np.sort(rng.uniform(-5, 5, size=s)) for s in sizes]).astype(np.float32)
    C = rng.uniform(-7, 7, size=(40, 6)).astype(np.float32)
    np.testing.assert_array_equal(orc.snap_to_valid(C, offsets, values), brute_snap(C, offsets, values))


def test_snap_integer_domains_round_half_down_and_clamp(orc):
    space = synth.conv2d_knob_space(64, 64, 56, 3)
    offsets, values = space.domains_csr()
    rng = np.random.default_rng(6)
    C = rng.uniform(-3, 90, size=(64, 8)).astype(np.float32)
    C[:8, :] = np.arange(8, dtype=np.float32)[:, None] + 0.5      # exact half-way cases
    got = orc.snap_to_valid(C, offsets, values)
    sizes = space.sizes
    want = np.clip(np.ceil(C.astype(np.float64) - 0.5), 0, sizes - 1).astype(np.int32)
    np.testing.assert_array_equal(got, want)
    assert np.all(got >= 0) and np.all(got < sizes)


def test_snap_is_idempotent_on_valid_configs(orc):
    p = synth.make_problem(synth.WORKLOADS["mid"], N=200)
    got = orc.snap_to_valid(p.X, p.dom_offsets, p.dom_values)      # first 8 columns are knob indices
    np.testing.assert_array_equal(got, p.X[:, :8].astype(np.int32))
