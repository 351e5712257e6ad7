"""Seeded synthetic inputs shaped like conv2d tuning spaces.

The adaptive-sampling step of the paper (Sec. 4.2, Algorithm 1) works on a
trajectory of knob configurations of a convolution template whose knobs are
listed in Table 1: tile_f, tile_y, tile_x (4-way splits), tile_rc, tile_ry,
tile_rx (2-way splits), auto_unroll_max_step and unroll_explicit.  The real
trajectories come from a tuner run and are not available, so this module
draws stand-ins with the same shape: integer knob indices in the product
space of the per-knob domains, optional derived loop-extent columns, and a
random forest standing in for the boosted-tree cost model.

This module is data only.  It holds none of the method's arithmetic (no
distances, no tree walks, no clustering) and is imported by the tests, the
benchmark and the smoke check to feed the same arrays to every
implementation.
"""
from __future__ import annotations

import dataclasses
from typing import List, Sequence, Tuple

import numpy as np

BASE_SEED = 12799

KNOB_NAMES = (
    "tile_f", "tile_y", "tile_x",
    "tile_rc", "tile_ry", "tile_rx",
    "auto_unroll_max_step", "unroll_explicit",
)
UNROLL_STEPS = (0, 512, 1500)
UNROLL_EXPLICIT = (0, 1)


def ordered_factorizations(n: int, parts: int) -> List[Tuple[int, ...]]:
    """All tuples of `parts` positive integers whose product is n, in lexicographic order."""
    if parts == 1:
        return [(n,)]
    out = []
    for a in range(1, n + 1):
        if n % a == 0:
            for rest in ordered_factorizations(n // a, parts - 1):
                out.append((a,) + rest)
    return out


@dataclasses.dataclass
class KnobSpace:
    """Per-knob domains of one conv2d template (Table 1). A knob's value is its index in its domain."""
    C: int
    K: int
    H: int
    r: int
    entries: List[list]            # per knob: the list of domain entries (factor tuples or scalars)

    @property
    def sizes(self) -> np.ndarray:
        return np.array([len(e) for e in self.entries], dtype=np.int64)

    @property
    def n_knobs(self) -> int:
        return len(self.entries)

    def domains_csr(self) -> Tuple[np.ndarray, np.ndarray]:
        """Domains as (offsets[n_knobs+1] int32, values[] fp32); the value of entry v of a knob is v itself."""
        sizes = self.sizes
        offsets = np.zeros(len(sizes) + 1, dtype=np.int32)
        offsets[1:] = np.cumsum(sizes)
        values = np.concatenate([np.arange(s, dtype=np.float32) for s in sizes])
        return offsets, values


def conv2d_knob_space(C: int, K: int, H: int, r: int) -> KnobSpace:
    entries = [
        ordered_factorizations(K, 4),      # tile_f: filters
        ordered_factorizations(H, 4),      # tile_y: output height
        ordered_factorizations(H, 4),      # tile_x: output width (square maps)
        ordered_factorizations(C, 2),      # tile_rc: input channels
        ordered_factorizations(r, 2),      # tile_ry
        ordered_factorizations(r, 2),      # tile_rx
        list(UNROLL_STEPS),
        list(UNROLL_EXPLICIT),
    ]
    return KnobSpace(C, K, H, r, entries)


def derived_extent_columns(space: KnobSpace, knobs: np.ndarray) -> np.ndarray:
    """Eight loop-extent columns (log2, fp32) looked up from integer knob indices [N, 8].

    For each of tile_f / tile_y / tile_x: log2 of the outermost (block) factor and of the third (thread)
    factor; then log2 of the inner factor of tile_rc and log2 of (inner tile_ry * inner tile_rx).
    """
    cols = []
    for j in range(3):
        tab = np.array(space.entries[j], dtype=np.float64)
        cols.append(np.log2(tab[:, 0])[knobs[:, j]])
        cols.append(np.log2(tab[:, 2])[knobs[:, j]])
    rc = np.array(space.entries[3], dtype=np.float64)
    cols.append(np.log2(rc[:, 1])[knobs[:, 3]])
    ry = np.array(space.entries[4], dtype=np.float64)
    rx = np.array(space.entries[5], dtype=np.float64)
    cols.append(np.log2(ry[:, 1][knobs[:, 4]] * rx[:, 1][knobs[:, 5]]))
    return np.stack(cols, axis=1).astype(np.float32)


def sample_knobs_mixture(space: KnobSpace, n: int, components: int, rng: np.random.Generator,
                         chunk: int = 1 << 20) -> Tuple[np.ndarray, np.ndarray]:
    """Knob indices [n, n_knobs] from an equal-weight Gaussian mixture in index space, rounded and clamped.

    Returns (knobs int64, component id int32).
    """
    sizes = space.sizes.astype(np.float64)
    means = rng.uniform(0.0, sizes - 1.0, size=(components, len(sizes)))
    sigma = np.maximum(0.5, 0.08 * sizes)
    comp = rng.integers(0, components, size=n).astype(np.int32)
    knobs = np.empty((n, len(sizes)), dtype=np.int64)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        z = rng.standard_normal(size=(e - s, len(sizes)))
        v = np.rint(means[comp[s:e]] + z * sigma)
        knobs[s:e] = np.clip(v, 0, sizes - 1).astype(np.int64)
    return knobs, comp


def sample_knobs_uniform(space: KnobSpace, n: int, rng: np.random.Generator) -> np.ndarray:
    sizes = space.sizes
    return np.stack([rng.integers(0, s, size=n) for s in sizes], axis=1).astype(np.int64)


def lognormal_extra_columns(comp: np.ndarray, components: int, n_cols: int, rng: np.random.Generator,
                            chunk: int = 1 << 20) -> np.ndarray:
    """Extent/stride-like columns: per-component centres ~ logNormal(0, 1), spread 10% of the centre."""
    centres = np.exp(rng.standard_normal(size=(components, n_cols)))
    n = comp.shape[0]
    out = np.empty((n, n_cols), dtype=np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        z = rng.standard_normal(size=(e - s, n_cols))
        out[s:e] = (centres[comp[s:e]] * (1.0 + 0.1 * z)).astype(np.float32)
    return out


@dataclasses.dataclass
class Forest:
    """Complete binary trees in level order: node n has children 2n+1 (left) and 2n+2 (right)."""
    n_trees: int
    depth: int
    n_features: int
    base: float
    feat: np.ndarray      # int32 [n_trees, 2**depth - 1]
    thr: np.ndarray       # fp32  [n_trees, 2**depth - 1]
    leaf: np.ndarray      # fp32  [n_trees, 2**depth]


def random_forest(X: np.ndarray, n_trees: int, depth: int, n_index_cols: int,
                  rng: np.random.Generator) -> Forest:
    """Random splits and N(0,1) leaves. Thresholds on index columns sit on half-integers (no equality hits)."""
    d = X.shape[1]
    n_int = (1 << depth) - 1
    lo = X.min(axis=0).astype(np.float64)
    hi = X.max(axis=0).astype(np.float64)
    feat = rng.integers(0, d, size=(n_trees, n_int)).astype(np.int32)
    u = rng.uniform(size=(n_trees, n_int))
    thr = lo[feat] + u * (hi[feat] - lo[feat])
    is_index = feat < n_index_cols
    thr = np.where(is_index, np.floor(thr) + 0.5, thr).astype(np.float32)
    leaf = rng.standard_normal(size=(n_trees, 1 << depth)).astype(np.float32)
    return Forest(n_trees, depth, d, 0.0, feat, thr, leaf)


@dataclasses.dataclass
class Workload:
    name: str
    N: int
    d: int
    conv: Tuple[int, int, int, int]     # (C, K, H, r)
    mixture: int                        # number of Gaussian components; 0 = uniform sampling
    n_trees: int
    depth: int
    k_min: int
    k_max: int
    iters: int
    seed: int
    batch: int = 1


WORKLOADS = {
    "tiny": Workload("tiny", 2_000, 8, (64, 64, 56, 3), 6, 64, 6, 1, 16, 20, BASE_SEED),
    "mid": Workload("mid", 65_536, 16, (128, 128, 28, 3), 32, 256, 8, 1, 64, 30, BASE_SEED),
    "whole_layer": Workload("whole_layer", 1_048_576, 16, (256, 256, 14, 3), 0, 512, 8, 1, 64, 30, BASE_SEED),
    "large": Workload("large", 8_388_608, 32, (512, 512, 28, 3), 128, 512, 10, 1, 128, 30, BASE_SEED),
    "batched": Workload("batched", 262_144, 16, (0, 0, 0, 0), 0, 256, 8, 1, 32, 30, BASE_SEED, batch=64),
}


def batched_conv_shapes(batch: int, seed: int = BASE_SEED) -> List[Tuple[int, int, int, int]]:
    """First `batch` of a seeded permutation of the 128 shapes C,K in {64..512} x H in {7..56} x r in {1,3}."""
    combos = [(C, K, H, r) for C in (64, 128, 256, 512) for K in (64, 128, 256, 512)
              for H in (7, 14, 28, 56) for r in (1, 3)]
    perm = np.random.default_rng(seed).permutation(len(combos))
    return [combos[i] for i in perm[:batch]]


@dataclasses.dataclass
class Problem:
    """One knob space's inputs: feature matrix, forest and knob domains."""
    X: np.ndarray                 # fp32 [N, d], C-contiguous
    forest: Forest
    dom_offsets: np.ndarray       # int32 [n_knobs + 1]
    dom_values: np.ndarray        # fp32
    space: KnobSpace
    component: np.ndarray | None  # planted mixture component per row (None for uniform sampling)


def make_problem(w: Workload, conv: Sequence[int] | None = None, seed: int | None = None,
                 N: int | None = None) -> Problem:
    """Build one knob space of workload `w` (for the batched workload pass conv and seed of the space)."""
    conv = tuple(conv) if conv is not None else w.conv
    seed = w.seed if seed is None else seed
    n = w.N if N is None else N
    rng = np.random.default_rng(seed)
    space = conv2d_knob_space(*conv)
    comp = None
    if w.mixture > 0:
        knobs, comp = sample_knobs_mixture(space, n, w.mixture, rng)
    else:
        knobs = sample_knobs_uniform(space, n, rng)
    cols = [knobs.astype(np.float32)]
    if w.d >= 16:
        cols.append(derived_extent_columns(space, knobs))
    if w.d > 16:
        cols.append(lognormal_extra_columns(comp if comp is not None else np.zeros(n, np.int32),
                                            max(w.mixture, 1), w.d - 16, rng))
    X = np.ascontiguousarray(np.concatenate(cols, axis=1), dtype=np.float32)
    assert X.shape == (n, w.d)
    forest = random_forest(X, w.n_trees, w.depth, space.n_knobs, rng)
    offs, vals = space.domains_csr()
    return Problem(X, forest, offs, vals, space, comp)


def visited_configs(p: Problem, n_visited: int, seed: int) -> np.ndarray:
    """Stand-in for the history v_Theta: int32 [n_visited][n_knobs] domain indices, half of them rows of the
    trajectory itself (configurations the search has been at), half uniform draws from the space."""
    rng = np.random.default_rng(seed)
    n_knobs = p.space.n_knobs
    n_traj = min(n_visited // 2, p.X.shape[0])
    rows = rng.choice(p.X.shape[0], size=n_traj, replace=False)
    sizes = np.diff(p.dom_offsets)
    traj = np.clip(np.rint(p.X[rows, :n_knobs]).astype(np.int64), 0, sizes[None, :] - 1)
    rest = sample_knobs_uniform(p.space, n_visited - n_traj, rng)
    return np.ascontiguousarray(np.concatenate([traj, rest], axis=0), dtype=np.int32)


def make_batched_problems(w: Workload, batch: int | None = None, N: int | None = None) -> List[Problem]:
    shapes = batched_conv_shapes(w.batch if batch is None else batch, w.seed)
    return [make_problem(w, conv=s, seed=w.seed + b, N=N) for b, s in enumerate(shapes)]


def planted_clusters(n_per: int, k: int, d: int, sep: float, sigma: float, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Well-separated planted clusters on a jittered grid of spacing `sep`: (X fp32 [k*n_per, d], truth int32)."""
    rng = np.random.default_rng(seed)
    side = int(np.ceil(k ** (1.0 / min(d, 3))))
    grid = np.array(np.meshgrid(*[np.arange(side)] * min(d, 3), indexing="ij")).reshape(min(d, 3), -1).T
    centres = np.zeros((k, d))
    centres[:, :min(d, 3)] = grid[:k] * sep
    truth = np.repeat(np.arange(k, dtype=np.int32), n_per)
    X = centres[truth] + sigma * rng.standard_normal(size=(k * n_per, d))
    perm = rng.permutation(k * n_per)
    return np.ascontiguousarray(X[perm], dtype=np.float32), truth[perm]
