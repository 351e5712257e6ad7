"""ctypes loader for the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package;
the GPU library and its Python binding never do.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rls_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

ORC_OK, ORC_ERR_ARG, ORC_ERR_RANGE, ORC_ERR_NOMEM = 0, -1, -2, -3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no FMA contraction, OpenMP for the one annotated loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_uniform.restype = ctypes.c_double
        _lib.orc_uniform.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        _lib.orc_splitmix64.restype = ctypes.c_uint64
        _lib.orc_splitmix64.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str) -> None:
    if rc != ORC_OK:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def threads() -> int:
    return int(lib().orc_threads())


def splitmix64(seed: int, j: int) -> int:
    return int(lib().orc_splitmix64(ctypes.c_uint64(seed), ctypes.c_uint64(j)))


def uniform(seed: int, j: int) -> float:
    return float(lib().orc_uniform(ctypes.c_uint64(seed), ctypes.c_uint64(j)))


def gbt_score(forest, X) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (fp32 tree-order sum, fp64 sum) per row of X. `forest` has n_trees, depth, base, feat, thr, leaf."""
    X = _f32(X)
    N, d = X.shape
    feat = np.ascontiguousarray(forest.feat, dtype=np.int32)
    thr = _f32(forest.thr)
    leaf = _f32(forest.leaf)
    s32 = np.empty(N, dtype=np.float32)
    s64 = np.empty(N, dtype=np.float64)
    rc = lib().orc_gbt_score(ctypes.c_int32(forest.n_trees), ctypes.c_int32(forest.depth),
                             ctypes.c_int32(forest.n_features), ctypes.c_float(forest.base),
                             _p(feat), _p(thr), _p(leaf), _p(X), ctypes.c_int64(N), ctypes.c_int32(d),
                             ctypes.c_int64(d), _p(s32), _p(s64))
    _check(rc, "gbt_score")
    return s32, s64


def kmeanspp_chain(X, k_max: int, seed: int) -> np.ndarray:
    X = _f32(X)
    N, d = X.shape
    idx = np.empty(k_max, dtype=np.int64)
    rc = lib().orc_kmeanspp_chain(_p(X), ctypes.c_int64(N), ctypes.c_int32(d), ctypes.c_int64(d),
                                  ctypes.c_int32(k_max), ctypes.c_uint64(seed), _p(idx))
    _check(rc, "kmeanspp_chain")
    return idx


def draw_index(D, r: float) -> int:
    """The D^2 draw of the seeding chain on a given distance array: first index whose prefix sum exceeds r."""
    D = np.ascontiguousarray(D, dtype=np.float64)
    fn = lib().orc_draw_index
    fn.restype = ctypes.c_int64
    return int(fn(_p(D), ctypes.c_int64(D.shape[0]), ctypes.c_double(r)))


def lloyd(X, k: int, iters: int, init_idx, want_trace: bool = False):
    """One k. Returns (labels int32 [N], centroids fp32 [k,d], inertia, half-step trace [2*iters+1] or None)."""
    X = _f32(X)
    N, d = X.shape
    init_idx = np.ascontiguousarray(init_idx, dtype=np.int64)
    assert init_idx.shape[0] >= k
    labels = np.empty(N, dtype=np.int32)
    C = np.empty((k, d), dtype=np.float32)
    J = np.zeros(1, dtype=np.float64)
    trace = np.zeros(2 * iters + 1, dtype=np.float64) if want_trace else None
    rc = lib().orc_lloyd(_p(X), ctypes.c_int64(N), ctypes.c_int32(d), ctypes.c_int64(d), ctypes.c_int32(k),
                         ctypes.c_int32(iters), _p(init_idx), _p(labels), _p(C), _p(J), _p(trace))
    _check(rc, "lloyd")
    return labels, C, float(J[0]), trace


def kmeans_sweep(X, k_min: int, k_max: int, iters: int, seed: int = 0, init_idx=None,
                 want_labels: bool = True, want_trace: bool = False):
    """Returns dict(labels [n_k,N] or None, centroids packed fp32, inertia [n_k], trace [n_k,iters+1] or None)."""
    X = _f32(X)
    N, d = X.shape
    n_k = k_max - k_min + 1
    rows = sum(range(k_min, k_max + 1))
    labels = np.empty((n_k, N), dtype=np.int32) if want_labels else None
    C = np.empty(rows * d, dtype=np.float32)
    J = np.zeros(n_k, dtype=np.float64)
    trace = np.zeros((n_k, iters + 1), dtype=np.float64) if want_trace else None
    if init_idx is not None:
        init_idx = np.ascontiguousarray(init_idx, dtype=np.int64)
        assert init_idx.shape[0] >= k_max
    rc = lib().orc_kmeans_sweep(_p(X), ctypes.c_int64(N), ctypes.c_int32(d), ctypes.c_int64(d),
                                ctypes.c_int32(k_min), ctypes.c_int32(k_max), ctypes.c_int32(iters),
                                ctypes.c_uint64(seed), _p(init_idx), _p(labels), _p(C), _p(J), _p(trace))
    _check(rc, "kmeans_sweep")
    return {"labels": labels, "centroids": C, "inertia": J, "trace": trace}


def pick_knee(inertia, k_min: int, k_max: int, knee_const: float) -> int:
    inertia = np.ascontiguousarray(inertia, dtype=np.float64)
    assert inertia.shape[0] >= k_max - k_min + 1
    out = ctypes.c_int32(0)
    rc = lib().orc_pick_knee(_p(inertia), ctypes.c_int32(k_min), ctypes.c_int32(k_max),
                             ctypes.c_double(knee_const), ctypes.byref(out))
    _check(rc, "pick_knee")
    return int(out.value)


def snap_to_valid(centroids, offsets, values) -> np.ndarray:
    C = _f32(centroids)
    k, d = C.shape
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    values = _f32(values)
    n_knobs = offsets.shape[0] - 1
    cfg = np.empty((k, n_knobs), dtype=np.int32)
    rc = lib().orc_snap_to_valid(_p(C), ctypes.c_int32(k), ctypes.c_int32(d), ctypes.c_int64(d),
                                 ctypes.c_int32(n_knobs), _p(offsets), _p(values), _p(cfg))
    _check(rc, "snap_to_valid")
    return cfg


def knob_modes(X, offsets, values) -> Tuple[np.ndarray, np.ndarray]:
    """mode(s_Theta): per knob the domain index most points take; also the counts of every domain entry."""
    X = _f32(X)
    N, d = X.shape
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    values = _f32(values)
    n_knobs = offsets.shape[0] - 1
    mode = np.empty(n_knobs, dtype=np.int32)
    hist = np.empty(int(offsets[-1]), dtype=np.int64)
    rc = lib().orc_knob_modes(_p(X), ctypes.c_int64(N), ctypes.c_int32(d), ctypes.c_int64(d), ctypes.c_int32(n_knobs),
                              _p(offsets), _p(values), _p(mode), _p(hist))
    _check(rc, "knob_modes")
    return mode, hist


def replace_visited(cfg, visited, mode_cfg) -> Tuple[np.ndarray, np.ndarray]:
    """Rows of cfg found among the visited rows become mode_cfg; returns (new cfg, replaced flags)."""
    cfg = np.array(cfg, dtype=np.int32, order="C", copy=True)
    k, n_knobs = cfg.shape
    visited = np.ascontiguousarray(visited, dtype=np.int32).reshape(-1, n_knobs)
    mode_cfg = np.ascontiguousarray(mode_cfg, dtype=np.int32)
    replaced = np.zeros(k, dtype=np.int32)
    rc = lib().orc_replace_visited(_p(cfg), ctypes.c_int32(k), ctypes.c_int32(n_knobs),
                                   _p(visited) if visited.shape[0] else None, ctypes.c_int64(visited.shape[0]),
                                   _p(mode_cfg), _p(replaced))
    _check(rc, "replace_visited")
    return cfg, replaced


def apply_actions(cfg, action, offsets, values, want_features: bool = True):
    """Configuration updater: cfg [m][n_knobs] domain indices + action in {-1, 0, +1} -> (new cfg, features or None)."""
    cfg = np.ascontiguousarray(cfg, dtype=np.int32)
    action = np.ascontiguousarray(action, dtype=np.int8)
    m, n_knobs = cfg.shape
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    values = _f32(values)
    out = np.empty_like(cfg)
    feats = np.zeros((m, n_knobs), dtype=np.float32) if want_features else None
    rc = lib().orc_apply_actions(_p(cfg), _p(action), ctypes.c_int64(m), ctypes.c_int32(n_knobs), _p(offsets), _p(values),
                                 _p(out), _p(feats), ctypes.c_int64(n_knobs))
    _check(rc, "apply_actions")
    return out, feats


def two_nearest(x, C) -> Tuple[float, float, int]:
    x = _f32(x)
    C = _f32(C)
    k, d = C.shape
    d1, d2, arg = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_int32(0)
    rc = lib().orc_two_nearest(_p(x), ctypes.c_int32(d), _p(C), ctypes.c_int32(k),
                               ctypes.byref(d1), ctypes.byref(d2), ctypes.byref(arg))
    _check(rc, "two_nearest")
    return d1.value, d2.value, int(arg.value)


def unpack_centroids(packed: np.ndarray, k_min: int, k: int, d: int) -> np.ndarray:
    """View of run k inside the packed centroid array of a sweep that starts at k_min."""
    off = sum(range(k_min, k)) * d
    return packed[off:off + k * d].reshape(k, d)
