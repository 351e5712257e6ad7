"""Thin ctypes binding over librls.so (the C ABI of include/rls.h).

Argument marshalling only: every step of the path runs in the HIP kernels behind the C calls.
PyTorch supplies device memory (tensors) and the current HIP stream; nothing here computes.
The library must have been built (python -m paper_1905_12799_amd.build, or __graft_entry__.build());
loading fails loudly when it is missing.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

from . import build as _build

RLS_OK = 0
RLS_STATUS_NONFINITE = 1
RLS_STATUS_RANGE = 2
MAX_D, MAX_K, MAX_DEPTH = 32, 128, 12


class RlsError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {error_string(code)} (code {code})")


class _Forest(ctypes.Structure):
    _fields_ = [("n_trees", ctypes.c_int32), ("depth", ctypes.c_int32), ("n_features", ctypes.c_int32),
                ("base", ctypes.c_float), ("feat_dev", ctypes.c_void_p), ("thr_dev", ctypes.c_void_p),
                ("leaf_dev", ctypes.c_void_p)]


class _Domains(ctypes.Structure):
    _fields_ = [("n_knobs", ctypes.c_int32), ("offsets_dev", ctypes.c_void_p), ("values_dev", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            raise ImportError(f"{_build.LIB} is missing: build it with `python -m paper_1905_12799_amd.build`")
        L = ctypes.CDLL(_build.LIB)
        L.rls_version.restype = ctypes.c_int32
        L.rls_error_string.restype = ctypes.c_char_p
        L.rls_error_string.argtypes = [ctypes.c_int32]
        L.rls_last_hip_error.restype = ctypes.c_int32
        L.rls_kmeans_sweep_workspace_bytes.restype = ctypes.c_int64
        L.rls_kmeans_sweep_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                       ctypes.c_int32]
        i32, i64, u64, vp, f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_double
        L.rls_gbt_score.restype = i32
        L.rls_gbt_score.argtypes = [ctypes.POINTER(_Forest), vp, i64, i32, i64, vp, vp]
        L.rls_gbt_score_batched.restype = i32
        L.rls_gbt_score_batched.argtypes = [ctypes.POINTER(_Forest), i32, vp, i64, i32, i64, i64, vp, vp]
        L.rls_kmeanspp_chain.restype = i32
        L.rls_kmeanspp_chain.argtypes = [vp, i64, i32, i64, i32, u64, vp, vp, i64, vp]
        L.rls_kmeans_sweep.restype = i32
        L.rls_kmeans_sweep.argtypes = [vp, i64, i32, i64, i32, i32, i32, u64, vp, vp, vp, vp, vp, vp, vp, i64, vp]
        L.rls_kmeans_sweep_batched.restype = i32
        L.rls_kmeans_sweep_static.restype = i32
        L.rls_kmeans_sweep_static.argtypes = [vp, i64, i32, i64, i32, i32, i32, u64, vp, vp, vp, vp, vp, vp, vp]
        L.rls_kmeans_sweep_batched.argtypes = [i32, vp, i64, i32, i64, i64, i32, i32, i32, ctypes.POINTER(u64), vp, vp,
                                               vp, vp, vp, vp, vp, i64, vp]
        L.rls_kmeans_sweep_until_knee_workspace_bytes.restype = ctypes.c_int64
        L.rls_kmeans_sweep_until_knee_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
        L.rls_kmeans_sweep_until_knee.restype = i32
        L.rls_kmeans_sweep_until_knee.argtypes = [vp, i64, i32, i64, i32, i32, i32, i32, u64, vp, f64, vp, vp, vp,
                                                  ctypes.POINTER(f64), ctypes.POINTER(i32), ctypes.POINTER(i32), vp, vp,
                                                  i64, vp]
        L.rls_pick_knee.restype = i32
        L.rls_pick_knee.argtypes = [ctypes.POINTER(f64), i32, i32, f64, ctypes.POINTER(i32)]
        L.rls_snap_to_valid.restype = i32
        L.rls_snap_to_valid.argtypes = [vp, i32, i32, i64, ctypes.POINTER(_Domains), vp, vp]
        L.rls_snap_to_valid_batched.restype = i32
        L.rls_snap_to_valid_batched.argtypes = [i32, vp, i32, i32, i64, i64, ctypes.POINTER(_Domains), vp, vp]
        L.rls_knob_modes.restype = i32
        L.rls_knob_modes.argtypes = [vp, i64, i32, i64, ctypes.POINTER(_Domains), i32, vp, vp, vp]
        L.rls_replace_visited.restype = i32
        L.rls_replace_visited.argtypes = [vp, i32, i32, vp, i64, vp, vp, vp]
        L.rls_apply_actions.restype = i32
        L.rls_apply_actions.argtypes = [vp, vp, i64, ctypes.POINTER(_Domains), vp, vp, i64, vp]
        L.rls_profile_enable.restype = i32
        L.rls_profile_enable.argtypes = [i32]
        L.rls_profile_read.restype = i32
        L.rls_profile_read.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(f64)]
        _lib = L
    return _lib


def version() -> int:
    return int(lib().rls_version())


def error_string(code: int) -> str:
    return lib().rls_error_string(ctypes.c_int32(code)).decode()


def profile_enable(on: bool) -> None:
    _check(lib().rls_profile_enable(1 if on else 0), "rls_profile_enable")


def profile_read():
    """(launches timed, total milliseconds) of the Lloyd step kernel since the last read."""
    n, ms = ctypes.c_int32(0), ctypes.c_double(0.0)
    _check(lib().rls_profile_read(ctypes.byref(n), ctypes.byref(ms)), "rls_profile_read")
    return int(n.value), float(ms.value)


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(None if t is None else t.data_ptr())


def _check(rc: int, what: str) -> None:
    if rc != RLS_OK:
        raise RlsError(rc, what)


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor of dtype {dtype}")
    return t


def _mat(t: torch.Tensor, name: str) -> torch.Tensor:
    """fp32 device matrix (optionally with a leading batch dimension) whose rows are contiguous."""
    if not t.is_cuda or t.dtype != torch.float32 or t.stride(-1) != 1:
        raise ValueError(f"{name} must be an fp32 device tensor with unit stride along the features")
    return t


class DeviceForest:
    """Device-resident forest (arrays as in rls_forest): feat int32 [T, 2^D-1], thr fp32, leaf fp32 [T, 2^D]."""

    def __init__(self, n_trees: int, depth: int, n_features: int, base: float, feat, thr, leaf, device="cuda"):
        self.n_trees, self.depth, self.n_features, self.base = int(n_trees), int(depth), int(n_features), float(base)
        self.feat = torch.as_tensor(feat, dtype=torch.int32).contiguous().to(device)
        self.thr = torch.as_tensor(thr, dtype=torch.float32).contiguous().to(device)
        self.leaf = torch.as_tensor(leaf, dtype=torch.float32).contiguous().to(device)

    @classmethod
    def from_host(cls, f, device="cuda") -> "DeviceForest":
        return cls(f.n_trees, f.depth, f.n_features, f.base, f.feat, f.thr, f.leaf, device)

    def struct(self) -> _Forest:
        return _Forest(self.n_trees, self.depth, self.n_features, self.base, self.feat.data_ptr(),
                       self.thr.data_ptr(), self.leaf.data_ptr())


class DeviceDomains:
    """Device-resident knob domains in CSR form (rls_knob_domains)."""

    def __init__(self, offsets, values, device="cuda"):
        self.offsets = torch.as_tensor(offsets, dtype=torch.int32).contiguous().to(device)
        self.values = torch.as_tensor(values, dtype=torch.float32).contiguous().to(device)
        self.n_knobs = int(self.offsets.numel()) - 1
        self.n_values = int(self.values.numel())

    def struct(self) -> _Domains:
        return _Domains(self.n_knobs, self.offsets.data_ptr(), self.values.data_ptr())


def gbt_score(forest: DeviceForest, X: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _mat(X, "X")
    N, d = X.shape
    out = torch.empty(N, dtype=torch.float32, device=X.device) if out is None else _dev(out, torch.float32, "out")
    st = forest.struct()
    _check(lib().rls_gbt_score(ctypes.byref(st), _ptr(X), N, d, X.stride(0), _ptr(out), _stream()), "rls_gbt_score")
    return out


def gbt_score_batched(forests: Sequence[DeviceForest], X: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _mat(X, "X")
    B, N, d = X.shape
    out = torch.empty((B, N), dtype=torch.float32, device=X.device) if out is None else _dev(out, torch.float32, "out")
    arr = (_Forest * B)(*[f.struct() for f in forests])
    _check(lib().rls_gbt_score_batched(arr, B, _ptr(X), N, d, X.stride(1), X.stride(0), _ptr(out), _stream()),
           "rls_gbt_score_batched")
    return out


def kmeans_sweep_workspace_bytes(N: int, d: int, k_min: int, k_max: int, batch: int = 1) -> int:
    n = int(lib().rls_kmeans_sweep_workspace_bytes(N, d, k_min, k_max, batch))
    if n < 0:
        raise RlsError(n, "rls_kmeans_sweep_workspace_bytes")
    return n


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(nbytes + 256, dtype=torch.uint8, device=device)


def _aligned_ptr(ws: torch.Tensor) -> int:
    return (ws.data_ptr() + 255) // 256 * 256


def kmeanspp_chain(X: torch.Tensor, k_max: int, seed: int, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _mat(X, "X")
    N, d = X.shape
    need = kmeans_sweep_workspace_bytes(N, d, k_max, k_max, 1)
    ws = _workspace(need, X.device) if workspace is None else workspace
    idx = torch.empty(k_max, dtype=torch.int64, device=X.device)
    base = _aligned_ptr(ws)
    avail = ws.numel() - (base - ws.data_ptr())
    _check(lib().rls_kmeanspp_chain(_ptr(X), N, d, X.stride(0), k_max, ctypes.c_uint64(seed), _ptr(idx),
                                    ctypes.c_void_p(base), avail, _stream()), "rls_kmeanspp_chain")
    return idx


class SweepResult:
    """Outputs of a sweep, all device tensors. centroids is packed; use centroids_of(k)."""

    def __init__(self, k_min, k_max, d, labels, centroids, inertia, trace, status):
        self.k_min, self.k_max, self.d = k_min, k_max, d
        self.labels, self.centroids, self.inertia, self.trace, self.status = labels, centroids, inertia, trace, status

    def centroids_of(self, k: int, b: Optional[int] = None) -> torch.Tensor:
        off = sum(range(self.k_min, k)) * self.d
        c = self.centroids if b is None else self.centroids[b]
        return c[off:off + k * self.d].view(k, self.d)


def kmeans_sweep(X: torch.Tensor, k_min: int, k_max: int, iters: int, seed: int = 0,
                 init_idx: Optional[torch.Tensor] = None, want_labels: bool = True, want_trace: bool = False,
                 workspace: Optional[torch.Tensor] = None, check_status: bool = True) -> SweepResult:
    _mat(X, "X")
    N, d = X.shape
    n_k = k_max - k_min + 1
    rows = sum(range(k_min, k_max + 1))
    need = kmeans_sweep_workspace_bytes(N, d, k_min, k_max, 1)
    ws = _workspace(need, X.device) if workspace is None else workspace
    dev = X.device
    labels = torch.empty((n_k, N), dtype=torch.int32, device=dev) if want_labels else None
    centroids = torch.empty(rows * d, dtype=torch.float32, device=dev)
    inertia = torch.empty(n_k, dtype=torch.float64, device=dev)
    trace = torch.empty((n_k, iters + 1), dtype=torch.float64, device=dev) if want_trace else None
    status = torch.empty(1, dtype=torch.int32, device=dev)
    if init_idx is not None:
        _dev(init_idx, torch.int64, "init_idx")
        if init_idx.numel() < k_max:
            raise ValueError("init_idx needs k_max entries")
    base = _aligned_ptr(ws)
    avail = ws.numel() - (base - ws.data_ptr())
    rc = lib().rls_kmeans_sweep(_ptr(X), N, d, X.stride(0), k_min, k_max, iters, ctypes.c_uint64(seed), _ptr(init_idx),
                                _ptr(labels), _ptr(centroids), _ptr(inertia), _ptr(trace), _ptr(status),
                                ctypes.c_void_p(base), avail, _stream())
    _check(rc, "rls_kmeans_sweep")
    if check_status:
        st = int(status.item())
        if st != 0:
            raise RuntimeError(f"rls_kmeans_sweep: data precondition violated, status bits {st}")
    return SweepResult(k_min, k_max, d, labels, centroids, inertia, trace, status)


STATIC_WORKSPACE_BYTES = 64 << 20


def kmeans_sweep_static(X: torch.Tensor, k_min: int, k_max: int, iters: int, seed: int = 0,
                        init_idx: Optional[torch.Tensor] = None, want_trace: bool = False,
                        out: Optional[SweepResult] = None) -> SweepResult:
    """rls_kmeans_sweep_static: the sweep on the library's own fixed workspace (the call allocates nothing).
    `out` supplies the output tensors (labels may be None); without it they are allocated here, before the call."""
    _mat(X, "X")
    N, d = X.shape
    n_k = k_max - k_min + 1
    rows = sum(range(k_min, k_max + 1))
    dev = X.device
    if out is None:
        out = SweepResult(k_min, k_max, d, torch.empty((n_k, N), dtype=torch.int32, device=dev),
                          torch.empty(rows * d, dtype=torch.float32, device=dev),
                          torch.empty(n_k, dtype=torch.float64, device=dev),
                          torch.empty((n_k, iters + 1), dtype=torch.float64, device=dev) if want_trace else None,
                          torch.empty(1, dtype=torch.int32, device=dev))
    if init_idx is not None:
        _dev(init_idx, torch.int64, "init_idx")
        if init_idx.numel() < k_max:
            raise ValueError("init_idx needs k_max entries")
    rc = lib().rls_kmeans_sweep_static(_ptr(X), N, d, X.stride(0), k_min, k_max, iters, ctypes.c_uint64(seed),
                                       _ptr(init_idx), _ptr(out.labels), _ptr(out.centroids), _ptr(out.inertia),
                                       _ptr(out.trace), _ptr(out.status), _stream())
    _check(rc, "rls_kmeans_sweep_static")
    return out


def kmeans_sweep_until_knee(X: torch.Tensor, k_min: int, k_max: int, k_wave: int, iters: int, knee_const: float,
                            seed: int = 0, init_idx: Optional[torch.Tensor] = None, want_labels: bool = True,
                            workspace: Optional[torch.Tensor] = None) -> Tuple[int, int, SweepResult]:
    """Algorithm 1's loop with its early exit: returns (chosen k, number of k computed, results).

    The result arrays are sized for the whole range; only the first `n_done` runs are written. Synchronises the
    current stream after every wave of k_wave values of k."""
    _mat(X, "X")
    N, d = X.shape
    n_k = k_max - k_min + 1
    rows = sum(range(k_min, k_max + 1))
    need = int(lib().rls_kmeans_sweep_until_knee_workspace_bytes(N, d, k_min, k_max, k_wave))
    if need < 0:
        _check(need, "rls_kmeans_sweep_until_knee_workspace_bytes")
    ws = _workspace(need, X.device) if workspace is None else workspace
    dev = X.device
    labels = torch.empty((n_k, N), dtype=torch.int32, device=dev) if want_labels else None
    centroids = torch.empty(rows * d, dtype=torch.float32, device=dev)
    inertia = torch.empty(n_k, dtype=torch.float64, device=dev)
    status = torch.empty(1, dtype=torch.int32, device=dev)
    if init_idx is not None:
        _dev(init_idx, torch.int64, "init_idx")
        if init_idx.numel() < k_max:
            raise ValueError("init_idx needs k_max entries")
    inertia_host = (ctypes.c_double * n_k)()
    k_out, n_done = ctypes.c_int32(0), ctypes.c_int32(0)
    base = _aligned_ptr(ws)
    avail = ws.numel() - (base - ws.data_ptr())
    rc = lib().rls_kmeans_sweep_until_knee(_ptr(X), N, d, X.stride(0), k_min, k_max, k_wave, iters, ctypes.c_uint64(seed),
                                           _ptr(init_idx), float(knee_const), _ptr(labels), _ptr(centroids), _ptr(inertia),
                                           inertia_host, ctypes.byref(k_out), ctypes.byref(n_done), _ptr(status),
                                           ctypes.c_void_p(base), avail, _stream())
    _check(rc, "rls_kmeans_sweep_until_knee")
    st = int(status.item())
    if st != 0:
        raise RuntimeError(f"rls_kmeans_sweep_until_knee: data precondition violated, status bits {st}")
    return int(k_out.value), int(n_done.value), SweepResult(k_min, k_max, d, labels, centroids, inertia, None, status)


def kmeans_sweep_batched(X: torch.Tensor, k_min: int, k_max: int, iters: int, seeds: Optional[Sequence[int]] = None,
                         init_idx: Optional[torch.Tensor] = None, want_labels: bool = True, want_trace: bool = False,
                         workspace: Optional[torch.Tensor] = None, check_status: bool = True) -> SweepResult:
    _mat(X, "X")
    B, N, d = X.shape
    n_k = k_max - k_min + 1
    rows = sum(range(k_min, k_max + 1))
    need = kmeans_sweep_workspace_bytes(N, d, k_min, k_max, B)
    ws = _workspace(need, X.device) if workspace is None else workspace
    dev = X.device
    labels = torch.empty((B, n_k, N), dtype=torch.int32, device=dev) if want_labels else None
    centroids = torch.empty((B, rows * d), dtype=torch.float32, device=dev)
    inertia = torch.empty((B, n_k), dtype=torch.float64, device=dev)
    trace = torch.empty((B, n_k, iters + 1), dtype=torch.float64, device=dev) if want_trace else None
    status = torch.empty(B, dtype=torch.int32, device=dev)
    seeds_arr = None
    if seeds is not None:
        seeds_arr = (ctypes.c_uint64 * B)(*[int(s) for s in seeds])
    if init_idx is not None:
        _dev(init_idx, torch.int64, "init_idx")
    base = _aligned_ptr(ws)
    avail = ws.numel() - (base - ws.data_ptr())
    rc = lib().rls_kmeans_sweep_batched(B, _ptr(X), N, d, X.stride(1), X.stride(0), k_min, k_max, iters, seeds_arr,
                                        _ptr(init_idx), _ptr(labels), _ptr(centroids), _ptr(inertia), _ptr(trace),
                                        _ptr(status), ctypes.c_void_p(base), avail, _stream())
    _check(rc, "rls_kmeans_sweep_batched")
    if check_status and bool((status != 0).any().item()):
        raise RuntimeError(f"rls_kmeans_sweep_batched: data precondition violated, status {status.tolist()}")
    return SweepResult(k_min, k_max, d, labels, centroids, inertia, trace, status)


def pick_knee(inertia_host: Sequence[float], k_min: int, k_max: int, knee_const: float) -> int:
    n = k_max - k_min + 1
    arr = (ctypes.c_double * n)(*[float(v) for v in inertia_host[:n]])
    out = ctypes.c_int32(0)
    _check(lib().rls_pick_knee(arr, k_min, k_max, ctypes.c_double(knee_const), ctypes.byref(out)), "rls_pick_knee")
    return int(out.value)


def snap_to_valid(centroids: torch.Tensor, domains: DeviceDomains, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _mat(centroids, "centroids")
    k, d = centroids.shape
    out = torch.empty((k, domains.n_knobs), dtype=torch.int32, device=centroids.device) if out is None else out
    st = domains.struct()
    _check(lib().rls_snap_to_valid(_ptr(centroids), k, d, centroids.stride(0), ctypes.byref(st), _ptr(out), _stream()),
           "rls_snap_to_valid")
    return out


def knob_modes(X: torch.Tensor, domains: DeviceDomains, hist: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """mode(s_Theta): per knob the domain index most rows take; returns (mode_cfg [n_knobs], hist [n_values])."""
    _mat(X, "X")
    N, d = X.shape
    mode = torch.empty(domains.n_knobs, dtype=torch.int32, device=X.device)
    hist = torch.empty(domains.n_values, dtype=torch.int32, device=X.device) if hist is None else _dev(hist, torch.int32, "hist")
    st = domains.struct()
    _check(lib().rls_knob_modes(_ptr(X), N, d, X.stride(0), ctypes.byref(st), domains.n_values, _ptr(mode), _ptr(hist),
                                _stream()), "rls_knob_modes")
    return mode, hist


def replace_visited(cfg: torch.Tensor, visited: Optional[torch.Tensor], mode_cfg: torch.Tensor) -> torch.Tensor:
    """Rows of cfg (int32 [k][n_knobs], updated in place) found among the visited rows become mode_cfg; returns flags [k]."""
    _dev(cfg, torch.int32, "cfg")
    k, n_knobs = cfg.shape
    if not cfg.is_contiguous():
        raise ValueError("cfg must be contiguous")
    n_visited = 0 if visited is None else int(visited.shape[0])
    if n_visited:
        _dev(visited, torch.int32, "visited")
        if not visited.is_contiguous() or visited.shape[1] != n_knobs:
            raise ValueError("visited must be contiguous [V][n_knobs]")
    replaced = torch.empty(k, dtype=torch.int32, device=cfg.device)
    _check(lib().rls_replace_visited(_ptr(cfg), k, n_knobs, _ptr(visited) if n_visited else None, n_visited,
                                     _ptr(_dev(mode_cfg, torch.int32, "mode_cfg")), _ptr(replaced), _stream()),
           "rls_replace_visited")
    return replaced


def apply_actions(cfg: torch.Tensor, action: torch.Tensor, domains: DeviceDomains, want_features: bool = True):
    """Configuration updater: cfg int32 [m][n_knobs] + action int8 in {-1, 0, +1} -> (new cfg, features [m][n_knobs] or None)."""
    _dev(cfg, torch.int32, "cfg")
    _dev(action, torch.int8, "action")
    m, n_knobs = cfg.shape
    if not (cfg.is_contiguous() and action.is_contiguous()) or action.shape != cfg.shape or n_knobs != domains.n_knobs:
        raise ValueError("cfg and action must be contiguous [m][n_knobs] with the domains' n_knobs")
    out = torch.empty_like(cfg)
    feats = torch.empty((m, n_knobs), dtype=torch.float32, device=cfg.device) if want_features else None
    st = domains.struct()
    _check(lib().rls_apply_actions(_ptr(cfg), _ptr(action), m, ctypes.byref(st), _ptr(out), _ptr(feats), n_knobs, _stream()),
           "rls_apply_actions")
    return out, feats


def snap_to_valid_batched(centroids: torch.Tensor, domains: Sequence[DeviceDomains],
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _mat(centroids, "centroids")
    B, k, d = centroids.shape
    n_knobs = domains[0].n_knobs
    out = torch.empty((B, k, n_knobs), dtype=torch.int32, device=centroids.device) if out is None else out
    arr = (_Domains * B)(*[dm.struct() for dm in domains])
    _check(lib().rls_snap_to_valid_batched(B, _ptr(centroids), k, d, centroids.stride(1), centroids.stride(0), arr,
                                           _ptr(out), _stream()), "rls_snap_to_valid_batched")
    return out
