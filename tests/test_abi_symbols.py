"""The C-ABI library loads and exports every symbol the headers under include/ declare (no compute calls: no GPU needed)."""
import ctypes
import glob
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert any(h.endswith("rls.h") for h in headers)
    for h in headers:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names.update(re.findall(r"\b(rls_[a-z_]+)\s*\(", text))
    return sorted(names)


@pytest.fixture(scope="module")
def library():
    from paper_1905_12799_amd import build
    if not os.path.exists(build.LIB):
        build.build_library()
    return ctypes.CDLL(build.LIB)


def test_every_declared_symbol_is_exported(library):
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(library, n), n


def test_version_and_error_strings(library):
    from paper_1905_12799_amd import binding
    assert binding.version() == 133
    assert binding.error_string(0) == "ok"
    for code in range(-6, 0):
        assert binding.error_string(code) not in ("ok", "unknown error code")
    assert binding.error_string(-99) == "unknown error code"


def test_host_side_argument_checks(library):
    """Argument errors are found on the host before anything is enqueued, so they can be forced without a GPU."""
    from paper_1905_12799_amd import binding
    L = binding.lib()
    wsb = L.rls_kmeans_sweep_workspace_bytes
    assert wsb(1000, 8, 1, 16, 1) > 0
    assert wsb(1000, 8, 1, 16, 1) % 256 == 0
    assert wsb(0, 8, 1, 16, 1) == -1            # N < 1
    assert wsb(1000, 33, 1, 16, 1) == -1        # d above the limit
    assert wsb(1000, 8, 0, 16, 1) == -1         # k_min < 1
    assert wsb(1000, 8, 5, 4, 1) == -1          # k_max < k_min
    assert wsb(10, 8, 1, 16, 1) == -1           # k_max > N
    assert wsb(1000, 8, 1, 129, 1) == -1        # k_max above the limit
    assert wsb(1000, 8, 1, 16, 0) == -1         # batch < 1
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(4096)                # never dereferenced: the checks below fail first
    f = binding._Forest(4, 3, 8, 0.0, 4096, 4096, 4096)
    assert L.rls_gbt_score(ctypes.byref(f), null, 10, 8, 8, fake, null) == -2
    assert L.rls_gbt_score(ctypes.byref(f), fake, 10, 9, 9, fake, null) == -3      # forest features != d
    assert L.rls_gbt_score(ctypes.byref(f), fake, 10, 8, 4, fake, null) == -3      # ldx < d
    f13 = binding._Forest(4, 13, 8, 0.0, 4096, 4096, 4096)
    assert L.rls_gbt_score(ctypes.byref(f13), fake, 10, 8, 8, fake, null) == -1    # depth above the limit
    seed = ctypes.c_uint64(1)
    # workspace too small / missing
    assert L.rls_kmeans_sweep(fake, 1000, 8, 8, 1, 16, 5, seed, null, null, fake, fake, null, fake, null, 0, null) == -4
    assert L.rls_kmeans_sweep(fake, 1000, 8, 8, 1, 16, 5, seed, null, null, fake, fake, null, fake, fake, 16, null) == -4
    assert L.rls_kmeans_sweep(fake, 1000, 8, 8, 1, 16, -1, seed, null, null, fake, fake, null, fake, fake, 1 << 40, null) == -1
    assert L.rls_kmeans_sweep(fake, 1000, 8, (1 << 24) + 1, 1, 16, 5, seed, null, null, fake, fake, null, fake, fake, 1 << 40, null) == -3
    assert L.rls_kmeans_sweep(fake, 1000, 8, 8, 1, 16, 5, seed, null, null, null, fake, null, fake, fake, 1 << 40, null) == -2
    out = ctypes.c_int32(0)
    assert L.rls_pick_knee(None, 1, 4, 1.05, ctypes.byref(out)) == -2
    assert L.rls_kmeans_sweep_until_knee_workspace_bytes(1000, 8, 1, 16, 0) == -1      # k_wave < 1
    assert 0 < L.rls_kmeans_sweep_until_knee_workspace_bytes(1000, 8, 1, 16, 8) <= wsb(1000, 8, 1, 16, 1) * 2
    d = binding._Domains(9, 4096, 4096)
    assert L.rls_snap_to_valid(fake, 4, 8, 8, ctypes.byref(d), fake, null) == -3   # more knobs than columns
    d8 = binding._Domains(8, 4096, 4096)
    assert L.rls_knob_modes(fake, 100, 8, 8, ctypes.byref(d), 40, fake, fake, null) == -3      # more knobs than columns
    assert L.rls_knob_modes(fake, 100, 8, 8, ctypes.byref(d8), 4, fake, fake, null) == -1      # fewer values than knobs
    assert L.rls_knob_modes(fake, 100, 8, 8, ctypes.byref(d8), 8193, fake, fake, null) == -1   # above RLS_MAX_DOMAIN_VALUES
    assert L.rls_knob_modes(fake, 100, 8, 8, ctypes.byref(d8), 40, null, fake, null) == -2
    assert L.rls_replace_visited(fake, 4, 8, null, 10, fake, fake, null) == -2                  # visited rows missing
    assert L.rls_replace_visited(fake, 0, 8, fake, 10, fake, fake, null) == -1
    assert L.rls_replace_visited(fake, 4, 33, fake, 10, fake, fake, null) == -1
    assert L.rls_apply_actions(fake, null, 10, ctypes.byref(d8), fake, null, 0, null) == -2
    assert L.rls_apply_actions(fake, fake, 0, ctypes.byref(d8), fake, null, 0, null) == -1
    assert L.rls_apply_actions(fake, fake, 10, ctypes.byref(d8), fake, fake, 4, null) == -3          # feature rows too short


def test_pick_knee_matches_golden_cases(library):
    from paper_1905_12799_amd import binding
    from tests.test_oracle_knee_snap import read_knee_cases
    for k_min, const, losses, want in read_knee_cases():
        assert binding.pick_knee(losses, k_min, k_min + len(losses) - 1, const) == want
