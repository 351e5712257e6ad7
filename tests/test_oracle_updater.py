"""Pins for the configuration updater of the search agent (Sec. 4.1: one direction per dimension)."""
import numpy as np
import pytest


def domains(sizes, rng):
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    values = np.concatenate([np.sort(rng.uniform(-9, 9, size=s)) for s in sizes]).astype(np.float32)
    return offsets, values


def test_updater_equals_clip_of_sum(orc):
    rng = np.random.default_rng(5)
    sizes = np.array([7, 1, 3, 12, 2])
    offsets, values = domains(sizes, rng)
    cfg = np.stack([rng.integers(0, s, size=500) for s in sizes], axis=1).astype(np.int32)
    act = rng.integers(-1, 2, size=cfg.shape).astype(np.int8)
    out, feats = orc.apply_actions(cfg, act, offsets, values)
    want = np.clip(cfg.astype(np.int64) + act, 0, sizes[None, :] - 1)
    np.testing.assert_array_equal(out, want)
    np.testing.assert_array_equal(feats, values[offsets[:-1][None, :] + want])


def test_updater_borders_and_stay(orc):
    offsets = np.array([0, 3, 4], dtype=np.int32)
    values = np.array([10.0, 20.0, 30.0, 5.0], dtype=np.float32)
    cfg = np.array([[0, 0], [2, 0], [1, 0], [1, 0]], dtype=np.int32)
    act = np.array([[-1, -1], [1, 1], [0, 0], [1, -1]], dtype=np.int8)
    out, feats = orc.apply_actions(cfg, act, offsets, values)
    np.testing.assert_array_equal(out, [[0, 0], [2, 0], [1, 0], [2, 0]])      # borders hold; a one-entry knob never moves
    np.testing.assert_array_equal(feats, [[10, 5], [30, 5], [20, 5], [30, 5]])
    # opposite actions undo each other away from the borders
    back, _ = orc.apply_actions(out[2:3], -act[2:3], offsets, values)
    np.testing.assert_array_equal(back, cfg[2:3])


def test_updater_rejects_bad_input(orc):
    offsets = np.array([0, 3], dtype=np.int32)
    values = np.array([1.0, 2.0, 3.0], dtype=np.float32)
    with pytest.raises(RuntimeError):
        orc.apply_actions(np.array([[3]], dtype=np.int32), np.array([[0]], dtype=np.int8), offsets, values)   # index outside
    with pytest.raises(RuntimeError):
        orc.apply_actions(np.array([[1]], dtype=np.int32), np.array([[2]], dtype=np.int8), offsets, values)   # not a direction
