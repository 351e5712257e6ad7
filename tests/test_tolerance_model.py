"""The Lloyd step kernel computes distances from two fp16 pieces per operand and re-decides every comparison that falls
inside an error bound with the exact arithmetic.  The part of that bound that covers what the pieces leave out is
checked here on the CPU against a model of the split (numpy only; no GPU, no oracle): per distance at most
24.5 * 2^-23 * (|x'|^2 + |c'|^2) plus 0.0781 * d for pieces below 2^-14 that may be lost altogether
(comment at `eps_a` in paper_1905_12799_amd/csrc/kmeans_lloyd.hip)."""
import numpy as np
import pytest


def rtz16(v):
    """fp32 -> fp16 rounded toward zero (as the packed conversion the kernel uses), returned as fp32."""
    h = v.astype(np.float16)
    away = np.abs(h.astype(np.float32)) > np.abs(v)
    return np.where(away, np.nextafter(h, np.float16(0)), h).astype(np.float32)


def lost_below_normal(v):
    return np.where(np.abs(v) < 2.0 ** -14, 0.0, v).astype(np.float32)


@pytest.mark.parametrize("flush", [False, True])
def test_two_piece_products_stay_inside_the_bound(flush):
    rng = np.random.default_rng(5 + int(flush))
    worst = 0.0
    for trial in range(80):
        d = int(rng.choice([8, 16, 32]))
        n = 2048
        scale = 2.0 ** rng.integers(-24, 14)
        x = (rng.standard_normal((n, d)) * scale).astype(np.float32)
        c = (rng.standard_normal((n, d)) * scale * rng.choice([1.0, 0.01, 30.0])).astype(np.float32)
        if trial % 3 == 0:                       # one column much larger than the rest
            x[:, 0] *= 2.0 ** 10
            c[:, 0] *= 2.0 ** 10
        x = np.clip(x, -2.0 ** 13, 2.0 ** 13)    # the kernel's scaling keeps |x'| < 2^13, |2c'| < 2^14
        c = np.clip(c, -2.0 ** 13, 2.0 ** 13)
        C = (-2.0 * c).astype(np.float32)
        xh, Ch = rtz16(x), rtz16(C)
        xl, Cl = rtz16(x - xh), rtz16(C - Ch)
        assert np.all((x - xh).astype(np.float64) == x.astype(np.float64) - xh.astype(np.float64))   # remainder is exact in fp32
        if flush:
            xh, xl, Ch, Cl = (lost_below_normal(a) for a in (xh, xl, Ch, Cl))
        f64 = np.float64
        approx = (xh.astype(f64) * Ch + xh.astype(f64) * Cl + xl.astype(f64) * Ch).sum(1)
        exact = (x.astype(f64) * C.astype(f64)).sum(1)
        S = (x.astype(f64) ** 2).sum(1) + (c.astype(f64) ** 2).sum(1)
        bound = 24.5 * 2.0 ** -23 * S + 0.0781 * d + d * 2.0 ** -27
        worst = max(worst, float((np.abs(approx - exact) / bound).max()))
    assert worst <= 1.0
    assert worst > 0.01      # the model is exercised: the errors are not orders of magnitude below the bound


def test_fp32_direct_form_first_stage_keeps_the_fp64_winner():
    """The exact argmin of the Lloyd step settles most calls in fp32: direct-form distances (difference, square, running
    sum with one rounding per multiply-add), then every centroid within 8 (d + 2) 2^-24 of the smallest stays a
    candidate and fp64 decides only among several.  Model of that stage in numpy: the relative error of the fp32 form
    against the exact distance is below (d + 2) 2^-24, and the fp64 winner (lowest index among equals) is always among
    the candidates - also with near-ties planted a few fp32 units apart."""
    rng = np.random.default_rng(41)
    worst = 0.0
    for trial in range(60):
        d = int(rng.choice([8, 16, 32]))
        k = int(rng.integers(2, 129))
        scale = 2.0 ** rng.integers(-30, 30)
        x = (rng.standard_normal(d) * scale).astype(np.float32)
        c = (rng.standard_normal((k, d)) * scale).astype(np.float32)
        if trial % 2 == 0:
            # near-ties: mirror a centroid in x along one feature (the same distance up to rounding), nudge another copy
            j, l = int(rng.integers(0, k - 1)), int(rng.integers(0, d))
            c[j + 1] = c[j]
            c[j + 1, l] = np.float32(2.0) * x[l] - c[j, l]
            if k > 3:
                c[(j + 2) % k] = np.nextafter(c[j], np.float32(np.inf))
        # fp32 stage: sequential multiply-adds (the product and the sum are rounded once together: emulate in fp64, round)
        acc = np.zeros(k, dtype=np.float32)
        for l in range(d):
            diff = (x[l] - c[:, l]).astype(np.float32)
            acc = (diff.astype(np.float64) * diff.astype(np.float64) + acc.astype(np.float64)).astype(np.float32)
        exact = ((x.astype(np.float64)[None, :] - c.astype(np.float64)) ** 2).sum(1)     # exact up to 2^-53 relative
        rel = np.abs(acc.astype(np.float64) - exact) / np.maximum(exact, 1e-300)
        worst = max(worst, float(rel.max() / ((d + 2) * 2.0 ** -24)))
        # the oracle's decision: fp64 direct form with separately rounded multiply and add, lowest index among equals
        d64 = np.zeros(k)
        for l in range(d):
            diff = x[l].astype(np.float64) - c[:, l].astype(np.float64)
            d64 = d64 + diff * diff
        winner = int(np.argmin(d64))
        wmin = acc.min()
        thr = np.float32(np.float64(wmin) * (8 * (d + 2)) * 2.0 ** -24 + np.float64(wmin))
        assert acc[winner] <= thr
    assert worst <= 1.0
    assert worst > 0.02


def test_seeding_skip_rule_never_skips_a_point_that_would_improve():
    """The seeding update leaves a point's row unread when D_i <= (1 - 2^-30) / 4 * |c_a - c_new|^2, a being the
    point's nearest earlier centre (triangle inequality).  Model of the rule in numpy, in the kernel's arithmetic
    (fp64 direct form on fp32 rows): no skipped point may have a strictly smaller distance to the new centre -
    on lattice data, where D_i = |c_a - c_new|^2 / 4 holds exactly for many points, on duplicates and on
    continuous data of very different scales."""
    rng = np.random.default_rng(77)
    cases = []
    for dims, span in ((2, 6), (3, 4), (8, 3), (16, 2)):
        cases.append(rng.integers(0, span + 1, size=(4000, dims)).astype(np.float32))
    cases.append((rng.standard_normal((4000, 16)) * 1e-6).astype(np.float32))
    cases.append((rng.standard_normal((4000, 32)) * 3e5 + 1e6).astype(np.float32))
    line = np.zeros((4001, 4), dtype=np.float32)
    line[:, 0] = np.arange(4001) * 0.5                         # midpoints between centres are data points
    cases.append(line)
    skipped_total = 0
    for X32 in cases:
        X = X32.astype(np.float64)
        n = X.shape[0]
        chain = [int(rng.integers(n))]
        D = ((X - X[chain[0]]) ** 2).sum(1)
        near = np.zeros(n, dtype=np.int64)
        for j in range(1, 24):
            pick = int(rng.integers(n))
            c = X[pick]
            dcc = ((X[chain] - c) ** 2).sum(1)
            thr = dcc * (0.25 * (1.0 - 2.0 ** -30))
            skip = D <= thr[near]
            dn = ((X - c) ** 2).sum(1)
            assert not np.any(skip & (dn < D))
            skipped_total += int(skip.sum())
            better = dn < D
            D = np.where(better, dn, D)
            near = np.where(better, j, near)
            chain.append(pick)
    assert skipped_total > 100000        # the rule does fire on these inputs
