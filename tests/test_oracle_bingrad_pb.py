"""Pins for the oracle's BinGrad-pb (Section 3.2, the partially biased two-level scheme)."""
from fractions import Fraction

import numpy as np

import oracle


def F(x):
    return Fraction(float(np.float32(x)))


def test_two_point_distribution_gives_its_magnitude():
    # +-a with equal counts: b_1 * n/2 = sum_{v >= b_1} v holds exactly at b_1 = a
    g = np.array([0.25, -0.25] * 50, np.float32)
    assert oracle.bingrad_pb_level(g) == np.float32(0.25)


def test_closed_form_roots_of_the_optimal_condition():
    # uniform on [-1, 1]:  b/2 = (1 - b^2)/4  ->  b = sqrt(2) - 1
    m = 4000
    grid = (np.arange(m) + 0.5) / m
    g = np.concatenate([grid, -grid]).astype(np.float32)
    assert abs(float(oracle.bingrad_pb_level(g)) - (np.sqrt(2) - 1)) < 2.0 / m
    # standard normal: b/2 = pdf(b) -> b = 0.6478...;  Laplace(0, 1): t = (t + 1) exp(-t) -> t = 0.8065...
    rng = np.random.default_rng(0)
    n = 20000
    normal_root, laplace_root = 0.64785, 0.80647
    assert abs(float(oracle.bingrad_pb_level(rng.normal(0, 1, n).astype(np.float32))) - normal_root) < 0.03
    assert abs(float(oracle.bingrad_pb_level(rng.laplace(0, 1, n).astype(np.float32))) - laplace_root) < 0.04
    # scaling the data scales the level
    g = rng.normal(0, 1, 2048).astype(np.float32)
    assert oracle.bingrad_pb_level(g * np.float32(2.0 ** -10)) == oracle.bingrad_pb_level(g) * np.float32(2.0 ** -10)


def test_level_sits_at_the_sign_change_of_the_condition_and_of_the_error_gradient():
    # f(b) = b * #{v > 0} - sum_{v >= b} v is half the derivative of the positive side's error
    # sum_{0<v<b} (b^2 - v^2) + sum_{v>=b} (v - b)^2 and grows with b: the chosen value is one of the two
    # candidates around its sign change, the one with the smaller |f| (the smaller value on a tie)
    rng = np.random.default_rng(1)
    for trial in range(150):
        n = int(rng.integers(1, 40))
        g = (rng.integers(-6, 7, n) if trial % 3 == 0 else rng.normal(0.1, 1, n)).astype(np.float32)
        b1 = oracle.bingrad_pb_level(g)
        pos = sorted(set(F(v) for v in g if v > 0))
        if not pos:
            assert b1 == 0
            continue
        npos = sum(1 for v in g if v > 0)

        def f(b):
            return b * npos - sum(F(v) for v in g if F(v) >= b)

        vals = [f(b) for b in pos]
        assert all(a < c for a, c in zip(vals[:-1], vals[1:]))          # strictly increasing over candidates
        assert vals[-1] >= 0                                             # so a sign change exists
        k = next(i for i, x in enumerate(vals) if x >= 0)
        choice = k if (k == 0 or abs(vals[k]) < abs(vals[k - 1])) else k - 1
        assert F(b1) == pos[choice]
        # error of the positive side: the chosen candidate is a minimiser among its neighbours up to one step
        def err(b):
            return sum((b * b - F(v) ** 2) if F(v) < b else (F(v) - b) ** 2 for v in g if v > 0)
        if 0 < choice < len(pos) - 1:
            assert err(pos[choice]) <= max(err(pos[choice - 1]), err(pos[choice + 1]))


def test_encoding_clamps_outside_and_rounds_without_bias_inside():
    rng = np.random.default_rng(2)
    base = rng.normal(0, 1, 400).astype(np.float32)
    M = 20000
    for probe in (np.float32(0.2), np.float32(-0.45), np.float32(3.0), np.float32(-3.0)):
        g = np.concatenate([base, np.full(M, probe, np.float32)])
        lv, codes, thr = oracle.quantize_codes(g, 1 << 15, 1, oracle.BINGRAD_PB, 0, seed=77)
        b1 = thr[0]
        assert lv[0] == -b1 and lv[1] == b1 and b1 > 0
        dec = lv[codes[400:]].astype(np.float64)
        if probe >= b1:
            assert np.all(dec == b1)
        elif probe < -b1:
            assert np.all(dec == -b1)
        else:
            var = (float(probe) + float(b1)) * (float(b1) - float(probe))
            assert abs(dec.mean() - float(probe)) < 4.5 * np.sqrt(var / M)
    # every element outside the levels goes to the nearer one, deterministically
    lv, codes, thr = oracle.quantize_codes(base, 512, 1, oracle.BINGRAD_PB, 0, seed=5)
    assert np.all(codes[base >= thr[0]] == 1) and np.all(codes[base < -thr[0]] == 0)


def test_degenerate_buckets():
    assert oracle.bingrad_pb_level(np.array([-1.0, -2.0, 0.0], np.float32)) == 0
    lv, codes, _ = oracle.quantize_codes(np.array([-1.0, -2.0, 0.0], np.float32), 64, 1, oracle.BINGRAD_PB)
    assert np.all(lv == 0) and np.all(lv[codes] == 0)
    assert oracle.bingrad_pb_level(np.array([5.0], np.float32)) == 5
    assert oracle.bingrad_pb_level(np.full(9, 2.0, np.float32)) == 2
