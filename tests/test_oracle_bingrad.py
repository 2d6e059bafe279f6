"""Pins for the oracle's BinGrad-b (Section 3.2: deterministic two-level quantization)."""
from fractions import Fraction

import numpy as np

import oracle


def F(x):
    return Fraction(float(np.float32(x)))


def bucket(rng, n, kind):
    if kind == "normal":
        return rng.normal(0, 1e-3, n).astype(np.float32)
    if kind == "laplace_tail":
        g = rng.laplace(0, 5e-4, n)
        g[rng.random(n) < 0.05] *= 20
        return g.astype(np.float32)
    if kind == "shifted":
        return (rng.normal(0.3, 1e-2, n)).astype(np.float32)
    raise ValueError(kind)


def exact_mse(g, b0, lo, hi):
    return sum((F(v) - (F(lo) if v < b0 else F(hi))) ** 2 for v in g)


def test_threshold_is_the_mean_and_levels_are_conditional_means():
    rng = np.random.default_rng(0)
    for kind in ("normal", "laplace_tail", "shifted"):
        for n in (1, 2, 5, 64, 513, 2048):
            g = bucket(rng, n, kind)
            lv, b0 = oracle.bingrad_bucket(g, 0)
            mean = sum(F(v) for v in g) / n
            assert b0 == np.float32(float(mean))
            lo = [F(v) for v in g if v < b0]
            hi = [F(v) for v in g if v >= b0]
            assert hi, "the side at or above the mean is never empty"
            want_hi = np.float32(float(sum(hi) / len(hi)))
            want_lo = np.float32(float(sum(lo) / len(lo))) if lo else want_hi
            assert lv[1] == want_hi and lv[0] == want_lo
            assert lv[0] <= b0 <= lv[1]


def test_decoded_bucket_keeps_the_bucket_sum():
    # n_lo * b_lo + n_hi * b_hi = sum(g): conditional means preserve the total
    rng = np.random.default_rng(1)
    g = bucket(rng, 2048, "laplace_tail")
    for iters in (0, 3):
        lv, b0 = oracle.bingrad_bucket(g, iters)
        n_lo = int((g < b0).sum())
        decoded = n_lo * float(lv[0]) + (g.size - n_lo) * float(lv[1])
        assert abs(decoded - float(g.astype(np.float64).sum())) <= 2048 * 2.0 ** -24 * np.abs(g).max()


def test_plus_minus_pairs_reduce_to_scaled_signsgd():
    # a bucket of +-a pairs has mean 0, so the levels are -+ ||G||_1 / dim(G) and the code is the sign
    rng = np.random.default_rng(2)
    a = np.abs(rng.normal(0, 1e-2, 500)).astype(np.float32) + np.float32(1e-6)
    g = np.concatenate([a, -a])
    rng.shuffle(g)
    lv, b0 = oracle.bingrad_bucket(g, 0)
    scale = np.float32(float(sum(F(v) for v in np.abs(g)) / g.size))
    assert b0 == 0
    assert lv[1] == scale and lv[0] == -scale
    levels, codes, thr = oracle.quantize_codes(g, 1024, 1, oracle.BINGRAD_B)
    assert np.array_equal(codes, (g > 0).astype(np.uint8))


def test_iterations_follow_the_optimal_condition_and_never_raise_the_error():
    rng = np.random.default_rng(3)
    for kind in ("normal", "laplace_tail"):
        for n in (6, 9, 12):
            for _ in range(10):
                g = bucket(rng, n, kind)
                x = np.sort(g)
                # exhaustive 1-D two-means: every contiguous split of the sorted bucket
                best = None
                for cut in range(1, n):
                    lo = sum(F(v) for v in x[:cut]) / cut
                    hi = sum(F(v) for v in x[cut:]) / (n - cut)
                    e = sum((F(v) - lo) ** 2 for v in x[:cut]) + sum((F(v) - hi) ** 2 for v in x[cut:])
                    best = e if best is None else min(best, e)
                prev = None
                for iters in range(0, 8):
                    lv, b0 = oracle.bingrad_bucket(g, iters)
                    # exact conditional means of this partition (levels are these, rounded to fp32)
                    lo = [F(v) for v in g if v < b0]
                    hi = [F(v) for v in g if v >= b0]
                    m_hi = sum(hi) / len(hi)
                    m_lo = sum(lo) / len(lo) if lo else m_hi
                    e = sum((v - m_lo) ** 2 for v in lo) + sum((v - m_hi) ** 2 for v in hi)
                    assert e >= best
                    if prev is not None:
                        assert e <= prev
                    prev = e
                # converged: the threshold is the midpoint of the two levels
                lv, b0 = oracle.bingrad_bucket(g, 60)
                lv2, b02 = oracle.bingrad_bucket(g, 61)
                assert b0 == b02 and np.array_equal(lv, lv2)
                lo = [F(v) for v in g if v < b0]
                hi = [F(v) for v in g if v >= b0]
                if lo:
                    mid = (sum(lo) / len(lo) + sum(hi) / len(hi)) / 2
                    assert b0 == np.float32(float(mid))


def test_two_separated_clusters_reach_the_global_two_means():
    rng = np.random.default_rng(4)
    g = np.concatenate([rng.normal(-1, 0.01, 40), rng.normal(2, 0.01, 25)]).astype(np.float32)
    rng.shuffle(g)
    lv, b0 = oracle.bingrad_bucket(g, 0)
    assert abs(lv[0] + 1) < 0.01 and abs(lv[1] - 2) < 0.01
    assert np.array_equal(g >= b0, g > 0)


def test_constant_bucket_has_equal_levels_and_all_codes_one():
    g = np.full(100, 0.25, np.float32)
    lv, b0 = oracle.bingrad_bucket(g, 2)
    assert lv[0] == lv[1] == np.float32(0.25)
    levels, codes, thr = oracle.quantize_codes(g, 64, 1, oracle.BINGRAD_B, 2)
    assert np.all(codes == 1) and np.all(levels == np.float32(0.25))


def test_strict_less_goes_down_equal_goes_up():
    # v < b0 -> lower level, v >= b0 -> upper level: an element equal to the threshold goes up
    g = np.array([-1.0, 0.0, 1.0], np.float32)  # mean 0 exactly
    levels, codes, thr = oracle.quantize_codes(g, 64, 1, oracle.BINGRAD_B)
    assert thr[0] == 0 and list(codes) == [0, 1, 1]
    assert levels[0] == -1.0 and levels[1] == 0.5


def test_buckets_are_independent_and_tail_bucket_is_short():
    rng = np.random.default_rng(6)
    g = bucket(rng, 64 * 5 + 17, "normal")
    levels, codes, thr = oracle.quantize_codes(g, 128, 1, oracle.BINGRAD_B)
    assert levels.size == 2 * 3 and thr.size == 3
    for b in range(3):
        lv, b0 = oracle.bingrad_bucket(g[128 * b:128 * (b + 1)], 0)
        assert np.array_equal(levels[2 * b:2 * b + 2], lv) and thr[b] == b0
