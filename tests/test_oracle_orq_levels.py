"""Pins for the ORQ level solver of the oracle (Theorem 1, its remarks, Corollary 1, Algorithm 1).

Everything is checked in exact rational arithmetic against exhaustive search on tiny buckets, so
that a wrong sign, a dropped term, an off-by-one rank or a swapped bound in the oracle fails.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle


def F(x):
    return Fraction(float(np.float32(x)))


def rounding_error(values, levels):
    """D = sum over elements of (v - b_k)(b_{k+1} - v), the variance of random rounding
    between the neighbouring levels (proof of Theorem 1).  Exact."""
    lv = sorted(F(b) for b in levels)
    total = Fraction(0)
    for v in values:
        v = F(v)
        assert lv[0] <= v <= lv[-1]
        best = None
        for a, b in zip(lv[:-1], lv[1:]):
            if a <= v <= b:
                e = (v - a) * (b - v)
                best = e if best is None else min(best, e)
        total += best
    return total


def tiny_bucket(rng, n, kind):
    if kind == "normal":
        return rng.normal(0, 1e-3, n).astype(np.float32)
    if kind == "ints":  # many duplicates
        return rng.integers(-4, 5, n).astype(np.float32)
    if kind == "heavy":
        return (rng.standard_t(3, n) * 1e-2).astype(np.float32)
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["normal", "ints", "heavy"])
def test_qstar_minimises_error_over_points_and_midpoints(kind):
    rng = np.random.default_rng(11)
    for trial in range(120):
        n = int(rng.integers(2, 13))
        g = tiny_bucket(rng, n, kind)
        x = np.sort(g)
        # outer levels: either the bucket ends or two inner data values
        if trial % 3 == 0 and n >= 4:
            i, j = sorted(rng.choice(n, 2, replace=False))
            L, R = x[i], x[j]
        else:
            L, R = x[0], x[-1]
        b = oracle.qstar(x, L, R)
        if not (L < R):
            assert b == L
            continue
        inside = [v for v in x if L <= v <= R]
        cands = sorted(set(F(v) for v in inside))
        cands += [(a + c) / 2 for a, c in zip(cands[:-1], cands[1:])]

        def D(mid):
            return sum((F(v) - F(L)) * (mid - F(v)) if F(v) <= mid else (F(v) - mid) * (F(R) - F(v))
                       for v in inside)

        best = min(D(c) for c in cands)
        assert L <= b <= R
        assert b in inside  # the solve returns a data value
        assert D(F(b)) == best, (kind, trial, x, L, R, b)


def test_qstar_takes_lower_end_of_a_flat_optimum():
    # L=0, R=4, inside {0,1,3,4}: S = 8, T = 2, slope is zero between 1 and 3 -> the lower end, 1
    x = np.array([0, 1, 3, 4], dtype=np.float32)
    assert oracle.qstar(x, 0, 4) == np.float32(1)


def test_qstar_sign_change_of_theorem1_residual():
    # Theorem 1 in discrete form: h(b) = L*#{L<=v<=b} + R*#{b<v<=R} - sum_{[L,R]} v is
    # non-increasing in b; the solve returns the first data value where h <= 0.
    rng = np.random.default_rng(5)
    for _ in range(100):
        n = int(rng.integers(3, 14))
        x = np.sort(tiny_bucket(rng, n, "normal"))
        L, R = x[0], x[-1]
        b = oracle.qstar(x, L, R)

        def h(mid):
            lo = sum(1 for v in x if v <= mid)
            hi = sum(1 for v in x if v > mid)
            return F(L) * lo + F(R) * hi - sum(F(v) for v in x)

        assert h(b) <= 0
        lower = [v for v in x if v < b]
        if lower:
            assert h(max(lower)) > 0


def test_uniform_data_gives_the_midpoint():
    # Remark after Theorem 1: for uniformly spread values b_k = (b_{k-1} + b_{k+1}) / 2
    for n, want_index in [(9, 4), (101, 50), (10, 4), (3, 1)]:
        x = np.arange(n, dtype=np.float32)
        b = oracle.qstar(x, x[0], x[-1])
        assert b == x[want_index]
    x = np.arange(65, dtype=np.float32)
    lv = oracle.orq_levels_bucket(x, 5, 0)
    assert list(lv) == [0, 16, 32, 48, 64]
    lv = oracle.orq_levels_bucket(x, 9, 3)
    assert list(lv) == [0, 8, 16, 24, 32, 40, 48, 56, 64]


def test_endpoints_are_min_and_max_and_levels_are_sorted_data_values():
    rng = np.random.default_rng(3)
    for s in (3, 4, 5, 8, 9):
        for sweeps in (0, 2):
            g = tiny_bucket(rng, 200, "heavy")
            lv = oracle.orq_levels_bucket(g, s, sweeps)
            assert lv[0] == g.min() and lv[-1] == g.max()  # Corollary 1
            assert np.all(np.diff(lv) >= 0)
            assert all(v in g for v in lv)


def test_three_levels_is_the_global_optimum():
    rng = np.random.default_rng(17)
    for kind in ("normal", "ints", "heavy"):
        for _ in range(40):
            n = int(rng.integers(3, 13))
            g = tiny_bucket(rng, n, kind)
            lv = oracle.orq_levels_bucket(g, 3, 0)
            got = rounding_error(g, lv)
            best = min(rounding_error(g, [g.min(), m, g.max()]) for m in g)
            assert got == best


@pytest.mark.parametrize("s", [4, 5, 8])
def test_greedy_plus_sweeps_against_exhaustive_placement(s):
    rng = np.random.default_rng(100 + s)
    hits = cases = 0
    for trial in range(30 if s < 8 else 12):
        n = int(rng.integers(s, 12 if s < 8 else 11))
        g = tiny_bucket(rng, n, "normal" if trial % 2 else "heavy")
        x = np.sort(g)
        # exhaustive optimum over placements on data values (D is affine in each level between
        # data points, so an optimum lies on data values)
        best = None
        for combo in itertools.combinations_with_replacement(range(n), s - 2):
            d = rounding_error(g, [x[0], *[x[i] for i in combo], x[-1]])
            best = d if best is None else min(best, d)
        prev = None
        for sweeps in range(0, 6):
            d = rounding_error(g, oracle.orq_levels_bucket(g, s, sweeps))
            assert d >= best
            if prev is not None:
                assert d <= prev  # a sweep never increases the error
            prev = d
        # converged state: no single interior level can be moved to another data value with gain
        lv = oracle.orq_levels_bucket(g, s, 40)
        d_conv = rounding_error(g, lv)
        for k in range(1, s - 1):
            for v in x:
                if lv[k - 1] <= v <= lv[k + 1]:
                    trial_lv = lv.copy()
                    trial_lv[k] = v
                    assert rounding_error(g, trial_lv) >= d_conv
        cases += 1
        hits += d_conv == best
    # coordinate descent usually, not always, reaches the global optimum
    assert hits / cases > (0.6 if s < 8 else 0.3)


def test_greedy_structure_for_2K_plus_1_levels():
    # Algorithm 1 for s = 5: b_2 from the ends, then b_1 from (b_0, b_2) and b_3 from (b_2, b_4)
    rng = np.random.default_rng(9)
    g = tiny_bucket(rng, 300, "heavy")
    x = np.sort(g)
    lv = oracle.orq_levels_bucket(g, 5, 0)
    b2 = oracle.qstar(x, x[0], x[-1])
    assert lv[2] == b2
    assert lv[1] == oracle.qstar(x, x[0], b2)
    assert lv[3] == oracle.qstar(x, b2, x[-1])


def test_degenerate_buckets():
    assert list(oracle.orq_levels_bucket(np.array([0.5], np.float32), 4, 2)) == [0.5] * 4
    assert list(oracle.orq_levels_bucket(np.full(7, -2.0, np.float32), 8, 1)) == [-2.0] * 8
    lv = oracle.orq_levels_bucket(np.array([1.0, 3.0], np.float32), 4, 2)  # fewer elements than levels
    assert lv[0] == 1.0 and lv[-1] == 3.0 and np.all(np.diff(lv) >= 0) and set(lv) <= {1.0, 3.0}


def test_ideal_compression_ratio_matches_the_paper_tables(golden_dir):
    import math, os
    with open(os.path.join(golden_dir, "paper_compression_ratios.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for s, ratio in rows:
        assert abs(32 / math.log2(int(s)) - float(ratio)) < 0.06


def test_greedy_structure_for_power_of_two_levels_rounds_the_middle_index_down():
    # s = 4 (not of the paper's 2^K + 1 form): b_1 is solved between the ends, then b_2 between b_1 and b_3
    rng = np.random.default_rng(19)
    g = tiny_bucket(rng, 300, "heavy")
    x = np.sort(g)
    lv = oracle.orq_levels_bucket(g, 4, 0)
    b1 = oracle.qstar(x, x[0], x[-1])
    assert lv[1] == b1 and lv[2] == oracle.qstar(x, b1, x[-1])
    # s = 8: b_3 first, then b_1 | b_5, then b_2 | b_4 | b_6
    lv = oracle.orq_levels_bucket(g, 8, 0)
    b3 = oracle.qstar(x, x[0], x[-1])
    b1 = oracle.qstar(x, x[0], b3)
    b5 = oracle.qstar(x, b3, x[-1])
    want = [x[0], b1, oracle.qstar(x, b1, b3), b3, oracle.qstar(x, b3, b5), b5, oracle.qstar(x, b5, x[-1]), x[-1]]
    assert list(lv) == want


# ------------------------------------------------------------------------------------------------
# floor(T) of the discrete optimal condition (second remark after Theorem 1) in exact arithmetic
# ------------------------------------------------------------------------------------------------
def _as_integer(v):
    """An fp32 value as an integer multiple of 2^-149 (exact)."""
    return int(Fraction(float(np.float32(v))) * 2 ** 149)


def test_exact_sums_against_rationals():
    """The oracle's multi-word sums: sign of sum c_i v_i for values anywhere in the fp32 range (subnormals, 1e-38 next to
    1e38, sums that cancel exactly or leave one unit of 2^-149) against Python integers."""
    rng = np.random.default_rng(5)
    for trial in range(400):
        k = int(rng.integers(1, 40))
        exponents = rng.integers(-149, 128, k)
        values = (rng.uniform(1, 2, k) * 2.0 ** exponents.astype(np.float64) * rng.choice([-1, 1], k)).astype(np.float32)
        values[~np.isfinite(values)] = np.float32(3.0e38)
        coeff = rng.integers(-(1 << 19), 1 << 19, k)
        if trial % 4 == 0:  # append the terms that cancel the sum exactly, then break the tie by one smallest unit
            values = np.concatenate([values, values])
            coeff = np.concatenate([coeff, -coeff])
            if trial % 8 == 0:
                values = np.concatenate([values, [np.float32(1e-45)]])
                coeff = np.concatenate([coeff, [(-1) ** (trial // 8)]])
        expected = sum(int(c) * _as_integer(v) for v, c in zip(values, coeff))
        assert oracle.exact_sign(values, coeff) == (expected > 0) - (expected < 0), trial
    assert oracle.exact_sign([0.0, -0.0], [5, -7]) == 0
    assert oracle.exact_sign([np.float32(1e-45)], [-1]) == -1
    big = np.full(32768, 3.0e38, np.float32)
    assert oracle.exact_sign(np.concatenate([big, -big, [np.float32(1e-45)]]), np.ones(65537, np.int64)) == 1


def _expected_qstar(x, L, R):
    """The solve with floor(T) in exact integers: x sorted fp32, L < R bucket values."""
    xi = [_as_integer(v) for v in x]
    Li, Ri = _as_integer(L), _as_integer(R)
    count_le_R = sum(1 for v in xi if v <= Ri)
    S = sum(v - Li for v in xi if Li <= v <= Ri)
    m = S // (Ri - Li)            # Python's floor division of integers is exact
    rank = max(1, count_le_R - m)
    b = x[rank - 1]
    return b if b >= L else L


@pytest.mark.parametrize("n", [2048, 4096, 8192, 32768])
def test_qstar_floor_is_exact_at_real_bucket_sizes(n):
    """At the bucket sizes of the hot path the level is the element of rank #{v <= R} - floor(T) with floor(T) exact,
    whatever a floating-point sum of the terms would give: buckets whose T is exactly an integer (where a sum that is one
    rounding low picks the neighbouring element), heavy tails with a dynamic range of 2^30 and more, values next to the
    ends of the fp32 range, and ordinary data."""
    rng = np.random.default_rng(n)
    cases = []
    # T exactly an integer: the only element above L is R, thousands of unlike large values below L
    x = (-1.0e6 * (1.0 + 1.0e-3 * rng.random(n))).astype(np.float32)
    x[0], x[1] = np.float32(rng.uniform(1, 9)), np.float32(rng.uniform(1, 2) * 1e20)
    x = np.sort(x)
    cases.append((x, x[-2], x[-1]))
    cases.append((x, x[0], x[-1]))
    # T exactly an integer with many unlike terms: inside [L,R] pairs (L + a_i, R - a_i) contribute R - L each
    a = np.sort(rng.uniform(0.01, 0.4, n // 4)).astype(np.float32)
    L, R = np.float32(1.0), np.float32(2.0)
    pairs = np.concatenate([L + a, R - a])          # exact in fp32 for these magnitudes? keep only exact pairs
    ok = np.array([_as_integer(p) + _as_integer(q) == _as_integer(L) + _as_integer(R) for p, q in zip(L + a, R - a)])
    pairs = np.concatenate([(L + a)[ok], (R - a)[ok]])
    below = (-rng.lognormal(0, 3, n - pairs.size - 2)).astype(np.float32)
    x = np.sort(np.concatenate([below, [L, R], pairs]).astype(np.float32))
    cases.append((x, L, R))
    # heavy tails
    for scale in (1.0, 1e-30, 1e25):
        x = np.sort((rng.lognormal(0, 4, n) * rng.choice([-1, 1], n) * scale).astype(np.float32))
        x = x[np.isfinite(x)]
        cases.append((x, x[0], x[-1]))
        i, j = sorted(rng.choice(x.size, 2, replace=False))
        cases.append((x, x[i], x[j]))
        cases.append((x, x[x.size // 2], x[-1]))
    # subnormal values next to ordinary ones
    x = np.sort(np.concatenate([rng.normal(0, 1e-40, n // 2), rng.normal(0, 1e-3, n - n // 2)]).astype(np.float32))
    cases.append((x, x[0], x[-1]))
    cases.append((x, x[n // 4], x[3 * n // 4]))
    # ordinary data and integers (ties)
    x = np.sort(rng.normal(0, 1e-3, n).astype(np.float32))
    cases.append((x, x[0], x[-1]))
    x = np.sort(rng.integers(-50, 51, n).astype(np.float32))
    cases.append((x, x[0], x[-1]))
    cases.append((x, np.float32(-7), np.float32(12)))
    for x, L, R in cases:
        if L < R:
            assert oracle.qstar(x, L, R) == _expected_qstar(x, L, R), (n, L, R)


def test_a_floating_point_sum_would_pick_the_neighbour():
    """Why the floor is exact: a bucket where T = 3 exactly, but the terms v - L added one by one in double precision
    (in sorted order) come out below 3 (R - L), so that floor(T) would be 2 and the level one element too high."""
    L, R = np.float32(0.0), np.float32(1.0)
    # 2^54 + 1 spread over terms that a running double sum cannot hold: many tiny terms after a large one
    tiny = np.full(4096, 2.0 ** -54, np.float32)           # 4096 * 2^-54 = 2^-42
    x = np.sort(np.concatenate([[L], tiny, [np.float32(1.0 - 2.0 ** -24)], [np.float32(2.0 ** -24 - 2.0 ** -42)],
                                [R, R]]).astype(np.float32))
    # S = 2^-42 + (1 - 2^-24) + (2^-24 - 2^-42) + 1 + 1 = 3 exactly
    assert sum(_as_integer(v) for v in x) == 3 * _as_integer(R)
    running = 0.0
    for v in x[::-1]:                                       # largest first: the tiny terms are lost one by one
        running += float(v)
    assert running < 3.0
    assert oracle.qstar(x, L, R) == _expected_qstar(x, L, R)
