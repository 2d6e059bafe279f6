"""Pins of the oracle's comparison level rules (Section 5, list of methods: Scaled SignSGD, QSGD-s /
TernGrad with evenly spaced levels, Linear-s) against closed forms, library routines and the ordering of
the quantization errors the paper reports (Section 5.1, discussion of the training curves)."""
import numpy as np
import pytest

import oracle


def _rounding_error(x, levels):
    """Expected squared error of random rounding: sum (b_{k+1} - v)(v - b_k) (variance term of Section 3.1)."""
    lv = np.asarray(levels, np.float64)
    x = np.asarray(x, np.float64)
    k = np.clip(np.searchsorted(lv, x, side="right") - 1, 0, lv.size - 2)
    return float(np.sum((lv[k + 1] - x) * (x - lv[k])))


def _two_level_error(x, levels, threshold):
    x = np.asarray(x, np.float64)
    q = np.where(x >= threshold, float(levels[1]), float(levels[0]))
    return float(np.sum((x - q) ** 2))


# ---- Scaled SignSGD ------------------------------------------------------------------------------
def test_scaled_sign_levels_are_the_mean_magnitude():
    rng = np.random.default_rng(0)
    for n in (1, 2, 63, 512, 2048):
        x = (rng.standard_t(3, n) * 1e-2).astype(np.float32)
        lv = oracle.scaled_sign_bucket(x)
        m = np.float32(np.abs(x.astype(np.float64)).sum() / n)
        assert lv[1] == m and lv[0] == -m


def test_scaled_sign_hand_example_and_reconstruction():
    x = np.array([3.0, -1.0, 0.5, -0.5, 0.0, 1.0], np.float32)  # ||x||_1 = 6, dim 6 -> m = 1
    lv, codes, thr = oracle.quantize_codes(x, 64, 1, oracle.SCALED_SIGN)
    assert lv.tolist() == [-1.0, 1.0]
    assert codes.tolist() == [1, 0, 1, 0, 1, 1]   # the zero goes to +m
    # Q(G) = m * sign(G) on the non-zero elements
    nz = x != 0
    assert np.array_equal(lv[codes][nz], np.sign(x)[nz])


def test_bingrad_b_on_sign_paired_data_is_scaled_sign():
    """For a bucket that holds every value with both signs the mean is 0 and both conditional means have
    the magnitude mean |v|: the two rules coincide (Section 3.2)."""
    rng = np.random.default_rng(1)
    a = np.abs(rng.normal(0, 1e-3, 300)).astype(np.float32) + np.float32(1e-6)
    x = np.concatenate([a, -a])
    rng.shuffle(x)
    lv_b, b0 = oracle.bingrad_bucket(x, 0)
    lv_s = oracle.scaled_sign_bucket(x)
    assert b0 == 0
    np.testing.assert_allclose(lv_b, lv_s, rtol=1e-6)


# ---- evenly spaced levels (QSGD-s, TernGrad) -----------------------------------------------------
def test_even_levels_hand_example_and_terngrad():
    assert oracle.even_levels_bucket(np.array([-4.0, 1.0, 2.0], np.float32), 5).tolist() == [-4.0, -2.0, 0.0, 2.0, 4.0]
    assert oracle.even_levels_bucket(np.array([0.25, -0.125, 3.0], np.float32), 3).tolist() == [-3.0, 0.0, 3.0]
    assert oracle.even_levels_bucket(np.zeros(7, np.float32), 9).tolist() == [0.0] * 9


@pytest.mark.parametrize("s", [3, 5, 9])
def test_even_levels_symmetric_equally_spaced(s):
    rng = np.random.default_rng(s)
    x = (rng.laplace(0, 5e-4, 2048)).astype(np.float32)
    lv = oracle.even_levels_bucket(x, s).astype(np.float64)
    M = float(np.abs(x).max())
    assert lv[0] == -M and lv[-1] == M and lv[(s - 1) // 2] == 0.0
    np.testing.assert_array_equal(lv, -lv[::-1])
    np.testing.assert_allclose(np.diff(lv), 2 * M / (s - 1), rtol=1e-6)
    # levels are the correctly rounded exact values M (2k - (s-1)) / (s-1)
    exact = [np.float32(M * (2 * k - (s - 1)) / (s - 1)) for k in range(s)]
    assert lv.astype(np.float32).tolist() == exact


# ---- Linear-s --------------------------------------------------------------------------------------
def test_linear_levels_hand_examples():
    x = np.array([5, 1, 3, 2, 4], np.float32)
    assert oracle.linear_levels_bucket(x, 3).tolist() == [1.0, 3.0, 5.0]
    assert oracle.linear_levels_bucket(x, 5).tolist() == [1.0, 2.0, 3.0, 4.0, 5.0]
    assert oracle.linear_levels_bucket(np.array([2, 1], np.float32), 3).tolist() == [1.0, 1.0, 2.0]
    assert oracle.linear_levels_bucket(np.array([7], np.float32), 5).tolist() == [7.0] * 5


@pytest.mark.parametrize("s", [3, 5, 9])
def test_linear_levels_are_numpy_lower_quantiles(s):
    rng = np.random.default_rng(10 + s)
    for n in (2, 17, 512, 2048, 4095):
        x = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
        ref = np.sort(x)[[(k * (n - 1)) // (s - 1) for k in range(s)]]
        assert oracle.linear_levels_bucket(x, s).tolist() == ref.tolist()
        if (n - 1) % (s - 1) == 0:  # fractions fall on ranks: every quantile definition agrees
            assert ref.tolist() == np.quantile(x, np.arange(s) / (s - 1), method="lower").tolist()
    x = rng.normal(0, 1, 4097).astype(np.float32)
    lv = oracle.linear_levels_bucket(x, 5)
    # equal mass between neighbouring levels
    counts = [int(((x >= lv[k]) & (x < lv[k + 1])).sum()) for k in range(4)]
    assert max(counts) - min(counts) <= 1


# ---- the encoder on the new level tables -----------------------------------------------------------
@pytest.mark.parametrize("scheme", [oracle.EVEN, oracle.LINEAR])
def test_random_rounding_on_comparison_levels_is_unbiased(scheme):
    rng = np.random.default_rng(int(scheme))
    x = rng.normal(0, 1e-3, 256).astype(np.float32)
    acc = np.zeros(x.size, np.float64)
    trials = 1500
    for seed in range(trials):
        lv, codes, _ = oracle.quantize_codes(x, 256, 2, scheme, seed=seed)
        assert codes.max() <= 2
        acc += lv[codes].astype(np.float64)
    spread = float(lv[-1] - lv[0])
    assert np.abs(acc / trials - x).max() < 5 * 0.5 * spread / np.sqrt(trials)


def test_level_counts_of_the_comparison_rules():
    for bits, s in ((2, 3), (3, 5), (4, 9)):
        assert oracle.levels_per_bucket(oracle.EVEN, bits) == s
        assert oracle.levels_per_bucket(oracle.LINEAR, bits) == s
    assert oracle.levels_per_bucket(oracle.SCALED_SIGN, 1) == 2
    for scheme, bits in ((oracle.SCALED_SIGN, 2), (oracle.EVEN, 1), (oracle.LINEAR, 1)):
        with pytest.raises(ValueError):
            oracle.levels_per_bucket(scheme, bits)


# ---- ordering of the quantization errors (Section 5.1) ---------------------------------------------
def _buckets():
    rng = np.random.default_rng(2020)
    n = 2048
    yield "normal", rng.normal(0, 1e-3, n).astype(np.float32)
    yield "laplace", rng.laplace(0, 5e-4, n).astype(np.float32)
    yield "student-t3", (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    yield "mixture", np.where(rng.random(n) < 0.9, rng.normal(0, 1e-4, n), rng.normal(0, 1e-2, n)).astype(np.float32)
    yield "shifted", rng.normal(3e-4, 1e-3, n).astype(np.float32)


@pytest.mark.parametrize("s", [3, 5, 9])
def test_orq_has_the_smallest_rounding_error_for_its_level_count(s):
    """ORQ-s beats the evenly spaced and the equal-mass levels with the same s on every distribution, and
    the gap widens on heavy tails."""
    for name, x in _buckets():
        e_orq = _rounding_error(x, oracle.orq_levels_bucket(x, s, 0))
        e_even = _rounding_error(x, oracle.even_levels_bucket(x, s))
        e_lin = _rounding_error(x, oracle.linear_levels_bucket(x, s))
        assert e_orq <= e_lin * (1 + 1e-9), (name, s)
        assert e_orq < e_even, (name, s)
        if s > 3 and name == "student-t3":
            assert e_orq < 0.5 * min(e_even, e_lin)


def test_bingrad_b_error_against_scaled_sign():
    """Same error on symmetric buckets (the rules nearly coincide), smaller once the bucket mean moves off 0."""
    for name, x in _buckets():
        lv_b, b0 = oracle.bingrad_bucket(x, 0)
        e_b = _two_level_error(x, lv_b, b0)
        e_s = _two_level_error(x, oracle.scaled_sign_bucket(x), 0.0)
        assert e_b <= e_s * 1.01, name
        if name == "shifted":
            assert e_b < 0.97 * e_s


def test_whole_gradient_driver_uses_the_rule_it_is_asked_for():
    """Per-bucket level tables of the gradient-level driver equal the per-bucket functions, bucket by bucket,
    the shorter last bucket included (hand values for the first bucket of the evenly spaced and Linear rules)."""
    rng = np.random.default_rng(5)
    d, n = 64, 64 * 3 + 17
    x = rng.normal(0, 1, n).astype(np.float32)
    x[:64] = np.arange(-32, 32, dtype=np.float32)          # first bucket: -32 .. 31
    for scheme, bits, per_bucket in ((oracle.EVEN, 3, lambda b: oracle.even_levels_bucket(b, 5)),
                                     (oracle.LINEAR, 3, lambda b: oracle.linear_levels_bucket(b, 5)),
                                     (oracle.SCALED_SIGN, 1, oracle.scaled_sign_bucket)):
        lv, codes, _ = oracle.quantize_codes(x, d, bits, scheme, seed=1)
        s = oracle.levels_per_bucket(scheme, bits)
        for b in range(4):
            assert lv[b * s:(b + 1) * s].tolist() == per_bucket(x[b * d:(b + 1) * d]).tolist(), (scheme, b)
    lv, _, _ = oracle.quantize_codes(x, d, 3, oracle.EVEN)
    assert lv[:5].tolist() == [-32.0, -16.0, 0.0, 16.0, 32.0]
    lv, _, _ = oracle.quantize_codes(x, d, 3, oracle.LINEAR)
    assert lv[:5].tolist() == [-32.0, -17.0, -1.0, 15.0, 31.0]   # ranks floor(k * 63 / 4) = 0, 15, 31, 47, 63
