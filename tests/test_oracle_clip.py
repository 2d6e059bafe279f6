"""Pins for the oracle's gradient clipping (Section 5: clip(v) = sign(v) * min(|v|, c * sigma))."""
import numpy as np

import oracle


def test_hand_example():
    # mean 0, variance (9+1+0+1+9)/5 = 4, sigma 2: c = 1 clips at +-2, c = 0.5 at +-1
    g = np.array([-3, -1, 0, 1, 3], np.float32)
    assert list(oracle.clip_bucket(g, 1.0)) == [-2, -1, 0, 1, 2]
    assert list(oracle.clip_bucket(g, 0.5)) == [-1, -1, 0, 1, 1]
    assert list(oracle.clip_bucket(g, 1.5)) == [-3, -1, 0, 1, 3]


def test_threshold_is_c_times_the_population_standard_deviation():
    rng = np.random.default_rng(0)
    for n in (7, 512, 2048):
        g = (rng.standard_t(3, n) * 1e-3 + 2e-4).astype(np.float32)
        for c in (1.7, 2.5):
            out = oracle.clip_bucket(g, c)
            limit = np.float32(np.float64(np.float32(c)) * np.std(g.astype(np.float64)))  # ddof = 0, about the mean
            want = np.clip(g, -limit, limit)
            assert np.array_equal(out, want)
            assert np.all(np.sign(out) == np.sign(g)) and np.all(np.abs(out) <= np.abs(g))
            if n >= 512:
                assert (out != g).any()  # a heavy tail of this length has something beyond 2.5 sigma


def test_limiting_cases():
    rng = np.random.default_rng(1)
    g = rng.normal(0, 1e-3, 1000).astype(np.float32)
    assert np.array_equal(oracle.clip_bucket(g, 0.0), g)        # off
    assert np.array_equal(oracle.clip_bucket(g, 1e6), g)        # nothing beyond a huge threshold
    # clipping is towards zero, not towards the mean: a constant bucket has sigma = 0
    assert np.all(oracle.clip_bucket(np.full(10, 3.0, np.float32), 2.5) == 0)
    # clipping twice with the same threshold value changes nothing more than the first time allows
    once = oracle.clip_bucket(g, 2.5)
    assert np.abs(once).max() <= np.float32(2.5 * g.astype(np.float64).std()) * (1 + 1e-6)


def test_quantizers_see_the_clipped_bucket():
    rng = np.random.default_rng(2)
    g = (rng.standard_t(3, 4 * 512 + 100) * 1e-3).astype(np.float32)
    for scheme, bits in ((oracle.BINGRAD_B, 1), (oracle.ORQ, 2)):
        lv_c, codes_c, thr_c = oracle.quantize_codes(g, 512, bits, scheme, 1, seed=3, clip_factor=2.5)
        clipped = np.concatenate([oracle.clip_bucket(g[i:i + 512], 2.5) for i in range(0, g.size, 512)])
        lv_p, codes_p, thr_p = oracle.quantize_codes(clipped, 512, bits, scheme, 1, seed=3)
        assert np.array_equal(lv_c, lv_p) and np.array_equal(codes_c, codes_p) and np.array_equal(thr_c, thr_p)
    # ORQ end levels of a clipped heavy-tailed bucket are -+ the threshold (Corollary 1 on the clipped values)
    lv, _, _ = oracle.quantize_codes(g[:512], 512, 2, oracle.ORQ, 0, clip_factor=1.0)
    limit = np.float32(np.std(g[:512].astype(np.float64)))
    assert lv[0] == -limit and lv[3] == limit
