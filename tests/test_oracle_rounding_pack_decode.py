"""Pins for the oracle's random rounding (Section 3.1), its bit packing and decode-average
(server step of Algorithm 2)."""
import os

import numpy as np

import oracle


def test_rounding_is_exact_on_levels_and_stays_in_the_interval():
    lv = np.array([-2.0, -0.5, 0.25, 3.0], np.float32)
    for u in (0.0, 0.3, 1 - 2.0 ** -24):
        assert oracle.orq_encode_element(-2.0, lv, u) == 0
        assert oracle.orq_encode_element(-0.5, lv, u) == 1
        assert oracle.orq_encode_element(0.25, lv, u) == 2
        assert oracle.orq_encode_element(3.0, lv, u) == 3  # the maximum always goes to the top level
        assert oracle.orq_encode_element(-1.0, lv, u) in (0, 1)
        assert oracle.orq_encode_element(1.0, lv, u) in (2, 3)
    # probability of going up is (v - b_k) / (b_{k+1} - b_k): v = -1.25 is halfway between -2 and -0.5
    assert oracle.orq_encode_element(-1.25, lv, 0.49) == 1
    assert oracle.orq_encode_element(-1.25, lv, 0.51) == 0
    # three quarters of the way up
    assert oracle.orq_encode_element(-0.875, lv, 0.74) == 1
    assert oracle.orq_encode_element(-0.875, lv, 0.76) == 0


def test_rounding_with_repeated_levels_decodes_exactly():
    lv = np.array([1.0, 2.0, 2.0, 5.0], np.float32)
    for u in (0.0, 0.5, 0.99):
        assert lv[oracle.orq_encode_element(2.0, lv, u)] == 2.0
        assert lv[oracle.orq_encode_element(1.0, lv, u)] == 1.0
        assert lv[oracle.orq_encode_element(5.0, lv, u)] == 5.0
    lv = np.array([1.0, 1.0, 5.0, 5.0], np.float32)
    for u in (0.0, 0.5, 0.99):
        assert lv[oracle.orq_encode_element(5.0, lv, u)] == 5.0
        assert lv[oracle.orq_encode_element(1.0, lv, u)] == 1.0
    flat = np.full(4, 7.0, np.float32)
    assert flat[oracle.orq_encode_element(7.0, flat, 0.3)] == 7.0


def test_quantized_gradient_is_unbiased_with_the_rounding_variance():
    # Assumption 1 / Section 3.1: E Q(v) = v;  Var Q(v) = (v - b_k)(b_{k+1} - v) (proof of Theorem 1).
    # One bucket whose data fix the levels; M copies of a probe value each get their own draw.
    M = 30000
    for bits, seed in ((2, 5), (3, 6)):
        s = 1 << bits
        rng = np.random.default_rng(seed)
        base = rng.normal(0, 1.0, 500).astype(np.float32)
        for probe in (np.float32(0.3137), np.float32(-1.234), np.float32(0.001)):
            g = np.concatenate([base, np.full(M, probe, np.float32)])
            # bucket large enough to hold everything, so all copies share the same levels
            levels, codes, _ = oracle.quantize_codes(g, 1 << 15, bits, oracle.ORQ, 2, seed=seed * 77)
            assert levels.size == s
            dec = levels[codes[500:]].astype(np.float64)
            below = levels[levels <= probe].max()
            above = levels[levels >= probe].min()
            if below == above:
                assert np.all(dec == probe)
                continue
            var = (float(probe) - float(below)) * (float(above) - float(probe))
            assert set(np.unique(dec)) <= {float(below), float(above)}
            assert abs(dec.mean() - float(probe)) < 4.5 * np.sqrt(var / M) + 2.0 ** -24 * (above - below)
            assert abs(dec.var() - var) < 0.05 * var + 1e-12


def test_whole_vector_mean_error_shrinks_like_one_over_sqrt_trials():
    # unbiasedness over seeds for every element of a bucket
    rng = np.random.default_rng(8)
    g = rng.normal(0, 1e-3, 256).astype(np.float32)
    trials = 400
    acc = np.zeros(g.size)
    var = None
    for t in range(trials):
        levels, codes, _ = oracle.quantize_codes(g, 256, 2, oracle.ORQ, 2, seed=1000 + t)
        acc += levels[codes].astype(np.float64)
        if var is None:
            lo = np.array([levels[levels <= v].max() for v in g], np.float64)
            hi = np.array([levels[levels >= v].min() for v in g], np.float64)
            var = (g - lo) * (hi - g)
    z = (acc / trials - g) / np.sqrt(np.maximum(var, 1e-30) / trials)
    z = z[var > 0]
    assert np.abs(z).max() < 5.0 and abs(z.mean()) < 0.3


def test_draws_follow_the_global_element_index():
    # a shard quantized with index_offset reproduces the codes of the full vector
    rng = np.random.default_rng(9)
    g = rng.normal(0, 1e-3, 1024).astype(np.float32)
    lv_full, c_full, _ = oracle.quantize_codes(g, 256, 3, oracle.ORQ, 1, seed=42)
    lv_part, c_part, _ = oracle.quantize_codes(g[512:], 256, 3, oracle.ORQ, 1, seed=42, index_offset=512)
    assert np.array_equal(c_full[512:], c_part) and np.array_equal(lv_full[16:], lv_part)
    _, c_other, _ = oracle.quantize_codes(g[512:], 256, 3, oracle.ORQ, 1, seed=42, index_offset=0)
    assert not np.array_equal(c_full[512:], c_other)


def test_pack_places_bit_p_of_element_i_at_word_group_times_bits_plus_p_bit_lane():
    codes = np.zeros(130, np.uint8)
    codes[0] = 0b101
    codes[63] = 0b010
    codes[64] = 0b111
    codes[129] = 0b100
    w = oracle.pack(codes, 3)
    assert w.size == 3 * 3
    assert w[0] == 1 and w[1] == (1 << 63) and w[2] == 1          # group 0: planes 0,1,2
    assert w[3] == 1 and w[4] == 1 and w[5] == 1                   # group 1: element 64 = lane 0
    assert w[6] == 0 and w[7] == 0 and w[8] == (1 << 1)            # group 2: element 129 = lane 1
    assert np.array_equal(oracle.unpack(w, 130, 3), codes)


def test_pack_round_trip_sizes_and_zero_padding():
    rng = np.random.default_rng(10)
    for bits in (1, 2, 3, 4):
        for n in (1, 63, 64, 65, 1000):
            codes = rng.integers(0, 1 << bits, n).astype(np.uint8)
            w = oracle.pack(codes, bits)
            assert w.size == ((n + 63) // 64) * bits
            assert np.array_equal(oracle.unpack(w, n, bits), codes)
            if n % 64:
                pad_mask = np.uint64(~((1 << (n % 64)) - 1) & (2 ** 64 - 1))
                assert all(int(x) & int(pad_mask) == 0 for x in w[-bits:])
    # one bit per element: N/8 bytes, the paper's x32 ratio for two levels
    assert oracle.pack(np.zeros(64000, np.uint8), 1).nbytes * 32 == 64000 * 4


def test_decode_average_special_cases():
    rng = np.random.default_rng(12)
    n, d, bits = 700, 128, 2
    gs = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(3)]
    q = [oracle.quantize(g, d, bits, oracle.ORQ, 2, seed=50 + i) for i, g in enumerate(gs)]
    # one worker: plain decode, level looked up per bucket
    lv, codes, _ = oracle.quantize_codes(gs[0], d, bits, oracle.ORQ, 2, seed=50)
    want = lv.reshape(-1, 4)[np.arange(n) // d, codes]
    got = oracle.dequantize_average([q[0][1]], [q[0][0]], n, d, bits)
    assert np.array_equal(got, want)
    # identical workers: same as one
    got3 = oracle.dequantize_average([q[0][1]] * 3, [q[0][0]] * 3, n, d, bits)
    assert np.allclose(got3, want, rtol=2e-7, atol=0)
    # the average of three different workers is the mean of their three decodes
    singles = [oracle.dequantize_average([w], [l], n, d, bits).astype(np.float64) for l, w in q]
    avg = oracle.dequantize_average([w for _, w in q], [l for l, _ in q], n, d, bits)
    assert np.array_equal(avg, ((singles[0] + singles[1] + singles[2]) / 3).astype(np.float32))
    # worker order does not matter beyond rounding
    avg_r = oracle.dequantize_average([w for _, w in q][::-1], [l for l, _ in q][::-1], n, d, bits)
    assert np.allclose(avg, avg_r, rtol=1e-7, atol=1e-12)


def test_decode_average_by_hand():
    # two workers, one bucket of 3 elements, 1 bit: levels (-1, 2) and (0, 4)
    w0 = np.array([0b101], np.uint64)   # codes 1,0,1
    w1 = np.array([0b110], np.uint64)   # codes 0,1,1
    out = oracle.dequantize_average([w0, w1], [np.array([-1, 2], np.float32), np.array([0, 4], np.float32)],
                                    3, 64, 1)
    assert list(out) == [1.0, 1.5, 3.0]


def test_table1_sizes_used_by_the_benchmark_configs(golden_dir):
    with open(os.path.join(golden_dir, "paper_comm_time_table1.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for model, millions, ms in rows:
        t = 32 * float(millions) * 1e6 / 10e9 * 1e3
        assert abs(t - float(ms)) < (3.0 if model == "GoogLeNet" else 0.6)


def test_paper_level_counts_three_five_nine():
    # s = 2^K + 1 levels (Algorithm 1's initialisation) coded with K + 1 bits; zero sweeps = the algorithm as printed
    rng = np.random.default_rng(21)
    g = (rng.standard_t(3, 3 * 256 + 40) * 1e-3).astype(np.float32)
    for bits, s in ((2, 3), (3, 5), (4, 9)):
        assert oracle.levels_per_bucket(oracle.ORQ_PAPER, bits) == s
        lv, codes, _ = oracle.quantize_codes(g, 256, bits, oracle.ORQ_PAPER, 0, seed=4)
        assert lv.size == 4 * s and codes.max() == s - 1 and codes.min() == 0
        for b in range(4):
            seg = g[256 * b:256 * (b + 1)]
            assert np.array_equal(lv[s * b:s * (b + 1)], oracle.orq_levels_bucket(seg, s, 0))
        dec = lv.reshape(4, s)[np.arange(g.size) // 256, codes]
        # each element decodes to one of its two neighbouring levels
        table = lv.reshape(4, s)[np.arange(g.size) // 256]
        below = np.max(np.where(table <= g[:, None], table, -np.inf), axis=1)
        above = np.min(np.where(table >= g[:, None], table, np.inf), axis=1)
        assert np.all((dec == below) | (dec == above))
        words = oracle.pack(codes, bits)
        out = oracle.dequantize_average([words], [lv], g.size, 256, bits, stride=s)
        assert np.array_equal(out, dec)


def test_three_level_rounding_is_unbiased():
    rng = np.random.default_rng(22)
    g = rng.normal(0, 1e-3, 128).astype(np.float32)
    acc = np.zeros(g.size)
    trials = 600
    for t in range(trials):
        lv, codes, _ = oracle.quantize_codes(g, 128, 2, oracle.ORQ_PAPER, 0, seed=5000 + t)
        acc += lv[codes].astype(np.float64)
    lo = np.array([lv[lv <= v].max() for v in g], np.float64)
    hi = np.array([lv[lv >= v].min() for v in g], np.float64)
    var = (g - lo) * (hi - g)
    z = (acc / trials - g)[var > 0] / np.sqrt(var[var > 0] / trials)
    assert np.abs(z).max() < 5.0
