"""Pins for the oracle's counter-based generator: published known answers and the keying."""
import os

import numpy as np

import oracle


def _read_kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            words = [int(w, 16) for w in line.split()]
            assert len(words) == 10
            rows.append((words[0:4], words[4:6], words[6:10]))
    return rows


def test_known_answer_vectors(golden_dir):
    rows = _read_kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = oracle.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def test_counter_words_are_not_interchangeable():
    # a transposed counter or key word must change the output (guards the operand order)
    base = oracle.philox4x32_10([1, 2, 3, 4], [5, 6])
    assert not np.array_equal(base, oracle.philox4x32_10([2, 1, 3, 4], [5, 6]))
    assert not np.array_equal(base, oracle.philox4x32_10([1, 2, 4, 3], [5, 6]))
    assert not np.array_equal(base, oracle.philox4x32_10([1, 2, 3, 4], [6, 5]))


def test_uniform_keying_by_seed_and_element_index():
    # element i takes word i%4 of the block with counter (lo32(i/4), hi32(i/4), 0, 0), key = seed halves
    seed = 0x0123456789ABCDEF
    for index in [0, 1, 2, 3, 4, 7, 1023, (1 << 34) + 5, (1 << 40) + 2]:
        block = index >> 2
        r = oracle.philox4x32_10([block & 0xFFFFFFFF, block >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        want = np.float32(int(r[index & 3]) >> 8) * np.float32(2.0 ** -24)
        assert np.float32(oracle.uniform(seed, index)) == want


def test_uniform_known_values_from_zero_block(golden_dir):
    # seed 0, elements 0..3 read the four words of the all-zero known answer
    _, _, want = _read_kat(golden_dir)[0]
    for i in range(4):
        assert oracle.uniform(0, i) == (want[i] >> 8) / float(1 << 24)


def test_uniform_range_grid_and_flatness():
    n = 40000
    u = np.array([oracle.uniform(7, i) for i in range(n)], dtype=np.float64)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * (1 << 24) == np.round(u * (1 << 24)))
    assert abs(u.mean() - 0.5) < 4 * (1 / np.sqrt(12 * n))
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    chi2 = ((hist - n / 16) ** 2 / (n / 16)).sum()
    assert chi2 < 50  # 15 degrees of freedom, p ~ 1e-5
