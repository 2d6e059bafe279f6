"""The C-ABI library loads on a machine without a GPU, exports every symbol the header declares,
and its host-side logic (size arithmetic, argument validation) behaves as documented.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

import paper_2002_11082_amd as ogq
from paper_2002_11082_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2002_11082_amd import build
        build.build()
    return ogq.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ogq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ogq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"ogq_quantize", "ogq_dequantize_average", "ogq_num_buckets", "ogq_levels_count", "ogq_codes_bytes",
            "ogq_strerror"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_params_struct_layout_matches_the_header():
    assert ctypes.sizeof(ogq.Params) == 40
    assert ogq.Params.seed.offset == 16 and ogq.Params.index_offset.offset == 24
    assert ogq.Params.clip_factor.offset == 32


def test_size_queries(lib):
    p = ogq.make_params(2048, 1, ogq.BINGRAD_B)
    assert ogq.ogq_num_buckets(25_600_000, p) == 12_500
    assert ogq.ogq_levels_count(25_600_000, p) == 25_000
    assert ogq.ogq_codes_bytes(25_600_000, p) == 3_200_000
    p = ogq.make_params(4096, 3, ogq.ORQ)
    assert ogq.ogq_num_buckets(143_700_000, p) == 35_084       # 35,083 full buckets + a tail of 32
    assert ogq.ogq_levels_count(143_700_000, p) == 35_084 * 8
    assert ogq.ogq_codes_bytes(143_700_000, p) == ((143_700_000 + 63) // 64) * 3 * 8
    p = ogq.make_params(2048, 2, ogq.ORQ)
    assert ogq.ogq_num_buckets(61_100_000, p) == 29_834
    assert ogq.ogq_codes_bytes(65, p) == 2 * 2 * 8
    assert ogq.ogq_num_buckets(0, p) == 0 and ogq.ogq_codes_bytes(0, p) == 0
    # the paper's level counts 3 / 5 / 9 need 2 / 3 / 4 index bits
    for bits, s in ((2, 3), (3, 5), (4, 9)):
        p = ogq.make_params(2048, bits, ogq.ORQ_PAPER)
        assert ogq.ogq_levels_per_bucket(p) == s
        assert ogq.ogq_levels_count(25_600_000, p) == 12_500 * s
        assert ogq.ogq_codes_bytes(25_600_000, p) == 400_000 * bits * 8
    assert ogq.ogq_levels_per_bucket(ogq.make_params(2048, 1, ogq.ORQ_PAPER)) == 0
    assert ogq.ogq_levels_per_bucket(ogq.make_params(2048, 3, ogq.ORQ)) == 8
    assert ogq.ogq_levels_per_bucket(ogq.make_params(2048, 1, ogq.BINGRAD_B)) == 2
    assert ogq.ogq_levels_per_bucket(ogq.make_params(2048, 1, ogq.BINGRAD_PB)) == 2
    assert ogq.ogq_levels_per_bucket(ogq.make_params(2048, 2, ogq.BINGRAD_PB)) == 0
    # one bit per element is the paper's x32 compression (level floats not counted)
    p = ogq.make_params(512, 1, ogq.BINGRAD_B)
    assert 4 * 1_048_576 / ogq.ogq_codes_bytes(1_048_576, p) == 32


def test_argument_validation_happens_before_any_launch(lib):
    A = 0x10000  # a fake, aligned, non-null device address: never dereferenced on these paths
    ok = ogq.make_params(2048, 1, ogq.BINGRAD_B)
    q = ogq.ogq_quantize_raw
    assert q(A, 0, ok, A, A) == 0                                       # n == 0 is a no-op
    assert q(0, 100, ok, A, A) == -1
    assert q(A, 100, ok, 0, A) == -1
    assert q(A, 100, ok, A, 0) == -1
    assert q(A + 4, 100, ok, A, A) == -6
    assert q(A, 100, ogq.make_params(0, 1, ogq.BINGRAD_B), A, A) == -2
    assert q(A, 100, ogq.make_params(100, 1, ogq.BINGRAD_B), A, A) == -2
    assert q(A, 100, ogq.make_params(32768 + 64, 1, ogq.BINGRAD_B), A, A) == -2
    assert q(A, 100, ogq.make_params(2048, 2, ogq.BINGRAD_B), A, A) == -3
    assert q(A, 100, ogq.make_params(2048, 4, ogq.ORQ), A, A) == -3
    assert q(A, 100, ogq.make_params(2048, 0, ogq.ORQ), A, A) == -3
    assert q(A, 100, ogq.make_params(2048, 2, 7), A, A) == -4
    assert q(A, 100, ogq.make_params(2048, 1, ogq.ORQ_PAPER), A, A) == -3
    assert q(A, 100, ogq.make_params(2048, 5, ogq.ORQ_PAPER), A, A) == -3
    assert q(A, 100, ogq.make_params(2048, 2, ogq.ORQ, index_offset=5), A, A) == -7
    assert q(A, 100, ogq.make_params(2048, 2, ogq.ORQ, clip_factor=-1.0), A, A) == -10
    assert q(A, 100, ogq.make_params(2048, 2, ogq.ORQ, clip_factor=float('nan')), A, A) == -10
    d = ogq.ogq_dequantize_average_raw
    assert d([A], [A], 0, ok, A) == 0
    assert d([], [], 100, ok, A) == -5
    assert d([A] * 65, [A] * 65, 100, ok, A) == -5
    assert d([A], [0], 100, ok, A) == -1
    assert d([A], [A], 100, ok, 0) == -1
    assert d([A + 8], [A], 100, ok, A) == -6
    assert d([A], [A], 100, ogq.make_params(2048, 5, ogq.ORQ), A) == -3
    bad = ogq.make_params(2048, 2, ogq.ORQ)
    bad.reserved = 1                                                    # documented as "must be 0"
    assert q(A, 100, bad, A, A) == -11 and d([A], [A], 100, bad, A) == -11
    for code in range(-11, 1):
        assert ogq.ogq_strerror(code) and ogq.ogq_strerror(code) != "unknown status"
    assert lib.ogq_quantize(A, 100, None, A, A, None) == -1


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.lib()


def test_tensor_wrappers_refuse_tensors_the_kernels_could_not_trust():
    """Host tensors, wrong dtypes and mismatched worker lists are turned into errors before any pointer is taken."""
    import torch
    p = ogq.make_params(2048, 1, ogq.BINGRAD_B)
    with pytest.raises(ValueError):
        ogq.ogq_quantize(torch.zeros(4096), p)                         # host memory
    with pytest.raises(ValueError):
        ogq.ogq_quantize(torch.zeros(2, 2048), p)                      # not 1-D
    with pytest.raises(ValueError):
        ogq.ogq_dequantize_average([], [], 4096, p)                    # no workers
    with pytest.raises(ValueError):
        ogq.ogq_dequantize_average([torch.zeros(64, dtype=torch.int64)], [], 4096, p)
    with pytest.raises(ValueError):
        ogq.ogq_dequantize_average([torch.zeros(64, dtype=torch.int64)], [torch.zeros(4)], 4096, p)  # host memory
