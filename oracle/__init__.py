"""CPU oracle for per-bucket optimal gradient quantization (arXiv 2002.11082).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's ``cpu_baseline``
leg may import this package; the product package never does.  The arithmetic lives in
``ogq_oracle.c`` (plain C, double precision); this module only compiles it with gcc, loads it
with ctypes and marshals numpy arrays.  Nothing here is shared with the HIP implementation.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ogq_oracle.c")
_LIB = os.path.join(_HERE, "libogq_oracle.so")
# A test may point the loader at another build of the same source (the sanitizer build of tests/test_sanitizers.py).
_OVERRIDE = os.environ.get("OGQ_ORACLE_LIBRARY")

BINGRAD_B = 0
ORQ = 1
BINGRAD_PB = 2
ORQ_PAPER = 3
SCALED_SIGN = 4
EVEN = 5
LINEAR = 6


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add contraction, OpenMP over buckets)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not _OVERRIDE:
            build()
        L = ctypes.CDLL(_OVERRIDE or _LIB)
        u32, u64, sz = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t
        vp = ctypes.c_void_p
        L.ogq_oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.ogq_oracle_philox4x32_10.restype = None
        L.ogq_oracle_uniform.argtypes = [u64, u64]
        L.ogq_oracle_uniform.restype = ctypes.c_float
        L.ogq_oracle_bingrad_bucket.argtypes = [vp, sz, u32, vp, vp]
        L.ogq_oracle_bingrad_bucket.restype = None
        L.ogq_oracle_bingrad_pb_level.argtypes = [vp, sz]
        L.ogq_oracle_bingrad_pb_level.restype = ctypes.c_float
        L.ogq_oracle_qstar.argtypes = [vp, sz, ctypes.c_float, ctypes.c_float]
        L.ogq_oracle_qstar.restype = ctypes.c_float
        L.ogq_oracle_exact_sign.argtypes = [vp, vp, sz]
        L.ogq_oracle_exact_sign.restype = ctypes.c_int
        L.ogq_oracle_orq_levels_bucket.argtypes = [vp, sz, u32, u32, vp]
        L.ogq_oracle_orq_levels_bucket.restype = None
        L.ogq_oracle_scaled_sign_bucket.argtypes = [vp, sz, vp]
        L.ogq_oracle_scaled_sign_bucket.restype = None
        L.ogq_oracle_even_levels_bucket.argtypes = [vp, sz, u32, vp]
        L.ogq_oracle_even_levels_bucket.restype = None
        L.ogq_oracle_linear_levels_bucket.argtypes = [vp, sz, u32, vp]
        L.ogq_oracle_linear_levels_bucket.restype = None
        L.ogq_oracle_orq_encode_element.argtypes = [ctypes.c_float, vp, u32, ctypes.c_float]
        L.ogq_oracle_orq_encode_element.restype = u32
        L.ogq_oracle_pack.argtypes = [vp, sz, u32, vp]
        L.ogq_oracle_pack.restype = None
        L.ogq_oracle_unpack.argtypes = [vp, sz, u32, vp]
        L.ogq_oracle_unpack.restype = None
        L.ogq_oracle_clip_bucket.argtypes = [vp, sz, ctypes.c_float, vp]
        L.ogq_oracle_clip_bucket.restype = None
        L.ogq_oracle_quantize_codes.argtypes = [vp, sz, u32, u32, u32, u32, u64, u64, ctypes.c_float, vp, vp, vp]
        L.ogq_oracle_quantize_codes.restype = ctypes.c_int
        L.ogq_oracle_quantize.argtypes = [vp, sz, u32, u32, u32, u32, u64, u64, ctypes.c_float, vp, vp]
        L.ogq_oracle_quantize.restype = ctypes.c_int
        L.ogq_oracle_dequantize_average.argtypes = [vp, vp, u32, sz, u32, u32, u32, vp]
        L.ogq_oracle_levels_per_bucket.argtypes = [u32, u32]
        L.ogq_oracle_levels_per_bucket.restype = u32
        L.ogq_oracle_dequantize_average.restype = ctypes.c_int
        L.ogq_oracle_threads.argtypes = []
        L.ogq_oracle_threads.restype = ctypes.c_int
        L.ogq_oracle_set_threads.argtypes = [ctypes.c_int]
        L.ogq_oracle_set_threads.restype = None
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    lib().ogq_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def uniform(seed: int, index: int) -> float:
    return float(lib().ogq_oracle_uniform(seed, index))


def bingrad_bucket(g, iters: int = 0):
    """Returns (levels[2] float32, b0 float32) of one bucket."""
    g = _f32(g)
    levels = np.zeros(2, dtype=np.float32)
    b0 = np.zeros(1, dtype=np.float32)
    lib().ogq_oracle_bingrad_bucket(_ptr(g), g.size, iters, _ptr(levels), _ptr(b0))
    return levels, np.float32(b0[0])


def bingrad_pb_level(g) -> np.float32:
    g = _f32(g)
    return np.float32(lib().ogq_oracle_bingrad_pb_level(_ptr(g), g.size))


def qstar(sorted_x, L, R) -> np.float32:
    x = _f32(sorted_x)
    return np.float32(lib().ogq_oracle_qstar(_ptr(x), x.size, float(np.float32(L)), float(np.float32(R))))


def exact_sign(values, coefficients) -> int:
    """Sign (-1, 0, +1) of sum_i coefficients[i] * values[i], exactly; |coefficient| < 2^20."""
    v = _f32(values)
    c = np.ascontiguousarray(coefficients, dtype=np.int64)
    assert v.shape == c.shape and v.ndim == 1
    return int(lib().ogq_oracle_exact_sign(_ptr(v), _ptr(c), v.size))


def orq_levels_bucket(g, s: int, sweeps: int = 0) -> np.ndarray:
    g = _f32(g)
    levels = np.zeros(s, dtype=np.float32)
    lib().ogq_oracle_orq_levels_bucket(_ptr(g), g.size, s, sweeps, _ptr(levels))
    return levels


def scaled_sign_bucket(g) -> np.ndarray:
    g = _f32(g)
    levels = np.zeros(2, dtype=np.float32)
    lib().ogq_oracle_scaled_sign_bucket(_ptr(g), g.size, _ptr(levels))
    return levels


def even_levels_bucket(g, s: int) -> np.ndarray:
    g = _f32(g)
    levels = np.zeros(s, dtype=np.float32)
    lib().ogq_oracle_even_levels_bucket(_ptr(g), g.size, s, _ptr(levels))
    return levels


def linear_levels_bucket(g, s: int) -> np.ndarray:
    g = _f32(g)
    levels = np.zeros(s, dtype=np.float32)
    lib().ogq_oracle_linear_levels_bucket(_ptr(g), g.size, s, _ptr(levels))
    return levels


def orq_encode_element(v, levels, u) -> int:
    lv = _f32(levels)
    return int(lib().ogq_oracle_orq_encode_element(float(np.float32(v)), _ptr(lv), lv.size, float(np.float32(u))))


def pack(codes, bits: int) -> np.ndarray:
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    words = np.zeros(((c.size + 63) // 64) * bits, dtype=np.uint64)
    lib().ogq_oracle_pack(_ptr(c), c.size, bits, _ptr(words))
    return words


def unpack(words, n: int, bits: int) -> np.ndarray:
    w = np.ascontiguousarray(words, dtype=np.uint64)
    assert w.size >= ((n + 63) // 64) * bits
    codes = np.zeros(n, dtype=np.uint8)
    lib().ogq_oracle_unpack(_ptr(w), n, bits, _ptr(codes))
    return codes


def levels_per_bucket(scheme: int, bits: int) -> int:
    s = int(lib().ogq_oracle_levels_per_bucket(scheme, bits))
    if s == 0:
        raise ValueError(f"bad scheme/bits combination ({scheme}, {bits})")
    return s


def clip_bucket(g, c: float) -> np.ndarray:
    g = _f32(g)
    out = np.zeros_like(g)
    lib().ogq_oracle_clip_bucket(_ptr(g), g.size, float(c), _ptr(out))
    return out


def quantize_codes(g, bucket_size: int, bits: int, scheme: int, level_iters: int = 0, seed: int = 0,
                   index_offset: int = 0, clip_factor: float = 0.0):
    """Returns (levels [num_buckets*levels_per_bucket] f32, codes [n] u8, thresholds [num_buckets] f32)."""
    g = _f32(g)
    n = g.size
    nb = (n + bucket_size - 1) // bucket_size
    levels = np.zeros(nb * levels_per_bucket(scheme, bits), dtype=np.float32)
    codes = np.zeros(n, dtype=np.uint8)
    thresholds = np.zeros(nb, dtype=np.float32)
    rc = lib().ogq_oracle_quantize_codes(_ptr(g), n, bucket_size, bits, scheme, level_iters, seed,
                                         index_offset, float(clip_factor), _ptr(levels), _ptr(codes), _ptr(thresholds))
    if rc != 0:
        raise ValueError(f"oracle quantize_codes rejected its arguments (rc={rc})")
    return levels, codes, thresholds


def quantize(g, bucket_size: int, bits: int, scheme: int, level_iters: int = 0, seed: int = 0,
             index_offset: int = 0, clip_factor: float = 0.0):
    """Returns (levels f32, packed code words u64)."""
    g = _f32(g)
    n = g.size
    nb = (n + bucket_size - 1) // bucket_size
    levels = np.zeros(nb * levels_per_bucket(scheme, bits), dtype=np.float32)
    words = np.zeros(((n + 63) // 64) * bits, dtype=np.uint64)
    rc = lib().ogq_oracle_quantize(_ptr(g), n, bucket_size, bits, scheme, level_iters, seed, index_offset,
                                   float(clip_factor), _ptr(levels), _ptr(words))
    if rc != 0:
        raise ValueError(f"oracle quantize rejected its arguments (rc={rc})")
    return levels, words


def dequantize_average(words_list, levels_list, n: int, bucket_size: int, bits: int, stride: int = 0) -> np.ndarray:
    """stride = levels per bucket (default 2^bits)."""
    W = len(words_list)
    stride = stride or (1 << bits)
    assert W == len(levels_list) and W > 0
    ws = [np.ascontiguousarray(w, dtype=np.uint64) for w in words_list]
    ls = [_f32(l) for l in levels_list]
    wp = (ctypes.c_void_p * W)(*[_ptr(w) for w in ws])
    lp = (ctypes.c_void_p * W)(*[_ptr(l) for l in ls])
    out = np.zeros(n, dtype=np.float32)
    rc = lib().ogq_oracle_dequantize_average(ctypes.addressof(wp), ctypes.addressof(lp), W, n, bucket_size,
                                             bits, stride, _ptr(out))
    if rc != 0:
        raise ValueError(f"oracle dequantize_average rejected its arguments (rc={rc})")
    return out


def threads() -> int:
    return int(lib().ogq_oracle_threads())


def set_threads(t: int) -> None:
    lib().ogq_oracle_set_threads(int(t))
