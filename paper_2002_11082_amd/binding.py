"""ctypes binding of libogq's C ABI (include/ogq.h).  Argument marshalling only: every step of the
path runs in the HIP kernels.  There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
# OGQ_LIBRARY names another build of the same C ABI (e.g. a host build with sanitizers for the argument checks).
LIB_PATH = os.environ.get("OGQ_LIBRARY") or os.path.join(_PKG, "libogq.so")

BINGRAD_B = 0
ORQ = 1
BINGRAD_PB = 2
ORQ_PAPER = 3
SCALED_SIGN = 4
EVEN = 5
LINEAR = 6
MAX_WORKERS = 64
PROBE_SINK_FLOATS = 8192


class Params(ctypes.Structure):
    """ogq_params_t"""
    _fields_ = [
        ("bucket_size", ctypes.c_uint32),
        ("bits", ctypes.c_uint32),
        ("scheme", ctypes.c_uint32),
        ("level_iters", ctypes.c_uint32),
        ("seed", ctypes.c_uint64),
        ("index_offset", ctypes.c_uint64),
        ("clip_factor", ctypes.c_float),
        ("reserved", ctypes.c_uint32),
    ]


class OgqError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libogq status {status}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2002_11082_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        sz, vp, u32 = ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint32
        pp = ctypes.POINTER(Params)
        L.ogq_levels_per_bucket.argtypes = [pp]
        L.ogq_levels_per_bucket.restype = sz
        for name in ("ogq_num_buckets", "ogq_levels_count", "ogq_codes_bytes"):
            f = getattr(L, name)
            f.argtypes = [sz, pp]
            f.restype = sz
        L.ogq_quantize.argtypes = [vp, sz, pp, vp, vp, vp]
        L.ogq_quantize.restype = ctypes.c_int
        L.ogq_dequantize_average.argtypes = [vp, vp, u32, sz, pp, vp, vp]
        L.ogq_dequantize_average.restype = ctypes.c_int
        L.ogq_probe_read.argtypes = [vp, sz, vp, vp]
        L.ogq_probe_read.restype = ctypes.c_int
        L.ogq_probe_copy.argtypes = [vp, vp, sz, vp]
        L.ogq_probe_copy.restype = ctypes.c_int
        L.ogq_strerror.argtypes = [ctypes.c_int]
        L.ogq_strerror.restype = ctypes.c_char_p
        L.ogq_last_hip_error.argtypes = []
        L.ogq_last_hip_error.restype = ctypes.c_int
        _lib = L
    return _lib


def make_params(bucket_size: int, bits: int, scheme: int, level_iters: int = 0, seed: int = 0,
                index_offset: int = 0, clip_factor: float = 0.0) -> Params:
    return Params(bucket_size, bits, scheme, level_iters, seed, index_offset, clip_factor, 0)


def ogq_strerror(status: int) -> str:
    return lib().ogq_strerror(status).decode()


def _check(status: int) -> None:
    if status != 0:
        raise OgqError(status, ogq_strerror(status))


def ogq_levels_per_bucket(params: Params) -> int:
    return lib().ogq_levels_per_bucket(ctypes.byref(params))


def ogq_num_buckets(n: int, params: Params) -> int:
    return lib().ogq_num_buckets(n, ctypes.byref(params))


def ogq_levels_count(n: int, params: Params) -> int:
    return lib().ogq_levels_count(n, ctypes.byref(params))


def ogq_codes_bytes(n: int, params: Params) -> int:
    return lib().ogq_codes_bytes(n, ctypes.byref(params))


def ogq_quantize_raw(d_grad: int, n: int, params: Params, d_levels: int, d_codes: int, stream: int = 0) -> int:
    """Raw call: device addresses as integers; returns the status code."""
    return lib().ogq_quantize(d_grad, n, ctypes.byref(params), d_levels, d_codes, stream)


def ogq_dequantize_average_raw(d_codes, d_levels, n: int, params: Params, d_out: int, stream: int = 0) -> int:
    """Raw call: d_codes / d_levels are sequences of device addresses; returns the status code."""
    W = len(d_codes)
    cp = (ctypes.c_void_p * max(W, 1))(*d_codes)
    lp = (ctypes.c_void_p * max(W, 1))(*d_levels)
    return lib().ogq_dequantize_average(ctypes.addressof(cp), ctypes.addressof(lp), W, n, ctypes.byref(params),
                                        d_out, stream)


def _stream_of(t) -> int:
    import torch
    return torch.cuda.current_stream(t.device).cuda_stream


def _require(ok: bool, what: str) -> None:
    if not ok:
        raise ValueError(what)


def _holds(t, dtype, elements: int, what: str) -> None:
    """A contiguous CUDA tensor of `dtype` with at least `elements` elements (the kernels trust these sizes)."""
    _require(t.is_cuda and t.dtype == dtype and t.is_contiguous(), f"{what}: expected a contiguous CUDA tensor of {dtype}")
    _require(t.numel() >= elements, f"{what}: {t.numel()} elements, at least {elements} needed")


def ogq_quantize(grad, params: Params, levels=None, codes=None):
    """grad: 1-D contiguous float32 CUDA tensor.  Returns (levels float32[levels_count],
    codes int64[codes_bytes/8]) on the same device, enqueued on torch's current stream."""
    import torch
    _require(grad.dim() == 1, "grad: expected a 1-D tensor")
    _holds(grad, torch.float32, 0, "grad")
    n = grad.numel()
    n_levels, n_words = ogq_levels_count(n, params), ogq_codes_bytes(n, params) // 8
    if levels is None:
        levels = torch.empty(max(n_levels, 4), dtype=torch.float32, device=grad.device)
    if codes is None:
        codes = torch.empty(max(n_words, 2), dtype=torch.int64, device=grad.device)
    _holds(levels, torch.float32, n_levels, "levels")
    _holds(codes, torch.int64, n_words, "codes")
    _require(levels.device == grad.device and codes.device == grad.device, "levels / codes: not on grad's device")
    _check(ogq_quantize_raw(grad.data_ptr(), n, params, levels.data_ptr(), codes.data_ptr(), _stream_of(grad)))
    return levels, codes


def ogq_dequantize_average(codes_list, levels_list, n: int, params: Params, out=None):
    """codes_list / levels_list: one CUDA tensor per worker as returned by ogq_quantize.
    Returns float32[n]."""
    import torch
    _require(len(codes_list) == len(levels_list) and len(codes_list) > 0, "one codes and one levels tensor per worker")
    dev = codes_list[0].device
    n_levels, n_words = ogq_levels_count(n, params), ogq_codes_bytes(n, params) // 8
    for w, (c, l) in enumerate(zip(codes_list, levels_list)):
        _holds(c, torch.int64, n_words, f"codes of worker {w}")
        _holds(l, torch.float32, n_levels, f"levels of worker {w}")
        _require(c.device == dev and l.device == dev, f"worker {w}: tensors on different devices")
    if out is None:
        out = torch.empty(max(n, 4), dtype=torch.float32, device=dev)[:n]
    _holds(out, torch.float32, n, "out")
    _require(out.device == dev, "out: not on the workers' device")
    _check(ogq_dequantize_average_raw([c.data_ptr() for c in codes_list], [l.data_ptr() for l in levels_list], n,
                                      params, out.data_ptr(), _stream_of(out)))
    return out


def ogq_probe_read(src, sink=None):
    import torch
    if sink is None:
        sink = torch.empty(PROBE_SINK_FLOATS, dtype=torch.float32, device=src.device)
    _check(lib().ogq_probe_read(src.data_ptr(), src.numel(), sink.data_ptr(), _stream_of(src)))
    return sink


def ogq_probe_copy(src, dst):
    _check(lib().ogq_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel(), _stream_of(src)))
    return dst
