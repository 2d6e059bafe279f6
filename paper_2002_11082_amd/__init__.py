"""Per-bucket optimal gradient quantization (BinGrad-b / ORQ, arXiv 2002.11082) on MI355X.

The product is libogq.so (HIP kernels behind the C ABI declared in include/ogq.h); this package
is the thin Python binding plus the seeded synthetic-input generators used by tests and bench.
"""
from .binding import (BINGRAD_B, BINGRAD_PB, EVEN, LINEAR, MAX_WORKERS, ORQ, ORQ_PAPER, SCALED_SIGN, OgqError, Params, lib, make_params, ogq_codes_bytes,
                      ogq_dequantize_average, ogq_dequantize_average_raw, ogq_levels_count, ogq_levels_per_bucket,
                      ogq_num_buckets,
                      ogq_probe_copy, ogq_probe_read, ogq_quantize, ogq_quantize_raw, ogq_strerror)

__all__ = [
    "BINGRAD_B", "BINGRAD_PB", "ORQ", "ORQ_PAPER", "SCALED_SIGN", "EVEN", "LINEAR", "MAX_WORKERS", "ogq_levels_per_bucket", "OgqError", "Params", "lib", "make_params", "ogq_codes_bytes",
    "ogq_dequantize_average", "ogq_dequantize_average_raw", "ogq_levels_count", "ogq_num_buckets", "ogq_probe_copy",
    "ogq_probe_read", "ogq_quantize", "ogq_quantize_raw", "ogq_strerror",
]
