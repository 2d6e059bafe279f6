"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, run the CPU oracle
on the same seeded input, and compare element by element under the acceptance rules:
  packed codes bit-exact except elements within 1e-6 relative of a decision boundary (counted),
  levels within 1e-5 relative, decoded averages within 1e-6 relative.
Expected values always come from the oracle, never from the HIP path."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2002_11082_amd as ogq

LEVEL_RTOL = 1e-5
BOUNDARY_RTOL = 1e-6
AVG_RTOL = 1e-6


def unpack_words(words: np.ndarray, n: int, bits: int) -> np.ndarray:
    """numpy-only unpacking of the bit-plane layout (independent of both implementations)."""
    w = words.view(np.uint64).reshape(-1, bits)
    lanes = np.arange(64, dtype=np.uint64)
    codes = np.zeros((w.shape[0], 64), dtype=np.uint8)
    for p in range(bits):
        codes |= (((w[:, p:p + 1] >> lanes) & np.uint64(1)).astype(np.uint8) << p)
    return codes.reshape(-1)[:n]


def gpu_quantize(g: np.ndarray, params, device="cuda:0"):
    dg = torch.from_numpy(g).to(device)
    levels, codes = ogq.ogq_quantize(dg, params)
    torch.cuda.synchronize()
    n = g.size
    nl = ogq.ogq_levels_count(n, params)
    nw = ogq.ogq_codes_bytes(n, params) // 8
    return levels[:nl].cpu().numpy(), codes[:nw].cpu().numpy().view(np.uint64), (levels, codes)


def check_quantize(g: np.ndarray, bucket_size: int, bits: int, scheme: int, level_iters: int = 0, seed: int = 0,
                   index_offset: int = 0, buckets=None, tag: str = "", clip_factor: float = 0.0):
    """Quantize g on the GPU and with the oracle and compare.  `buckets`: optional list of bucket
    indices to check (sampled comparison at full sizes); None = every bucket.
    Returns (device levels, device codes, report dict)."""
    n = g.size
    params = ogq.make_params(bucket_size, bits, scheme, level_iters, seed, index_offset, clip_factor)
    s = ogq.ogq_levels_per_bucket(params)
    assert s == oracle.levels_per_bucket(scheme, bits)
    print(f"[parity] {tag} n={n} d={bucket_size} bits={bits} scheme={scheme} iters={level_iters} seed={seed} "
          f"offset={index_offset} clip={clip_factor}", flush=True)
    lv_gpu, words_gpu, dev = gpu_quantize(g, params)
    nb = (n + bucket_size - 1) // bucket_size
    assert lv_gpu.size == nb * s and words_gpu.size == ((n + 63) // 64) * bits
    codes_gpu = unpack_words(words_gpu, n, bits)
    # pad bits of the last group are zero
    if n % 64:
        pad = np.uint64((~((1 << (n % 64)) - 1)) & (2 ** 64 - 1))
        assert all(int(x) & int(pad) == 0 for x in words_gpu[-bits:])

    if buckets is None:
        lv_ref, codes_ref, thr_ref = oracle.quantize_codes(g, bucket_size, bits, scheme, level_iters, seed,
                                                           index_offset, clip_factor)
        sel = np.arange(nb)
        lv_g = lv_gpu.reshape(nb, s)
        lv_r = lv_ref.reshape(nb, s)
        cg, cr = codes_gpu, codes_ref
        gv = g if clip_factor == 0 else np.concatenate(
            [oracle.clip_bucket(g[i:i + bucket_size], clip_factor) for i in range(0, n, bucket_size)])
        thr = np.repeat(thr_ref, bucket_size)[:n]
        lvl_ok_elem = None
    else:
        sel = np.array(sorted(set(int(b) for b in buckets)))
        lv_r = np.zeros((sel.size, s), np.float32)
        parts_c, parts_g, parts_v, parts_t = [], [], [], []
        for i, b in enumerate(sel):
            lo, hi = b * bucket_size, min((b + 1) * bucket_size, n)
            l, c, t = oracle.quantize_codes(g[lo:hi], bucket_size, bits, scheme, level_iters, seed,
                                            index_offset + lo, clip_factor)
            lv_r[i] = l
            parts_c.append(c)
            parts_g.append(codes_gpu[lo:hi])
            parts_v.append(g[lo:hi] if clip_factor == 0 else oracle.clip_bucket(g[lo:hi], clip_factor))
            parts_t.append(np.full(hi - lo, t[0], np.float32))
        lv_g = lv_gpu.reshape(nb, s)[sel]
        cr, cg = np.concatenate(parts_c), np.concatenate(parts_g)
        gv, thr = np.concatenate(parts_v), np.concatenate(parts_t)

    # levels
    scale = np.maximum(np.abs(lv_g), np.abs(lv_r))
    lv_bad = np.abs(lv_g.astype(np.float64) - lv_r.astype(np.float64)) > LEVEL_RTOL * scale
    bad_buckets = np.flatnonzero(lv_bad.any(axis=1))
    # codes
    diff = np.flatnonzero(cg != cr)
    excused = 0
    if diff.size:
        if scheme == ogq.BINGRAD_B:
            v, t = gv[diff].astype(np.float64), thr[diff].astype(np.float64)
            near = np.abs(v - t) <= BOUNDARY_RTOL * np.maximum(np.abs(v), np.abs(t))
            excused = int(near.sum())
        else:
            excused = 0  # same fp32 operations on equal levels leave no boundary cases
    report = {"buckets_checked": int(sel.size), "level_mismatch_buckets": int(bad_buckets.size),
              "code_mismatches": int(diff.size), "code_mismatches_at_boundary": excused,
              "levels_bit_equal": bool(np.array_equal(lv_g, lv_r))}
    print(f"[parity] {tag} report {report}", flush=True)
    if buckets is None:
        report["oracle_levels"], report["oracle_codes"] = lv_ref, codes_ref  # what the oracle computed, for reuse
    assert bad_buckets.size == 0, (tag, "levels differ in buckets", sel[bad_buckets][:10],
                                   lv_g[bad_buckets][:3], lv_r[bad_buckets][:3])
    assert diff.size == excused, (tag, "code mismatches away from a decision boundary", diff[:10])
    return dev[0], dev[1], report


def term_scale(levels_list, codes_list, n, bucket_size, bits, stride=0):
    """mean over workers of |decoded term| per element (denominator of the averaging tolerance)."""
    acc = np.zeros(n, np.float64)
    for lv, w in zip(levels_list, codes_list):
        acc += np.abs(oracle.dequantize_average([w], [lv], n, bucket_size, bits, stride).astype(np.float64))
    return acc / len(levels_list)


def check_average(out_gpu: np.ndarray, ref: np.ndarray, scale: np.ndarray, tag: str = "", skip=None):
    denom = np.maximum(np.abs(ref.astype(np.float64)), scale)
    err = np.abs(out_gpu.astype(np.float64) - ref.astype(np.float64))
    bad = err > AVG_RTOL * denom
    if skip is not None:
        bad &= ~skip
    worst = float((err / np.maximum(denom, 1e-300)).max()) if err.size else 0.0
    print(f"[parity] {tag} decode-average worst relative error {worst:.3e}, bad {int(bad.sum())}", flush=True)
    assert not bad.any(), (tag, np.flatnonzero(bad)[:10])
