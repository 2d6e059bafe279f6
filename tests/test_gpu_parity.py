"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2002_11082_amd as ogq
from paper_2002_11082_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _rng_bucket(rng, n, kind):
    if kind == "normal":
        return rng.normal(0, 1e-3, n).astype(np.float32)
    if kind == "ints":
        return rng.integers(-3, 4, n).astype(np.float32)
    if kind == "heavy":
        return (rng.standard_t(3, n) * 1e-2).astype(np.float32)
    if kind == "shifted":
        return rng.normal(5.0, 1e-3, n).astype(np.float32)
    if kind == "const":
        return np.full(n, -0.75, np.float32)
    if kind == "zeros":
        g = np.zeros(n, np.float32)
        g[::7] = -0.0
        return g
    raise ValueError(kind)


# ------------------------------------------------------------------------------------------------
# small sizes: every element compared; several tiles and ragged tails
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d", [64, 128, 192, 256, 512, 1024, 2048, 3072, 4096])
@pytest.mark.parametrize("kind", ["normal", "ints", "heavy", "shifted", "const", "zeros"])
def test_bingrad_small(d, kind):
    rng = np.random.default_rng(d + len(kind))
    # bucket sizes dividing 2048 send whole 2048-element chunks and the rest to different kernels
    for n in (1, 63, 64, 65, d - 1, d, d + 1, 5 * d + 37, 16 * d, 3 * 2048 + 2 * d + 11, 9 * 2048):
        if n < 1:
            continue
        g = _rng_bucket(rng, n, kind)
        for iters in (0, 1, 4):
            parity.check_quantize(g, d, 1, ogq.BINGRAD_B, iters, tag=f"bingrad-{kind}-d{d}-n{n}-it{iters}")


@pytest.mark.parametrize("d", [64, 128, 256, 512, 1024])
def test_bingrad_unlike_buckets_in_one_wavefront(d):
    """Neighbouring buckets of one 2048-element chunk with nothing in common: constant, all equal but one,
    one huge outlier, integers (the per-bucket special cases of the level solve)."""
    rng = np.random.default_rng(77 + d)
    kinds = ["const", "normal", "zeros", "heavy", "ints", "shifted"]
    nb = (5 if d <= 256 else 2050) * (2048 // d) + 3
    parts = []
    for b in range(nb):
        kind = kinds[int(rng.integers(len(kinds)))]
        x = _rng_bucket(rng, d, kind)
        r = b % 7
        if r == 3:
            x = np.full(d, 1e-3, np.float32)
            x[int(rng.integers(d))] = 2.0
        elif r == 5:
            x = rng.normal(0, 1e-3, d).astype(np.float32)
            x[int(rng.integers(d))] = -3000.0  # upper-side sum far below the largest magnitude
        parts.append(x)
    g = np.concatenate(parts)[: nb * d - 17]
    for iters in (0, 3):
        parity.check_quantize(g, d, 1, ogq.BINGRAD_B, iters, tag=f"bingrad-unlike-d{d}-it{iters}")


@pytest.mark.parametrize("d", [512, 1024])
def test_bingrad_several_buckets_per_wavefront_above_four_million_elements(d):
    """Buckets of 512 and 1024 elements are packed several to a wavefront only for long gradients."""
    rng = np.random.default_rng(d)
    n = 2100 * 2048 + d + 77
    g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    g[5 * d:6 * d] = 0.25          # a constant bucket
    g[9 * d:10 * d] = rng.normal(0, 1e-3, d).astype(np.float32)
    g[9 * d + 3] = -3000.0         # upper-side sum far below the largest magnitude
    for iters in (0, 2):
        parity.check_quantize(g, d, 1, ogq.BINGRAD_B, iters, tag=f"bingrad-long-d{d}-it{iters}")


@pytest.mark.parametrize("bits", [1, 2, 3])
@pytest.mark.parametrize("d", [64, 128, 256, 320, 2048, 4096])
def test_orq_small(bits, d):
    rng = np.random.default_rng(100 * bits + d)
    for kind in ("normal", "ints", "heavy", "shifted", "const", "zeros"):
        # (the longer ones: whole and cut-off groups of the 64- and 128-element buckets that share a wavefront)
        for n in (1, 2, 3, 65, d - 1, d, d + 1, 3 * d + 129, 1024 + 5 * d, 2048 + 3 * d + 4):
            if n < 1:
                continue
            g = _rng_bucket(rng, n, kind)
            for sweeps in (0, 2):
                parity.check_quantize(g, d, bits, ogq.ORQ, sweeps, seed=1234 + n, index_offset=64 * (n % 3),
                                      tag=f"orq{bits}-{kind}-d{d}-n{n}")


@pytest.mark.parametrize("d", [64, 128, 256, 320, 512, 2048, 4096])
def test_bingrad_pb_small(d):
    rng = np.random.default_rng(1000 + d)
    for kind in ("normal", "ints", "heavy", "shifted", "const", "zeros"):
        # (the longer ones: whole and cut-off groups of the 64- and 128-element buckets that share a wavefront)
        for n in (1, 2, 3, 65, d - 1, d, d + 1, 3 * d + 129, 1024 + 5 * d, 2048 + 3 * d + 4):
            g = _rng_bucket(rng, n, kind)
            parity.check_quantize(g, d, 1, ogq.BINGRAD_PB, 0, seed=31 + n, index_offset=64 * (n % 3),
                                  tag=f"bingradpb-{kind}-d{d}-n{n}")
            parity.check_quantize(-g, d, 1, ogq.BINGRAD_PB, 0, seed=31 + n, tag=f"bingradpb-neg-{kind}-d{d}-n{n}")
    g = _rng_bucket(rng, 4 * d + 3, "heavy")
    parity.check_quantize(g, d, 1, ogq.BINGRAD_PB, 0, seed=5, clip_factor=2.5, tag=f"bingradpb-clip-d{d}")


def test_bingrad_pb_resnet50_size_sampled():
    wl = synth.WORKLOADS["cfg2"]
    g = wl.gradient()
    d = 2048
    nb = (g.size + d - 1) // d
    lv, codes, rep = parity.check_quantize(g, d, 1, ogq.BINGRAD_PB, 0, seed=9, buckets=_sample(nb, 120, 4),
                                           tag="bingradpb-cfg2")
    out = ogq.ogq_dequantize_average([codes], [lv], g.size, ogq.make_params(d, 1, ogq.BINGRAD_PB))
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    for b in _sample(nb, 40, 2):
        lo, hi = b * d, min((b + 1) * d, g.size)
        l, w = oracle.quantize(g[lo:hi], d, 1, ogq.BINGRAD_PB, 0, 9, lo)
        assert np.array_equal(out[lo:hi], oracle.dequantize_average([w], [l], hi - lo, d, 1, 2))


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("d", [64, 128, 512, 2048, 4096])
def test_orq_paper_level_counts_small(bits, d):
    # s = 3, 5, 9 levels; zero sweeps is Algorithm 1 as printed
    rng = np.random.default_rng(7 * bits + d)
    for kind in ("normal", "ints", "heavy", "shifted", "const", "zeros"):
        # (with three levels and 64 or 128 elements per bucket a wavefront sorts several buckets in its registers:
        # whole and cut-off groups of them)
        for n in (1, 2, 3, 65, d - 1, d, d + 1, 3 * d + 129, 1024 + 5 * d, 2048 + 3 * d + 4, 4096 + d + 62):
            g = _rng_bucket(rng, n, kind)
            for sweeps in (0, 1):
                parity.check_quantize(g, d, bits, ogq.ORQ_PAPER, sweeps, seed=99 + n, index_offset=64 * (n % 5),
                                      tag=f"orqpaper{bits}-{kind}-d{d}-n{n}-sw{sweeps}")


def test_orq_paper_five_levels_resnet50_size():
    # ORQ-5 as in the paper's tables (bucket 2048, no clipping; and bucket 512 with clipping 2.5 as on ImageNet)
    wl = synth.WORKLOADS["cfg3"]
    g = wl.gradient()
    for d, clip in ((2048, 0.0), (512, 2.5)):
        nb = (g.size + d - 1) // d
        lv, codes, rep = parity.check_quantize(g, d, 3, ogq.ORQ_PAPER, 0, seed=8, clip_factor=clip,
                                               tag=f"orq5-d{d}-clip{clip}")
        assert rep["buckets_checked"] == nb
        params = ogq.make_params(d, 3, ogq.ORQ_PAPER)
        out = ogq.ogq_dequantize_average([codes], [lv], g.size, params)
        torch.cuda.synchronize()
        out = out.cpu().numpy()
        for b in _sample(nb, 60, 1):
            lo, hi = b * d, min((b + 1) * d, g.size)
            l, w = oracle.quantize(g[lo:hi], d, 3, ogq.ORQ_PAPER, 0, 8, lo, clip)
            ref = oracle.dequantize_average([w], [l], hi - lo, d, 3, 5)
            assert np.array_equal(out[lo:hi], ref)


# ------------------------------------------------------------------------------------------------
# the comparison level rules of the paper's Section 5 on the same kernels
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d", [64, 128, 192, 512, 1024, 2048, 3072, 4096])
def test_scaled_sign_small(d):
    rng = np.random.default_rng(4000 + d)
    for kind in ("normal", "ints", "heavy", "shifted", "const", "zeros"):
        for n in (1, 65, d - 1, d, 3 * d + 129, 3 * 2048 + 2 * d + 11):
            g = _rng_bucket(rng, n, kind)
            parity.check_quantize(g, d, 1, ogq.SCALED_SIGN, 0, tag=f"sign-{kind}-d{d}-n{n}")
        g = _rng_bucket(rng, 4 * d + 3, kind)
        parity.check_quantize(g, d, 1, ogq.SCALED_SIGN, 0, clip_factor=2.5, tag=f"sign-clip-{kind}-d{d}")


@pytest.mark.parametrize("d", [512, 1024])
def test_scaled_sign_several_buckets_per_wavefront_above_four_million_elements(d):
    rng = np.random.default_rng(d + 1)
    n = 2100 * 2048 + d + 77
    g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    g[5 * d:6 * d] = -0.0
    parity.check_quantize(g, d, 1, ogq.SCALED_SIGN, 0, tag=f"sign-long-d{d}")


@pytest.mark.parametrize("scheme", [ogq.EVEN, ogq.LINEAR])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("d", [64, 128, 320, 512, 2048, 4096])
def test_even_and_linear_levels_small(scheme, bits, d):
    rng = np.random.default_rng(17 * bits + d + scheme)
    for kind in ("normal", "ints", "heavy", "shifted", "const", "zeros"):
        # (with 64 and 128 elements per bucket a wavefront holds several buckets: whole and cut-off groups of them)
        for n in (1, 2, 3, 65, d - 1, d, 3 * d + 129, 1024 + 5 * d, 2048 + 3 * d + 4, 4096 + d + 62):
            g = _rng_bucket(rng, n, kind)
            parity.check_quantize(g, d, bits, scheme, 0, seed=7 + n, index_offset=64 * (n % 7),
                                  tag=f"rule{scheme}-b{bits}-{kind}-d{d}-n{n}")
        g = _rng_bucket(rng, 4 * d + 3, kind)
        parity.check_quantize(g, d, bits, scheme, 0, seed=3, clip_factor=2.5, index_offset=64 * 12345,
                              tag=f"rule{scheme}-b{bits}-clip-{kind}-d{d}")


def _rounding_error(x, levels):
    lv = np.asarray(levels, np.float64)
    x = np.asarray(x, np.float64)
    k = np.clip(np.searchsorted(lv, x, side="right") - 1, 0, lv.size - 2)
    return float(np.sum((lv[k + 1] - x) * (x - lv[k])))


def test_comparison_rules_resnet50_size_and_error_ordering():
    """The three multi-level rules at full size on one gradient (every bucket against the oracle, decode on a sample), and the ordering of their expected rounding errors from the device's own level tables
    (Section 5.1: ORQ has the smallest error for its number of levels)."""
    wl = synth.WORKLOADS["cfg3"]
    g = wl.gradient()
    d, bits, s = 2048, 3, 5
    nb = (g.size + d - 1) // d
    tables = {}
    for scheme in (ogq.ORQ_PAPER, ogq.EVEN, ogq.LINEAR):
        lv, codes, rep = parity.check_quantize(g, d, bits, scheme, 0, seed=21, tag=f"rule{scheme}-cfg3")
        assert rep["buckets_checked"] == nb
        tables[scheme] = lv[:nb * s].cpu().numpy().reshape(nb, s)
        if scheme != ogq.ORQ_PAPER:
            out = ogq.ogq_dequantize_average([codes], [lv], g.size, ogq.make_params(d, bits, scheme))
            torch.cuda.synchronize()
            out = out.cpu().numpy()
            for b in _sample(nb, 30, 1):
                lo, hi = b * d, min((b + 1) * d, g.size)
                l, w = oracle.quantize(g[lo:hi], d, bits, scheme, 0, 21, lo)
                assert np.array_equal(out[lo:hi], oracle.dequantize_average([w], [l], hi - lo, d, bits, s))
    err = {k: 0.0 for k in tables}
    for b in _sample(nb, 300, 9):
        x = g[b * d:min((b + 1) * d, g.size)]
        for k in tables:
            err[k] += _rounding_error(x, tables[k][b])
    print(f"[parity] expected rounding error, 300 buckets of cfg3: ORQ-5 {err[ogq.ORQ_PAPER]:.4e}, "
          f"evenly spaced {err[ogq.EVEN]:.4e}, Linear-5 {err[ogq.LINEAR]:.4e}", flush=True)
    assert err[ogq.ORQ_PAPER] < err[ogq.EVEN] and err[ogq.ORQ_PAPER] < err[ogq.LINEAR]


def test_scaled_sign_resnet50_size():
    wl = synth.WORKLOADS["cfg2"]
    g = wl.gradient()
    d = 2048
    lv, codes, rep = parity.check_quantize(g, d, 1, ogq.SCALED_SIGN, 0, tag="sign-cfg2-all")
    assert rep["code_mismatches"] == 0
    # two-level error against BinGrad-b on the same gradient, from the device's outputs
    out_s = ogq.ogq_dequantize_average([codes], [lv], g.size, ogq.make_params(d, 1, ogq.SCALED_SIGN)).cpu().numpy()
    lv_b, codes_b = ogq.ogq_quantize(torch.from_numpy(g).to(DEV), ogq.make_params(d, 1, ogq.BINGRAD_B))
    out_b = ogq.ogq_dequantize_average([codes_b], [lv_b], g.size, ogq.make_params(d, 1, ogq.BINGRAD_B)).cpu().numpy()
    e_s = float(np.sum((g.astype(np.float64) - out_s) ** 2))
    e_b = float(np.sum((g.astype(np.float64) - out_b) ** 2))
    print(f"[parity] squared error on cfg2: BinGrad-b {e_b:.6e}, Scaled SignSGD {e_s:.6e}", flush=True)
    assert e_b <= e_s * 1.001


# ------------------------------------------------------------------------------------------------
# buckets above 4096 elements (the paper's bucket-size sweep goes to 32768): several wavefronts per bucket
# ------------------------------------------------------------------------------------------------
LARGE_SCHEMES = [(ogq.BINGRAD_B, 1), (ogq.SCALED_SIGN, 1), (ogq.BINGRAD_PB, 1), (ogq.ORQ, 1), (ogq.ORQ, 2), (ogq.ORQ, 3),
                 (ogq.ORQ_PAPER, 2), (ogq.ORQ_PAPER, 3), (ogq.ORQ_PAPER, 4), (ogq.EVEN, 2), (ogq.EVEN, 4),
                 (ogq.LINEAR, 2), (ogq.LINEAR, 3)]


@pytest.mark.parametrize("scheme,bits", LARGE_SCHEMES)
@pytest.mark.parametrize("d", [4160, 6144, 8192, 16384, 20480, 32768])
def test_buckets_above_4096(scheme, bits, d):
    rng = np.random.default_rng(d + 31 * scheme + bits)
    stride = oracle.levels_per_bucket(scheme, bits)
    cases = [("normal", d), ("heavy", 2 * d + 777), ("ints", d + 4097), ("const", d - 1), ("zeros", 65),
             ("shifted", 3 * d)]
    for kind, n in cases:
        g = _rng_bucket(rng, n, kind)
        for iters in ((0, 2) if kind in ("normal", "heavy") else (1,)):
            lv, codes, rep = parity.check_quantize(g, d, bits, scheme, iters, seed=n + 5, index_offset=64 * 77,
                                                   tag=f"large-s{scheme}b{bits}-{kind}-d{d}-n{n}-it{iters}")
        out = ogq.ogq_dequantize_average([codes], [lv], n, ogq.make_params(d, bits, scheme))
        torch.cuda.synchronize()
        l, w = oracle.quantize(g, d, bits, scheme, iters, n + 5, 64 * 77)
        assert np.array_equal(out.cpu().numpy(), oracle.dequantize_average([w], [l], n, d, bits, stride)), (kind, n)
    g = _rng_bucket(rng, 2 * d + 5, "heavy")
    parity.check_quantize(g, d, bits, scheme, 1, seed=3, clip_factor=2.5, tag=f"large-clip-s{scheme}b{bits}-d{d}")


def test_bucket_size_sweep_of_the_paper_at_resnet50_size():
    """ORQ-3 and TernGrad-noclip over the bucket sizes of the paper's CIFAR-10 sweep (128 .. 32768), every
    bucket against the oracle; the expected rounding error per element must grow with the bucket size for
    both and stay lower for ORQ-3 (the trend behind the accuracy table of Section 5.1)."""
    wl = synth.WORKLOADS["cfg3"]
    g = wl.gradient()[:8_000_000]
    err = {ogq.ORQ_PAPER: [], ogq.EVEN: []}
    sizes = (128, 512, 1024, 2048, 4096, 8192, 16384, 32768)
    for d in sizes:
        nb = (g.size + d - 1) // d
        for scheme in err:
            picks = _sample(nb, max(8, 65536 // d), d + scheme)
            lv, codes, rep = parity.check_quantize(g, d, 2, scheme, 0, seed=13, tag=f"sweep-s{scheme}-d{d}")
            assert rep["buckets_checked"] == nb
            table = lv[:nb * 3].cpu().numpy().reshape(nb, 3)
            e, cnt = 0.0, 0
            for b in picks:
                x = g[b * d:min((b + 1) * d, g.size)]
                e += _rounding_error(x, table[b])
                cnt += x.size
            err[scheme].append(e / cnt)
    print("[parity] expected rounding error per element by bucket size", sizes, {k: [f"{x:.3e}" for x in v] for k, v in err.items()},
          flush=True)
    for i in range(len(sizes)):
        assert err[ogq.ORQ_PAPER][i] < err[ogq.EVEN][i]
    assert err[ogq.ORQ_PAPER][-1] > err[ogq.ORQ_PAPER][0] and err[ogq.EVEN][-1] > err[ogq.EVEN][0]


@pytest.mark.parametrize("scheme,bits", [(ogq.ORQ, 2), (ogq.ORQ, 3), (ogq.ORQ_PAPER, 2), (ogq.ORQ_PAPER, 4), (ogq.LINEAR, 3),
                                         (ogq.BINGRAD_PB, 1)])
@pytest.mark.parametrize("d", [512, 2048, 4096, 16384])
def test_crowded_bins_of_distinct_values(scheme, bits, d):
    """Buckets whose values crowd a few bins of the in-bucket grouping without being equal: a shifted normal puts
    65 .. 256 distinct values (selection on register-held keys) or many hundreds (selection over LDS) into one bin,
    for the rank picks of every rule."""
    rng = np.random.default_rng(d + 7 * bits + scheme)
    n = 6 * d + 200
    for mean, sigma in ((5.0, 0.5), (-3.0, 0.2), (5.0, 0.02), (0.75, 0.1)):
        g = rng.normal(mean, sigma, n).astype(np.float32)
        g[::97] *= np.float32(-1.0)   # a few values on the other side of zero
        for iters in (0, 2):
            parity.check_quantize(g, d, bits, scheme, iters, seed=d + 3, tag=f"crowded-s{scheme}b{bits}-d{d}-m{mean}-sd{sigma}-it{iters}")


def test_orq_sweeps_and_offsets():
    rng = np.random.default_rng(77)
    g = _rng_bucket(rng, 8 * 1024 + 100, "heavy")
    for sweeps in (0, 1, 3, 5):
        parity.check_quantize(g, 1024, 3, ogq.ORQ, sweeps, seed=9, tag=f"orq-sweeps{sweeps}")
    # shard with an index offset, including one above 2^34 (second counter word in use)
    for off in (1024, 64 * 12345, (1 << 36) + 64):
        parity.check_quantize(g, 1024, 2, ogq.ORQ, 2, seed=(1 << 40) + 17, index_offset=off, tag=f"orq-offset{off}")
    # a shard reproduces the full vector's codes
    params = ogq.make_params(1024, 2, ogq.ORQ, 2, 5, 0)
    _, words_full, _ = parity.gpu_quantize(g, params)
    params_s = ogq.make_params(1024, 2, ogq.ORQ, 2, 5, 4096)
    _, words_shard, _ = parity.gpu_quantize(g[4096:], params_s)
    assert np.array_equal(words_full[4096 // 64 * 2:], words_shard)


@pytest.mark.parametrize("clip", [1.0, 1.7, 2.5])
def test_clipping_before_quantization(clip):
    rng = np.random.default_rng(int(clip * 10))
    for kind in ("normal", "heavy", "shifted", "const", "ints"):
        for d, n in ((64, 200), (512, 5 * 512 + 77), (2048, 3 * 2048), (3072, 3 * 3072 + 2500), (4096, 2 * 4096 + 5)):
            g = _rng_bucket(rng, n, kind)
            parity.check_quantize(g, d, 1, ogq.BINGRAD_B, 1, clip_factor=clip, tag=f"clip{clip}-bingrad-{kind}-d{d}")
            for bits in (2, 3):
                parity.check_quantize(g, d, bits, ogq.ORQ, 2, seed=11, clip_factor=clip,
                                      tag=f"clip{clip}-orq{bits}-{kind}-d{d}")


def test_random_shapes_and_parameters():
    # many small random problems: sizes, bucket sizes (every multiple of 64 is legal), schemes, widths, iterations,
    # clipping, value distributions, including buckets dominated by repeated values
    rng = np.random.default_rng(20260101)
    kinds = ("normal", "ints", "heavy", "shifted", "const", "zeros")
    for trial in range(390):
        d = int(rng.choice([64, 128, 192, 256, 448, 512, 1024, 1536, 2048, 3072, 4096]))
        n = int(rng.integers(1, 5 * d + 2))
        scheme, bits = [(ogq.BINGRAD_B, 1), (ogq.BINGRAD_PB, 1), (ogq.ORQ, 1), (ogq.ORQ, 2), (ogq.ORQ, 3),
                        (ogq.ORQ_PAPER, 2), (ogq.ORQ_PAPER, 3), (ogq.ORQ_PAPER, 4), (ogq.SCALED_SIGN, 1),
                        (ogq.EVEN, 2), (ogq.EVEN, 4), (ogq.LINEAR, 2), (ogq.LINEAR, 3)][trial % 13]
        g = _rng_bucket(rng, n, kinds[int(rng.integers(len(kinds)))])
        if trial % 5 == 0:  # mixed magnitudes inside one bucket
            g = (g * np.float32(10.0) ** rng.integers(-6, 4, n).astype(np.float32)).astype(np.float32)
        clip = float(rng.choice([0.0, 0.0, 1.7, 2.5]))
        iters = int(rng.integers(0, 4))
        off = 64 * int(rng.integers(0, 1 << 20))
        parity.check_quantize(g, d, bits, scheme, iters, seed=int(rng.integers(1 << 62)), index_offset=off,
                              clip_factor=clip, tag=f"random-{trial}")


def test_random_value_distributions():
    """Distributions the other tests do not draw: log-normal with a dynamic range of 2^30, Cauchy, subnormal values,
    70 % zeros, sorted input, a handful of distinct values, scaled integers; random bucket sizes up to 32768, schemes,
    sweeps, clipping and index offsets (under the acceptance rules; an earlier run of 15,000 such cases had levels one
    fp32 ulp apart in one clipped log-normal bucket and equal everywhere else)."""
    rng = np.random.default_rng(77)

    def draw(n):
        k = int(rng.integers(0, 8))
        if k == 0:
            return (rng.lognormal(0, 3, n) * rng.choice([-1, 1], n)).astype(np.float32)
        if k == 1:
            return rng.choice(rng.normal(0, 1, 17).astype(np.float32), n)
        if k == 2:
            return (rng.standard_cauchy(n) * 1e-3).astype(np.float32)
        if k == 3:
            return rng.normal(0, 1e-40, n).astype(np.float32)
        if k == 4:
            g = rng.normal(0, 1e-3, n).astype(np.float32)
            g[rng.random(n) < 0.7] = 0
            return g
        if k == 5:
            return rng.normal(rng.uniform(-10, 10), 10.0 ** rng.uniform(-4, 0), n).astype(np.float32)
        if k == 6:
            return np.sort(rng.normal(0, 1, n).astype(np.float32))
        return (rng.integers(-1000, 1000, n) * np.float32(2.0 ** rng.integers(-20, 20))).astype(np.float32)

    schemes = [(ogq.BINGRAD_B, 1), (ogq.ORQ, 1), (ogq.ORQ, 2), (ogq.ORQ, 3), (ogq.BINGRAD_PB, 1), (ogq.ORQ_PAPER, 2),
               (ogq.ORQ_PAPER, 3), (ogq.ORQ_PAPER, 4), (ogq.SCALED_SIGN, 1), (ogq.EVEN, 3), (ogq.LINEAR, 2), (ogq.LINEAR, 4)]
    for trial in range(360):
        scheme, bits = schemes[trial % len(schemes)]
        d = 64 * int(rng.choice([1, 2, 3, 4, 8, 12, 16, 32, 33, 48, 64, 96, 128, 200, 256, 512]))
        n = int(rng.integers(1, 4 * d + 100))
        parity.check_quantize(draw(n), d, bits, scheme, int(rng.integers(0, 4)), seed=int(rng.integers(1 << 62)),
                              index_offset=64 * int(rng.integers(0, 1 << 30)), clip_factor=float(rng.choice([0.0, 0.0, 2.5, 1.7])),
                              tag=f"dist-{trial}")


def test_integer_t_where_the_prefix_sums_cancel():
    """A level solve whose T = S / (R - L) is an integer while S, taken as a difference of prefix sums, carries their
    rounding: floor(T) must not follow that error.  Built so that the second solve of a four-level bucket lies
    between the second largest and the largest value (T = 1 exactly: the only element above L is R) with thousands of
    unlike values of large magnitude below L; also the heavy-tailed buckets of a working-file search for solves whose
    T is an integer in the oracle's arithmetic."""
    for seed in range(40):
        rng = np.random.default_rng(500 + seed)
        d = int(rng.choice([128, 512, 2048, 3072, 4096, 8192]))
        bucket = (-1.0e6 * (1.0 + 1.0e-3 * rng.random(d))).astype(np.float32)
        bucket[rng.integers(0, d)] = np.float32(rng.uniform(1.0, 9.0))
        where = rng.integers(0, d)
        bucket[where] = np.float32(rng.uniform(1.0, 2.0) * 10.0 ** rng.integers(6, 31))
        g = np.concatenate([bucket, bucket[::-1], bucket[: d // 2 + 7]])
        for scheme, bits, sweeps in ((ogq.ORQ, 2, 0), (ogq.ORQ, 2, 2), (ogq.ORQ, 3, 1), (ogq.ORQ_PAPER, 3, 1)):
            parity.check_quantize(g, d, bits, scheme, sweeps, seed=seed, tag=f"integer-T-built{seed}-s{scheme}b{bits}-d{d}")
    for seed in (1, 11, 14, 41, 77, 95, 120, 122):
        rng = np.random.default_rng(seed)
        d = int(rng.choice([128, 512, 2048, 3072, 4096]))
        bucket = (rng.lognormal(0, 3, d) * rng.choice([-1, 1], d)).astype(np.float32)
        g = np.concatenate([bucket, bucket[::-1], bucket[: d // 2 + 7]])
        for scheme, bits in ((ogq.ORQ, 3), (ogq.ORQ, 2), (ogq.ORQ_PAPER, 3)):
            parity.check_quantize(g, d, bits, scheme, 1, seed=seed, tag=f"integer-T-seed{seed}-s{scheme}b{bits}-d{d}")


@pytest.mark.parametrize("d", [64, 128, 512, 2048, 4096, 8192, 32768])
def test_symmetric_buckets_where_t_is_exactly_an_integer(d):
    """A bucket that holds -v for every v has S = (len / 2) (R - L) between its extremes: T is an integer, the optimum is
    flat and the lower end must be taken whatever a floating-point sum of the terms gives.  With values spread over
    more binades than the fp64 sums hold exactly (log-normal, tiny values next to large ones) the kernels have to decide
    floor(T) with their exact sums; with a narrow spread the fp64 sums are exact themselves.  Both against the oracle,
    whose floor(T) is exact by construction."""
    rng = np.random.default_rng(900 + d)
    halves = [
        rng.lognormal(0, 4, d // 2),                                              # dynamic range far beyond 2^30
        np.concatenate([rng.normal(0, 1, d // 2 - 8), rng.normal(0, 1e-30, 8)]),  # a few tiny values
        rng.normal(0, 1e-3, d // 2),                                              # narrow: exact fp64 sums
        rng.integers(1, 40, d // 2).astype(np.float64),                           # many equal values
        np.concatenate([rng.normal(0, 1e-40, d // 4), rng.normal(0, 1e-3, d // 2 - d // 4)]),  # subnormals
    ]
    # magnitudes spread over just as many binades as the fp64 sums of a bucket of this size hold exactly, and two more
    safe = 28 - int(np.ceil(np.log2(max(d, 64))))
    for span in (safe, safe + 2):
        halves.append(rng.uniform(1, 2, d // 2) * 2.0 ** (-rng.integers(0, span + 1, d // 2).astype(np.float64)))
    buckets = []
    for h in halves:
        h = np.abs(h).astype(np.float32)
        bucket = np.concatenate([h, -h])
        rng.shuffle(bucket)
        buckets.append(bucket)
    g = np.concatenate(buckets + [buckets[0][: d // 2 + 6]])
    for scheme, bits, sweeps in ((ogq.ORQ_PAPER, 2, 0), (ogq.ORQ, 2, 2), (ogq.ORQ, 3, 1), (ogq.ORQ_PAPER, 3, 1), (ogq.ORQ_PAPER, 4, 0)):
        parity.check_quantize(g, d, bits, scheme, sweeps, seed=d, tag=f"symmetric-s{scheme}b{bits}-d{d}")


def test_non_finite_values_stay_inside_their_bucket():
    """NaN and infinities give unspecified levels and codes for their own bucket only: every call returns, and the
    buckets without them still match the oracle (every kernel family and bucket-size class)."""
    rng = np.random.default_rng(99)
    cases = [(ogq.BINGRAD_B, 1, 512, 2100 * 2048 + 700), (ogq.BINGRAD_B, 1, 2048, 40 * 2048 + 5),
             (ogq.BINGRAD_B, 1, 8192, 9 * 8192), (ogq.SCALED_SIGN, 1, 256, 30 * 2048 + 64),
             (ogq.ORQ, 2, 2048, 40 * 2048 + 5), (ogq.ORQ, 3, 4096, 12 * 4096), (ogq.ORQ_PAPER, 2, 16384, 5 * 16384 + 9),
             (ogq.BINGRAD_PB, 1, 1024, 33 * 1024), (ogq.EVEN, 2, 512, 70 * 512), (ogq.LINEAR, 3, 2048, 21 * 2048),
             # several buckets per wavefront: the neighbours of a poisoned bucket share its registers' lanes
             (ogq.EVEN, 2, 64, 41 * 64 + 7), (ogq.ORQ, 2, 128, 37 * 128 + 50), (ogq.ORQ, 1, 64, 29 * 64),
             (ogq.ORQ_PAPER, 2, 64, 53 * 64 + 1), (ogq.ORQ_PAPER, 4, 128, 19 * 128 + 127),
             (ogq.BINGRAD_PB, 1, 128, 26 * 128 + 3), (ogq.LINEAR, 3, 64, 44 * 64 + 63)]
    for scheme, bits, d, n in cases:
        g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
        nb = (n + d - 1) // d
        poisoned = sorted(set(int(b) for b in rng.choice(nb, size=min(6, nb // 2), replace=False)))
        for i, b in enumerate(poisoned):
            lo, hi = b * d, min((b + 1) * d, n)
            if i % 3 == 2:
                g[lo:hi] = np.nan                          # a bucket of nothing but NaN
            else:
                where = rng.choice(hi - lo, size=min(5, hi - lo), replace=False) + lo
                g[where] = [np.nan, np.inf, -np.inf, np.nan, np.inf][:where.size] if i % 3 == 0 else np.inf
        clean = [b for b in range(nb) if b not in poisoned]
        for clip in (0.0, 2.5):
            lv, codes, rep = parity.check_quantize(g, d, bits, scheme, 2, seed=4, buckets=clean, clip_factor=clip,
                                                   tag=f"nonfinite-s{scheme}b{bits}-d{d}-clip{clip}")
            out = ogq.ogq_dequantize_average([codes], [lv], n, ogq.make_params(d, bits, scheme))
            torch.cuda.synchronize()
            assert out.shape[0] >= n


def test_calls_can_be_captured_in_a_graph():
    """The entry points only enqueue kernels, so a quantize + decode-average pair can be captured once and replayed
    on new inputs: every replay must give what the eager calls give (several kernel families, a gradient that takes
    two launches, several replays with other work in between)."""
    rng = np.random.default_rng(31)
    cases = [(ogq.BINGRAD_B, 1, 512, 2100 * 2048 + 700, 0), (ogq.ORQ, 2, 2048, 9 * 2048 + 100, 2),
             (ogq.ORQ_PAPER, 2, 8192, 3 * 8192 + 5, 0)]
    for scheme, bits, d, n, iters in cases:
        params = ogq.make_params(d, bits, scheme, iters, seed=17)
        g_dev = torch.empty(n, dtype=torch.float32, device=DEV)
        lv = torch.zeros(ogq.ogq_levels_count(n, params) + 4, dtype=torch.float32, device=DEV)
        codes = torch.zeros(ogq.ogq_codes_bytes(n, params) // 8 + 2, dtype=torch.int64, device=DEV)
        out = torch.zeros(n, dtype=torch.float32, device=DEV)
        inputs = [(rng.standard_t(3, n) * 1e-3).astype(np.float32) for _ in range(3)]
        g_dev.copy_(torch.from_numpy(inputs[0]))
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):  # warm-up outside the capture
            ogq.ogq_quantize(g_dev, params, lv, codes)
            ogq.ogq_dequantize_average([codes], [lv], n, params, out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ogq.ogq_quantize(g_dev, params, lv, codes)
            ogq.ogq_dequantize_average([codes], [lv], n, params, out)
        for x in inputs[::-1]:
            g_dev.copy_(torch.from_numpy(x))
            graph.replay()
            torch.cuda.synchronize()
            replayed = (lv.clone(), codes.clone(), out.clone())
            lv_e, codes_e = ogq.ogq_quantize(torch.from_numpy(x).to(DEV), params)   # eager, fresh buffers
            out_e = ogq.ogq_dequantize_average([codes_e], [lv_e], n, params)
            torch.cuda.synchronize()
            nl, nw = ogq.ogq_levels_count(n, params), ogq.ogq_codes_bytes(n, params) // 8
            assert torch.equal(replayed[0][:nl], lv_e[:nl]) and torch.equal(replayed[1][:nw], codes_e[:nw])
            assert torch.equal(replayed[2], out_e[:n])


@pytest.mark.parametrize("scheme,bits,d,iters", [(ogq.BINGRAD_B, 1, 2048, 1), (ogq.BINGRAD_B, 1, 512, 0), (ogq.ORQ, 2, 2048, 2),
                                                  (ogq.ORQ_PAPER, 2, 8192, 0)])
def test_gradient_longer_than_2_pow_32_elements(scheme, bits, d, iters):
    """Element and word indices beyond 32 bits: a gradient of 2^32 + 5 d + 77 elements (17 GB), built on the device
    from a seeded host block that is repeated with a different scale per repetition, so that buckets 2^32 elements
    apart differ.  Buckets at both ends, on both sides of element 2^32 and the short last bucket are checked
    against the oracle (levels, codes, decoded values), which gets the bucket contents read back from the device."""
    free, _ = torch.cuda.mem_get_info()
    if free < 48 * 2 ** 30:
        pytest.skip("needs 48 GB of free device memory")
    block = 1 << 24
    n = (1 << 32) + 5 * d + 77
    base = torch.from_numpy(synth.laplace_heavy_tail(block, 5e-4, 77)).to(DEV)
    g = torch.empty(n, dtype=torch.float32, device=DEV)
    for t, lo in enumerate(range(0, n, block)):
        hi = min(lo + block, n)
        torch.mul(base[:hi - lo], 1.0 + t / 1024.0, out=g[lo:hi])
    seed, offset = 11, 64 * 3
    params = ogq.make_params(d, bits, scheme, iters, seed, offset)
    s = ogq.ogq_levels_per_bucket(params)
    print(f"[parity] beyond-2^32 n={n} d={d} bits={bits} scheme={scheme} iters={iters}", flush=True)
    levels, codes = ogq.ogq_quantize(g, params)
    out = ogq.ogq_dequantize_average([codes], [levels], n, params)
    torch.cuda.synchronize()
    nb = (n + d - 1) // d
    assert ogq.ogq_num_buckets(n, params) == nb and n % d != 0
    edge = (1 << 32) // d
    picks = sorted({0, 1, edge - 2, edge - 1, edge, edge + 1, nb - 3, nb - 2, nb - 1, nb // 3, edge // 2 + 7})
    for b in picks:
        lo, hi = b * d, min((b + 1) * d, n)
        x = g[lo:hi].cpu().numpy()
        lv_ref, codes_ref, _ = oracle.quantize_codes(x, d, bits, scheme, iters, seed, offset + lo)
        lv_gpu = levels[b * s:(b + 1) * s].cpu().numpy()
        words = codes[lo // 64 * bits:(hi + 63) // 64 * bits].cpu().numpy().view(np.uint64)
        assert np.array_equal(lv_gpu, lv_ref), (b, lv_gpu, lv_ref)
        assert np.array_equal(parity.unpack_words(words, hi - lo, bits), codes_ref), b
        l, w = oracle.quantize(x, d, bits, scheme, iters, seed, offset + lo)
        assert np.array_equal(out[lo:hi].cpu().numpy(), oracle.dequantize_average([w], [l], hi - lo, d, bits, s)), b
    # every decoded value is one of its bucket's levels (whole array, compared on the device)
    full = n // d
    table = levels[:full * s].view(full, s)
    view = out[:full * d].view(full, d)
    hit = torch.zeros_like(view, dtype=torch.bool)
    for k in range(s):
        hit |= view == table[:, k:k + 1]
    assert bool(hit.all())
    del g, out, hit, levels, codes
    torch.cuda.empty_cache()


def test_empty_input_is_a_noop():
    p = ogq.make_params(512, 1, ogq.BINGRAD_B)
    x = torch.zeros(4, device=DEV)
    assert ogq.ogq_quantize_raw(x.data_ptr(), 0, p, x.data_ptr(), x.data_ptr()) == 0
    assert ogq.ogq_dequantize_average_raw([x.data_ptr()], [x.data_ptr()], 0, p, x.data_ptr()) == 0
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------------
# decode + average
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits,scheme", [(1, ogq.BINGRAD_B), (1, ogq.BINGRAD_PB), (1, ogq.ORQ), (2, ogq.ORQ), (3, ogq.ORQ),
                                         (2, ogq.ORQ_PAPER), (3, ogq.ORQ_PAPER), (4, ogq.ORQ_PAPER),
                                         (1, ogq.SCALED_SIGN), (2, ogq.EVEN), (4, ogq.LINEAR)])
@pytest.mark.parametrize("d", [64, 128, 192, 256, 512, 1024, 1536, 2048, 4096])
def test_decode_average_small(bits, scheme, d):
    rng = np.random.default_rng(bits * 1000 + d)
    stride = oracle.levels_per_bucket(scheme, bits)
    # a wavefront decodes 1024 elements: whole spans and a ragged last one for every bucket size
    for n in (1, 65, d, 2 * d + 63, 7 * d + 1, 3 * 1024 + 2 * d + 65):
        for W in (1, 2, 3, 8):
            gs = [_rng_bucket(rng, n, "heavy" if w % 2 else "normal") for w in range(W)]
            # oracle streams decoded by the oracle = expected; the same streams uploaded and decoded on the GPU
            q = [oracle.quantize(g, d, bits, scheme, 1, seed=40 + w) for w, g in enumerate(gs)]
            ref = oracle.dequantize_average([w for _, w in q], [l for l, _ in q], n, d, bits, stride)
            scale = parity.term_scale([l for l, _ in q], [w for _, w in q], n, d, bits, stride)
            dl = [torch.from_numpy(np.concatenate([l, np.zeros(4, np.float32)])).to(DEV) for l, _ in q]
            dc = [torch.from_numpy(np.concatenate([w, np.zeros(2, np.uint64)]).view(np.int64)).to(DEV) for _, w in q]
            params = ogq.make_params(d, bits, scheme)
            out = ogq.ogq_dequantize_average(dc, dl, n, params)
            torch.cuda.synchronize()
            parity.check_average(out.cpu().numpy(), ref, scale, tag=f"avg-b{bits}-d{d}-n{n}-W{W}")


@pytest.mark.parametrize("bits,scheme,d", [(1, ogq.BINGRAD_B, 2048), (2, ogq.ORQ, 1024), (3, ogq.ORQ, 4096), (4, ogq.ORQ_PAPER, 512),
                                           (3, ogq.ORQ_PAPER, 128), (2, ogq.EVEN, 192)])
def test_decode_average_many_distinct_workers(bits, scheme, d):
    """More workers than the decoder fetches at once (4 or 8), every one with its own gradient, levels and codes:
    worker counts that end inside a batch and on a batch boundary, whole spans and a ragged last one."""
    rng = np.random.default_rng(17 * bits + d)
    stride = oracle.levels_per_bucket(scheme, bits)
    n = 5 * 1024 + 2 * d + 65
    for W in (5, 9, 16, 33):
        gs = [_rng_bucket(rng, n, "heavy" if w % 3 else "normal") * np.float32(1 + w) for w in range(W)]
        q = [oracle.quantize(g, d, bits, scheme, 1, seed=90 + w) for w, g in enumerate(gs)]
        ref = oracle.dequantize_average([w for _, w in q], [l for l, _ in q], n, d, bits, stride)
        scale = parity.term_scale([l for l, _ in q], [w for _, w in q], n, d, bits, stride)
        dl = [torch.from_numpy(np.concatenate([l, np.zeros(4, np.float32)])).to(DEV) for l, _ in q]
        dc = [torch.from_numpy(np.concatenate([w, np.zeros(2, np.uint64)]).view(np.int64)).to(DEV) for _, w in q]
        out = ogq.ogq_dequantize_average(dc, dl, n, ogq.make_params(d, bits, scheme))
        torch.cuda.synchronize()
        parity.check_average(out.cpu().numpy(), ref, scale, tag=f"avg-distinct-b{bits}-s{scheme}-d{d}-W{W}")


def test_decode_average_many_identical_workers():
    rng = np.random.default_rng(5)
    n, d, bits = 5000, 512, 2
    g = _rng_bucket(rng, n, "normal")
    lv, w = oracle.quantize(g, d, bits, ogq.ORQ, 2, seed=3)
    single = oracle.dequantize_average([w], [lv], n, d, bits)
    dl = torch.from_numpy(np.concatenate([lv, np.zeros(4, np.float32)])).to(DEV)
    dc = torch.from_numpy(np.concatenate([w, np.zeros(2, np.uint64)]).view(np.int64)).to(DEV)
    for W in (1, 7, 64):
        out = ogq.ogq_dequantize_average([dc] * W, [dl] * W, n, ogq.make_params(d, bits, ogq.ORQ))
        torch.cuda.synchronize()
        ref = oracle.dequantize_average([w] * W, [lv] * W, n, d, bits)
        parity.check_average(out.cpu().numpy(), ref, np.abs(single).astype(np.float64), tag=f"avg-identical-W{W}")


# ------------------------------------------------------------------------------------------------
# the benchmark configurations at full size
# ------------------------------------------------------------------------------------------------
def _end_to_end(wl, g_list, sample_buckets):
    """Quantize every worker's gradient, decode-average the packed streams, compare both with the oracle.
    sample_buckets = None compares every bucket (whole-vector oracle calls); a list compares those buckets."""
    n, d, bits = g_list[0].size, wl.bucket_size, wl.bits
    dev_levels, dev_codes, q = [], [], []
    nb = (n + d - 1) // d
    for w, g in enumerate(g_list):
        lv, codes, rep = parity.check_quantize(g, d, bits, wl.scheme, wl.level_iters, wl.philox_seed(w),
                                               buckets=sample_buckets, tag=f"{wl.name}-w{w}", clip_factor=wl.clip_factor)
        assert rep["buckets_checked"] == (nb if sample_buckets is None else len(set(sample_buckets)))
        dev_levels.append(lv)
        dev_codes.append(codes)
        if sample_buckets is None:  # the oracle's own levels and packed words of this worker
            q.append((rep["oracle_levels"], oracle.pack(rep["oracle_codes"], bits)))
    params = ogq.make_params(d, bits, wl.scheme)
    stride = ogq.ogq_levels_per_bucket(params)
    out = ogq.ogq_dequantize_average(dev_codes, dev_levels, n, params)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    if sample_buckets is None:
        # expected average of the whole vector, from oracle streams only
        ref = oracle.dequantize_average([x[1] for x in q], [x[0] for x in q], n, d, bits, stride)
        scale = parity.term_scale([x[0] for x in q], [x[1] for x in q], n, d, bits, stride)
        parity.check_average(out, ref, scale, tag=f"{wl.name}-all-{nb}-buckets")
        return
    sel = sorted(set(sample_buckets))
    for b in sel:
        lo, hi = b * d, min((b + 1) * d, n)
        q = [oracle.quantize(g[lo:hi], d, bits, wl.scheme, wl.level_iters, wl.philox_seed(w), lo, wl.clip_factor)
             for w, g in enumerate(g_list)]
        ref = oracle.dequantize_average([x[1] for x in q], [x[0] for x in q], hi - lo, d, bits, stride)
        scale = parity.term_scale([x[0] for x in q], [x[1] for x in q], hi - lo, d, bits, stride)
        denom = np.maximum(np.abs(ref.astype(np.float64)), scale)
        err = np.abs(out[lo:hi].astype(np.float64) - ref.astype(np.float64))
        assert np.all(err <= parity.AVG_RTOL * denom), (wl.name, b, np.flatnonzero(err > parity.AVG_RTOL * denom)[:5])
    print(f"[parity] {wl.name} decode-average checked on {len(sel)} buckets", flush=True)


def _sample(nb, count, seed):
    rng = np.random.default_rng(seed)
    picks = set(rng.choice(nb, size=min(count, nb), replace=False).tolist())
    picks |= {0, 1, nb - 2, nb - 1} & set(range(nb))
    return sorted(picks)


def test_cfg1_bingrad_1m_full_compare():
    wl = synth.WORKLOADS["cfg1"]
    _end_to_end(wl, [wl.gradient()], None)


def test_cfg2_bingrad_resnet50_size():
    wl = synth.WORKLOADS["cfg2"]
    _end_to_end(wl, [wl.gradient()], None)


def test_cfg3_orq2_mixture():
    """Every one of the 12,500 buckets: levels, codes and the decoded average."""
    wl = synth.WORKLOADS["cfg3"]
    _end_to_end(wl, [wl.gradient()], None)


def test_cfg4_orq3_vgg19_shape():
    """Every one of the 35,084 buckets (the last one holds 32 elements)."""
    wl = synth.WORKLOADS["cfg4"]
    _end_to_end(wl, [wl.gradient()], None)


def test_cfg5_eight_workers_decode_average():
    """Every one of the 8 x 29,834 buckets, and the average of the eight decoded streams."""
    wl = synth.WORKLOADS["cfg5"]
    _end_to_end(wl, [wl.gradient(w) for w in range(wl.workers)], None)


@pytest.mark.parametrize("name", ["orq5", "orq3clip", "tern3", "linear5", "orq3d32k", "orq3d128", "sign2", "cfg2clip", "bin512"])
def test_further_bench_workloads_every_bucket(name):
    """The other workloads bench.py knows, whose oracle is linear in the bucket size: every bucket of the gradient."""
    wl = synth.WORKLOADS[name]
    _end_to_end(wl, [wl.gradient(w) for w in range(wl.workers)], None)


def test_pb2_bench_workload_sampled():
    """BinGrad-pb on the ResNet-50-sized gradient.  The oracle's level search is quadratic in the bucket size
    (every positive value is tried against a full pass over the bucket), so 400 of the 12,500 buckets are compared."""
    wl = synth.WORKLOADS["pb2"]
    nb = (wl.n + wl.bucket_size - 1) // wl.bucket_size
    _end_to_end(wl, [wl.gradient()], _sample(nb, 400, 6))
