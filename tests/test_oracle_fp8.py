"""Pins for the oracle's FP8 codec and scale rules (CPU only).

Each test checks the oracle against something other than itself: the format
facts of the cited standard (tests/golden/fp8_formats.txt), PyTorch's CPU
float8 casts (an independent library), closed forms, or a brute-force scan.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import fp8, quant

FMTS = [fp8.E4M3, fp8.E5M2]
TORCH_DT = {"e4m3": torch.float8_e4m3fn, "e5m2": torch.float8_e5m2}


def _golden(golden_dir):
    rows = {}
    with open(os.path.join(golden_dir, "fp8_formats.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows[p[0]] = dict(exp_bits=int(p[1]), man_bits=int(p[2]), bias=int(p[3]), max_code=int(p[4], 16),
                              max_finite=float(p[5]), min_normal=float(p[6]), min_sub=float(p[7]),
                              n_nan=int(p[8]), n_inf=int(p[9]))
    return rows


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_format_facts(fmt, golden_dir):
    g = _golden(golden_dir)[fmt.name]
    assert (fmt.exp_bits, fmt.man_bits, fmt.bias, fmt.max_code) == (g["exp_bits"], g["man_bits"], g["bias"], g["max_code"])
    assert 1 + fmt.exp_bits + fmt.man_bits == 8
    tab = fp8.decode_table(fmt)
    assert tab[fmt.max_code] == g["max_finite"] == fp8.max_finite(fmt)
    assert tab[1] == g["min_sub"]
    assert tab[1 << fmt.man_bits] == g["min_normal"]
    assert np.isnan(tab).sum() == g["n_nan"]
    assert np.isinf(tab).sum() == g["n_inf"]
    finite = tab[: fmt.max_code + 1]
    assert np.all(np.diff(finite) > 0)                      # code order = value order
    assert np.array_equal(tab[128:128 + fmt.max_code + 1], -finite)
    assert tab[0] == 0 and math.copysign(1, tab[128]) == -1


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_decode_matches_torch_float8(fmt):
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(TORCH_DT[fmt.name]).to(torch.float64).numpy()
    tab = fp8.decode_table(fmt)
    assert np.array_equal(np.isnan(ref), np.isnan(tab))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], tab[ok])


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_round_trip_every_code(fmt):
    tab = fp8.decode_table(fmt)
    for c in range(256):
        v = tab[c]
        if math.isnan(v) or math.isinf(v):
            continue
        assert fp8.satcast(np.array([v]), fmt)[0] == c
        assert fp8.satcast_scalar(float(v), fmt) == c


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_midpoints_go_to_even_and_neighbours_split(fmt):
    tab = fp8.decode_table(fmt)
    for c in range(fmt.max_code):
        lo, hi = tab[c], tab[c + 1]
        mid = (lo + hi) / 2
        even = c if c % 2 == 0 else c + 1
        assert fp8.satcast(np.array([mid]), fmt)[0] == even
        assert fp8.satcast(np.array([-mid]), fmt)[0] == (even | 0x80)
        # one binary32 step either side of the midpoint decides the other way
        below = np.nextafter(np.float32(mid), np.float32(-np.inf))
        above = np.nextafter(np.float32(mid), np.float32(np.inf))
        assert fp8.satcast(np.array([below]), fmt)[0] == c
        assert fp8.satcast(np.array([above]), fmt)[0] == c + 1


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_saturation_underflow_specials(fmt):
    fmax = fp8.max_finite(fmt)
    big = np.array([np.nextafter(np.float32(fmax), np.float32(np.inf)), 1e30, np.inf, 3.4e38], dtype=np.float32)
    assert np.all(fp8.satcast(big, fmt) == fmt.max_code)
    assert np.all(fp8.satcast(-big, fmt) == (fmt.max_code | 0x80))
    sub = fp8.decode_table(fmt)[1]
    assert fp8.satcast(np.array([sub / 2]), fmt)[0] == 0              # exact half: even = 0
    assert fp8.satcast(np.array([np.nextafter(np.float32(sub / 2), np.float32(1))]), fmt)[0] == 1
    assert fp8.satcast(np.array([sub / 4, 1e-30, 0.0]), fmt).tolist() == [0, 0, 0]
    assert fp8.satcast(np.array([-1e-30, -0.0]), fmt).tolist() == [0x80, 0x80]
    nan = fp8.satcast(np.array([np.nan]), fmt)[0]
    assert math.isnan(fp8.code_value(fmt, int(nan)))


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_satcast_matches_torch_cast_in_range(fmt):
    # torch's CPU cast is an independent round-to-nearest-even implementation;
    # it does not saturate, so compare on |v| <= fmax only.
    rng = np.random.default_rng(7)
    fmax = fp8.max_finite(fmt)
    v = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(fmax / 4),
        rng.standard_normal(200000).astype(np.float32),
        (rng.standard_normal(100000) * 4 * fp8.decode_table(fmt)[1]).astype(np.float32),   # subnormal range
        np.exp(rng.uniform(np.log(1e-8), np.log(fmax), 200000)).astype(np.float32),
    ])
    v = v[np.abs(v) <= fmax]
    ref = torch.from_numpy(v).to(TORCH_DT[fmt.name]).view(torch.uint8).numpy()
    got = fp8.satcast(v, fmt)
    assert np.array_equal(ref, got)


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_vector_and_scalar_definitions_agree(fmt):
    rng = np.random.default_rng(3)
    v = (rng.standard_normal(3000) * rng.choice([1e-5, 1e-2, 1, 100, 1e5], 3000)).astype(np.float32)
    got = fp8.satcast(v, fmt)
    ref = np.array([fp8.satcast_scalar(float(t), fmt) for t in v], dtype=np.uint8)
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- scale rules

@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
def test_per_tensor_fills_the_format(fmt):
    rng = np.random.default_rng(11)
    v = rng.standard_normal(4096).astype(np.float32) * np.float32(0.37)
    codes, scale, a = quant.quantize_per_tensor(v, fmt)
    assert a == np.abs(v).max()
    assert (codes & 0x7F).max() == fmt.max_code                    # the max element maps to fmax
    assert scale == np.float32(np.float32(fp8.max_finite(fmt)) / a)
    # dequantized error is bounded by half a spacing at the top binade
    deq = fp8.decode(codes, fmt) / float(scale)
    top_spacing = 2.0 ** (math.floor(math.log2(fp8.max_finite(fmt))) - fmt.man_bits)
    assert np.abs(deq - v).max() <= 0.5 * top_spacing / float(scale) * 1.001


@pytest.mark.parametrize("fmt", FMTS, ids=lambda f: f.name)
@pytest.mark.parametrize("k", [-7, -1, 3, 10])
def test_power_of_two_invariance(fmt, k):
    rng = np.random.default_rng(5)
    v = rng.standard_normal(2048).astype(np.float32)
    c0, s0, _ = quant.quantize_per_tensor(v, fmt)
    c1, s1, _ = quant.quantize_per_tensor(v * np.float32(2.0 ** k), fmt)
    assert np.array_equal(c0, c1)
    assert s1 == np.float32(s0 * np.float32(2.0 ** -k))


def test_scale_guards_and_pow2():
    assert quant.scale_from_amax(np.float32(0), fp8.E4M3) == 1.0
    assert quant.scale_from_amax(np.float32(1e-40), fp8.E4M3) == np.finfo(np.float32).max
    c, s, a = quant.quantize_per_tensor(np.zeros(8, np.float32), fp8.E4M3)
    assert s == 1 and a == 0 and not c.any()
    for amax in [0.3, 1.0, 5.5, 448.0, 1000.0]:
        s = float(quant.scale_from_amax(np.float32(amax), fp8.E4M3, pow2=True))
        exact = 448.0 / amax
        assert s == 2.0 ** math.floor(math.log2(float(np.float32(448) / np.float32(amax))))
        assert s <= exact * (1 + 1e-6) and s > exact / 2
    # NaN is ignored by amax
    assert quant.amax(np.array([1.0, np.nan, -3.0], np.float32)) == 3.0


def test_given_scale_saturation_and_flush_counts():
    v = np.array([1.0, 100.0, -1000.0, 1e-6, 0.0], np.float32)
    scale = np.float32(4.0)          # stale scale: 100*4 fits, 1000*4 does not
    codes, s, _ = quant.quantize_per_tensor(v, fp8.E4M3, scale=scale)
    assert s == scale
    assert codes.tolist() == [fp8.satcast_scalar(4.0, fp8.E4M3), fp8.satcast_scalar(400.0, fp8.E4M3), 0xFE, 0, 0]
    assert quant.count_saturated(v, scale, fp8.E4M3) == 1
    assert quant.count_flushed(v, codes) == 1
