"""Pins for the oracle's FP8 codec, bf16 rounding and per-tensor quantizer.

Nothing here calls the GPU path.  The oracle is checked against: hand-worked codes
(tests/golden/fp8_encode_pins.txt), a brute-force nearest-value search written here
from the format definition, PyTorch's CPU float8 casts (an independent library
routine), and closed forms of the quantizer.
"""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fp8_encode_pins.txt")
FMT = {"E4M3": oracle.E4M3, "E5M2": oracle.E5M2}
FMAX = {oracle.E4M3: 448.0, oracle.E5M2: 57344.0}


def _value_table(fmt):
    """All finite code values, built here from the format definition (not from the oracle)."""
    mbits, bias = (3, 7) if fmt == oracle.E4M3 else (2, 15)
    vals = {}
    for code in range(128):
        field, mant = code >> mbits, code & ((1 << mbits) - 1)
        if fmt == oracle.E4M3 and code == 0x7F:
            continue
        if fmt == oracle.E5M2 and field == 31:
            continue
        if field == 0:
            v = mant * 2.0 ** (1 - bias - mbits)
        else:
            v = (1 + mant / (1 << mbits)) * 2.0 ** (field - bias)
        vals[code] = v
    return vals


def _brute_force_encode(v, fmt, table):
    """Nearest representable magnitude by exhaustive search; ties -> even code; saturating."""
    a = min(abs(float(v)), max(table.values()))          # saturating
    sign = 0x80 if np.signbit(np.float32(v)) else 0
    best, best_d = None, None
    for code, val in table.items():
        d = abs(val - a)
        if best is None or d < best_d or (d == best_d and code % 2 == 0 and best % 2 == 1):
            best, best_d = code, d
    return sign | best


def test_golden_pins():
    n = 0
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, val, code = line.split()[:3]
            got = int(oracle.fp8_encode([float.fromhex(val)], FMT[name])[0])
            assert got == int(code, 16), (line, hex(got))
            n += 1
    assert n >= 40


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_decode_matches_definition(fmt):
    table = _value_table(fmt)
    dec = oracle.fp8_decode(np.arange(256, dtype=np.uint8), fmt)
    for code, val in table.items():
        assert dec[code] == val
        assert dec[code | 0x80] == -val
    assert max(table.values()) == FMAX[fmt] == oracle.fp8_max(fmt)
    if fmt == oracle.E4M3:
        assert np.isnan(dec[0x7F]) and np.isnan(dec[0xFF])
    else:
        assert np.isinf(dec[0x7C]) and np.isnan(dec[0x7D]) and np.isnan(dec[0x7F])


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_round_trip_every_finite_code(fmt):
    table = _value_table(fmt)
    codes = np.array(sorted(table) + [c | 0x80 for c in sorted(table)], np.uint8)
    back = oracle.fp8_encode(oracle.fp8_decode(codes, fmt).astype(np.float32), fmt)
    assert np.array_equal(back, codes)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_encode_vs_brute_force_search(fmt):
    """Every representable value, every midpoint between neighbours, and values one fp32 ulp
    either side of each, against a nearest-value search over the whole code table."""
    table = _value_table(fmt)
    vals = np.array(sorted(table.values()), np.float64)
    mids = (vals[:-1] + vals[1:]) / 2
    pts = np.concatenate([vals, mids]).astype(np.float32)      # all exactly representable in fp32
    pts = np.concatenate([pts, np.nextafter(pts, np.float32(np.inf)), np.nextafter(pts, np.float32(-np.inf))])
    pts = pts[pts >= 0]
    pts = np.concatenate([pts, -pts, np.float32([FMAX[fmt] * 1.01, FMAX[fmt] * 4, 3e38])])
    got = oracle.fp8_encode(pts, fmt)
    for v, c in zip(pts, got):
        assert c == _brute_force_encode(v, fmt, table), (float(v), hex(c))


@pytest.mark.parametrize("fmt,tdtype", [(oracle.E4M3, torch.float8_e4m3fn), (oracle.E5M2, torch.float8_e5m2)])
def test_encode_vs_torch_cpu_cast(fmt, tdtype):
    """PyTorch's CPU cast is round-to-nearest-even but not saturating: clamp first."""
    g = np.random.default_rng(7)
    # every bf16 bit pattern (finite), plus random fp32 bit patterns, plus log-uniform magnitudes
    bf = (np.arange(65536, dtype=np.uint32) << 16).view(np.float32)
    rnd = g.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32).view(np.float32)
    logu = (np.exp(g.uniform(np.log(1e-8), np.log(1e6), size=1 << 20)) * g.choice([-1, 1], size=1 << 20)).astype(np.float32)
    v = np.concatenate([bf, rnd, logu])
    v = v[np.isfinite(v)]
    t = torch.from_numpy(v).clamp(-FMAX[fmt], FMAX[fmt]).to(tdtype).view(torch.uint8).numpy()
    got = oracle.fp8_encode(v, fmt)
    assert np.array_equal(got, t)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_monotone_and_sign_symmetric(fmt):
    g = np.random.default_rng(11)
    v = np.sort(np.exp(g.uniform(np.log(1e-7), np.log(1e5), size=200000)).astype(np.float32))
    c = oracle.fp8_encode(v, fmt).astype(np.int32)
    assert np.all(np.diff(c) >= 0)                 # positive codes order like their values
    assert np.array_equal(oracle.fp8_encode(-v, fmt), (c | 0x80).astype(np.uint8))
    d = oracle.fp8_decode(c.astype(np.uint8), fmt)
    # nearest: error at most half the local spacing (checked through the neighbours)
    table = np.array(sorted(_value_table(fmt).values()))
    pos = np.searchsorted(table, np.minimum(v.astype(np.float64), FMAX[fmt]))
    lo = table[np.maximum(pos - 1, 0)]
    hi = table[np.minimum(pos, len(table) - 1)]
    best = np.minimum(np.abs(lo - np.minimum(v, FMAX[fmt])), np.abs(hi - np.minimum(v, FMAX[fmt])))
    assert np.all(np.abs(d - np.minimum(v.astype(np.float64), FMAX[fmt])) <= best + 0.0)


def test_round_bf16_vs_torch():
    g = np.random.default_rng(3)
    v = np.concatenate([g.normal(size=100000) * 10.0 ** g.integers(-20, 20, size=100000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 1 + 2 ** -8, 1 + 3 * 2 ** -8]])
    f32 = v.astype(np.float32).astype(np.float64)             # exactly representable in fp32
    want = torch.from_numpy(f32.astype(np.float32)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.round_bf16(f32), want)
    # hand-worked ties: 1 + 2^-8 is halfway 1 | 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.round_bf16([1 + 2 ** -8])[0] == 1.0
    assert oracle.round_bf16([1 + 3 * 2 ** -8])[0] == 1 + 2 ** -6


# ---------------------------------------------------------------------------------------
# quantizer
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("fmt,maxcode", [(oracle.E4M3, 0x7E), (oracle.E5M2, 0x7B)])
def test_quantize_amax_maps_to_max_code(fmt, maxcode):
    g = np.random.default_rng(5)
    x = g.normal(size=(37, 53)).astype(np.float32)
    x[11, 17] = -7.25                                   # the largest magnitude, negative
    q, s, amax = oracle.quantize(x, fmt)
    assert amax == np.float32(7.25)
    assert s == np.float32(FMAX[fmt]) / np.float32(7.25)
    assert q[11, 17] == (maxcode | 0x80)
    assert np.all((q & 0x7F) <= maxcode)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_quantize_power_of_two_scale_reproduces_pins(fmt):
    """amax = fmt_max / 4 gives scale exactly 4, so codes are the plain encodings of 4x."""
    vals = np.array([1.0, 0.5, 1.0625, 1.1875, 17, 19, 0.1, 0.3, 3.14159, -2.5, 0.0], np.float32)
    x = np.concatenate([vals / 4, [FMAX[fmt] / 4]]).astype(np.float32)
    q, s, amax = oracle.quantize(x, fmt)
    assert s == 4.0 and amax == np.float32(FMAX[fmt] / 4)
    assert np.array_equal(q[:-1], oracle.fp8_encode((vals / 4) * np.float32(4), fmt))


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_quantize_idempotent_with_exact_scale(fmt):
    g = np.random.default_rng(9)
    codes = g.integers(0, 256, size=4096).astype(np.uint8)
    dec = oracle.fp8_decode(codes, fmt)
    keep = np.isfinite(dec)
    codes, dec = codes[keep], dec[keep]
    s = np.float32(8.0)
    q, s_out, _ = oracle.quantize((dec / 8.0).astype(np.float32), fmt, scale_in=s)
    assert s_out == s
    assert np.array_equal(q, codes)


def test_quantize_all_zero_tensor():
    q, s, amax = oracle.quantize(np.zeros((4, 8), np.float32), oracle.E4M3)
    assert amax == 0 and np.all(q == 0)
    assert s == np.float32(448.0) / np.float32(1e-12)
    q, s, _ = oracle.quantize(np.zeros(5, np.float32), oracle.E5M2)
    assert s == np.float32(57344.0) / np.float32(1e-12) and np.all(q == 0)


def test_quantize_supplied_scale_saturates():
    """Adapter rows are cast with the backbone's scale; entries beyond its range clip."""
    a = np.array([0.01, -0.2, 0.5, 3.0], np.float32)
    q, s, amax = oracle.quantize(a, oracle.E4M3, scale_in=np.float32(1000.0))
    assert s == np.float32(1000.0) and amax == np.float32(3.0)
    assert list(q) == [int(oracle.fp8_encode([10.0], 0)[0]), int(oracle.fp8_encode([-200.0], 0)[0]), 0x7E, 0x7E]


def test_quantize_product_is_rounded_to_fp32_before_the_cast():
    """The cast sees fl32(x*s), not the exact product.  Find inputs where the two round to
    different codes (the fp32 product lands exactly on a halfway point that the exact product
    misses) and check the quantizer follows the fp32 product."""
    table = _value_table(oracle.E4M3)
    vals = np.array(sorted(table.values()))
    mids = (vals[:-1] + vals[1:]) / 2
    s = np.float32(448.0) / np.float32(3.0)           # 149.33333, inexact
    # candidates: the fp32 numbers within a few ulps of mid/s, for every halfway point and a
    # family of scales' worth of neighbours
    x0 = (mids[mids > 0.01] / np.float64(s)).astype(np.float32)
    cand = [x0]
    for _ in range(6):
        cand.append(np.nextafter(cand[-1], np.float32(np.inf)))
    lo = x0
    for _ in range(6):
        lo = np.nextafter(lo, np.float32(0))
        cand.append(lo)
    x = np.unique(np.concatenate(cand))
    x = x[x < 3.0]
    p32 = (x * s).astype(np.float64)                  # numpy fp32 multiply, widened
    p64 = x.astype(np.float64) * np.float64(s)        # exact product (24 x 24 bits fit in fp64)
    on_mid = np.isin(p32, mids) & (p64 != p32)
    assert on_mid.sum() > 0
    xs = x[on_mid]
    want = np.array([_brute_force_encode(v, oracle.E4M3, table) for v in p32[on_mid]], np.uint8)
    other = np.array([_nearest_no_tie(v, table) for v in p64[on_mid]], np.uint8)
    assert np.any(want != other)                      # the distinction is real for these inputs
    q, s_out, _ = oracle.quantize(np.concatenate([xs, [3.0]]).astype(np.float32), oracle.E4M3)
    assert s_out == s
    assert np.array_equal(q[:-1], want)


def _nearest_no_tie(a, table):
    return min(table, key=lambda c: abs(table[c] - a))
