"""Pins for the reference implementation's element formats (CPU only).

The paper names the element formats (Table 1) and defers their bit layouts to
the OCP FP8 / MX documents.  The decode tables are pinned here against an
independent library (PyTorch's float8 dtypes), against the well-known literal
values of the small formats, and against structural facts that follow from
"sign / x exponent bits / y mantissa bits, bias 2^(x-1)-1".  The encoder is
pinned against the definition "nearest representable value, ties by mode,
finite overflow clamps" evaluated by brute force in exact rational arithmetic,
and against PyTorch's float8 conversion where that applies.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

E4M3, E5M2, E3M2, E2M3, E2M1, INT8 = range(6)
RNE, AWAY = 0, 1
BITS = {E4M3: 8, E5M2: 8, E3M2: 6, E2M3: 6, E2M1: 4, INT8: 8}


def test_widths_and_emax(oracle):
    # Table 1: element bit-widths; emax = exponent of the largest normal
    assert [oracle.elem_bits(f) for f in range(6)] == [8, 8, 6, 6, 4, 8]
    assert [oracle.emax(f) for f in range(6)] == [8, 15, 4, 2, 2, 0]
    assert oracle.elem_bits(6) == -1


def test_decode_fp8_against_torch(oracle):
    codes = torch.arange(256, dtype=torch.uint8)
    for fmt, dt in ((E4M3, torch.float8_e4m3fn), (E5M2, torch.float8_e5m2)):
        ref = codes.view(dt).to(torch.float64).numpy()
        got = np.array([oracle.decode(fmt, c) for c in range(256)])
        assert np.array_equal(np.isnan(ref), np.isnan(got))
        ok = ~np.isnan(ref)
        assert np.array_equal(ref[ok], got[ok])
        assert np.array_equal(np.signbit(ref[ok]), np.signbit(got[ok]))


def test_decode_literals(oracle):
    # FP4 E2M1: the eight magnitudes of a 1-2-1 format with bias 1
    assert [oracle.decode(E2M1, c) for c in range(8)] == [0, 0.5, 1, 1.5, 2, 3, 4, 6]
    assert [oracle.decode(E2M1, c) for c in range(9, 16)] == [-0.5, -1, -1.5, -2, -3, -4, -6]
    assert math.copysign(1, oracle.decode(E2M1, 8)) == -1 and oracle.decode(E2M1, 8) == 0
    # extreme values of each format
    assert oracle.decode(E4M3, 0x7E) == 448 and oracle.decode(E4M3, 0x08) == 2.0**-6
    assert oracle.decode(E4M3, 0x01) == 2.0**-9 and math.isnan(oracle.decode(E4M3, 0x7F))
    assert math.isnan(oracle.decode(E4M3, 0xFF)) and oracle.decode(E4M3, 0x78) == 256
    assert oracle.decode(E5M2, 0x7B) == 57344 and oracle.decode(E5M2, 0x7C) == math.inf
    assert oracle.decode(E5M2, 0xFC) == -math.inf and oracle.decode(E5M2, 0x01) == 2.0**-16
    assert all(math.isnan(oracle.decode(E5M2, c)) for c in (0x7D, 0x7E, 0x7F, 0xFD, 0xFE, 0xFF))
    assert oracle.decode(E3M2, 0x1F) == 28 and oracle.decode(E3M2, 0x01) == 0.0625
    assert oracle.decode(E3M2, 0x04) == 0.25 and oracle.decode(E3M2, 0x3F) == -28
    assert oracle.decode(E2M3, 0x1F) == 7.5 and oracle.decode(E2M3, 0x01) == 0.125
    assert oracle.decode(E2M3, 0x08) == 1.0 and oracle.decode(E2M3, 0x3F) == -7.5
    assert oracle.decode(INT8, 0x40) == 1.0 and oracle.decode(INT8, 0x7F) == 1.984375
    assert oracle.decode(INT8, 0xFF) == -1.0 / 64 and oracle.decode(INT8, 0x80) == -2.0
    # codes are masked to the element width
    assert oracle.decode(E2M1, 0x17) == 6 and oracle.decode(E3M2, 0x5F) == 28


@pytest.mark.parametrize("fmt,ebits,mbits", [(E4M3, 4, 3), (E5M2, 5, 2), (E3M2, 3, 2), (E2M3, 2, 3), (E2M1, 2, 1)])
def test_decode_structure(oracle, fmt, ebits, mbits):
    """Facts any sign/exponent/mantissa format obeys: positive finite codes are
    strictly increasing; negative codes mirror them; spacing is constant inside
    a binade (2^mbits codes), equal in the two lowest binades (subnormals share
    the first normal binade's step) and doubles from one binade to the next;
    code 2^mbits (first normal) equals 2^(1-bias)."""
    half = 1 << (BITS[fmt] - 1)
    vals = [oracle.decode(fmt, c) for c in range(half)]
    fin = [v for v in vals if math.isfinite(v)]
    assert all(b > a for a, b in zip(fin, fin[1:]))
    for c in range(half):
        n = oracle.decode(fmt, c | half)
        assert (math.isnan(n) and math.isnan(vals[c])) or n == -vals[c]
    m = 1 << mbits
    bias = (1 << (ebits - 1)) - 1
    assert vals[m] == 2.0 ** (1 - bias)
    steps = [fin[i + 1] - fin[i] for i in range(len(fin) - 1)]
    for i, s in enumerate(steps):
        binade = i // m
        expect = steps[0] * 2.0 ** max(binade - 1, 0)
        assert s == expect, (i, s, expect)
    assert steps[0] == 2.0 ** (1 - bias - mbits)


def test_decode_int8_is_twos_complement(oracle):
    ref = np.arange(256, dtype=np.uint8).view(np.int8).astype(np.float64) / 64.0
    got = np.array([oracle.decode(INT8, c) for c in range(256)])
    assert np.array_equal(ref, got)


# ---------------------------------------------------------------- encoder ----
def _finite_table(oracle, fmt):
    """(magnitude as Fraction, code) for the non-negative finite codes that the
    encoder may emit, in increasing order."""
    half = 1 << (BITS[fmt] - 1)
    out = []
    for c in range(half):
        v = oracle.decode(fmt, c)
        if math.isfinite(v):
            out.append((Fraction(v), c))
    return out


def _nearest(table, x: Fraction, rnd):
    """Brute-force definition: the table entry closest to |x|; a tie goes to the
    entry with even code (ties-to-even) or the larger one (ties-away); anything
    beyond the largest entry clamps to it."""
    a = abs(x)
    if a >= table[-1][0]:
        return table[-1][1]
    best = min(abs(a - v) for v, _ in table)
    cands = [(v, c) for v, c in table if abs(a - v) == best]
    if len(cands) == 1:
        return cands[0][1]
    assert len(cands) == 2
    if rnd == AWAY:
        return max(cands)[1]
    return [c for _, c in cands if c % 2 == 0][0]


def _sweep(table, rng, n_random):
    """Every table value, every midpoint, both neighbours of every midpoint at
    several distances, and random points across and beyond the range."""
    xs = []
    vals = [v for v, _ in table]
    for a, b in zip(vals, vals[1:]):
        mid = (a + b) / 2
        xs += [a, mid]
        for k in (20, 40, 52):
            d = (b - a) * Fraction(1, 2**k)
            xs += [mid - d, mid + d, a + d, b - d]
    top = vals[-1]
    xs += [top, top * Fraction(17, 16), top * 2 - Fraction(1, 2**30), top * 1000, Fraction(1, 2**60), Fraction(0)]
    xs += [Fraction(float(top) * 1.2 * rng.random()) for _ in range(n_random)]
    xs += [Fraction(float(vals[1]) * 4 * rng.random()) for _ in range(n_random // 4)]
    # only values a double holds exactly can be passed to the C function
    return [x for x in xs if Fraction(float(x)) == x]


@pytest.mark.parametrize("fmt", [E4M3, E5M2, E3M2, E2M3, E2M1])
@pytest.mark.parametrize("rnd", [RNE, AWAY])
def test_encode_is_nearest_value_fp(oracle, fmt, rnd):
    rng = np.random.default_rng(100 + fmt)
    table = _finite_table(oracle, fmt)
    half = 1 << (BITS[fmt] - 1)
    xs = _sweep(table, rng, 4000)
    assert len(xs) > 4000
    for x in xs:
        want = _nearest(table, x, rnd)
        assert oracle.encode(fmt, rnd, float(x)) == want, (float(x), want)
        if x != 0:
            assert oracle.encode(fmt, rnd, -float(x)) == (want | half), float(x)
    # signed zero keeps its sign
    assert oracle.encode(fmt, rnd, 0.0) == 0 and oracle.encode(fmt, rnd, -0.0) == half


@pytest.mark.parametrize("rnd", [RNE, AWAY])
def test_encode_is_nearest_value_int8(oracle, rnd):
    rng = np.random.default_rng(7)
    table = [(Fraction(k, 64), k) for k in range(128)]  # 0x80 (-2.0) is never emitted
    for x in _sweep(table, rng, 4000):
        k = _nearest(table, x, rnd)
        assert oracle.encode(INT8, rnd, float(x)) == k
        assert oracle.encode(INT8, rnd, -float(x)) == (-k) & 0xFF
    assert oracle.encode(INT8, rnd, -0.0) == 0
    assert oracle.encode(INT8, rnd, -5.0) == 0x81  # symmetric clamp, never 0x80


@pytest.mark.parametrize("fmt", range(6))
def test_encode_roundtrips_every_code(oracle, fmt):
    for c in range(1 << BITS[fmt]):
        v = oracle.decode(fmt, c)
        if math.isnan(v) or (fmt == INT8 and c == 0x80):
            continue
        for rnd in (RNE, AWAY):
            assert oracle.encode(fmt, rnd, v) == c, (c, v)


@pytest.mark.parametrize("fmt,dt,top", [(E4M3, torch.float8_e4m3fn, 448.0), (E5M2, torch.float8_e5m2, 57344.0)])
def test_encode_rne_against_torch_float8(oracle, fmt, dt, top):
    """PyTorch's float32 -> float8 conversion rounds to nearest even; inside the
    finite range it must agree with the reference encoder bit for bit."""
    rng = np.random.default_rng(11 + fmt)
    x = np.concatenate([
        rng.uniform(-top, top, 40000),
        rng.standard_normal(40000) * top / 50,
        rng.standard_normal(20000) * (2.0**-8 if fmt == E4M3 else 2.0**-15),
        rng.integers(-1800, 1800, 4000) / 4096.0,
    ]).astype(np.float32)
    x = x[np.abs(x) <= top]
    ref = torch.from_numpy(x).to(dt).view(torch.uint8).numpy()
    got = np.array([oracle.encode(fmt, RNE, float(v)) for v in x], dtype=np.uint8)
    assert np.array_equal(ref, got)


@pytest.mark.parametrize("fmt", range(6))
@pytest.mark.parametrize("rnd", [RNE, AWAY])
def test_encode_monotone(oracle, fmt, rnd):
    top = {E4M3: 600, E5M2: 70000, E3M2: 40, E2M3: 10, E2M1: 8, INT8: 3}[fmt]
    xs = np.sort(np.random.default_rng(5).uniform(0, top, 20000))
    vals = [oracle.decode(fmt, oracle.encode(fmt, rnd, float(x))) for x in xs]
    assert all(b >= a for a, b in zip(vals, vals[1:]))


def test_encode_nonfinite(oracle):
    for rnd in (RNE, AWAY):
        assert oracle.encode(E4M3, rnd, math.nan) == 0x7F
        assert oracle.encode(E4M3, rnd, math.inf) == 0x7F      # no Inf code, never clamped
        assert oracle.encode(E4M3, rnd, -math.inf) == 0xFF
        assert oracle.encode(E5M2, rnd, math.nan) == 0x7E
        assert oracle.encode(E5M2, rnd, math.inf) == 0x7C
        assert oracle.encode(E5M2, rnd, -math.inf) == 0xFC
        # huge finite values clamp instead
        assert oracle.encode(E4M3, rnd, 1e300) == 0x7E and oracle.encode(E5M2, rnd, -1e300) == 0xFB
