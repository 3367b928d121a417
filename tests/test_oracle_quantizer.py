"""Pins for the oracle's conversions, row scale, scalar quantizer and packing.

None of these re-types the oracle's formula: the quantizer is checked against exact rational
arithmetic over every bf16 bit pattern, the conversions against an independent library
(torch CPU), the row scale against closed forms and an exactly rounded sum.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch


def frac_of_f32(f):
    return Fraction(float(np.float32(f)))


def bf16_fraction(bits):
    """Exact rational value of a finite bf16 bit pattern, decoded field by field."""
    sign = -1 if bits >> 15 else 1
    e = (bits >> 7) & 0xFF
    m = bits & 0x7F
    if e == 0xFF:
        return None
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(2) ** (-126)
    return sign * (1 + Fraction(m, 1 << 7)) * Fraction(2) ** (e - 127)


def round_half_even(fr):
    fl = math.floor(fr)
    d = fr - fl
    if d > Fraction(1, 2):
        return fl + 1
    if d < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def clamp(v):
    return max(-8, min(7, v))


# ------------------------------------------------------------------ conversions
def test_bf16_widening_matches_field_decode(oracle):
    L = oracle.lib()
    for bits in list(range(0, 0x10000, 7)) + [0x0000, 0x8000, 0x0001, 0x007F, 0x0080, 0x7F7F, 0xFF7F]:
        fr = bf16_fraction(bits)
        if fr is None:
            continue
        assert Fraction(float(L.oracle_bf16_to_f32(bits))) == fr


def test_bf16_rounding_roundtrip_and_ties(oracle):
    L = oracle.lib()
    # every finite bf16 value converts back to itself
    for bits in range(0x10000):
        if (bits >> 7) & 0xFF == 0xFF:
            continue
        f = L.oracle_bf16_to_f32(bits)
        assert L.oracle_f32_to_bf16(f) == bits
    # exact ties go to the even neighbour: 1 + 2^-8 is halfway between 1.0 (0x3F80, even) and 0x3F81
    assert L.oracle_f32_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert L.oracle_f32_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    assert L.oracle_f32_to_bf16(float(np.float32(1.0 + 2.0 ** -8 + 2.0 ** -20))) == 0x3F81
    assert L.oracle_f32_to_bf16(-(1.0 + 2.0 ** -8)) == 0xBF80
    assert L.oracle_f32_to_bf16(float("inf")) == 0x7F80
    nan_bits = L.oracle_f32_to_bf16(float("nan"))
    assert (nan_bits & 0x7F80) == 0x7F80 and (nan_bits & 0x7F) != 0


def test_bf16_rounding_matches_torch(oracle):
    rng = np.random.default_rng(5)
    vals = np.concatenate([rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 6, 20000).astype(np.float32),
                           np.array([0.0, -0.0, 1e-40, -1e-40, 3.3895e38, 65504.0], np.float32)])
    want = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    L = oracle.lib()
    got = np.array([L.oracle_f32_to_bf16(float(v)) for v in vals], np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ scalar quantizer, brute force
C_VALUES = [1.0, 0.5, 1.0 / 3.0, 0.7310586, 2.718281828, 13.37, 1.0 / 6.1234, 123.456]


@pytest.mark.parametrize("c", C_VALUES)
def test_quantizer_brute_force_all_bf16(oracle, c):
    """Every bf16 input against exact rational arithmetic: equal, except where the exact product
    sits within fp32 rounding distance of a half-integer; there it must be one of the two
    neighbours."""
    L = oracle.lib()
    c32 = float(np.float32(c))
    cf = Fraction(c32)
    near_tie = 0
    for bits in range(0x10000):
        xf = bf16_fraction(bits)
        got = L.oracle_quantize_scalar(bits, c32)
        if xf is None:
            continue
        p = xf * cf
        ideal = clamp(round_half_even(p))
        lo, hi = clamp(math.floor(p)), clamp(math.ceil(p))
        if abs(p) >= 9:                       # far outside the grid: fp32 rounding cannot matter
            assert got == ideal, (hex(bits), c, got, ideal)
            continue
        # distance of p to the nearest half-integer
        nearest_odd = 2 * math.floor(p) + 1
        dist = abs(p * 2 - nearest_odd) / 2
        exact_in_f32 = Fraction(float(np.float32(float(p)))) == p
        if exact_in_f32 or dist > abs(p) * Fraction(1, 1 << 23):
            assert got == ideal, (hex(bits), c, got, ideal)
        else:
            near_tie += 1
            assert got in (lo, hi), (hex(bits), c, got, lo, hi)
    # the excluded band is tiny: a handful of inputs per multiplier
    assert near_tie < 200


def test_quantizer_explicit_ties_clamp_and_specials(oracle):
    L = oracle.lib()
    from fptq_workloads import f32_to_bf16_bits
    b = lambda v: int(f32_to_bf16_bits(np.array([v], np.float32))[0])
    q = lambda v, c: L.oracle_quantize_scalar(b(v), float(np.float32(c)))
    # x * 0.5 is exact: ties go to even
    assert [q(v, 0.5) for v in (1.0, 3.0, 5.0, 7.0, -1.0, -3.0, -5.0)] == [0, 2, 2, 4, 0, -2, -2]
    # clamp edges: 7.5 -> 8 -> 7 ; -8.5 -> -8 ; 6.5 -> 6 ; -7.5 -> -8
    assert [q(v, 0.5) for v in (15.0, -17.0, 13.0, -15.0, 14.0, -16.0, 100.0, -100.0)] == [7, -8, 6, -8, 7, -8, 7, -8]
    # zeros, subnormals, infinities, NaN
    assert q(0.0, 3.0) == 0
    assert L.oracle_quantize_scalar(0x8000, 3.0) == 0           # -0.0
    assert L.oracle_quantize_scalar(0x0001, 1e30) == 0          # smallest subnormal * 1e30 = 9.2e-11
    assert L.oracle_quantize_scalar(0x7F80, 1.0) == 7           # +inf
    assert L.oracle_quantize_scalar(0xFF80, 1.0) == -8          # -inf
    assert L.oracle_quantize_scalar(0x7FC0, 1.0) == 0           # NaN
    assert L.oracle_quantize_scalar(0x7F80, 0.0) == 0           # inf * 0 = NaN -> 0


def test_row_multiplier_is_one_division_then_one_multiply(oracle):
    """c_t = S_t * (1 / s_a), every step rounded to fp32: checked with exact rationals."""
    L = oracle.lib()
    rng = np.random.default_rng(11)
    for _ in range(2000):
        s_a = float(np.float32(rng.uniform(0.01, 10)))
        r = float(np.float32(rng.uniform(0.01, 10)))
        inv = np.float32(Fraction(1) / Fraction(s_a))          # correctly rounded 1/s_a
        want = np.float32(Fraction(float(inv)) * Fraction(r))   # correctly rounded product
        assert L.oracle_row_multiplier(r, s_a, 1) == float(want)
        assert L.oracle_row_multiplier(r, s_a, 0) == float(inv)


# ------------------------------------------------------------------ row scale (Sec. 3.1.3)
def test_row_scale_closed_forms(oracle):
    from fptq_workloads import f32_to_bf16_bits
    K = 256
    # constant row x = c -> S = 1/|c|
    for c in (1.0, -2.0, 0.5, 3.0, -1.5, 0.0078125):
        x = f32_to_bf16_bits(np.full((1, K), c, np.float32))
        r = oracle.row_scale(x, oracle.MODE_RMS, 0.0)
        assert r[0] == np.float32(1.0 / abs(c))
    # a single non-zero a in a row of K = 256 -> RMS = |a| / 16 -> S = 16 / |a|
    for a in (3.0, -5.0, 0.75, 96.0):
        row = np.zeros((1, K), np.float32)
        row[0, 17] = a
        r = oracle.row_scale(f32_to_bf16_bits(row), oracle.MODE_RMS, 0.0)
        assert r[0] == np.float32(16.0 / abs(a))
    # eps enters under the root: zero row with eps -> 1/sqrt(eps)
    r = oracle.row_scale(np.zeros((1, K), np.uint16), oracle.MODE_RMS, 0.25)
    assert r[0] == np.float32(2.0)
    # modes NONE and GIVEN
    x = f32_to_bf16_bits(np.ones((3, K), np.float32))
    assert np.array_equal(oracle.row_scale(x, oracle.MODE_NONE), np.ones(3, np.float32))
    g = np.array([0.5, 2.0, 7.0], np.float32)
    assert np.array_equal(oracle.row_scale(x, oracle.MODE_GIVEN, 0.0, g), g)


def test_row_scale_against_exact_sum(oracle):
    """Random rows: within one fp32 ulp of the value computed from an exactly rounded sum."""
    from fptq_workloads import f32_to_bf16_bits, bf16_bits_to_f32
    rng = np.random.default_rng(3)
    x = rng.standard_normal((64, 1000)).astype(np.float32)
    x[:, 5] *= 40
    bits = f32_to_bf16_bits(x)
    xv = bf16_bits_to_f32(bits).astype(np.float64)
    eps = 1e-5
    r = oracle.row_scale(bits, oracle.MODE_RMS, eps)
    for t in range(64):
        ss = math.fsum(float(v) * float(v) for v in xv[t])
        want = 1.0 / math.sqrt(ss / 1000 + eps)
        assert abs(float(r[t]) - want) <= np.spacing(np.float32(want))


# ------------------------------------------------------------------ packing (App. J)
def test_pack_known_bytes(oracle):
    v = np.array([[-8, 7, -1, 1, 0, -2, 5, 3]], np.int8)
    assert oracle.pack(v).tolist() == [[0x78, 0x1F, 0xE0, 0x35]]


def test_pack_unpack_exhaustive(oracle):
    # all 16 x 16 nibble pairs
    pairs = np.array([[a, b] for a in range(-8, 8) for b in range(-8, 8)], np.int8)
    packed = oracle.pack(pairs)
    assert packed.shape == (256, 1)
    assert sorted(packed[:, 0].tolist()) == list(range(256))      # a bijection onto the byte values
    assert np.array_equal(oracle.unpack(packed, 2), pairs)
    # every byte value round-trips the other way
    allbytes = np.arange(256, dtype=np.uint8).reshape(1, 256)
    assert np.array_equal(oracle.pack(oracle.unpack(allbytes, 512)), allbytes)
    # sign extension spelled out: nibble 0xF is -1, 0x8 is -8, 0x7 is 7
    assert oracle.unpack(np.array([[0x8F, 0x07]], np.uint8), 4).tolist() == [[-1, -8, 7, 0]]


def test_quantize_tensor_uses_the_scalar_rule(oracle):
    """The tensor routine equals the brute-forced scalar rule element by element (ragged sizes)."""
    from fptq_workloads import f32_to_bf16_bits
    rng = np.random.default_rng(9)
    x = f32_to_bf16_bits(rng.standard_normal((7, 34)).astype(np.float32) * 5)
    r = rng.uniform(0.5, 2, 7).astype(np.float32)
    s_a = np.float32(0.83)
    q = oracle.quantize(x, s_a, r)
    L = oracle.lib()
    for t in range(7):
        c = L.oracle_row_multiplier(float(r[t]), float(s_a), 1)
        for k in range(34):
            assert q[t, k] == L.oracle_quantize_scalar(int(x[t, k]), c)
    q0 = oracle.quantize(x, s_a, None)
    c0 = L.oracle_row_multiplier(1.0, float(s_a), 0)
    assert q0[3, 5] == L.oracle_quantize_scalar(int(x[3, 5]), c0)
