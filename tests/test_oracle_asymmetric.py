"""Pins for the oracle's asymmetric (zero-point) activation grid (App. D: scale and offset are parameters)."""
import math
from fractions import Fraction

import numpy as np
import pytest

import fptq_workloads as synth


def test_zero_point_zero_is_the_symmetric_quantizer(oracle):
    rng = np.random.default_rng(0)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((5, 70)).astype(np.float32) * 4)
    r = rng.uniform(0.5, 2, 5).astype(np.float32)
    assert np.array_equal(oracle.quantize_zp(xb, np.float32(0.7), 0, r), oracle.quantize(xb, np.float32(0.7), r))
    acc = rng.integers(-1000, 1000, (5, 6)).astype(np.int32)
    s_w = rng.uniform(0.005, 0.02, 6).astype(np.float32)
    ws = rng.integers(-100, 100, 6).astype(np.int32)
    assert np.array_equal(oracle.epilogue_zp(acc, np.float32(0.3), s_w, 0, ws), oracle.epilogue(acc, np.float32(0.3), s_w))


@pytest.mark.parametrize("zp", [-8, -5, 3, 7])
def test_scalar_rule_against_exact_arithmetic(oracle, zp):
    L = oracle.lib()
    c32 = float(np.float32(0.7310586))
    for bits in range(0, 0x10000, 3):
        if (bits >> 7) & 0xFF == 0xFF:
            continue
        x = Fraction(float(L.oracle_bf16_to_f32(bits)))
        u = Fraction(float(np.float32(float(x * Fraction(c32)))))      # the one fp32 rounding
        fl = math.floor(u)
        d = u - fl
        rne = fl + 1 if d > Fraction(1, 2) else fl if d < Fraction(1, 2) else fl + (fl % 2)
        assert L.oracle_quantize_scalar_zp(bits, c32, zp) == max(-8, min(7, rne + zp))
    assert L.oracle_quantize_scalar_zp(0x7FC0, 1.0, zp) == zp                 # NaN -> the code of zero
    assert L.oracle_quantize_scalar_zp(0x0000, 1.0, zp) == zp


def test_accumulator_identity_and_row_sums(oracle):
    """sum_k (v - z) w = acc - z * sum_k w, exactly."""
    rng = np.random.default_rng(1)
    v = rng.integers(-8, 8, (7, 96), dtype=np.int8)
    w = rng.integers(-8, 8, (9, 96), dtype=np.int8)
    ws = oracle.weight_row_sums(w)
    assert np.array_equal(ws, w.astype(np.int64).sum(1))
    acc = oracle.gemm_i64(v, w)
    for z in (-8, -3, 0, 7):
        want = (v.astype(np.int64) - z) @ w.astype(np.int64).T
        assert np.array_equal(acc - z * ws[None, :].astype(np.int64), want)
        y = synth.bf16_bits_to_f32(oracle.epilogue_zp(acc.astype(np.int32), np.float32(1.0), np.ones(9, np.float32), z, ws))
        assert np.array_equal(y, synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(want.astype(np.float32))))


def test_asymmetric_grid_halves_the_error_on_one_sided_activations(oracle):
    """Non-negative activations (what a gated unit emits): the symmetric grid wastes its negative half."""
    rng = np.random.default_rng(2)
    x = np.abs(rng.standard_normal((16, 256))).astype(np.float32)
    xb = synth.f32_to_bf16_bits(x)
    xv = synth.bf16_bits_to_f32(xb).astype(np.float64)
    amax = xv.max()
    s_sym, s_asym = np.float32(amax / 7.0), np.float32(amax / 15.0)
    q0 = oracle.quantize_zp(xb, s_sym, 0)
    q1 = oracle.quantize_zp(xb, s_asym, -8)
    e0 = np.abs(xv - float(s_sym) * q0).mean()
    e1 = np.abs(xv - float(s_asym) * (q1.astype(np.float64) + 8)).mean()
    assert q1.min() == -8 and q1.max() == 7 and q0.min() >= 0
    assert e1 < 0.6 * e0
    with pytest.raises(ValueError):
        oracle.quantize_zp(xb, s_sym, 8)
