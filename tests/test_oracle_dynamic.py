"""Pins for the oracle's dynamic (per-token, run-time) activation quantizer (App. B)."""
import math
from fractions import Fraction

import numpy as np

import fptq_workloads as synth


def test_scale_is_absmax_over_seven_and_codes_follow_exact_arithmetic(oracle):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((6, 40)).astype(np.float32) * np.array([[1], [10], [0.01], [300], [1], [5]], np.float32)
    xb = synth.f32_to_bf16_bits(x)
    xv = synth.bf16_bits_to_f32(xb)
    q, s = oracle.quantize_dynamic(xb)
    for t in range(6):
        amax = np.abs(xv[t]).max()
        want_s = np.float32(Fraction(float(amax)) / 7)               # correctly rounded division
        assert s[t] == want_s
        c = np.float32(Fraction(1) / Fraction(float(s[t])))          # correctly rounded reciprocal
        for k in range(40):
            p = Fraction(float(xv[t, k])) * Fraction(float(c))
            u = Fraction(float(np.float32(float(p))))                # one fp32 rounding of the product
            fl = math.floor(u)
            d = u - fl
            want = fl + 1 if d > Fraction(1, 2) else fl if d < Fraction(1, 2) else fl + (fl % 2)
            assert q[t, k] == max(-8, min(7, want))
        assert np.abs(q[t]).max() == 7                               # the largest element lands on the grid's end
        assert np.all(np.abs(xv[t] - s[t] * q[t]) <= s[t] * 0.5 * (1 + 1e-3))   # dequantization error at most half a step


def test_power_of_two_row_scaling_only_moves_the_scale(oracle):
    rng = np.random.default_rng(1)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((5, 64)).astype(np.float32))
    f = (2.0 ** rng.integers(-5, 6, 5)).astype(np.float32)
    xs = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(xb) * f[:, None])
    q1, s1 = oracle.quantize_dynamic(xb)
    q2, s2 = oracle.quantize_dynamic(xs)
    assert np.array_equal(q1, q2) and np.array_equal(s2, s1 * f)


def test_degenerate_rows(oracle):
    x = np.zeros((3, 16), np.float32)
    x[1, 3] = np.inf
    x[2, 2] = 5.0
    xb = synth.f32_to_bf16_bits(x)
    xb[2, 7] = 0x7FC0                                                # a NaN does not enter the maximum
    q, s = oracle.quantize_dynamic(xb)
    assert s[0] == 1.0 and not q[0].any()
    assert s[1] == 1.0 and q[1, 3] == 7
    assert s[2] == np.float32(5.0) / np.float32(7.0) and q[2, 2] == 7 and q[2, 7] == 0


def test_dynamic_linear_equals_float_layer_within_the_grid_error(oracle):
    """acc * s_t * s_w reproduces x (s_w w)^T up to the per-token half-step bound."""
    rng = np.random.default_rng(2)
    M, N, K = 12, 20, 128
    xb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.standard_normal((M, 1))).astype(np.float32))
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    q, s = oracle.quantize_dynamic(xb)
    acc = oracle.gemm_i64(q, w).astype(np.int32)
    y = synth.bf16_bits_to_f32(oracle.epilogue(acc, np.float32(1.0), s_w, s)).astype(np.float64)
    wf = w.astype(np.float64) * s_w.astype(np.float64)[:, None]
    y_fp = synth.bf16_bits_to_f32(xb).astype(np.float64) @ wf.T
    bound = np.abs(wf).sum(axis=1)[None, :] * (s.astype(np.float64)[:, None] / 2)
    assert np.all(np.abs(y - y_fp) <= bound * 1.001 + np.abs(y_fp) * 2.0 ** -7)
