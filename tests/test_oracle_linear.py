"""Pins for the oracle's integer matmul, epilogue and the path end to end.

Checks against things the oracle does not contain: NumPy's own int64 matmul, worst-case closed
forms, exact rational arithmetic for the epilogue, invariances the method must have.
"""
from fractions import Fraction

import numpy as np
import pytest

import fptq_workloads as synth


def test_gemm_matches_numpy_int64(oracle):
    rng = np.random.default_rng(0)
    for (M, N, K) in [(1, 1, 2), (3, 5, 34), (17, 9, 130), (33, 70, 258)]:
        q = rng.integers(-8, 8, (M, K), dtype=np.int8)
        w = rng.integers(-8, 8, (N, K), dtype=np.int8)
        want = q.astype(np.int64) @ w.astype(np.int64).T
        assert np.array_equal(oracle.gemm_i64(q, w), want)
        assert np.array_equal(oracle.gemm_i32(q, w), want.astype(np.int32))


def test_gemm_is_not_transposed_or_shifted(oracle):
    """Asymmetric operands: a one-hot weight row picks exactly one activation column."""
    q = np.arange(-8, 8, dtype=np.int8).reshape(2, 8)
    w = np.zeros((3, 8), np.int8)
    w[0, 1] = 1
    w[1, 6] = -2
    w[2, 7] = 7
    acc = oracle.gemm_i64(q, w)
    assert acc.tolist() == [[-7, -2 * -2, 7 * -1], [1, -2 * 6, 7 * 7]]


def test_gemm_worst_case_reaches_64K(oracle):
    for K in (2, 512, 28672):
        q = np.full((2, K), -8, np.int8)
        w = np.full((3, K), -8, np.int8)
        assert np.all(oracle.gemm_i64(q, w) == 64 * K)
        w[:] = 7
        assert np.all(oracle.gemm_i64(q, w) == -56 * K)
    assert 64 * 28672 < 2 ** 24 < 2 ** 31   # largest config: exact in int32 and in fp32


def test_gemm_samples_agree_with_full(oracle):
    rng = np.random.default_rng(1)
    q = rng.integers(-8, 8, (20, 64), dtype=np.int8)
    w = rng.integers(-8, 8, (30, 64), dtype=np.int8)
    rows = rng.integers(0, 20, 50)
    cols = rng.integers(0, 30, 50)
    full = q.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(oracle.gemm_i64_samples(q, w, rows, cols), full[rows, cols])


def test_epilogue_against_exact_rationals(oracle):
    """y is acc * s_a * s_w[o] * d_t rounded three times (fp32, fp32, bf16): it must sit within one
    bf16 step of the exact product and reproduce it when every factor is a power of two."""
    rng = np.random.default_rng(2)
    M, N = 6, 9
    acc = rng.integers(-(1 << 20), 1 << 20, (M, N)).astype(np.int32)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    d = rng.uniform(0.5, 2.0, M).astype(np.float32)
    s_a = np.float32(0.37)
    for dd in (None, d):
        y = synth.bf16_bits_to_f32(oracle.epilogue(acc, s_a, s_w, dd))
        for t in range(M):
            for o in range(N):
                exact = Fraction(int(acc[t, o])) * Fraction(float(s_a)) * Fraction(float(s_w[o]))
                if dd is not None:
                    exact *= Fraction(float(d[t]))
                assert abs(Fraction(float(y[t, o])) - exact) <= abs(exact) * Fraction(1, 1 << 8) * Fraction(101, 100)
    # powers of two: no rounding anywhere
    acc2 = np.array([[3, -5, 96]], np.int32)
    y = synth.bf16_bits_to_f32(oracle.epilogue(acc2, np.float32(0.5), np.array([2.0, 0.25, 1.0], np.float32),
                                               np.array([4.0], np.float32)))
    assert y.tolist() == [[12.0, -2.5, 192.0]]
    # per-channel scale indexes the output channel, row scale the token
    acc3 = np.ones((2, 3), np.int32)
    y = synth.bf16_bits_to_f32(oracle.epilogue(acc3, np.float32(1.0), np.array([1.0, 2.0, 4.0], np.float32),
                                               np.array([1.0, 8.0], np.float32)))
    assert y.tolist() == [[1.0, 2.0, 4.0], [8.0, 16.0, 32.0]]


def test_integer_special_case_equals_plain_matmul(oracle):
    """s_a = 1, s_w = 1, integer-valued X inside the grid: the layer is a plain integer matmul."""
    rng = np.random.default_rng(3)
    M, N, K = 5, 7, 8
    x = rng.integers(-2, 3, (M, K)).astype(np.float32)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    out = oracle.w4a4_linear(synth.f32_to_bf16_bits(x), w, np.float32(1.0), np.ones(N, np.float32), oracle.MODE_NONE)
    want = x.astype(np.int64) @ w.astype(np.int64).T      # |.| <= 8*2*8 = 128: exact in bf16
    assert np.array_equal(out["q"], x.astype(np.int8))
    assert np.array_equal(out["acc"], want)
    assert np.array_equal(synth.bf16_bits_to_f32(out["y"]), want.astype(np.float32))


def test_row_rescaling_invariance(oracle):
    """RMS mode, eps = 0: scaling a token by a power of two changes nothing downstream
    (Sec. 3.1.3: the normalised representation does not depend on the token's scale)."""
    rng = np.random.default_rng(4)
    M, N, K = 8, 16, 96
    x = rng.standard_normal((M, K)).astype(np.float32)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    xb = synth.f32_to_bf16_bits(x)
    scale = (2.0 ** rng.integers(-6, 7, M)).astype(np.float32)
    xs = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(xb) * scale[:, None])   # exact
    a = oracle.w4a4_linear(xb, w, np.float32(0.4), s_w, oracle.MODE_RMS, 0.0)
    b = oracle.w4a4_linear(xs, w, np.float32(0.4), s_w, oracle.MODE_RMS, 0.0)
    assert np.array_equal(a["q"], b["q"]) and np.array_equal(a["acc"], b["acc"]) and np.array_equal(a["y"], b["y"])
    assert np.array_equal(a["r"], b["r"] * scale)
    assert a["q"].min() < 0 < a["q"].max()


def test_input_channel_permutation_invariance(oracle):
    rng = np.random.default_rng(5)
    M, N, K = 6, 10, 64
    xb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32) * 3)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    r = rng.uniform(0.5, 2.0, M).astype(np.float32)
    perm = rng.permutation(K)
    a = oracle.w4a4_linear(xb, w, np.float32(0.9), s_w, oracle.MODE_GIVEN, 0.0, r)
    b = oracle.w4a4_linear(xb[:, perm], w[:, perm], np.float32(0.9), s_w, oracle.MODE_GIVEN, 0.0, r)
    assert np.array_equal(a["q"][:, perm], b["q"])
    assert np.array_equal(a["acc"], b["acc"]) and np.array_equal(a["y"], b["y"])


def test_dequantised_output_tracks_the_float_layer(oracle):
    """With the undo scale d_t = 1 / S_t the layer approximates the float linear x (s_w w)^T, and the
    error is bounded by the quantization step: |y - y_fp| <= sum_k |s_w w| * s_a / (2 S_t) + bf16."""
    rng = np.random.default_rng(6)
    M, N, K = 16, 24, 256
    xb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    r = oracle.row_scale(xb, oracle.MODE_RMS, 0.0)
    xt = synth.bf16_bits_to_f32(xb).astype(np.float64) * r.astype(np.float64)[:, None]
    s_a = np.float32(np.abs(xt).max() / 7.0)
    out = oracle.w4a4_linear(xb, w, s_a, s_w, oracle.MODE_RMS, 0.0, None, (1.0 / r).astype(np.float32))
    y = synth.bf16_bits_to_f32(out["y"]).astype(np.float64)
    wf = w.astype(np.float64) * s_w.astype(np.float64)[:, None]
    y_fp = synth.bf16_bits_to_f32(xb).astype(np.float64) @ wf.T
    bound = (np.abs(wf).sum(axis=1)[None, :] * float(s_a) / 2.0) / r.astype(np.float64)[:, None]
    assert np.all(np.abs(y - y_fp) <= bound * 1.001 + np.abs(y_fp) * 2.0 ** -7)
    # and it is a real approximation, not noise: relative error small on aggregate
    assert np.linalg.norm(y - y_fp) / np.linalg.norm(y_fp) < 0.2


def test_timed_build_equals_checked_build(oracle):
    case = synth.config_cases("c1")[1]
    inp = synth.draw(case, M=9)
    a = oracle.w4a4_linear(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, case.mode, case.eps)
    y = oracle.w4a4_linear_timed(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, case.mode, case.eps)
    assert np.array_equal(a["y"], y)


def test_synth_configs_have_the_published_shapes():
    shapes = {c.key: (c.M, c.N, c.K) for cfg in synth.ALL_CONFIGS for c in synth.config_cases(cfg)}
    assert shapes["c1.tiny_none.M128"] == (128, 512, 512)
    assert shapes["c2.gate.M2048"] == (2048, 11008, 4096) and shapes["c2.down.M2048"] == (2048, 4096, 11008)
    assert shapes["c3.qkv.M4096"] == (4096, 6144, 4096) and shapes["c3.gate_up.M4096"] == (4096, 28672, 4096)
    assert shapes["c3.down.M4096"] == (4096, 4096, 14336) and shapes["c3.o.M4096"] == (4096, 4096, 4096)
    assert shapes["c4.down.M8"] == (8, 4096, 14336) and shapes["c4.qkv.M32"] == (32, 6144, 4096)
    assert shapes["c5.qkv.M8192"] == (8192, 10240, 8192) and shapes["c5.gate_up.M8192"] == (8192, 57344, 8192)
    assert shapes["c5.down.M8192"] == (8192, 8192, 28672) and shapes["c5.o.M8192"] == (8192, 8192, 8192)
    inp = synth.draw(synth.config_cases("c1")[0])
    assert inp.x_bits.shape == (128, 512) and inp.w_int.shape == (512, 512) and len(inp.channels) == 4
    assert inp.w_int.min() == -8 and inp.w_int.max() == 7
    assert 0.005 <= inp.s_w.min() and inp.s_w.max() <= 0.02
    # gate and up read the same X but different weights
    g, u = synth.config_cases("c2")[:2]
    wg, _ = synth.draw_weights(LinearCaseSmall(g))
    wu, _ = synth.draw_weights(LinearCaseSmall(u))
    assert not np.array_equal(wg, wu)


def LinearCaseSmall(case):
    import dataclasses
    return dataclasses.replace(case, N=8, K=64)
