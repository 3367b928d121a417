"""Pins for the oracle's fused residual step (Sec. 3.1.3, Eq. 5-7): residual add, norm, S_n update, quantizer."""
import numpy as np

from oracle import transforms as T
import fptq_workloads as synth


def test_closed_forms(oracle):
    K = 256
    # y = 0, constant residual c: RMS = |c| -> new residual +-1, S_n = S_{n-1} / |c|
    for c in (2.0, -0.5, 3.0):
        x = synth.f32_to_bf16_bits(np.full((1, K), c, np.float32))
        y = np.zeros((1, K), np.uint16)
        out = oracle.residual_norm_quantize(x, y, np.float32(0.25), np.array([4.0], np.float32))
        assert np.all(synth.bf16_bits_to_f32(out["x_next"]) == np.float32(np.sign(c)))
        assert out["s_next"][0] == np.float32(4.0) * np.float32(1.0 / abs(c))
        assert np.all(out["q"] == int(np.clip(np.sign(c) * 4, -8, 7)))          # 1 / 0.25 = 4
    # x = -y: zero row with eps -> 1 / sqrt(eps)
    x = synth.f32_to_bf16_bits(np.full((1, K), 1.5, np.float32))
    y = synth.f32_to_bf16_bits(np.full((1, K), -1.5, np.float32))
    out = oracle.residual_norm_quantize(x, y, np.float32(1.0), None, 0.25)
    assert out["s_next"][0] == np.float32(2.0) and not out["q"].any()


def test_one_step_of_the_recursion_matches_the_fp64_definition(oracle):
    """Against the FP64 recursion of the transforms module (itself pinned to S_n = 1 / RMS(X_n))."""
    rng = np.random.default_rng(0)
    L, D = 12, 128
    W = rng.standard_normal((D, D)) / 8
    blocks = [lambda h: np.tanh(h @ W)]
    X1 = rng.standard_normal((L, D)) * np.exp(rng.standard_normal((L, 1)))
    # scaled stream after block 1: X~_1 = X_1 / RMS, Y~_1 = S_1 F(X~_1)
    Ss, Zts = T.scaled_residual_stack(X1, blocks + blocks)
    S1 = Ss[0]
    Xt1 = X1 * S1
    Yt1 = Zts[0] - Xt1
    xb, yb = synth.f32_to_bf16_bits(Xt1.astype(np.float32)), synth.f32_to_bf16_bits(Yt1.astype(np.float32))
    out = oracle.residual_norm_quantize(xb, yb, np.float32(0.5), S1[:, 0].astype(np.float32))
    # S_2 and X~_2 from the FP64 reference, up to the bf16 storage of the inputs
    assert np.allclose(out["s_next"], Ss[1][:, 0], rtol=2e-2)
    Xt2 = Zts[0] / T.rms(Zts[0])
    assert np.abs(synth.bf16_bits_to_f32(out["x_next"]) - Xt2).max() < 5e-2
    # exact relations on the bf16 inputs themselves
    z = synth.bf16_bits_to_f32(xb).astype(np.float64) + synth.bf16_bits_to_f32(yb).astype(np.float64)
    inv = 1.0 / np.sqrt((z * z).mean(1))
    assert np.allclose(out["s_next"], S1[:, 0].astype(np.float32) * inv, rtol=1e-6)
    assert np.abs(synth.bf16_bits_to_f32(out["x_next"]) - z * inv[:, None]).max() <= 2.0 ** -8 * np.abs(z * inv[:, None]).max()
    qf = z * inv[:, None] / 0.5
    near_tie = np.abs(qf - np.floor(qf) - 0.5) < 1e-4
    assert np.array_equal(out["q"][~near_tie], np.clip(np.rint(qf), -8, 7)[~near_tie])
    # the new residual has unit RMS (that is the point of the transform)
    assert np.allclose(T.rms(synth.bf16_bits_to_f32(out["x_next"]).astype(np.float64)), 1.0, atol=5e-3)


def test_power_of_two_invariance(oracle):
    rng = np.random.default_rng(1)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((6, 96)).astype(np.float32))
    yb = synth.f32_to_bf16_bits(rng.standard_normal((6, 96)).astype(np.float32) * 0.3)
    f = (2.0 ** rng.integers(-4, 5, 6)).astype(np.float32)[:, None]
    a = oracle.residual_norm_quantize(xb, yb, np.float32(0.4))
    b = oracle.residual_norm_quantize(synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(xb) * f),
                                      synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(yb) * f), np.float32(0.4))
    assert np.array_equal(a["q"], b["q"]) and np.array_equal(a["x_next"], b["x_next"])
    assert np.array_equal(a["s_next"], b["s_next"] * f[:, 0])


def test_equals_add_then_unfused_quantizer_when_the_sum_is_exact_in_bf16(oracle):
    """If x + y is representable in bf16, the fused step quantizes exactly like fptq's plain RMS-mode quantizer
    applied to the stored sum."""
    rng = np.random.default_rng(2)
    x = rng.integers(-20, 21, (5, 64)).astype(np.float32)
    y = rng.integers(-20, 21, (5, 64)).astype(np.float32)       # sums are small integers: exact in bf16
    xb, yb, zb = (synth.f32_to_bf16_bits(v) for v in (x, y, x + y))
    fused = oracle.residual_norm_quantize(xb, yb, np.float32(0.3), None, 1e-5)
    r = oracle.row_scale(zb, oracle.MODE_RMS, 1e-5)
    assert np.array_equal(fused["s_next"], r)
    assert np.array_equal(fused["q"], oracle.quantize(zb, np.float32(0.3), r))
