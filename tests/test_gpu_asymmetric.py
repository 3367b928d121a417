"""GPU parity of the asymmetric (zero-point) activation grid: quantizer, weight row sums, corrected epilogue."""
import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq
import fptq_workloads as synth

from gpu_util import Y_TOL, dev, dev_bf16, host_bits, y_error

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("zp", [-8, -3, 0, 5, 7])
@pytest.mark.parametrize("M,K,mode", [(3, 34, 0), (17, 512, 1), (9, 4096, 2), (2, 28672, 0), (5, 1001, 2)])
def test_asymmetric_quantizer_bit_exact(oracle, M, K, mode, zp):
    case = synth.LinearCase("a", "q", M, 8, K, "normal", 0.0, 2, 4.0, mode, M + K)
    inp = synth.draw(case, with_weights=False)
    xq, r = fptq.fptq_quantize_act_asym(dev_bf16(inp.x_bits), float(inp.s_a), zp, mode, 1e-5, dev(inp.row_scale_in))
    r_ref = oracle.row_scale(inp.x_bits, mode, 1e-5, inp.row_scale_in)
    q_ref = oracle.quantize_zp(inp.x_bits, inp.s_a, zp, None if mode == 0 else r_ref)
    assert np.array_equal(fptq.fptq_unpack(xq, M, K).cpu().numpy(), q_ref)
    assert np.array_equal(r.cpu().numpy().view(np.uint32), r_ref.view(np.uint32))


@pytest.mark.parametrize("zp", [-8, -3, 0, 5, 7])
@pytest.mark.parametrize("s_a", [0.731, 1e-30, 3e30])
def test_asymmetric_quantizer_every_bf16_pattern(oracle, zp, s_a):
    """All 65536 bit patterns (NaNs, infinities, subnormals, huge and tiny magnitudes), also with scales that drive the
    product to infinity or to zero: the saturating integer path must agree with clamping in float."""
    allbits = np.arange(65536, dtype=np.uint16).reshape(8, 8192)
    r = np.array([1.0, 0.5, 0.3333, 2.7, 13.37, 1e-3, 100.0, 7.0], np.float32)
    xq, _ = fptq.fptq_quantize_act_asym(dev_bf16(allbits), s_a, zp, synth.MODE_GIVEN, 0.0, dev(r))
    q = fptq.fptq_unpack(xq, 8, 8192).cpu().numpy()
    assert np.array_equal(q, oracle.quantize_zp(allbits, np.float32(s_a), zp, r))


@pytest.mark.parametrize("M", [5, 200])
def test_asymmetric_linear_long_k(oracle, M):
    """K > 65535 with a zero point: the staged correction 256 * z * wsum of the MFMA kernel could overflow, so that
    kernel hands over to the simple one; extreme operands (all codes -8, zero point -8, weights -8)."""
    N, K, zp = 24, 65536 + 320, -8
    q = np.full((M, K), -8, np.int8)
    w = np.full((N, K), -8, np.int8)
    rng = np.random.default_rng(M)
    w[1::2] = rng.integers(-8, 8, (len(w[1::2]), K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    wsum = fptq.fptq_weight_row_sums(dev(w))
    y, acc = fptq.fptq_w4a4_linear_zp(fptq.fptq_pack_weights(dev(q)), fptq.fptq_pack_weights(dev(w)), M, N, K, 0.125, dev(s_w), zp,
                                      wsum, want_acc=True)
    acc_ref = oracle.gemm_i64(q, w).astype(np.int32)
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    assert np.array_equal(host_bits(y), oracle.epilogue_zp(acc_ref, np.float32(0.125), s_w, zp, oracle.weight_row_sums(w)))


def test_weight_row_sums(oracle):
    rng = np.random.default_rng(0)
    for N, K in [(1, 1), (5, 34), (300, 4096), (64, 11008)]:
        w = rng.integers(-8, 8, (N, K), dtype=np.int8)
        assert np.array_equal(fptq.fptq_weight_row_sums(dev(w)).cpu().numpy(), oracle.weight_row_sums(w))


@pytest.mark.parametrize("M,N,K", [(1, 512, 512), (8, 700, 1024), (32, 17000, 256), (100, 300, 640), (300, 520, 2048),
                                   (513, 260, 4096)])
@pytest.mark.parametrize("zp", [-8, 4])
def test_asymmetric_linear_matches_oracle(oracle, M, N, K, zp):
    """One-sided (non-negative) activations on the shifted grid, through the few-token and the MFMA kernels."""
    rng = np.random.default_rng(M + N + K)
    x = np.abs(rng.standard_normal((M, K))).astype(np.float32) if zp < 0 else rng.standard_normal((M, K)).astype(np.float32)
    xb = synth.f32_to_bf16_bits(x)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    s_a = np.float32(np.abs(x).max() / (15.0 if zp == -8 else 7.0))
    xq, _ = fptq.fptq_quantize_act_asym(dev_bf16(xb), float(s_a), zp)
    wsum = fptq.fptq_weight_row_sums(dev(w))
    y, acc = fptq.fptq_w4a4_linear_zp(xq, fptq.fptq_pack_weights(dev(w)), M, N, K, float(s_a), dev(s_w), zp, wsum, want_acc=True)
    q_ref = oracle.quantize_zp(xb, s_a, zp)
    acc_ref = oracle.gemm_i64(q_ref, w).astype(np.int32)
    y_ref = oracle.epilogue_zp(acc_ref, s_a, s_w, zp, oracle.weight_row_sums(w))
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    assert y_error(host_bits(y), y_ref) <= Y_TOL
    assert np.array_equal(host_bits(y), y_ref)
    if zp == -8:    # and it is a real improvement over the symmetric grid on one-sided data
        y_fp = synth.bf16_bits_to_f32(xb).astype(np.float64) @ (w.astype(np.float64) * s_w[:, None].astype(np.float64)).T
        sym = oracle.w4a4_linear(xb, w, np.float32(np.abs(x).max() / 7.0), s_w, oracle.MODE_NONE)
        e_asym = np.linalg.norm(synth.bf16_bits_to_f32(host_bits(y)).astype(np.float64) - y_fp)
        e_sym = np.linalg.norm(synth.bf16_bits_to_f32(sym["y"]).astype(np.float64) - y_fp)
        assert e_asym < 0.7 * e_sym


def test_asymmetric_argument_errors():
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fptq.FptqError) as e:
        fptq.fptq_quantize_act_asym(x, 1.0, 8)
    assert e.value.code == -6
    xq, _ = fptq.fptq_quantize_act_asym(x, 1.0, 3)
    w = torch.zeros((8, 128), dtype=torch.int8, device="cuda")
    L = fptq.lib()
    import ctypes
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    y = torch.empty((4, 8), dtype=torch.bfloat16, device="cuda")
    s_w = torch.ones(8, device="cuda")
    wq = fptq.fptq_pack_weights(w)
    assert L.fptq_w4a4_linear_zp(p(xq), p(wq), 4, 8, 128, 1.0, p(s_w), None, 3, None, p(y), None, None) == -6
