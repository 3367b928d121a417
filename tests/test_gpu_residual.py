"""GPU parity of the fused residual step (Sec. 3.1.3, Eq. 5-7) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq
import fptq_workloads as synth

from gpu_util import dev, dev_bf16, host_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("with_prev", [False, True])
@pytest.mark.parametrize("M,K", [(1, 8), (3, 34), (5, 129), (17, 512), (9, 4096), (6, 8192), (3, 11008), (130, 1000), (2, 28672),
                                 # every launch shape: a workgroup per row at each width class, a wave per row (many short rows)
                                 (5, 2048), (4, 5120), (3, 12288), (2, 16384), (800, 2048), (1000, 4096), (770, 520)])
def test_residual_step_bit_exact(oracle, M, K, with_prev):
    rng = np.random.default_rng(M * 11 + K)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.standard_normal((M, 1))).astype(np.float32))
    yb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32) * 0.5)
    sp = rng.uniform(0.2, 3, M).astype(np.float32) if with_prev else None
    s_a = np.float32(0.45)
    for eps in (0.0, 1e-5):
        x_next, s_next, xq = fptq.fptq_residual_norm_quantize(dev_bf16(xb), dev_bf16(yb), float(s_a), dev(sp), eps)
        ref = oracle.residual_norm_quantize(xb, yb, s_a, sp, eps)
        assert np.array_equal(s_next.cpu().numpy().view(np.uint32), ref["s_next"].view(np.uint32))
        assert np.array_equal(host_bits(x_next), ref["x_next"])
        assert np.array_equal(fptq.fptq_unpack(xq, M, K).cpu().numpy(), ref["q"])
    assert ref["q"].min() == -8 or ref["q"].max() == 7 or M * K < 3000


def test_residual_step_in_place_and_then_linear(oracle):
    """x_next may alias the residual input; the packed result feeds the linear layer."""
    rng = np.random.default_rng(5)
    M, K, N = 64, 1024, 384
    xb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32) * 3)
    yb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    xd = dev_bf16(xb)
    x_next, s_next, xq = fptq.fptq_residual_norm_quantize(xd, dev_bf16(yb), 0.5, None, 1e-5, x_next=xd)
    assert x_next.data_ptr() == xd.data_ptr()
    y, acc = fptq.fptq_w4a4_linear(xq, fptq.fptq_pack_weights(dev(w)), M, N, K, 0.5, dev(s_w), want_acc=True)
    ref = oracle.residual_norm_quantize(xb, yb, np.float32(0.5), None, 1e-5)
    assert np.array_equal(host_bits(xd), ref["x_next"])
    acc_ref = oracle.gemm_i64(ref["q"], w).astype(np.int32)
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    assert np.array_equal(host_bits(y), oracle.epilogue(acc_ref, np.float32(0.5), s_w))


@pytest.mark.parametrize("alias", ["x_res", "y"])
@pytest.mark.parametrize("M,K", [(5, 129), (130, 1000), (3, 16390), (2, 20000)])
def test_residual_step_in_place_on_the_two_pass_path(oracle, M, K, alias):
    """K not a multiple of 8, or above 16384: the kernel that reads its inputs twice.  The output may be either input."""
    rng = np.random.default_rng(M + K)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32) * 2)
    yb = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    sp = rng.uniform(0.2, 3, M).astype(np.float32)
    xd, yd = dev_bf16(xb), dev_bf16(yb)
    target = xd if alias == "x_res" else yd
    x_next, s_next, xq = fptq.fptq_residual_norm_quantize(xd, yd, 0.45, dev(sp), 1e-5, x_next=target)
    ref = oracle.residual_norm_quantize(xb, yb, np.float32(0.45), sp, 1e-5)
    assert x_next.data_ptr() == target.data_ptr()
    assert np.array_equal(host_bits(target), ref["x_next"])
    assert np.array_equal(s_next.cpu().numpy().view(np.uint32), ref["s_next"].view(np.uint32))
    assert np.array_equal(fptq.fptq_unpack(xq, M, K).cpu().numpy(), ref["q"])
