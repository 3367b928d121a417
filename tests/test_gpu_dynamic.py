"""GPU parity of the dynamic (per-token, run-time scale) quantizer and the linear layer fed by it."""
import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq
import fptq_workloads as synth

from gpu_util import Y_TOL, dev, dev_bf16, host_bits, y_error

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,K", [(1, 8), (3, 34), (5, 129), (17, 512), (9, 4096), (4, 11008), (2, 28672), (3, 1001),
                                 (2, 40000), (300, 640),
                                 # every launch shape: a workgroup per row (all widths), a wave per row (many short rows)
                                 (3, 2048), (5, 8192), (4, 12288), (3, 14336), (2, 16384), (2, 24576), (2, 32768),
                                 (800, 2048), (1000, 4096), (770, 520)])
def test_dynamic_quantizer_bit_exact(oracle, M, K):
    rng = np.random.default_rng(M * 5 + K)
    x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.standard_normal((M, 1))).astype(np.float32)
    xb = synth.f32_to_bf16_bits(x)
    xq, s = fptq.fptq_quantize_act_dynamic(dev_bf16(xb))
    q = fptq.fptq_unpack(xq, M, K).cpu().numpy()
    q_ref, s_ref = oracle.quantize_dynamic(xb)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(q, q_ref)
    assert np.abs(q_ref).max(axis=1).min() == 7


def test_dynamic_degenerate_rows(oracle):
    x = np.zeros((4, 128), np.float32)
    x[1, 3] = np.inf
    x[2, 2] = -5.0
    x[3, :] = 1e-30
    xb = synth.f32_to_bf16_bits(x)
    xb[2, 7] = 0x7FC0
    xq, s = fptq.fptq_quantize_act_dynamic(dev_bf16(xb))
    q_ref, s_ref = oracle.quantize_dynamic(xb)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(fptq.fptq_unpack(xq, 4, 128).cpu().numpy(), q_ref)


@pytest.mark.parametrize("M,N,K", [(8, 300, 1024), (200, 520, 2048), (32, 4096, 4096), (300, 260, 640)])
def test_dynamic_linear_matches_oracle(oracle, M, N, K):
    """Dynamic activations through the same linear entry point: s_a = 1 and the per-token scale as the
    output row scale give y = bf16(acc * s_w[o] * s_t)."""
    rng = np.random.default_rng(M + N + K)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 4, replace=False)] *= 20
    xb = synth.f32_to_bf16_bits(x)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    xq, s = fptq.fptq_quantize_act_dynamic(dev_bf16(xb))
    y, acc = fptq.fptq_w4a4_linear(xq, fptq.fptq_pack_weights(dev(w)), M, N, K, 1.0, dev(s_w), row_out_scale=s, want_acc=True)
    q_ref, s_ref = oracle.quantize_dynamic(xb)
    acc_ref = oracle.gemm_i64(q_ref, w).astype(np.int32)
    y_ref = oracle.epilogue(acc_ref, np.float32(1.0), s_w, s_ref)
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    assert y_error(host_bits(y), y_ref) <= Y_TOL
    assert np.array_equal(host_bits(y), y_ref)


def test_dynamic_needs_the_scale_buffer():
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    L = fptq.lib()
    out = torch.empty(fptq.fptq_packed_bytes(4, 128), dtype=torch.uint8, device="cuda")
    import ctypes
    assert L.fptq_quantize_act_dynamic(ctypes.c_void_p(x.data_ptr()), 4, 128, ctypes.c_void_p(out.data_ptr()), out.numel(), None, None) == -1
