"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Sizes here are the ones the oracle recomputes whole in seconds: the tiny configuration, ragged
and degenerate shapes, several tiles plus a tail.  Full-size configurations are in
test_gpu_configs.py.
"""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq
import fptq_workloads as synth

from gpu_util import Y_TOL, dev, dev_bf16, host_bits, layout_from_canonical, run_gpu_linear, y_error

pytestmark = pytest.mark.gpu


def small_case(M, N, K, mode, seed=7, dist="normal", count=2, mult=4.0):
    return synth.LinearCase("t", f"m{M}n{N}k{K}", M, N, K, dist, 0.0, count, mult, mode, seed)


# ------------------------------------------------------------------ packing
@pytest.mark.parametrize("N,K", [(1, 2), (5, 34), (16, 128), (33, 130), (300, 512), (257, 1000), (64, 4096)])
def test_pack_weights_layout_and_roundtrip(oracle, N, K):
    rng = np.random.default_rng(N * 1000 + K)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    packed = fptq.fptq_pack_weights(dev(w))
    assert packed.numel() == fptq.fptq_packed_bytes(N, K) == ((K + 127) // 128) * N * 64
    back = fptq.fptq_unpack(packed, N, K).cpu().numpy()
    assert np.array_equal(back, w)
    # the documented byte layout, rebuilt from the oracle's canonical packing
    want = layout_from_canonical(oracle.pack(w), N, K)
    assert np.array_equal(packed.cpu().numpy(), want)


def test_pack_weights_odd_K():
    rng = np.random.default_rng(1)
    w = rng.integers(-8, 8, (7, 129), dtype=np.int8)
    packed = fptq.fptq_pack_weights(dev(w))
    assert np.array_equal(fptq.fptq_unpack(packed, 7, 129).cpu().numpy(), w)


# ------------------------------------------------------------------ activation quantizer
@pytest.mark.parametrize("mode", [synth.MODE_NONE, synth.MODE_RMS, synth.MODE_GIVEN])
@pytest.mark.parametrize("M,K", [(1, 8), (3, 34), (5, 129), (17, 512), (128, 512), (9, 4096), (4, 11008), (2, 28672),
                                 (2, 40000), (3, 1001),
                                 # every launch shape: a workgroup per row (all widths), a wave per row (many short rows)
                                 (3, 2048), (5, 8192), (4, 12288), (3, 14336), (2, 16384), (2, 24576), (2, 32768),
                                 (800, 2048), (1000, 4096), (770, 520)])
def test_quantize_act_bit_exact(oracle, mode, M, K):
    case = small_case(M, 8, K, mode, seed=M + K)
    inp = synth.draw(case, with_weights=False)
    for eps in (0.0, 1e-5):
        xq, r = fptq.fptq_quantize_act(dev_bf16(inp.x_bits), float(inp.s_a), mode, eps, dev(inp.row_scale_in))
        q = fptq.fptq_unpack(xq, M, K).cpu().numpy()
        r_ref = oracle.row_scale(inp.x_bits, mode, eps, inp.row_scale_in)
        q_ref = oracle.quantize(inp.x_bits, inp.s_a, None if mode == synth.MODE_NONE else r_ref)
        assert np.array_equal(r.cpu().numpy().view(np.uint32), r_ref.view(np.uint32))
        assert np.array_equal(q, q_ref)
        if M * K >= 512:
            assert q_ref.min() < 0 < q_ref.max()
        if K % 2 == 0:   # padded bytes beyond K are zero and the layout is the documented one
            want = layout_from_canonical(oracle.pack(q_ref), M, K)
            assert np.array_equal(xq.cpu().numpy(), want)


@pytest.mark.parametrize("M,K,mode", [(16512, 8192, synth.MODE_RMS), (5000, 28672, synth.MODE_GIVEN)])
def test_quantize_act_larger_than_the_last_level_cache(oracle, M, K, mode):
    """Inputs above 256 MB take the streaming-load path of both quantizer kernels: sampled rows against the oracle,
    every row against the same kernel on the two halves of the tensor (each small enough for the ordinary path)."""
    torch.manual_seed(M)
    x = (torch.randn((M, K), device="cuda") * 1.5).to(torch.bfloat16)
    x[:, 7] *= 30.0
    r_in = (torch.rand(M, device="cuda") + 0.5) if mode == synth.MODE_GIVEN else None
    xq, r = fptq.fptq_quantize_act(x, 0.4, mode, 1e-5, r_in)
    q = fptq.fptq_unpack(xq, M, K)
    h = M // 2
    for lo, hi in ((0, h), (h, M)):
        xq2, r2 = fptq.fptq_quantize_act(x[lo:hi].contiguous(), 0.4, mode, 1e-5, None if r_in is None else r_in[lo:hi].contiguous())
        assert torch.equal(fptq.fptq_unpack(xq2, hi - lo, K), q[lo:hi]) and torch.equal(r2, r[lo:hi])
    rows = np.random.default_rng(M).choice(M, 48, replace=False)
    bits = x[torch.from_numpy(rows).cuda()].view(torch.int16).cpu().numpy().view(np.uint16)
    rin = None if r_in is None else r_in.cpu().numpy()[rows]
    r_ref = oracle.row_scale(bits, mode, 1e-5, rin)
    assert np.array_equal(r.cpu().numpy()[rows].view(np.uint32), r_ref.view(np.uint32))
    assert np.array_equal(q.cpu().numpy()[rows], oracle.quantize(bits, np.float32(0.4), r_ref))


def test_quantize_act_special_values(oracle):
    """Ties, clamp edges, infinities, NaN, signed zero, subnormals: same decisions as the oracle."""
    vals = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 7.5, -8.5, 6.5, -7.5, 100.0, -100.0, 0.0, -0.0,
                     np.inf, -np.inf, np.nan, 1e-40, -1e-40, 3.0, -3.0], np.float32)
    x = np.zeros((2, 128), np.float32)
    x[0, :len(vals)] = vals
    x[1, :len(vals)] = vals * 2
    bits = synth.f32_to_bf16_bits(x)
    bits[0, 15] = 0x7FC0
    for s_a in (1.0, 2.0, 0.37):
        xq, _ = fptq.fptq_quantize_act(dev_bf16(bits), s_a, synth.MODE_NONE)
        q = fptq.fptq_unpack(xq, 2, 128).cpu().numpy()
        assert np.array_equal(q, oracle.quantize(bits, np.float32(s_a), None))
    # every bf16 bit pattern once, with a row scale
    allbits = np.arange(65536, dtype=np.uint16).reshape(8, 8192)
    r = np.array([1.0, 0.5, 0.3333, 2.7, 13.37, 1e-3, 100.0, 7.0], np.float32)
    xq, r_out = fptq.fptq_quantize_act(dev_bf16(allbits), 0.731, synth.MODE_GIVEN, 0.0, dev(r))
    q = fptq.fptq_unpack(xq, 8, 8192).cpu().numpy()
    assert np.array_equal(q, oracle.quantize(allbits, np.float32(0.731), r))
    assert np.array_equal(r_out.cpu().numpy(), r)


# ------------------------------------------------------------------ the linear layer
SHAPES = [(1, 1, 2), (3, 5, 34), (128, 512, 512), (100, 300, 640), (257, 513, 1024), (33, 1000, 130),
          (300, 260, 4096), (64, 64, 128), (1, 512, 512), (8, 700, 1024), (32, 256, 4096), (31, 33, 258),
          (16, 300, 2048), (17, 48, 14336), (5, 1030, 4096), (2, 16, 128), (32, 17, 896), (9, 2000, 11008),
          (32, 16400, 256), (20, 16390, 384), (3, 70, 8200),
          # 33 .. 64 tokens: every launch shape of the few-token kernel (narrow matrices) and the hand-over to the
          # prefill kernel's small tiles (wide ones, and everything from 65 tokens on)
          (64, 10200, 256), (50, 6200, 4096), (48, 100, 4096), (40, 3000, 4096), (40, 5000, 2048), (64, 16400, 256), (33, 10240, 384),
          (128, 16400, 256), (100, 6150, 640), (127, 300, 4224), (65, 200, 4100), (129, 300, 640)]


@pytest.mark.parametrize("use_ref", [False, True], ids=["tuned", "ref"])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_matches_oracle(oracle, M, N, K, use_ref):
    mode = (synth.MODE_RMS, synth.MODE_GIVEN, synth.MODE_NONE)[(M + N + K) % 3]
    inp = synth.draw(small_case(M, N, K, mode, seed=M * 7 + N * 3 + K))
    ref = oracle.w4a4_linear(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, mode, inp.case.eps, inp.row_scale_in)
    got = run_gpu_linear(inp, use_ref=use_ref)
    assert np.array_equal(got["r"].view(np.uint32), ref["r"].view(np.uint32))
    assert np.array_equal(got["q"], ref["q"])
    assert np.array_equal(got["acc"], ref["acc"])
    assert y_error(got["y"], ref["y"]) <= Y_TOL
    assert np.array_equal(got["y"], ref["y"])          # same fp32 recipe on both sides: expected identical


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("M,N,K", [(128, 512, 512), (257, 513, 1024), (300, 260, 4096), (100, 300, 640), (33, 1000, 130),
                                   (520, 390, 896)])
def test_every_prefill_tile_shape(oracle, M, N, K, tile):
    """Each tile shape of the MFMA kernel, forced, on shapes with ragged edges in M, N and K."""
    inp = synth.draw(small_case(M, N, K, synth.MODE_RMS, seed=M + N + K + tile))
    ref = oracle.w4a4_linear(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, synth.MODE_RMS, inp.case.eps)
    fptq.fptq_set_gemm_tile(tile)
    try:
        got = run_gpu_linear(inp)
    finally:
        fptq.fptq_set_gemm_tile(0)
    assert np.array_equal(got["acc"], ref["acc"])
    assert np.array_equal(got["y"], ref["y"])


def test_config1_tiny(oracle):
    for case in synth.config_cases("c1"):
        inp = synth.draw(case)
        ref = oracle.w4a4_linear(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, case.mode, case.eps)
        for use_ref in (False, True):
            got = run_gpu_linear(inp, use_ref=use_ref)
            assert np.array_equal(got["q"], ref["q"]) and np.array_equal(got["acc"], ref["acc"])
            assert y_error(got["y"], ref["y"]) <= Y_TOL


def test_linear_with_output_row_scale(oracle):
    inp = synth.draw(small_case(70, 200, 384, synth.MODE_RMS, seed=21))
    got = run_gpu_linear(inp, undo_scale=True)
    ref = oracle.w4a4_linear(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, synth.MODE_RMS, inp.case.eps, None, got["d"])
    assert np.array_equal(got["acc"], ref["acc"])
    assert y_error(got["y"], ref["y"]) <= Y_TOL


def test_linear_worst_case_accumulator(oracle):
    """All operands -8 at the largest K of the configurations: acc = 64 K exactly."""
    M, N, K = 40, 48, 28672
    w = np.full((N, K), -8, np.int8)
    x = synth.f32_to_bf16_bits(np.full((M, K), -8.0, np.float32))
    xq, _ = fptq.fptq_quantize_act(dev_bf16(x), 1.0, synth.MODE_NONE)
    wq = fptq.fptq_pack_weights(dev(w))
    s_w = torch.ones(N, device="cuda")
    for fn in (fptq.fptq_w4a4_linear, fptq.fptq_w4a4_linear_ref):
        y, acc = fn(xq, wq, M, N, K, 1.0, s_w, want_acc=True)
        assert torch.all(acc == 64 * K)
    w[:] = 7
    wq = fptq.fptq_pack_weights(dev(w))
    y, acc = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 1.0, s_w, want_acc=True)
    assert torch.all(acc == -56 * K)


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5, 6, 7, 8, "workspace"])
def test_largest_k_of_the_widened_accumulator(oracle, tile):
    """K = 131071, all operands -8 (and a block of +7 weights): 256 * acc = 2^31 - 16384 is the largest value the
    widened accumulator ever holds; every tile shape, the K groups' exchange and the split over workgroups keep it."""
    M, N, K = 200, 130, 131071
    x = np.full((M, K), -8, np.int8)
    w = np.full((N, K), -8, np.int8)
    w[5:40] = 7
    s_w = np.random.default_rng(9).uniform(0.005, 0.02, N).astype(np.float32)
    xq, wq = fptq.fptq_pack_weights(dev(x)), fptq.fptq_pack_weights(dev(w))
    want = np.full((M, N), 64 * K, np.int32)
    want[:, 5:40] = -56 * K
    if tile == "workspace":
        nbytes = fptq.fptq_linear_workspace_bytes(M, N, K)
        assert nbytes > 0
        ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        y, acc = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, 0.25, dev(s_w), ws, want_acc=True)
    else:
        fptq.fptq_set_gemm_tile(tile)
        try:
            y, acc = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.25, dev(s_w), want_acc=True)
        finally:
            fptq.fptq_set_gemm_tile(0)
    assert np.array_equal(acc.cpu().numpy(), want)
    assert np.array_equal(host_bits(y), oracle.epilogue(want, np.float32(0.25), s_w))


@pytest.mark.parametrize("M", [3, 200])
def test_k_beyond_the_widened_accumulator_limit(oracle, M):
    """K > 131071: 256 * acc no longer fits int32, so both tuned kernels hand over to the simple one.  All operands
    -8: the largest accumulator there is."""
    N, K = 40, 131072 + 192
    x = np.full((M, K), -8, np.int8)
    w = np.full((N, K), -8, np.int8)
    rng = np.random.default_rng(M)
    w[::3] = rng.integers(-8, 8, (len(w[::3]), K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    xq, wq = fptq.fptq_pack_weights(dev(x)), fptq.fptq_pack_weights(dev(w))
    y, acc = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.25, dev(s_w), want_acc=True)
    acc_ref = oracle.gemm_i64(x, w)
    assert acc_ref.max() == 64 * K
    assert np.array_equal(acc.cpu().numpy(), acc_ref.astype(np.int32))
    assert np.array_equal(host_bits(y), oracle.epilogue(acc_ref.astype(np.int32), np.float32(0.25), s_w))


@pytest.mark.parametrize("M,N,K", [((1 << 24) + 3, 3, 6), (2, (1 << 24) + 5, 4)])
def test_dimension_beyond_16_million(oracle, M, N, K):
    """More than 2^24 rows (beyond the prefill kernel's buffer descriptors: the simple kernel answers) and more
    than 2^24 channels against two tokens (the few-token kernel's 64-bit addressing)."""
    rng = np.random.default_rng(N)
    x = rng.integers(-8, 8, (M, K), dtype=np.int8)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    xq, wq = fptq.fptq_pack_weights(dev(x)), fptq.fptq_pack_weights(dev(w))
    y, acc = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.25, dev(s_w), want_acc=True)
    want = (x.astype(np.int32) @ w.astype(np.int32).T).astype(np.int32)
    assert np.array_equal(acc.cpu().numpy(), want)
    assert np.array_equal(host_bits(y), oracle.epilogue(want, np.float32(0.25), s_w))


def test_linear_is_deterministic():
    inp = synth.draw(small_case(300, 520, 2048, synth.MODE_RMS, seed=5))
    a = run_gpu_linear(inp)
    b = run_gpu_linear(inp)
    assert np.array_equal(a["acc"], b["acc"]) and np.array_equal(a["y"], b["y"])


def test_acc_dump_is_optional(oracle):
    inp = synth.draw(small_case(50, 260, 256, synth.MODE_NONE, seed=3))
    a = run_gpu_linear(inp, want_acc=False)
    b = run_gpu_linear(inp, want_acc=True)
    assert a["acc"] is None and np.array_equal(a["y"], b["y"])


# ------------------------------------------------------------------ error returns
def test_error_codes():
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fptq.FptqError) as e:
        fptq.fptq_quantize_act(x, 0.0)
    assert e.value.code == -6
    with pytest.raises(fptq.FptqError) as e:
        fptq.fptq_quantize_act(x, 1.0, 7)
    assert e.value.code == -4
    with pytest.raises(fptq.FptqError) as e:
        fptq.fptq_quantize_act(x, 1.0, synth.MODE_GIVEN, 0.0, None)
    assert e.value.code == -4
    with pytest.raises(fptq.FptqError) as e:
        fptq.fptq_quantize_act(x, 1.0, out=torch.zeros(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    L = fptq.lib()
    assert L.fptq_packed_bytes(0, 128) == -2 and L.fptq_packed_bytes(4, -1) == -2
    assert L.fptq_w4a4_linear(None, None, 1, 1, 2, 1.0, None, None, None, None, None) == -1
    assert b"NULL" in L.fptq_last_error()
