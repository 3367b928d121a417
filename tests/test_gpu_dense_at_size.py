"""Full-size parity on operands that fill the 4-bit grid.

The configurations' own activations quantize to mostly zeros (absmax calibration with outlier channels), so a K tile
that the kernel dropped, duplicated or mis-addressed could hide behind them.  Here the activations are uniform random
INT4 codes (every K tile contributes to every accumulator), at the shapes and through the entry point the benchmark
times, compared with the oracle: whole tensors for the Llama-2-7B and Llama-3-8B shapes (prefill and decode), sampled
rows, columns and entries plus a full-coverage Freivalds check for the Llama-3-70B shapes.  A second family of cases
confines the non-zero activations to ONE K tile at a time, so each K tile's contribution is checked by itself.
"""
import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq
import fptq_workloads as synth

from gpu_util import dev, host_bits
from test_gpu_configs import freivalds_rhs

pytestmark = pytest.mark.gpu


def dense_inputs(M, N, K, seed):
    rng = np.random.default_rng([seed, M, N, K])
    x = rng.integers(-8, 8, size=(M, K), dtype=np.int8)
    w = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, N).astype(np.float32)
    d = rng.uniform(0.5, 2.0, M).astype(np.float32)
    return x, w, s_w, d


def gpu_linear(x, w, s_w, d, s_a, entry=None):
    M, K = x.shape
    N = w.shape[0]
    xq, wq = fptq.fptq_pack_weights(dev(x)), fptq.fptq_pack_weights(dev(w))     # one packed layout for both operands
    entry = entry or fptq.fptq_w4a4_linear
    y, acc = entry(xq, wq, M, N, K, s_a, dev(s_w), dev(d), want_acc=True)
    y_plain = entry(xq, wq, M, N, K, s_a, dev(s_w), dev(d))                     # the timed variant: no accumulator dump
    assert torch.equal(y.view(torch.int16), y_plain.view(torch.int16))
    return y, acc, xq, wq


PREFILL_WHOLE = [("c2 gate+up as one launch", 2048, 22016, 4096), ("c2 gate", 2048, 11008, 4096), ("c2 down", 2048, 4096, 11008),
                 ("c3 qkv", 4096, 6144, 4096), ("c3 o", 4096, 4096, 4096), ("c3 gate+up", 4096, 28672, 4096),
                 ("c3 down", 4096, 4096, 14336)]


@pytest.mark.parametrize("name,M,N,K", PREFILL_WHOLE, ids=[c[0] for c in PREFILL_WHOLE])
def test_dense_prefill_whole_tensor(oracle, name, M, N, K):
    x, w, s_w, d = dense_inputs(M, N, K, 1)
    y, acc, _, _ = gpu_linear(x, w, s_w, d, 0.31)
    acc_ref = oracle.gemm_i32(x, w)
    assert np.array_equal(acc.cpu().numpy(), acc_ref), name
    assert (acc_ref != 0).mean() > 0.99                       # dense operands: hardly a sum is zero, unlike the sparse cases
    assert np.array_equal(host_bits(y), oracle.epilogue(acc_ref, np.float32(0.31), s_w, d)), name


@pytest.mark.parametrize("M", [1, 8, 32])
@pytest.mark.parametrize("name,N,K", [("qkv", 6144, 4096), ("o", 4096, 4096), ("gate_up", 28672, 4096), ("down", 4096, 14336)])
def test_dense_decode_whole_tensor(oracle, name, N, K, M):
    x, w, s_w, d = dense_inputs(M, N, K, 2)
    y, acc, _, _ = gpu_linear(x, w, s_w, d, 0.27)
    acc_ref = oracle.gemm_i32(x, w)
    assert np.array_equal(acc.cpu().numpy(), acc_ref), (name, M)
    assert np.array_equal(host_bits(y), oracle.epilogue(acc_ref, np.float32(0.27), s_w, d)), (name, M)


PREFILL_SAMPLED = [("c5 qkv", 8192, 10240, 8192), ("c5 o", 8192, 8192, 8192), ("c5 gate+up", 8192, 57344, 8192),
                   ("c5 down", 8192, 8192, 28672)]


@pytest.mark.parametrize("name,M,N,K", PREFILL_SAMPLED, ids=[c[0] for c in PREFILL_SAMPLED])
def test_dense_prefill_sampled_and_freivalds(oracle, name, M, N, K):
    x, w, s_w, d = dense_inputs(M, N, K, 3)
    y, acc, _, _ = gpu_linear(x, w, s_w, d, 0.31)
    rng = np.random.default_rng(K + N)
    ns = 16
    rs, cs = rng.choice(M, ns, replace=False), rng.choice(N, ns, replace=False)
    # one row and one column out of every tile row / tile column of the largest tile, so no tile escapes the sample
    rs = np.concatenate([rs, np.arange(0, M, 256) + rng.integers(0, 256, (M + 255) // 256)]) % M
    cs = np.concatenate([cs, np.arange(0, N, 256) + rng.integers(0, 256, (N + 255) // 256)]) % N
    acc_rows = acc[torch.from_numpy(rs).cuda()].cpu().numpy()
    assert np.array_equal(acc_rows, oracle.gemm_i32(x[rs], w)), name
    acc_cols = acc[:, torch.from_numpy(cs).cuda()].cpu().numpy()
    assert np.array_equal(acc_cols, oracle.gemm_i32(x, w[cs])), name
    rows, cols = rng.integers(0, M, 8192), rng.integers(0, N, 8192)
    got = acc[torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.int64)
    assert np.array_equal(oracle.gemm_i64_samples(x, w, rows, cols), got), name
    for _ in range(2):          # Freivalds: every entry enters, exact integer arithmetic
        v = rng.integers(-8, 9, N).astype(np.int64)
        lhs = (acc.to(torch.int64) * torch.from_numpy(v).cuda()).sum(dim=1).cpu().numpy()
        assert np.array_equal(lhs, freivalds_rhs(x, w, v)), name
    # the epilogue on the sampled rows
    y_rows = host_bits(y[torch.from_numpy(rs).cuda()])
    assert np.array_equal(y_rows, oracle.epilogue(acc_rows, np.float32(0.31), s_w, d[rs])), name


ONE_TILE = [("c2 gate+up as one launch", 2048, 22016, 4096, 1), ("c2 down", 2048, 4096, 11008, 1), ("c3 qkv", 4096, 6144, 4096, 1),
            ("c3 down", 4096, 4096, 14336, 3), ("c5 o", 8192, 8192, 8192, 5), ("c4 down, 8 tokens", 8, 4096, 14336, 1),
            ("c4 gate+up, 32 tokens", 32, 28672, 4096, 1)]


@pytest.mark.parametrize("name,M,N,K,stride", ONE_TILE, ids=[c[0] for c in ONE_TILE])
def test_one_k_tile_at_a_time(oracle, name, M, N, K, stride):
    """Activations that are zero outside one 128-value K tile: the accumulators are that tile's contribution alone, which
    the oracle computes on the sliced operands.  Every K tile (every stride-th on the largest shapes, the first and last
    six always: the pipeline's prologue and drain) is checked on the whole output."""
    x, w, s_w, d = dense_inputs(M, N, K, 4)
    wq = fptq.fptq_pack_weights(dev(w))
    s_w_d = dev(s_w)
    ktiles = (K + 127) // 128
    picked = sorted(set(range(0, ktiles, stride)) | set(range(min(6, ktiles))) | set(range(max(0, ktiles - 6), ktiles)))
    xd = torch.zeros((M, K), dtype=torch.int8, device="cuda")
    x_dev = dev(x)
    for j in picked:
        k0, k1 = j * 128, min(K, (j + 1) * 128)
        xd.zero_()
        xd[:, k0:k1] = x_dev[:, k0:k1]
        xq = fptq.fptq_pack_weights(xd)
        y, acc = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.5, s_w_d, want_acc=True)
        acc_ref = oracle.gemm_i32(np.ascontiguousarray(x[:, k0:k1]), np.ascontiguousarray(w[:, k0:k1]))
        assert torch.equal(acc, torch.from_numpy(acc_ref).cuda()), (name, j)
    assert np.array_equal(host_bits(y), oracle.epilogue(acc_ref, np.float32(0.5), s_w)), name


@pytest.mark.parametrize("M,N,K", [(256, 1024, 8192), (256, 2048, 12288), (512, 1024, 14336), (200, 1000, 28672)])
def test_dense_split_k_whole_tensor(oracle, M, N, K):
    """The workspace path (K split over several workgroups per 64 x 64 tile) and the same through the library's built-in
    scratch area, on dense operands against the oracle."""
    x, w, s_w, d = dense_inputs(M, N, K, 5)
    nbytes = fptq.fptq_linear_workspace_bytes(M, N, K)
    assert nbytes > 0
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    acc_ref = oracle.gemm_i32(x, w)
    y_ref = oracle.epilogue(acc_ref, np.float32(0.29), s_w, d)
    for entry in (lambda *a, **k: fptq.fptq_w4a4_linear_ws(*a[:7], ws, *a[7:], **k), fptq.fptq_w4a4_linear_noalloc):
        y, acc, _, _ = gpu_linear(x, w, s_w, d, 0.29, entry)
        assert np.array_equal(acc.cpu().numpy(), acc_ref), (M, N, K)
        assert np.array_equal(host_bits(y), y_ref), (M, N, K)
    assert int(ws[: 4 * 1024].max()) == 0


@pytest.mark.parametrize("M,N,K", [(2048, 11008, 4096), (2000, 11001, 4100)], ids=["c2 gate", "ragged"])
def test_every_tile_shape_at_size_dense(oracle, M, N, K):
    """Every tile shape of the prefill kernel forced on a full-size problem (several rounds of workgroups for the large
    tiles, thousands of tiles for the small ones, so the tile -> XCD mapping and the partial last round are exercised),
    dense operands, whole tensor against the oracle.  The ragged case has partial tiles on every edge and a padded last
    K tile."""
    x, w, s_w, d = dense_inputs(M, N, K, 6)
    acc_ref = torch.from_numpy(oracle.gemm_i32(x, w)).cuda()
    y_ref = torch.from_numpy(oracle.epilogue(acc_ref.cpu().numpy(), np.float32(0.33), s_w, d).view(np.int16)).cuda()
    xq, wq = fptq.fptq_pack_weights(dev(x)), fptq.fptq_pack_weights(dev(w))
    s_w_d, d_d = dev(s_w), dev(d)
    for tile in range(1, 9):
        fptq.fptq_set_gemm_tile(tile)
        try:
            y, acc = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.33, s_w_d, d_d, want_acc=True)
            y2 = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.33, s_w_d, d_d)
        finally:
            fptq.fptq_set_gemm_tile(0)
        assert torch.equal(acc, acc_ref), (tile, M, N, K)
        assert torch.equal(y.view(torch.int16), y_ref) and torch.equal(y2.view(torch.int16), y_ref), (tile, M, N, K)
