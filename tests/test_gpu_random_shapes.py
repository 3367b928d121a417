"""Seeded random shapes through every kernel choice of the linear layer (few-token kernel, each prefill tile shape,
split K with a workspace), against the independent one-thread-per-output kernel, which the other tests pin to the
oracle.  Shapes are ragged on purpose: M, N and K are rarely multiples of any tile."""
import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq

pytestmark = pytest.mark.gpu


def random_case(rng):
    kind = rng.integers(0, 4)
    if kind == 0:        # few tokens
        M, N, K = int(rng.integers(1, 129)), int(rng.integers(1, 3000)), int(rng.integers(1, 3000)) * 2
    elif kind == 1:      # ragged prefill
        M, N, K = int(rng.integers(129, 700)), int(rng.integers(1, 1500)), int(rng.integers(1, 2500)) * 2
    elif kind == 2:      # long K, few tiles (split K when a workspace is given)
        M, N, K = int(rng.integers(129, 400)), int(rng.integers(1, 700)), int(rng.integers(4096, 9000)) * 2
    else:                # wide
        M, N, K = int(rng.integers(33, 300)), int(rng.integers(16000, 20000)), int(rng.integers(1, 300)) * 2
    return M, N, K


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_against_the_simple_kernel(seed):
    rng = np.random.default_rng(1000 + seed)
    for _ in range(12):
        M, N, K = random_case(rng)
        x = torch.from_numpy(rng.integers(-8, 8, (M, K), dtype=np.int8)).cuda()
        w = torch.from_numpy(rng.integers(-8, 8, (N, K), dtype=np.int8)).cuda()
        xq, wq = fptq.fptq_pack_weights(x), fptq.fptq_pack_weights(w)       # the packed layout is the same for both operands
        s_w = torch.from_numpy(rng.uniform(0.005, 0.02, N).astype(np.float32)).cuda()
        d = torch.from_numpy(rng.uniform(0.5, 2.0, M).astype(np.float32)).cuda() if rng.integers(0, 2) else None
        s_a = float(rng.uniform(0.01, 1.0))
        y_ref, a_ref = fptq.fptq_w4a4_linear_ref(xq, wq, M, N, K, s_a, s_w, d, want_acc=True)
        tile = int(rng.integers(0, 9))
        fptq.fptq_set_gemm_tile(tile)
        try:
            y, a = fptq.fptq_w4a4_linear(xq, wq, M, N, K, s_a, s_w, d, want_acc=True)
        finally:
            fptq.fptq_set_gemm_tile(0)
        where = f"M={M} N={N} K={K} tile={tile}"
        assert torch.equal(a, a_ref), where
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), where
        nbytes = fptq.fptq_linear_workspace_bytes(M, N, K)
        if nbytes:
            ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            for _ in range(2):
                y2 = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, s_a, s_w, ws, d)
                assert torch.equal(y2.view(torch.int16), y_ref.view(torch.int16)), where + " (workspace)"


def test_launch_order_tile_mapping_gives_the_same_results():
    """The measurement aid that maps workgroups to tiles in launch order changes which workgroup computes which tile,
    nothing else."""
    rng = np.random.default_rng(77)
    for M, N, K, tile in [(700, 1500, 512, 4), (1100, 2100, 384, 1), (300, 4000, 256, 3), (513, 777, 1024, 0), (260, 900, 12288, 0)]:
        xq = fptq.fptq_pack_weights(torch.from_numpy(rng.integers(-8, 8, (M, K), dtype=np.int8)).cuda())
        wq = fptq.fptq_pack_weights(torch.from_numpy(rng.integers(-8, 8, (N, K), dtype=np.int8)).cuda())
        s_w = torch.from_numpy(rng.uniform(0.005, 0.02, N).astype(np.float32)).cuda()
        y_ref, a_ref = fptq.fptq_w4a4_linear_ref(xq, wq, M, N, K, 0.3, s_w, want_acc=True)
        fptq.fptq_set_gemm_tile(tile)
        fptq.fptq_set_gemm_map(1)
        try:
            y, a = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.3, s_w, want_acc=True)
        finally:
            fptq.fptq_set_gemm_map(0)
            fptq.fptq_set_gemm_tile(0)
        assert torch.equal(a, a_ref) and torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), (M, N, K, tile)
