"""The entry point that allocates nothing (fptq_w4a4_linear_noalloc): the split-K exchange through the library's
built-in scratch area gives what fptq_w4a4_linear_ws gives with a caller workspace, bit for bit, on calls in a row
that share the area -- a larger problem first, then a smaller one, then one that does not split at all."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq

pytestmark = pytest.mark.gpu


def operands(M, N, K, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    rnd = lambda n: torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda", generator=g)
    xq, wq = rnd(fptq.fptq_packed_bytes(M, K)), rnd(fptq.fptq_packed_bytes(N, K))
    if K % 128:          # keep the K padding of both operands zero, as the packers do
        xq = fptq.fptq_pack_weights(fptq.fptq_unpack(xq, M, K))
        wq = fptq.fptq_pack_weights(fptq.fptq_unpack(wq, N, K))
    s_w = torch.rand(N, device="cuda", generator=g) * 0.015 + 0.005
    d = torch.rand(M, device="cuda", generator=g) + 0.5
    return xq, wq, s_w, d


def test_two_calls_in_a_row_match_the_workspace_entry_point():
    shapes = [(512, 1024, 14336), (256, 512, 6272), (300, 1000, 12290), (200, 260, 28672), (256, 4096, 4096), (8, 4096, 4096)]
    prepared = []
    for i, (M, N, K) in enumerate(shapes):
        xq, wq, s_w, d = operands(M, N, K, 100 + i)
        nbytes = fptq.fptq_linear_workspace_bytes(M, N, K)
        ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None
        y_ws, a_ws = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, 0.37, s_w, ws, d, want_acc=True)
        y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        prepared.append((M, N, K, xq, wq, s_w, d, y_ws, a_ws, y, acc, nbytes))
    assert [p[-1] > 0 for p in prepared] == [True, True, True, True, False, False]
    assert prepared[0][-1] > prepared[1][-1]          # the second call is the smaller one
    torch.cuda.synchronize()
    # all outputs exist: from here on nothing is allocated by anybody
    before = torch.cuda.memory_allocated()
    for rep in range(3):
        for M, N, K, xq, wq, s_w, d, y_ws, a_ws, y, acc, _ in prepared:
            y.zero_(), acc.zero_()
            fptq.fptq_w4a4_linear_noalloc(xq, wq, M, N, K, 0.37, s_w, d, out=y, acc=acc)
            assert torch.equal(acc, a_ws), (rep, M, N, K)
            assert torch.equal(y.view(torch.int16), y_ws.view(torch.int16)), (rep, M, N, K)
            fptq.fptq_w4a4_linear_noalloc(xq, wq, M, N, K, 0.37, s_w, d, out=y)      # and without the accumulator dump
            assert torch.equal(y.view(torch.int16), y_ws.view(torch.int16)), (rep, M, N, K)
    assert torch.cuda.memory_allocated() == before


def test_same_validation_as_the_plain_entry_point():
    L = fptq.lib()
    dummy = ctypes.c_void_p(4096)
    assert L.fptq_w4a4_linear_noalloc(None, dummy, 256, 1024, 14336, 1.0, dummy, None, dummy, None, None) == -1
    assert L.fptq_w4a4_linear_noalloc(dummy, dummy, 0, 1024, 14336, 1.0, dummy, None, dummy, None, None) == -2
    assert L.fptq_w4a4_linear_noalloc(dummy, dummy, 256, 1024, 14336, -1.0, dummy, None, dummy, None, None) == -6
    assert L.fptq_w4a4_linear_noalloc(dummy, dummy, 256, 1024, 1 << 25, 1.0, dummy, None, dummy, None, None) == -2
