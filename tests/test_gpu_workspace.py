"""The linear layer with a workspace: K split over workgroups for problems with few output tiles.  Same results as
without, bit for bit, against the oracle on the small shapes and against the unsplit kernel on the large ones."""
import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq
import fptq_workloads as synth

from gpu_util import dev, dev_bf16, host_bits

pytestmark = pytest.mark.gpu


def zero_ws(M, N, K, extra=0):
    n = fptq.fptq_linear_workspace_bytes(M, N, K)
    return n, (torch.zeros(n + extra, dtype=torch.uint8, device="cuda") if n + extra > 0 else None)


def test_workspace_size_rules():
    assert fptq.fptq_linear_workspace_bytes(2048, 11008, 4096) == 0          # enough tiles already
    assert fptq.fptq_linear_workspace_bytes(8, 4096, 4096) == 0              # few-token kernel
    assert fptq.fptq_linear_workspace_bytes(256, 1024, 4096) == 0            # K too short to split
    assert fptq.fptq_linear_workspace_bytes(256, 4096, 14336) == 0           # a 64 x 64 tile for every CU already
    n = fptq.fptq_linear_workspace_bytes(256, 1024, 14336)                   # 64 tiles, 4 ranges of 28 K tiles
    assert n == (1024 + 4 * 64 * 64 * 64) * 4
    assert fptq.fptq_linear_workspace_bytes(256, 2048, 14336) == (1024 + 2 * 128 * 64 * 64) * 4
    with pytest.raises(fptq.FptqError):
        fptq.fptq_linear_workspace_bytes(0, 4096, 4096)


@pytest.mark.parametrize("M,N,K", [(129, 300, 12288), (200, 260, 12416), (257, 130, 12290), (300, 1000, 12288), (512, 128, 14336),
                                   (130, 2100, 12288)])
def test_split_matches_oracle(oracle, M, N, K):
    case = synth.LinearCase("ws", f"m{M}", M, N, K, "normal", 0.0, 3, 4.0, synth.MODE_RMS, M + N + K)
    inp = synth.draw(case)
    ref = oracle.w4a4_linear(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, synth.MODE_RMS, case.eps)
    nbytes, ws = zero_ws(M, N, K)
    assert nbytes > 0
    xq, _ = fptq.fptq_quantize_act(dev_bf16(inp.x_bits), float(inp.s_a), synth.MODE_RMS, case.eps)
    wq = fptq.fptq_pack_weights(dev(inp.w_int))
    for _ in range(3):                       # the workspace is reused: every call must leave it usable
        y, acc = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, float(inp.s_a), dev(inp.s_w), ws, want_acc=True)
        assert np.array_equal(acc.cpu().numpy(), ref["acc"])
        assert np.array_equal(host_bits(y), ref["y"])
    counters = ws[: 4 * 1024]
    assert int(counters.max()) == 0          # arrival counters are back to zero


@pytest.mark.parametrize("M,N,K", [(256, 2048, 12288), (512, 1024, 14336), (1024, 512, 16384), (129, 2048, 6144), (384, 1030, 12296),
                                   (300, 1500, 28672), (256, 1024, 6272)])
def test_split_equals_unsplit_at_size(M, N, K):
    torch.manual_seed(M + N + K)
    xq = torch.randint(0, 256, (fptq.fptq_packed_bytes(M, K),), dtype=torch.uint8, device="cuda")
    wq = torch.randint(0, 256, (fptq.fptq_packed_bytes(N, K),), dtype=torch.uint8, device="cuda")
    if K % 128:                              # keep the K padding of both operands zero, as the packers do
        w8 = fptq.fptq_unpack(wq, N, K)
        wq = fptq.fptq_pack_weights(w8)
        x8 = fptq.fptq_unpack(xq, M, K)
        xq = fptq.fptq_pack_weights(x8)
    s_w = torch.rand(N, device="cuda") * 0.015 + 0.005
    d = torch.rand(M, device="cuda") + 0.5
    y0, a0 = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.37, s_w, d, want_acc=True)
    nbytes, ws = zero_ws(M, N, K, extra=1024)
    assert nbytes > 0
    for _ in range(5):
        y1, a1 = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, 0.37, s_w, ws, d, want_acc=True)
        assert torch.equal(a0, a1) and torch.equal(y0.view(torch.int16), y1.view(torch.int16))
    y2 = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, 0.37, s_w, ws, d)          # without the accumulator dump
    assert torch.equal(y0.view(torch.int16), y2.view(torch.int16))


def test_split_never_reads_a_previous_call_s_partials():
    """The same workspace under alternating inputs: a partial tile left over from the previous call (a stale cache
    line on another XCD, say) would show up as a wrong sum."""
    M, N, K = 256, 1024, 14336
    torch.manual_seed(5)
    wq = torch.randint(0, 256, (fptq.fptq_packed_bytes(N, K),), dtype=torch.uint8, device="cuda")
    s_w = torch.rand(N, device="cuda") * 0.015 + 0.005
    xs = [torch.randint(0, 256, (fptq.fptq_packed_bytes(M, K),), dtype=torch.uint8, device="cuda") for _ in range(3)]
    want = [fptq.fptq_w4a4_linear(x, wq, M, N, K, 0.5, s_w, want_acc=True)[1] for x in xs]
    _, ws = zero_ws(M, N, K)
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    bad = 0
    for it in range(150):
        i = it % 3
        fptq.fptq_w4a4_linear_ws(xs[i], wq, M, N, K, 0.5, s_w, ws, acc=acc)
        bad += int((acc != want[i]).sum())
    assert bad == 0


def test_workspace_too_small_or_absent_falls_back():
    M, N, K = 256, 1024, 12288
    torch.manual_seed(1)
    xq = torch.randint(0, 256, (fptq.fptq_packed_bytes(M, K),), dtype=torch.uint8, device="cuda")
    wq = torch.randint(0, 256, (fptq.fptq_packed_bytes(N, K),), dtype=torch.uint8, device="cuda")
    s_w = torch.rand(N, device="cuda") * 0.015 + 0.005
    y0 = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.5, s_w)
    small = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    for ws in (None, small):
        y1 = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, 0.5, s_w, ws)
        assert torch.equal(y0.view(torch.int16), y1.view(torch.int16))
    assert int(small.max()) == 0             # an unusable workspace is not touched


def test_calls_of_different_shapes_share_one_workspace():
    """One workspace, sized for the largest, serves problems of different tile counts in turn: the arrival counters
    sit in a region of fixed size, so a smaller problem's partial sums never land where a larger one counts."""
    shapes = [(512, 1024, 14336), (256, 512, 6272), (300, 1000, 12290), (129, 128, 12288), (512, 1024, 14336)]
    torch.manual_seed(9)
    ws = torch.zeros(max(fptq.fptq_linear_workspace_bytes(*s) for s in shapes), dtype=torch.uint8, device="cuda")
    for rep in range(2):
        for M, N, K in shapes:
            xq = fptq.fptq_pack_weights(torch.randint(-8, 8, (M, K), dtype=torch.int8, device="cuda"))
            wq = fptq.fptq_pack_weights(torch.randint(-8, 8, (N, K), dtype=torch.int8, device="cuda"))
            s_w = torch.rand(N, device="cuda") * 0.015 + 0.005
            y0, a0 = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.4, s_w, want_acc=True)
            y1, a1 = fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, 0.4, s_w, ws, want_acc=True)
            assert torch.equal(a0, a1) and torch.equal(y0.view(torch.int16), y1.view(torch.int16)), (rep, M, N, K)
            assert int(ws[: 4 * 1024].max()) == 0
