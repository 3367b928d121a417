"""The library under HIP graph capture: a block's worth of calls captured once and replayed on changing inputs, with
eager work and synchronisations between the replays; every replay must equal the eager result on the same inputs
(this includes the split-K workspace, whose arrival counters must be back to zero after every launch)."""
import pytest
import torch

from paper_2506_04985_amd import binding as fptq

pytestmark = pytest.mark.gpu


def run_block(t):
    """quantize -> prefill linear (MFMA tiles); residual step -> few-token linear; Hadamard quantizer -> split-K linear."""
    fptq.fptq_quantize_act(t["x"], 0.3, 1, 1e-5, None, out=t["xq"], row_scale_out=t["r"])
    fptq.fptq_w4a4_linear(t["xq"], t["w1"], t["M"], t["N1"], t["K"], 0.3, t["s1"], out=t["y1"])
    fptq.fptq_residual_norm_quantize(t["xs"], t["ys"], 0.3, None, 1e-5, x_next=t["xn"], s_next=t["sn"], out=t["xqs"])
    fptq.fptq_w4a4_linear(t["xqs"], t["w1"], t["Ms"], t["N1"], t["K"], 0.3, t["s1"], t["sn"], out=t["y2"])
    fptq.fptq_quantize_act_hadamard(t["h"], 0.3, 256, 2, 1e-5, t["rin"], out=t["hq"], row_scale_out=t["r"])
    fptq.fptq_w4a4_linear_ws(t["hq"], t["w2"], t["M"], t["N2"], t["K2"], 0.3, t["s2"], t["ws"], out=t["y3"])


def test_replays_match_eager_results():
    dev = "cuda"
    torch.manual_seed(11)
    M, Ms, K, N1, K2, N2 = 200, 8, 1024, 1536, 6400, 512
    assert fptq.fptq_linear_workspace_bytes(M, N2, K2) > 0
    t = {"M": M, "Ms": Ms, "K": K, "N1": N1, "K2": K2, "N2": N2}
    t["w1"] = torch.randint(0, 256, (fptq.fptq_packed_bytes(N1, K),), dtype=torch.uint8, device=dev)
    t["w2"] = torch.randint(0, 256, (fptq.fptq_packed_bytes(N2, K2),), dtype=torch.uint8, device=dev)
    t["s1"] = torch.rand(N1, device=dev) * 0.015 + 0.005
    t["s2"] = torch.rand(N2, device=dev) * 0.015 + 0.005
    t["rin"] = torch.rand(M, device=dev) + 0.5
    t["ws"] = torch.zeros(fptq.fptq_linear_workspace_bytes(M, N2, K2), dtype=torch.uint8, device=dev)
    bf = lambda *s: torch.empty(s, dtype=torch.bfloat16, device=dev)
    t.update(x=bf(M, K), xs=bf(Ms, K), ys=bf(Ms, K), xn=bf(Ms, K), h=bf(M, K2), y1=bf(M, N1), y2=bf(Ms, N1), y3=bf(M, N2))
    t.update(xq=torch.empty(fptq.fptq_packed_bytes(M, K), dtype=torch.uint8, device=dev),
             xqs=torch.empty(fptq.fptq_packed_bytes(Ms, K), dtype=torch.uint8, device=dev),
             hq=torch.empty(fptq.fptq_packed_bytes(M, K2), dtype=torch.uint8, device=dev),
             r=torch.empty(M, dtype=torch.float32, device=dev), sn=torch.empty(Ms, dtype=torch.float32, device=dev))
    inputs, outputs = ("x", "xs", "ys", "h"), ("y1", "y2", "y3", "xn", "sn", "xq", "hq")

    def fresh_inputs(seed):
        g = torch.Generator(device=dev).manual_seed(seed)
        for k in inputs:
            t[k].copy_((torch.randn(t[k].shape, device=dev, generator=g) * 1.5).to(torch.bfloat16))

    def snapshot():
        return {k: t[k].clone() for k in outputs}

    fresh_inputs(0)
    fptq.fptq_init()                               # the device is set up; no kernel of the block has to run before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        run_block(t)
    for seed in (1, 2, 3, 4):
        fresh_inputs(seed)
        run_block(t)
        torch.cuda.synchronize()
        want = snapshot()
        for k in outputs:
            t[k].zero_()
        junk = torch.randn(1 << 20, device=dev).sum()        # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = snapshot()
        for k in outputs:
            assert torch.equal(got[k].view(torch.uint8), want[k].view(torch.uint8)), (seed, k)
        assert int(t["ws"][: 4 * 1024].max()) == 0 and junk.isfinite()


def test_the_entry_point_that_allocates_nothing_under_capture():
    """What fptq_w4a4_linear_noalloc is for: a split-K linear captured without any workspace in sight; every replay, on
    new activations, equals the eager result of the plain entry point."""
    dev = "cuda"
    torch.manual_seed(3)
    M, N, K = 256, 1024, 8192
    assert fptq.fptq_linear_workspace_bytes(M, N, K) > 0
    wq = torch.randint(0, 256, (fptq.fptq_packed_bytes(N, K),), dtype=torch.uint8, device=dev)
    s_w = torch.rand(N, device=dev) * 0.015 + 0.005
    xq = torch.empty(fptq.fptq_packed_bytes(M, K), dtype=torch.uint8, device=dev)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    fptq.fptq_init()
    xq.random_(0, 256)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        fptq.fptq_w4a4_linear_noalloc(xq, wq, M, N, K, 0.4, s_w, out=y)
    for seed in range(4):
        g = torch.Generator(device=dev).manual_seed(seed)
        xq.random_(0, 256, generator=g)
        want = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.4, s_w)
        y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), want.view(torch.int16)), seed
