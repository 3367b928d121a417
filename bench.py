#!/usr/bin/env python3
"""Benchmark of the W4A4 static-quantized linear path on one MI355X.

A step is one pass of the whole hot path over the Llama-2-7B-shaped MLP of the second benchmark
configuration (2048 tokens): quantize X (per-token RMS scale) -> gate and up GEMM (one launch on the
concatenated weights) -> quantize the down-projection input (given per-token scale) -> down GEMM.  Inputs are synthetic,
seeded, and resident in HBM before the timed region.  One JSON line is printed:

  value      whole-step throughput in TOP/s (2*M*N*K of the three GEMMs / step time, quantize
             kernels included in the time)
  roofline   the MFMA GEMM kernel: algorithmic ops per launch / average launch duration (HIP
             events on the launch stream) against the 5.0 POP/s dense INT8 MFMA peak
  cpu_baseline  the CPU oracle (never tuned) on the same workload, timed on the host cores
  decode     few-token (M = 1, 8, 32) GB/s over the Llama-3-8B layer matrices, graph-replayed and
             cycled over > 256 MB of distinct weight copies so nothing is served from cache
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense INT8 MFMA, TOP/s
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, GB/s


# HBM-side bytes per GEMM launch of the timed region (mean of the gate+up and the down launch), from the
# FETCH_SIZE and WRITE_SIZE counter passes summarised in profiles/bench_c2_mlp_and_decode.md (reads scaled by
# 2.0, writes by 1.0, the factors a 1 GiB elementwise add calibrates).  Offline figures: counters cannot be
# read from inside this script.  The algorithmic bytes are the packed operands, the scales and the bf16 output.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 224.8e6
GEMM_ALGORITHMIC_BYTES_PER_LAUNCH = 95079424


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode summary")
    ap.add_argument("--shapes-out", default=None,
                    help="also time every prefill linear of configs c2, c3, c5 (their own synthetic activations and "
                         "uniform random INT4 activations) and write the table to this JSON file")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one elementwise kernel that reads 1 GiB and writes 1 GiB: under rocprofv3 --pmc "
                         "its FETCH_SIZE / WRITE_SIZE readings give the counter scale for a known byte count")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_04985_amd import binding as fptq
    from paper_2506_04985_amd import probe
    import fptq_workloads as synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    fptq.lib()          # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    if args.calibrate_copy:
        # an elementwise kernel that reads 1 GiB and writes 1 GiB (a plain tensor copy may go through
        # the DMA engines and would not show up as a kernel)
        src = torch.full((1 << 28,), 3, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ workload: config c2
    gate, up, down = synth.config_cases("c2")
    in_gu = synth.draw(gate, with_weights=False)             # X shared by gate and up
    in_dn = synth.draw(down, with_weights=False)
    M = gate.M
    x_gu, x_dn = dev_bf16(in_gu.x_bits), dev_bf16(in_dn.x_bits)
    r_dn = torch.from_numpy(in_dn.row_scale_in).to(dev)
    # gate and up read the same quantized X, so their weights are concatenated along N when they are packed
    # (offline, like every other weight preparation) and one launch computes both: Y[:, :11008] is the gate
    # output, Y[:, 11008:] the up output.
    layers = []
    w_g, s_g = synth.draw_weights(gate)
    w_u, s_u = synth.draw_weights(up)
    w_gu = torch.from_numpy(np.concatenate([w_g, w_u], axis=0)).to(dev)
    layers.append(("gate_up", gate.N + up.N, gate.K, fptq.fptq_pack_weights(w_gu), torch.from_numpy(np.concatenate([s_g, s_u])).to(dev)))
    separate = [(c, fptq.fptq_pack_weights(torch.from_numpy(w).to(dev)), torch.from_numpy(sw).to(dev)) for c, w, sw in ((gate, w_g, s_g), (up, w_u, s_u))]
    del w_g, w_u, w_gu
    w_d, s_d = synth.draw_weights(down)
    layers.append(("down", down.N, down.K, fptq.fptq_pack_weights(torch.from_numpy(w_d).to(dev)), torch.from_numpy(s_d).to(dev)))
    del w_d
    xq_gu = torch.empty(fptq.fptq_packed_bytes(M, gate.K), dtype=torch.uint8, device=dev)
    xq_dn = torch.empty(fptq.fptq_packed_bytes(M, down.K), dtype=torch.uint8, device=dev)
    r_out = torch.empty(M, dtype=torch.float32, device=dev)
    ys = [torch.empty((M, n), dtype=torch.bfloat16, device=dev) for _, n, _, _, _ in layers]
    s_gu, s_dn = float(in_gu.s_a), float(in_dn.s_a)
    gemm_events = []

    def step(record=-1):
        """One pass of the hot path; record = index of the GEMM to bracket with events (-1: none).  Every event
        leaves a bubble of 3-6 us on the stream (the kernel trace shows it in front of the next kernel), so one
        GEMM of every fourth step is bracketed, the two GEMMs in turn."""
        for i, (name, n, k, wq, s_w) in enumerate(layers):
            if i == 0:
                fptq.fptq_quantize_act(x_gu, s_gu, gate.mode, gate.eps, None, out=xq_gu, row_scale_out=r_out)
            else:
                fptq.fptq_quantize_act(x_dn, s_dn, down.mode, down.eps, r_dn, out=xq_dn, row_scale_out=r_out)
            xq, s_a = (xq_gu, s_gu) if i == 0 else (xq_dn, s_dn)
            if record == i:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            fptq.fptq_w4a4_linear(xq, wq, M, n, k, s_a, s_w, out=ys[i])
            if record == i:
                e1.record()
                gemm_events.append((2 * M * n * k, e0, e1))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(record=(k // 4) % 2 if k % 4 == 0 else -1)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    ops_step = sum(2 * M * n * k for _, n, k, _, _ in layers)
    value = ops_step / (ms_per_step * 1e-3) / 1e12

    per_launch = {}
    for (name, _, _, _, _), idx in zip(layers, range(len(layers))):
        t_us = sorted(e0.elapsed_time(e1) * 1e3 for ops, e0, e1 in gemm_events if ops == 2 * M * layers[idx][1] * layers[idx][2])
        if t_us:          # with fewer steps than launches per step some launch is never bracketed
            per_launch[name] = {"n": len(t_us), "median_us": round(t_us[len(t_us) // 2], 2), "best_us": round(t_us[0], 2)}
    # one launch of each kind per step: the average launch is the mean of the kinds' means, however many of each were bracketed
    kinds = {}
    for ops, e0, e1 in gemm_events:
        kinds.setdefault(ops, []).append(e0.elapsed_time(e1))
    gemm_ops = list(kinds)
    avg_ms = float(np.mean([np.mean(v) for v in kinds.values()]))
    achieved = float(np.mean(gemm_ops)) / (avg_ms * 1e-3) / 1e12
    roofline = {"kernel": "linear_mfma_kernel", "bound": "mfma", "achieved": round(achieved, 1),
                "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4),
                "avg_launch_us": round(avg_ms * 1e3, 2), "ops_per_launch": int(np.mean(gemm_ops)),
                "launches": per_launch, "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH, "traffic_unit": "bytes per launch (algorithmic: %d)" % GEMM_ALGORITHMIC_BYTES_PER_LAUNCH}

    # the same three GEMMs on uniform random INT4 activations (dense operands draw more power)
    dense = {}
    for name, rows, K in (("gate_up_input", M, gate.K), ("down_input", M, down.K)):
        dense[name] = torch.randint(0, 256, (fptq.fptq_packed_bytes(rows, K),), dtype=torch.uint8, device=dev)
    def dense_pass():
        for i, (name, n, k, wq, s_w) in enumerate(layers):
            fptq.fptq_w4a4_linear(dense["gate_up_input" if i == 0 else "down_input"], wq, M, n, k, 1.0, s_w, out=ys[i])
    for _ in range(3):
        dense_pass()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        dense_pass()
    e1.record()
    torch.cuda.synchronize()
    dense_tops = ops_step / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e12

    # gate and up as two launches of 11008 channels each (what the single fused launch replaces)
    y_sep = torch.empty((M, gate.N), dtype=torch.bfloat16, device=dev)
    def separate_pass():
        for case, wq, s_w in separate:
            fptq.fptq_w4a4_linear(xq_gu, wq, M, case.N, case.K, s_gu, s_w, out=y_sep)
    sep_us = graph_time_us(torch, separate_pass, iters=10, replays=3)
    fused_us = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear(xq_gu, layers[0][3], M, layers[0][1], layers[0][2], s_gu, layers[0][4], out=ys[0]), iters=10, replays=3)
    del y_sep, separate

    out = {"metric": "W4A4 linear TOPS (prefill)", "value": round(value, 1), "unit": "TOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8 MFMA on int4 operands, int32 accumulate",
           "data": "synthetic",
           "config": {"workload": "c2: Llama-2-7B-shaped MLP, prefill 2048 tokens: quantize X, gate and up [11008x4096 each, "
                                  "packed as one 22016x4096 weight, one launch], quantize X_down, down [4096x11008]",
                      "tokens": M, "ops_per_step": ops_step},
           "pct_int8_mfma_peak": round(value / INT8_MFMA_PEAK_TOPS * 100, 2),
           "gemm_only_dense_int4_activations_tops": round(dense_tops, 1),
           "gate_up_us": {"one_launch_22016": round(fused_us, 1), "two_launches_11008": round(sep_us, 1)},
           "roofline": roofline}

    # ------------------------------------------------------------------ what the device sustains with nothing else going on
    out["attainable"] = attainable_summary(torch, probe, dev)

    # ------------------------------------------------------------------ activation-side kernels and the widened rows
    out["activation_kernels"] = activation_summary(torch, fptq, dev, x_gu, x_dn, r_dn, s_gu, s_dn, gate, down, layers, xq_dn, ys)

    # ------------------------------------------------------------------ few output tiles: the split over K with a workspace
    out["few_tile_linear"] = few_tile_summary(torch, fptq, dev)

    # ------------------------------------------------------------------ decode summary (config c4)
    if not args.no_decode:
        out["decode"] = decode_summary(torch, fptq, dev)

    # ------------------------------------------------------------------ CPU oracle beside it
    if not args.no_cpu:
        from oracle import linear as oracle
        oracle.lib()
        cpu_s = 0.0
        for case, inp in ((gate, in_gu), (up, in_gu), (down, in_dn)):
            w, s_w = synth.draw_weights(case)
            t1 = time.perf_counter()
            oracle.w4a4_linear_timed(inp.x_bits, w, inp.s_a, s_w, case.mode, case.eps, inp.row_scale_in)
            cpu_s += time.perf_counter() - t1
        out["cpu_baseline"] = {"value": round(ops_step / cpu_s / 1e12, 4), "unit": "TOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "seconds": round(cpu_s, 2),
                               "sample": "the full c2 step once (2048 tokens, three linears, quantizer included; weight "
                                         "generation excluded)"}
    if args.shapes_out:
        del layers, ys, x_gu, x_dn, xq_gu, xq_dn
        torch.cuda.empty_cache()
        with open(args.shapes_out, "w") as f:
            json.dump(all_prefill_shapes(torch, fptq, synth, dev, dev_bf16), f, indent=1)
    print(json.dumps(out))


def all_prefill_shapes(torch, fptq, synth, dev, dev_bf16):
    """Every prefill linear of c2, c3, c5: TOP/s of fptq_w4a4_linear on the configuration's own quantized
    activations and on uniform random INT4 activations (graph replay, 10 calls)."""
    rows = []
    for cfg in ("c2", "c3", "c5"):
        for case in synth.config_cases(cfg):
            inp = synth.draw(case, with_weights=False)
            x = dev_bf16(inp.x_bits)
            r_in = None if inp.row_scale_in is None else torch.from_numpy(inp.row_scale_in).to(dev)
            xq, _ = fptq.fptq_quantize_act(x, float(inp.s_a), case.mode, case.eps, r_in)
            nonzero = float((fptq.fptq_unpack(xq, case.M, case.K) != 0).float().mean())
            del x, inp
            wq = torch.randint(0, 256, (fptq.fptq_packed_bytes(case.N, case.K),), dtype=torch.uint8, device=dev)
            s_w = torch.rand(case.N, device=dev) * 0.015 + 0.005
            y = torch.empty((case.M, case.N), dtype=torch.bfloat16, device=dev)
            us_own = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear(xq, wq, case.M, case.N, case.K, 0.5, s_w, out=y), iters=10, replays=3)
            xd = torch.randint(0, 256, (xq.numel(),), dtype=torch.uint8, device=dev)
            us_dense = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear(xd, wq, case.M, case.N, case.K, 0.5, s_w, out=y), iters=10, replays=3)
            rows.append({"case": case.key, "M": case.M, "N": case.N, "K": case.K, "nonzero_activation_fraction": round(nonzero, 4),
                         "own_activations": {"us": round(us_own, 1), "TOPS": round(case.ops / us_own / 1e6, 1),
                                             "pct_peak": round(case.ops / us_own / 1e6 / INT8_MFMA_PEAK_TOPS * 100, 1)},
                         "uniform_int4_activations": {"us": round(us_dense, 1), "TOPS": round(case.ops / us_dense / 1e6, 1),
                                                      "pct_peak": round(case.ops / us_dense / 1e6 / INT8_MFMA_PEAK_TOPS * 100, 1)}})
            del xq, xd, wq, y
            torch.cuda.empty_cache()
    return rows


def attainable_summary(torch, probe, dev):
    """Rates of the library's MFMA-only loop (zero and random INT4 operands) and of a streaming read, measured in
    this run: the published peaks are the roofline denominators, these say what the board delivers under load."""
    res = {}
    chk = torch.empty(65536, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for name, dense in (("mfma_loop_zero_operands_tops", 0), ("mfma_loop_random_int4_operands_tops", 1)):
        probe.mfma_rate(500, dense, chk)
        torch.cuda.synchronize()
        e0.record()
        ops, _ = probe.mfma_rate(2000, dense, chk)
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 256)
    x4 = torch.zeros(4, dtype=torch.int32, device=dev)
    probe.read(src, x4)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        probe.read(src, x4)
    e1.record()
    torch.cuda.synchronize()
    res["stream_read_1GiB_GBps"] = round(5 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    return res


def few_tile_summary(torch, fptq, dev):
    """256 tokens, where the large tiles would leave most CUs idle: the Llama-3-8B down projection (N = 4096,
    K = 14336; a 64 x 64 tile per CU) and the Llama-3-70B key projection (N = 1024, K = 8192; 64 such tiles), the
    latter also through fptq_w4a4_linear_ws, which splits K over four workgroups per tile through a caller workspace."""
    res = []
    for M, N, K in ((256, 4096, 14336), (256, 1024, 8192)):
        xq = torch.randint(0, 256, (fptq.fptq_packed_bytes(M, K),), dtype=torch.uint8, device=dev)
        wq = torch.randint(0, 256, (fptq.fptq_packed_bytes(N, K),), dtype=torch.uint8, device=dev)
        s_w = torch.rand(N, device=dev) * 0.015 + 0.005
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ops = 2 * M * N * K
        plain = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.5, s_w, out=y), iters=10, replays=3)
        row = {"shape": f"M {M} x N {N} x K {K}", "plain_us": round(plain, 1), "plain_TOPS": round(ops / plain / 1e6, 1)}
        nbytes = fptq.fptq_linear_workspace_bytes(M, N, K)
        if nbytes:
            ws = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
            split = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear_ws(xq, wq, M, N, K, 0.5, s_w, ws, out=y), iters=10, replays=3)
            row.update({"workspace_us": round(split, 1), "workspace_TOPS": round(ops / split / 1e6, 1), "workspace_MiB": round(nbytes / 2**20, 1)})
        res.append(row)
    return res


def graph_time_us(torch, fn, iters=20, replays=5):
    """Average time of one call of fn, launch overhead removed by replaying a captured graph."""
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=st):
        for _ in range(iters):
            fn()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (iters * replays)


def activation_summary(torch, fptq, dev, x_gu, x_dn, r_dn, s_gu, s_dn, gate, down, layers, xq_dn, ys):
    """GB/s of the bandwidth-bound activation kernels on the c2 tensors (algorithmic bytes / time), and the
    down projection through the zero-point epilogue."""
    M = gate.M
    res = {}

    def entry(name, us, nbytes):
        res[name] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1), "pct_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS * 100, 1)}

    xq_a = torch.empty(fptq.fptq_packed_bytes(M, gate.K), dtype=torch.uint8, device=dev)
    xq_b = torch.empty(fptq.fptq_packed_bytes(M, down.K), dtype=torch.uint8, device=dev)
    r_out = torch.empty(M, dtype=torch.float32, device=dev)
    b_a = M * gate.K * 2.5 + 4 * M
    b_b = M * down.K * 2.5 + 8 * M
    entry("quantize_rms_2048x4096", graph_time_us(torch, lambda: fptq.fptq_quantize_act(x_gu, s_gu, gate.mode, gate.eps, None, out=xq_a, row_scale_out=r_out)), b_a)
    entry("quantize_given_2048x11008", graph_time_us(torch, lambda: fptq.fptq_quantize_act(x_dn, s_dn, down.mode, down.eps, r_dn, out=xq_b, row_scale_out=r_out)), b_b)
    # the same two quantizers on inputs that are not in any cache: cycled over > 320 MB of copies of X.  (Behind its
    # producer the input is usually still in the 256 MB last-level cache, which is what the figures above see.)
    def cold(x, fn):
        copies = [x.clone() for _ in range((320 << 20) // (x.numel() * 2) + 1)]
        state = {"i": 0}
        def call():
            fn(copies[state["i"] % len(copies)])
            state["i"] += 1
        return graph_time_us(torch, call, iters=2 * len(copies), replays=3)
    entry("quantize_rms_2048x4096_cold_input", cold(x_gu, lambda xx: fptq.fptq_quantize_act(xx, s_gu, gate.mode, gate.eps, None, out=xq_a, row_scale_out=r_out)), b_a)
    entry("quantize_given_2048x11008_cold_input", cold(x_dn, lambda xx: fptq.fptq_quantize_act(xx, s_dn, down.mode, down.eps, r_dn, out=xq_b, row_scale_out=r_out)), b_b)
    entry("hadamard256_quantize_given_2048x11008", graph_time_us(torch, lambda: fptq.fptq_quantize_act_hadamard(x_dn, s_dn, 256, down.mode, down.eps, r_dn, out=xq_b, row_scale_out=r_out)), b_b)
    # the Llama-3-8B down-projection input (4096 tokens x 14336), whose largest power-of-two block is 2048
    x_l3 = torch.randn((4096, 14336), device=dev).to(torch.bfloat16)
    xq_l3 = torch.empty(fptq.fptq_packed_bytes(4096, 14336), dtype=torch.uint8, device=dev)
    r_l3 = torch.rand(4096, device=dev) + 0.5
    r_o3 = torch.empty(4096, dtype=torch.float32, device=dev)
    b_l3 = 4096 * 14336 * 2.5 + 8 * 4096
    entry("quantize_given_4096x14336", graph_time_us(torch, lambda: fptq.fptq_quantize_act(x_l3, 0.3, down.mode, down.eps, r_l3, out=xq_l3, row_scale_out=r_o3)), b_l3)
    entry("hadamard2048_quantize_given_4096x14336", graph_time_us(torch, lambda: fptq.fptq_quantize_act_hadamard(x_l3, 0.3, 2048, down.mode, down.eps, r_l3, out=xq_l3, row_scale_out=r_o3)), b_l3)
    entry("hadamard256_quantize_given_4096x14336", graph_time_us(torch, lambda: fptq.fptq_quantize_act_hadamard(x_l3, 0.3, 256, down.mode, down.eps, r_l3, out=xq_l3, row_scale_out=r_o3)), b_l3)
    del x_l3, xq_l3
    entry("dynamic_quantize_2048x11008", graph_time_us(torch, lambda: fptq.fptq_quantize_act_dynamic(x_dn, out=xq_b, token_scale_out=r_out)), b_b)
    x_next = torch.empty_like(x_gu)
    y_blk = (torch.randn(x_gu.shape, device=dev) * 0.5).to(torch.bfloat16)
    entry("residual_norm_quantize_2048x4096", graph_time_us(torch, lambda: fptq.fptq_residual_norm_quantize(x_gu, y_blk, s_gu, None, gate.eps, x_next=x_next, s_next=r_out, out=xq_a)), M * gate.K * 6.5 + 4 * M)
    _, n_dn, k_dn, wq, s_w = layers[1]
    wsum = torch.zeros(n_dn, dtype=torch.int32, device=dev)
    us = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear_zp(xq_dn, wq, M, n_dn, k_dn, s_dn, s_w, 3, wsum, out=ys[1]))
    res["down_linear_zero_point_epilogue"] = {"us": round(us, 2), "TOPS": round(2 * M * n_dn * k_dn / us / 1e6, 1)}
    us = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear(xq_dn, wq, M, n_dn, k_dn, s_dn, s_w, out=ys[1]))
    res["down_linear_symmetric"] = {"us": round(us, 2), "TOPS": round(2 * M * n_dn * k_dn / us / 1e6, 1)}
    return res


def decode_summary(torch, fptq, dev):
    """GB/s of fptq_w4a4_linear at M = 1, 8, 32 over the four Llama-3-8B layer matrices."""
    layers = {"qkv": (6144, 4096), "o": (4096, 4096), "gate_up": (28672, 4096), "down": (4096, 14336)}
    res = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    weights = {}
    for name, (N, K) in layers.items():
        wbytes = fptq.fptq_packed_bytes(N, K)
        copies = max(2, (320 << 20) // wbytes + 1)
        weights[name] = [torch.randint(0, 256, (wbytes,), dtype=torch.uint8, device=dev) for _ in range(copies)]
    for M in (1, 8, 32):
        tot_b, tot_ms, per = 0, 0.0, {}
        for name, (N, K) in layers.items():
            ws = weights[name]
            xq = torch.randint(0, 256, (fptq.fptq_packed_bytes(M, K),), dtype=torch.uint8, device=dev)
            s_w = torch.rand(N, device=dev) * 0.015 + 0.005
            y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            iters = 2 * len(ws)
            fptq.fptq_w4a4_linear(xq, ws[0], M, N, K, 0.5, s_w, out=y)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            st = torch.cuda.Stream()
            st.wait_stream(torch.cuda.current_stream())
            with torch.cuda.graph(g, stream=st):
                for i in range(iters):
                    fptq.fptq_w4a4_linear(xq, ws[i % len(ws)], M, N, K, 0.5, s_w, out=y)
            g.replay()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(5):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / (5 * iters)
            nbytes = len(ws[0]) + 4 * N + M * K // 2 + 2 * M * N
            per[name] = {"us": round(ms * 1e3, 2), "GBps": round(nbytes / ms / 1e6, 1)}
            tot_b += nbytes
            tot_ms += ms
            del g
        gbs = tot_b / tot_ms / 1e6
        res[f"M{M}"] = {"layer_us": round(tot_ms * 1e3, 2), "GBps": round(gbs, 1),
                        "pct_hbm_peak": round(gbs / HBM_PEAK_GBS * 100, 2), "per_matrix": per,
                        "layer_with_activation_kernels_us": round(decode_layer_us(torch, fptq, dev, M, layers, weights), 2)}
    return res


def decode_layer_us(torch, fptq, dev, M, layers, weights):
    """The eight launches of one block in their order, the linears on cold weights: residual step -> QKV, quantizer
    -> O, residual step -> gate+up, Hadamard quantizer (block 2048) -> down.  Attention and the gated activation
    between them are not part of this library; their outputs are stand-in tensors."""
    d, f = layers["qkv"][1], layers["down"][1]
    bf = lambda *shape: torch.randn(shape, device=dev).to(torch.bfloat16)
    x_res, y_blk, attn, hid = bf(M, d), bf(M, d), bf(M, d), bf(M, f)
    x_next = torch.empty_like(x_res)
    s_n, r_out, r_in = (torch.empty(M, dtype=torch.float32, device=dev) for _ in range(3))
    r_in.fill_(0.8)
    xq_d = torch.empty(fptq.fptq_packed_bytes(M, d), dtype=torch.uint8, device=dev)
    xq_f = torch.empty(fptq.fptq_packed_bytes(M, f), dtype=torch.uint8, device=dev)
    s_w = {n: torch.rand(N, device=dev) * 0.015 + 0.005 for n, (N, K) in layers.items()}
    y = {n: torch.empty((M, N), dtype=torch.bfloat16, device=dev) for n, (N, K) in layers.items()}
    state = {"i": 0}

    def lin(name, xq):
        N, K = layers[name]
        ws = weights[name]
        fptq.fptq_w4a4_linear(xq, ws[state["i"] % len(ws)], M, N, K, 0.5, s_w[name], out=y[name])

    def layer():
        fptq.fptq_residual_norm_quantize(x_res, y_blk, 0.3, None, 1e-5, x_next=x_next, s_next=s_n, out=xq_d)
        lin("qkv", xq_d)
        fptq.fptq_quantize_act(attn, 0.3, 2, 1e-5, r_in, out=xq_d, row_scale_out=r_out)
        lin("o", xq_d)
        fptq.fptq_residual_norm_quantize(x_res, y_blk, 0.3, s_n, 1e-5, x_next=x_next, s_next=s_n, out=xq_d)
        lin("gate_up", xq_d)
        fptq.fptq_quantize_act_hadamard(hid, 0.3, 2048, 2, 1e-5, r_in, out=xq_f, row_scale_out=r_out)
        lin("down", xq_f)
        state["i"] += 1
    return graph_time_us(torch, layer, iters=12, replays=3)


if __name__ == "__main__":
    main()
