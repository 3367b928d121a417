#!/usr/bin/env python3
"""Benchmark of the W4A4 static-quantized linear path on one MI355X.

A step is one pass of the whole hot path over the linear layers of one Llama-3-70B-shaped decoder layer at 8192
prefill tokens (the largest single-GPU benchmark configuration, "c5"): for each of QKV, O, gate+up and down,
quantize the layer's bf16 input (per-token scale, static INT4 grid, packing) and run the INT4 x INT4 linear with its
dequantizing epilogue.  Inputs are synthetic, seeded, and resident in HBM before the timed region.  One JSON line:

  value        whole-step throughput in TOP/s (2 M N K of the four linears / step time, quantizers in the time),
               on the configuration's own activations
  roofline     the dominant launch (the gate+up GEMM): algorithmic ops per launch / average launch duration from
               HIP events on the launch stream, against the 5.0 POP/s dense INT8 MFMA peak.  The configuration's own
               activations quantize to > 99 % zeros (absmax calibration with outlier channels), which lets the part
               clock higher, so the same launches are also timed on uniform random INT4 activations and the LOWER of
               the two rates is the one reported as achieved / frac; both are in the object
  configs      the same two regions for every benchmark configuration with prefill shapes (c2, c3, c5), per launch
  decode       few-token (M = 1, 8, 32) GB/s over the Llama-3-8B layer matrices on cold weights, next to a pure
               streaming read launched the same way (the ceiling of this launch pattern on this board)
  cpu_baseline the CPU oracle (never tuned) on the first rows of the same workload, timed on the host cores
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense INT8 MFMA, TOP/s
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, GB/s
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "linear_mfma_traffic.md")
CPU_SAMPLE_ROWS = 4096           # token rows of the headline workload the oracle is timed on
WARM_SECONDS = 1.0               # untimed stepping before each timed region, beyond --warmup (clock and power settle)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode summary")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the headline workload (c5): no c2 / c3 regions, no activation-kernel, few-tile or attainable-rate sections")
    ap.add_argument("--warm-seconds", type=float, default=WARM_SECONDS,
                    help="untimed stepping before each timed region beyond --warmup (0 for counter passes, where every dispatch is slow)")
    ap.add_argument("--gemm-map", type=int, default=0, choices=(0, 1),
                    help="workgroup -> tile mapping of the prefill kernel: 0 = the library's XCD-aware default, 1 = launch order "
                         "(to measure what the mapping is worth)")
    ap.add_argument("--gemm-tile", type=int, default=0, choices=range(0, 9),
                    help="force one tile shape of the prefill kernel (0 = the library's choice): for A/B runs of the launcher's rule")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one elementwise kernel that reads 1 GiB and writes 1 GiB: under rocprofv3 --pmc "
                         "its FETCH_SIZE / WRITE_SIZE readings give the counter scale for a known byte count")
    return ap.parse_args()


def read_traffic_table(path=TRAFFIC_TABLE):
    """Rows of the committed counter summary: launch name -> dict(M, N, K, kernel, grid, bytes).  Each row is
    | name | M | N | K | kernel | grid threads | FETCH_SIZE KiB | WRITE_SIZE KiB | fetch scale | write scale |."""
    rows = {}
    if not os.path.exists(path):
        return rows
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) != 10 or not re.fullmatch(r"[0-9]+", cells[1] or ""):
            continue
        name, M, N, K, kernel, grid, fetch, write, fs, ws = cells
        rows[name] = {"M": int(M), "N": int(N), "K": int(K), "kernel": kernel.strip("`"), "grid": int(grid),
                      "fetch_kib": float(fetch), "write_kib": float(write), "fetch_scale": float(fs), "write_scale": float(ws),
                      "bytes": 1024.0 * (float(fetch) * float(fs) + float(write) * float(ws))}
    return rows


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
    fptq.fptq_init()
    fptq.fptq_set_gemm_map(args.gemm_map)
    fptq.fptq_set_gemm_tile(args.gemm_tile)
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

    traffic = read_traffic_table()
    keep_host = {}       # first rows of the headline inputs and its weights, for the CPU leg

    def build(cfg):
        """Device-resident layers of one configuration in call order.  The Llama-2 MLP's gate and up read the same
        quantized X, so their weights are concatenated along N when they are packed (offline, like every other weight
        preparation) and one launch computes both."""
        cases = synth.config_cases(cfg)
        layers = []
        if cfg == "c2":
            gate, up, down = cases
            inp = synth.draw(gate, with_weights=False)
            (w_g, s_g), (w_u, s_u) = synth.draw_weights(gate), synth.draw_weights(up)
            layers.append(make_layer("gate_up", gate, inp, np.concatenate([w_g, w_u], axis=0), np.concatenate([s_g, s_u])))
            inp = synth.draw(down, with_weights=False)
            layers.append(make_layer("down", down, inp, *synth.draw_weights(down)))
            return layers
        for case in cases:
            inp = synth.draw(case, with_weights=False)
            w, s_w = synth.draw_weights(case)
            if cfg == "c5" and not args.no_cpu:
                keep_host[case.name] = (case, inp.x_bits[:CPU_SAMPLE_ROWS].copy(), w, s_w, inp.s_a,
                                        None if inp.row_scale_in is None else inp.row_scale_in[:CPU_SAMPLE_ROWS].copy())
            layers.append(make_layer(case.name, case, inp, w, s_w))
        return layers

    def make_layer(name, case, inp, w, s_w):
        M, K, N = case.M, case.K, w.shape[0]
        L = {"name": name, "cfg": case.config, "M": M, "N": N, "K": K, "ops": 2 * M * N * K, "mode": case.mode, "eps": case.eps,
             "s_a": float(inp.s_a), "x": dev_bf16(inp.x_bits),
             "r_in": None if inp.row_scale_in is None else torch.from_numpy(inp.row_scale_in).to(dev),
             "wq": fptq.fptq_pack_weights(torch.from_numpy(w).to(dev)), "s_w": torch.from_numpy(s_w).to(dev),
             "xq": torch.empty(fptq.fptq_packed_bytes(M, K), dtype=torch.uint8, device=dev),
             "r_out": torch.empty(M, dtype=torch.float32, device=dev),
             "y": torch.empty((M, N), dtype=torch.bfloat16, device=dev)}
        # uniform random INT4 codes in the packed layout (any byte is two valid codes; K is a multiple of 128 at these shapes)
        L["xq_dense"] = torch.randint(0, 256, (L["xq"].numel(),), dtype=torch.uint8, device=dev)
        L["plan"] = fptq.fptq_linear_launch_plan(M, N, K)
        torch.cuda.synchronize()
        return L

    def run_regions(layers, steps, warmup):
        """The timed region on the configuration's own activations, then the same on dense INT4 codes.  Every GEMM
        launch is bracketed by a pair of HIP events on the launch stream (each pair leaves a few microseconds of
        bubble, which is part of the step time reported)."""
        ops_step = sum(L["ops"] for L in layers)

        def step(dense, events=None):
            for L in layers:
                fptq.fptq_quantize_act(L["x"], L["s_a"], L["mode"], L["eps"], L["r_in"], out=L["xq"], row_scale_out=L["r_out"])
                if events is not None:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                fptq.fptq_w4a4_linear(L["xq_dense"] if dense else L["xq"], L["wq"], L["M"], L["N"], L["K"], L["s_a"], L["s_w"], out=L["y"])
                if events is not None:
                    e1.record()
                    events.setdefault(L["name"], []).append((e0, e1))
            if events is not None:      # a bracket around nothing: what the pair of events itself costs
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                e1.record()
                events.setdefault("", []).append((e0, e1))

        res = {}
        for dense in (False, True):
            # --warmup steps, then keep stepping until WARM_SECONDS have passed: the clock under load settles
            # over hundreds of milliseconds, far more than a handful of steps of a small configuration
            n_warm = 0
            t_w = time.perf_counter()
            while n_warm < warmup or time.perf_counter() - t_w < args.warm_seconds:
                step(dense)
                n_warm += 1
                if n_warm % 8 == 0:
                    torch.cuda.synchronize()
            torch.cuda.synchronize()
            events = {}
            t0 = time.perf_counter()
            for _ in range(steps):
                step(dense, events)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) / steps * 1e3
            # A bracket holds the launch between two event packets; the bracket around nothing measures what the second
            # packet adds (about 5 us), which is subtracted: what remains is the kernel plus the launch latency any stream of
            # kernels pays (with it the averages agree with a kernel trace of the same run to about 1 us).  Negligible for the
            # headline launches, 10 % of the shortest ones.
            pair_us = float(np.mean([a.elapsed_time(b) * 1e3 for a, b in events[""]]))
            launches = {}
            for L in layers:
                t_us = [a.elapsed_time(b) * 1e3 - pair_us for a, b in events[L["name"]]]
                avg = float(np.mean(t_us))
                launches[L["name"]] = {"avg_us": round(avg, 2), "min_us": round(min(t_us), 2), "n": len(t_us),
                                       "TOPS": round(L["ops"] / avg / 1e6, 1),
                                       "pct_peak": round(L["ops"] / avg / 1e6 / INT8_MFMA_PEAK_TOPS * 100, 2)}
            gemm_us = sum(v["avg_us"] for v in launches.values())
            res["dense_int4_activations" if dense else "own_activations"] = {
                "ms_per_step": round(ms, 4), "step_TOPS": round(ops_step / ms / 1e9, 1), "warmup_steps_run": n_warm,
                "gemm_launches_TOPS": round(ops_step / gemm_us / 1e6, 1), "event_pair_overhead_us": round(pair_us, 2),
                "launches": launches}
        return ops_step, res

    def config_entry(layers, ops_step, res):
        shapes = {L["name"]: {"M": L["M"], "N": L["N"], "K": L["K"], "GOP": round(L["ops"] / 1e9, 2), "kernel": L["plan"][0],
                              "grid_threads": L["plan"][1] * L["plan"][2]} for L in layers}
        worst = min((min(res[k]["launches"][n]["pct_peak"] for k in res), n) for n in shapes)
        return {"ops_per_step": ops_step, "shapes": shapes, **res, "lowest_launch_pct_peak": {"launch": worst[1], "pct_peak": worst[0]}}

    # ------------------------------------------------------------------ headline workload: config c5
    t_gen = time.perf_counter()
    layers = build("c5")
    gen_s = time.perf_counter() - t_gen
    M = layers[0]["M"]
    ops_step, res = run_regions(layers, args.steps, args.warmup)
    own, dense = res["own_activations"], res["dense_int4_activations"]
    configs = {"c5": config_entry(layers, ops_step, res)}

    dom = max(layers, key=lambda L: L["ops"])                # the gate+up GEMM: 55 % of the step's operations
    d_own, d_dense = own["launches"][dom["name"]], dense["launches"][dom["name"]]
    low = d_dense if d_dense["avg_us"] >= d_own["avg_us"] else d_own
    alg_bytes = dom["N"] * dom["K"] // 2 + dom["M"] * dom["K"] // 2 + 4 * dom["N"] + 2 * dom["M"] * dom["N"]
    trow = traffic.get("c5." + dom["name"])
    stale = trow is not None and (trow["kernel"], trow["grid"]) != (dom["plan"][0], dom["plan"][1] * dom["plan"][2])
    roofline = {"kernel": "linear_mfma_kernel<%s>, c5 %s %dx%dx%d" % (dom["plan"][0], dom["name"], dom["M"], dom["N"], dom["K"]),
                "bound": "mfma", "achieved": low["TOPS"], "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(low["TOPS"] / INT8_MFMA_PEAK_TOPS, 4),
                "region": "dense_int4_activations" if low is d_dense else "own_activations (the timed region)",
                "avg_launch_us": low["avg_us"], "ops_per_launch": dom["ops"],
                "event_pair_overhead_us": dense["event_pair_overhead_us"] if low is d_dense else own["event_pair_overhead_us"],
                "own_activations": d_own, "dense_int4_activations": d_dense,
                "traffic": None if trow is None or stale else round(trow["bytes"]),
                "traffic_source": "profiles/linear_mfma_traffic.md (FETCH_SIZE and WRITE_SIZE counter passes, scaled by a 1 GiB "
                                  "copy kernel)" + (" -- STALE: the launcher now picks another kernel or grid" if stale else ""),
                "algorithmic_bytes_per_launch": alg_bytes}

    out = {"metric": "W4A4 linear TOPS (prefill)", "value": own["step_TOPS"], "unit": "TOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": own["ms_per_step"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "int8 MFMA on int4 operands, int32 accumulate", "data": "synthetic",
           "config": {"workload": "c5: Llama-3-70B-shaped layer linears, prefill 8192 tokens: for QKV [10240x8192], O [8192x8192], "
                                  "gate+up [57344x8192] and down [8192x28672]: quantize the bf16 input (per-token scale, static "
                                  "INT4, packing), INT4 x INT4 linear with dequantizing epilogue to bf16",
                      "tokens": M, "ops_per_step": ops_step, "input_generation_s": round(gen_s, 1)},
           "pct_int8_mfma_peak": round(own["step_TOPS"] / INT8_MFMA_PEAK_TOPS * 100, 2),
           "value_dense_int4_activations": dense["step_TOPS"],
           "pct_int8_mfma_peak_dense_int4_activations": round(dense["step_TOPS"] / INT8_MFMA_PEAK_TOPS * 100, 2),
           "warmup_note": "after --warmup steps every region keeps stepping untimed until %.1f s have passed" % args.warm_seconds,
           "gemm_map": args.gemm_map, "gemm_tile": args.gemm_tile,
           "roofline": roofline}

    # ------------------------------------------------------------------ the other prefill configurations, same two regions
    if not args.headline_only:
        del layers
        torch.cuda.empty_cache()
        for cfg in ("c2", "c3"):
            ls = build(cfg)
            o, r = run_regions(ls, max(args.steps, 50), args.warmup)
            configs[cfg] = config_entry(ls, o, r)
            if cfg == "c2":
                act_layers = ls
            else:
                del ls
            torch.cuda.empty_cache()
    out["configs"] = configs

    if not args.headline_only:
        out["attainable"] = attainable_summary(torch, probe, dev)
        out["activation_kernels"] = activation_summary(torch, fptq, dev, act_layers)
        del act_layers
        torch.cuda.empty_cache()
        out["few_tile_linear"] = few_tile_summary(torch, fptq, dev)

    # ------------------------------------------------------------------ decode summary (config c4)
    if not args.no_decode:
        out["decode"] = decode_summary(torch, fptq, probe, dev)

    # ------------------------------------------------------------------ CPU oracle beside it
    if not args.no_cpu:
        from oracle import linear as oracle
        from oracle import build as oracle_build
        oracle.lib()
        cpu_s, cpu_ops = 0.0, 0
        for name, (case, x_bits, w, s_w, s_a, r_in) in keep_host.items():
            t1 = time.perf_counter()
            oracle.w4a4_linear_timed(x_bits, w, s_a, s_w, case.mode, case.eps, r_in)
            cpu_s += time.perf_counter() - t1
            cpu_ops += 2 * x_bits.shape[0] * case.N * case.K
        out["cpu_baseline"] = {"value": round(cpu_ops / cpu_s / 1e12, 4), "unit": "TOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "seconds": round(cpu_s, 2),
                               "sample": "the first %d of the 8192 token rows of the same c5 step (four linears, quantizer and "
                                         "epilogue included; input generation excluded); the rate is per operation, so the "
                                         "whole step extrapolates to %.0f s" % (CPU_SAMPLE_ROWS, ops_step / (cpu_ops / cpu_s)),
                               "extrapolated": True, "compiler_flags": "gcc " + " ".join(oracle_build.CFLAGS)}
    print(json.dumps(out))


def warm_graph_time_us(torch, fn, iters=10, replays=5, warm_s=0.25):
    """Average time of one call of fn from a replayed graph, after replaying it untimed for warm_s seconds."""
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=st):
        for _ in range(iters):
            fn()
    t0 = time.perf_counter()
    while True:
        g.replay()
        torch.cuda.synchronize()
        if time.perf_counter() - t0 >= warm_s:
            break
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (iters * replays)


def graph_time_us(torch, fn, iters=20, replays=5):
    """Average time of one call of fn, launch overhead removed by replaying a captured graph."""
    return warm_graph_time_us(torch, fn, iters, replays, warm_s=0.0)


def attainable_summary(torch, probe, dev):
    """Rates of an MFMA-only loop and of a streaming read, measured in this run: the published peaks are the roofline
    denominators, these say what the board delivers under sustained load with nothing else going on.  The MFMA loop
    runs on zero operands, on random INT4 operands (the prefill kernel's operand form) that never change, on such
    operands redrawn every iteration in registers (4 VALU instructions pinned behind every MFMA, no memory traffic:
    the rate the power limit leaves a kernel that feeds the matrix pipe fresh dense data), and with that instruction
    stream on operands that stay zero (what the VALU instructions cost by themselves)."""
    res = {}
    chk = torch.empty(65536, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for name, mode in (("mfma_loop_zero_operands_tops", 0), ("mfma_loop_random_int4_operands_tops", 1),
                       ("mfma_loop_fresh_random_int4_operands_tops", 2), ("mfma_loop_fresh_instruction_stream_zero_operands_tops", 3)):
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.5:          # half a second of the same loop first: the rate under sustained load
            probe.mfma_rate_ex(20000, mode, 1, chk)
            torch.cuda.synchronize()
        e0.record()
        ops = probe.mfma_rate_ex(20000, mode, 1, chk)
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
    latter also with K split over four workgroups per tile: through a caller workspace and through the library's
    built-in scratch area."""
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
            if hasattr(fptq, "fptq_w4a4_linear_noalloc"):
                na = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear_noalloc(xq, wq, M, N, K, 0.5, s_w, out=y), iters=10, replays=3)
                row.update({"builtin_scratch_us": round(na, 1)})
        res.append(row)
    return res


def activation_summary(torch, fptq, dev, c2_layers):
    """GB/s of the bandwidth-bound activation kernels on the c2 tensors (algorithmic bytes / time), and the
    down projection through the zero-point epilogue."""
    gu, dn = c2_layers
    M = gu["M"]
    x_gu, x_dn, r_dn, s_gu, s_dn = gu["x"], dn["x"], dn["r_in"], gu["s_a"], dn["s_a"]
    res = {}

    def entry(name, us, nbytes):
        res[name] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1), "pct_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS * 100, 1)}

    xq_a, xq_b, r_out = gu["xq"], dn["xq"], gu["r_out"]
    b_a = M * gu["K"] * 2.5 + 4 * M
    b_b = M * dn["K"] * 2.5 + 8 * M
    entry("quantize_rms_2048x4096", graph_time_us(torch, lambda: fptq.fptq_quantize_act(x_gu, s_gu, gu["mode"], gu["eps"], None, out=xq_a, row_scale_out=r_out)), b_a)
    entry("quantize_given_2048x11008", graph_time_us(torch, lambda: fptq.fptq_quantize_act(x_dn, s_dn, dn["mode"], dn["eps"], r_dn, out=xq_b, row_scale_out=r_out)), b_b)
    # the same two quantizers on inputs that are not in any cache: cycled over > 320 MB of copies of X.  (Behind its
    # producer the input is usually still in the 256 MB last-level cache, which is what the figures above see.)
    def cold(x, fn):
        copies = [x.clone() for _ in range((320 << 20) // (x.numel() * 2) + 1)]
        state = {"i": 0}
        def call():
            fn(copies[state["i"] % len(copies)])
            state["i"] += 1
        return graph_time_us(torch, call, iters=2 * len(copies), replays=3)
    entry("quantize_rms_2048x4096_cold_input", cold(x_gu, lambda xx: fptq.fptq_quantize_act(xx, s_gu, gu["mode"], gu["eps"], None, out=xq_a, row_scale_out=r_out)), b_a)
    entry("quantize_given_2048x11008_cold_input", cold(x_dn, lambda xx: fptq.fptq_quantize_act(xx, s_dn, dn["mode"], dn["eps"], r_dn, out=xq_b, row_scale_out=r_out)), b_b)
    entry("hadamard256_quantize_given_2048x11008", graph_time_us(torch, lambda: fptq.fptq_quantize_act_hadamard(x_dn, s_dn, 256, dn["mode"], dn["eps"], r_dn, out=xq_b, row_scale_out=r_out)), b_b)
    # the Llama-3-8B down-projection input (4096 tokens x 14336), whose largest power-of-two block is 2048
    x_l3 = torch.randn((4096, 14336), device=dev).to(torch.bfloat16)
    xq_l3 = torch.empty(fptq.fptq_packed_bytes(4096, 14336), dtype=torch.uint8, device=dev)
    r_l3 = torch.rand(4096, device=dev) + 0.5
    r_o3 = torch.empty(4096, dtype=torch.float32, device=dev)
    b_l3 = 4096 * 14336 * 2.5 + 8 * 4096
    entry("quantize_given_4096x14336", graph_time_us(torch, lambda: fptq.fptq_quantize_act(x_l3, 0.3, dn["mode"], dn["eps"], r_l3, out=xq_l3, row_scale_out=r_o3)), b_l3)
    entry("hadamard2048_quantize_given_4096x14336", graph_time_us(torch, lambda: fptq.fptq_quantize_act_hadamard(x_l3, 0.3, 2048, dn["mode"], dn["eps"], r_l3, out=xq_l3, row_scale_out=r_o3)), b_l3)
    entry("hadamard256_quantize_given_4096x14336", graph_time_us(torch, lambda: fptq.fptq_quantize_act_hadamard(x_l3, 0.3, 256, dn["mode"], dn["eps"], r_l3, out=xq_l3, row_scale_out=r_o3)), b_l3)
    del x_l3, xq_l3
    entry("dynamic_quantize_2048x11008", graph_time_us(torch, lambda: fptq.fptq_quantize_act_dynamic(x_dn, out=xq_b, token_scale_out=r_out)), b_b)
    x_next = torch.empty_like(x_gu)
    y_blk = (torch.randn(x_gu.shape, device=dev) * 0.5).to(torch.bfloat16)
    entry("residual_norm_quantize_2048x4096", graph_time_us(torch, lambda: fptq.fptq_residual_norm_quantize(x_gu, y_blk, s_gu, None, gu["eps"], x_next=x_next, s_next=r_out, out=xq_a)), M * gu["K"] * 6.5 + 4 * M)
    wsum = torch.zeros(dn["N"], dtype=torch.int32, device=dev)
    us = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear_zp(dn["xq_dense"], dn["wq"], M, dn["N"], dn["K"], s_dn, dn["s_w"], 3, wsum, out=dn["y"]))
    res["down_linear_zero_point_epilogue_dense"] = {"us": round(us, 2), "TOPS": round(dn["ops"] / us / 1e6, 1)}
    us = graph_time_us(torch, lambda: fptq.fptq_w4a4_linear(dn["xq_dense"], dn["wq"], M, dn["N"], dn["K"], s_dn, dn["s_w"], out=dn["y"]))
    res["down_linear_symmetric_dense"] = {"us": round(us, 2), "TOPS": round(dn["ops"] / us / 1e6, 1)}
    return res


def decode_summary(torch, fptq, probe, dev):
    """GB/s of fptq_w4a4_linear at M = 1, 8, 32 over the four Llama-3-8B layer matrices, every launch on weights that
    are in no cache (cycled over > 320 MB of copies per matrix), next to the ceiling of that launch pattern: a kernel
    that only streams the same bytes, launched the same way (one launch per matrix, same cold copies)."""
    layers = {"qkv": (6144, 4096), "o": (4096, 4096), "gate_up": (28672, 4096), "down": (4096, 14336)}
    res = {}
    weights = {}
    for name, (N, K) in layers.items():
        wbytes = fptq.fptq_packed_bytes(N, K)
        copies = max(2, (320 << 20) // wbytes + 1)
        weights[name] = [torch.randint(0, 256, (wbytes,), dtype=torch.uint8, device=dev) for _ in range(copies)]

    def cycled_us(call, n_copies):
        state = {"i": 0}
        def fn():
            call(state["i"] % n_copies)
            state["i"] += 1
        return graph_time_us(torch, fn, iters=2 * n_copies, replays=5)

    # the ceiling: a pure read of each matrix's bytes as one burst of streaming loads, the best of a few launch shapes
    x4 = torch.zeros(1024, dtype=torch.int32, device=dev)
    ceil_us = {name: min(cycled_us(lambda i, ws=ws: probe.read_burst(ws[i], x4, th, ld), len(ws)) for th, ld in ((256, 4), (256, 8), (1024, 4)))
               for name, ws in weights.items()}
    tiny = torch.zeros(16, dtype=torch.uint8, device=dev)
    empty_us = graph_time_us(torch, lambda: probe.read_burst(tiny, x4, 256, 1), iters=50, replays=5)      # the launch floor of this replay pattern
    wsum_b = sum(len(ws[0]) for ws in weights.values())
    ceil_layer_us = sum(ceil_us.values())
    res["streaming_read_ceiling"] = {"per_matrix_us": {k: round(v, 2) for k, v in ceil_us.items()}, "layer_us": round(ceil_layer_us, 2),
                                     "near_empty_kernel_us": round(empty_us, 2),
                                     "GBps": round(wsum_b / ceil_layer_us / 1e3, 1), "pct_hbm_peak": round(wsum_b / ceil_layer_us / 1e3 / HBM_PEAK_GBS * 100, 2),
                                     "what": "a kernel that only reads each matrix's packed bytes (contiguous, one burst of streaming loads, best of three launch "
                                             "shapes), one launch per matrix on cold copies, graph-replayed like the linears"}
    for M in (1, 8, 32):
        tot_b, tot_us, per = 0, 0.0, {}
        for name, (N, K) in layers.items():
            ws = weights[name]
            xq = torch.randint(0, 256, (fptq.fptq_packed_bytes(M, K),), dtype=torch.uint8, device=dev)
            s_w = torch.rand(N, device=dev) * 0.015 + 0.005
            y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            us = cycled_us(lambda i: fptq.fptq_w4a4_linear(xq, ws[i], M, N, K, 0.5, s_w, out=y), len(ws))
            nbytes = len(ws[0]) + 4 * N + M * K // 2 + 2 * M * N
            per[name] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1), "pct_of_read_ceiling": round(ceil_us[name] / us * 100, 1)}
            tot_b += nbytes
            tot_us += us
        gbs = tot_b / tot_us / 1e3
        res[f"M{M}"] = {"layer_us": round(tot_us, 2), "GBps": round(gbs, 1),
                        "pct_hbm_peak": round(gbs / HBM_PEAK_GBS * 100, 2), "pct_of_read_ceiling": round(ceil_layer_us / tot_us * 100, 1),
                        "per_matrix": per,
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
