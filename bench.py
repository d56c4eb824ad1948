#!/usr/bin/env python3
"""Benchmark of the PEQA quantized-linear hot path on one MI355X.

One "step" = one training pass over the seven linears of a LLaMA-7B decoder block
(4-bit per-channel codes, T = 2048 tokens): forward Y, backward dX, scale gradient d_ds
and the AdamW scale update, all through the C-ABI library.  Quantization is the method's
one-time decomposition step and is done (and timed) once before the loop.  The layers of the block
that read one input (q, k, v; gate, up) run stacked along their output channels as one layer each,
which is a property of the packed layout, not another kernel (--separate runs the seven one by one).

Prints ONE JSON line: fwd+bwd TFLOP/s counting 6*T*N*K flops per layer (three dense
contractions: forward, dX, and the product recomputed for the scale gradient), with
  roofline     - the dominant kernel against the bf16 MFMA peak, timed with HIP events
  cpu_baseline - the CPU oracle timed on a bounded sample of the same workload
  small_batch  - the deployment forward (T = 1 and 16) of the same block against the HBM peak,
                 rotating through more than 256 MB of distinct weights so that every read is from HBM
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="workload index (see synth.CONFIGS)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-small-batch", action="store_true")
    ap.add_argument("--no-kept-product", action="store_true",
                    help="skip the secondary timing of the variant that keeps the forward's product")
    ap.add_argument("--separate", action="store_true",
                    help="run q, k, v and gate, up as separate layers (7 forward and 7 backward contractions "
                         "of each kind) instead of stacked along their output channels (4 of each kind)")
    ap.add_argument("--graph", action="store_true",
                    help="replay a HIP graph of the forward and backward calls instead of launching them one by "
                         "one (measured about 1 %% slower than the direct launches on this workload)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three 256 MiB device copies, a kernel of known traffic against which "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


class Layer:
    def __init__(self, torch, peqa, N, K, bits, group, T, seed, w_std, dy_std):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        self.N, self.K, self.T = N, K, T
        self.L = peqa.layout(N, K, bits, group)
        G = self.L.groups
        W0 = torch.randn((N, K), generator=g, device="cuda", dtype=torch.float32) * w_std
        self.packed = torch.empty(peqa.packed_words(self.L), dtype=torch.int32, device="cuda")
        self.s0 = torch.empty((N, G), dtype=torch.float32, device="cuda")
        self.z0 = torch.empty((N, G), dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        peqa.quantize(self.L, W0, self.packed, self.s0, self.z0)
        torch.cuda.synchronize()
        self.quantize_ms = (time.perf_counter() - t0) * 1e3
        del W0
        self.ds = torch.zeros((N, G), dtype=torch.float32, device="cuda")
        self.m = torch.zeros_like(self.ds)
        self.v = torch.zeros_like(self.ds)
        self.dds = torch.empty_like(self.ds)
        self.X = torch.randn((T, K), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        self.dY = (torch.randn((T, N), generator=g, device="cuda", dtype=torch.float32) * dy_std).to(torch.bfloat16)
        self.Y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
        self.dX = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
        self.ws_fwd = peqa.workspace_bytes(self.L, T, peqa.PEQA_OP_FWD)
        self.ws_bwd = peqa.workspace_bytes(self.L, T, peqa.PEQA_OP_BWD)


def stack_layers(torch, peqa, members, bits, group):
    """One layer out of layers that read the same input, stacked along the output channels.  Packed
    codes are stored by rows of 128-channel tiles and s0, z0, ds by channel, so the stacked layer's
    arrays are the members' arrays one after the other: Y and dY become [T, sum N] (each member a
    column slice), and the backward returns the gradient of the shared input, i.e. the sum of the
    members' dX, from one contraction over all sum N channels."""
    first = members[0]
    st = Layer.__new__(Layer)
    st.N, st.K, st.T = sum(m.N for m in members), first.K, first.T
    st.L = peqa.layout(st.N, st.K, bits, group)
    st.packed = torch.cat([m.packed for m in members])
    st.s0 = torch.cat([m.s0 for m in members])
    st.z0 = torch.cat([m.z0 for m in members])
    assert st.packed.numel() == peqa.packed_words(st.L)
    st.quantize_ms = 0.0
    st.ds = torch.zeros_like(st.s0)
    st.m = torch.zeros_like(st.s0)
    st.v = torch.zeros_like(st.s0)
    st.dds = torch.empty_like(st.s0)
    st.X = first.X
    st.dY = torch.cat([m.dY for m in members], dim=1).contiguous()
    st.Y = torch.empty((st.T, st.N), dtype=torch.bfloat16, device="cuda")
    st.dX = torch.empty((st.T, st.K), dtype=torch.bfloat16, device="cuda")
    st.ws_fwd = peqa.workspace_bytes(st.L, st.T, peqa.PEQA_OP_FWD)
    st.ws_bwd = peqa.workspace_bytes(st.L, st.T, peqa.PEQA_OP_BWD)
    return st


def shared_input_groups(cfg):
    """Indices of the block's layers grouped by the input they read: the first three of a run of four
    equal layers are q, k, v (the fourth, o, reads the attention output); a run of two is gate, up."""
    groups, i = [], 0
    for (_, _, count) in cfg["layers"]:
        fuse = count - 1 if count == 4 else count
        groups.append(list(range(i, i + fuse)))
        if fuse != count:
            groups.append([i + fuse])
        i += count
    return groups


def small_batch(torch, peqa, layers, cfg, ws, ws_bytes, stream, reps=20):
    """Forward of the block at T = 1 and T = 16 through the matrix-vector path.  Algorithmic bytes per
    layer: packed codes + s0, ds (fp32) and z0 (uint8) per scale + X and Y (bf16).  `wall` is the
    stream time per block (what a caller sees); `kernels` sums the event-bracketed launches, which
    includes the events' own gaps."""
    bits = cfg["bits"]
    block_packed = sum(l.packed.numel() * 4 for l in layers)
    nsets = max(2, -(-(300 << 20) // block_packed))            # > 256 MB of distinct weight bytes
    g = torch.Generator(device="cuda")
    g.manual_seed(12345)
    sets = [[l.packed for l in layers]]
    for _ in range(nsets - 1):
        sets.append([torch.randint(-2 ** 31, 2 ** 31 - 1, (l.packed.numel(),), generator=g, device="cuda",
                                   dtype=torch.int32) for l in layers])
    out = {"weight_sets": nsets, "hbm_peak_GBs": HBM_PEAK_GBS}
    for T in (1, 16):
        need = max(peqa.workspace_bytes(l.L, T, peqa.PEQA_OP_FWD) for l in layers)
        assert need <= ws_bytes
        bytes_block = sum(l.N * l.K * bits / 8 + l.N * l.L.groups * 9 + 2 * T * (l.K + l.N) for l in layers)

        def run():
            for packed_set in sets:
                for l, pk in zip(layers, packed_set):
                    peqa.linear_fwd(l.L, pk, l.s0, l.ds, l.z0, l.X, T, l.Y, ws, ws_bytes, stream)

        for _ in range(3):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        wall_us = (time.perf_counter() - t0) / (reps * nsets) * 1e6
        peqa.trace_begin(2 * len(layers) * nsets * reps + 16)
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        tr = peqa.trace_end(16)
        kern_us = sum(ms for (_, ms) in tr.values()) * 1e3 / (reps * nsets)
        main_us = tr["gemv"][1] * 1e3 / (reps * nsets)
        # the same block with the layers that read one X fused into one call each:
        # (q, k, v), o, (gate, up), down -- 4 calls instead of 7
        groups = shared_input_groups(cfg)
        need_f = max(peqa.workspace_bytes_fused([(layers[j].L, layers[j].packed, layers[j].s0, layers[j].ds,
                                                  layers[j].z0, layers[j].Y) for j in grp], T) for grp in groups)
        assert need_f <= ws_bytes
        bytes_fused = sum(l.N * l.K * bits / 8 + l.N * l.L.groups * 9 + 2 * T * l.N for l in layers) + \
            sum(2 * T * layers[grp[0]].K for grp in groups)

        def run_fused():
            for packed_set in sets:
                for grp in groups:
                    items = [(layers[j].L, packed_set[j], layers[j].s0, layers[j].ds, layers[j].z0, layers[j].Y)
                             for j in grp]
                    peqa.linear_fwd_fused(items, layers[grp[0]].X, T, ws, ws_bytes, stream)

        for _ in range(3):
            run_fused()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            run_fused()
        torch.cuda.synchronize()
        fused_us = (time.perf_counter() - t0) / (reps * nsets) * 1e6
        # the same calls replayed as one HIP graph (how a decode loop would launch them)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=torch.cuda.Stream()):
            cap = torch.cuda.current_stream().cuda_stream
            for packed_set in sets:
                for grp in groups:
                    items = [(layers[j].L, packed_set[j], layers[j].s0, layers[j].ds, layers[j].z0, layers[j].Y)
                             for j in grp]
                    peqa.linear_fwd_fused(items, layers[grp[0]].X, T, ws, ws_bytes, cap)
        for _ in range(3):
            gr.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            gr.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / (reps * nsets) * 1e6
        del gr
        out["T%d" % T] = {
            "fused_shared_x": {"calls_per_block": len(groups), "bytes_per_block": int(bytes_fused),
                               "block_us_wall": round(fused_us, 2), "GBs_wall": round(bytes_fused / fused_us / 1e3, 1),
                               "frac_of_hbm_peak_wall": round(bytes_fused / fused_us / 1e3 / HBM_PEAK_GBS, 4),
                               "block_us_hip_graph": round(graph_us, 2),
                               "frac_of_hbm_peak_hip_graph": round(bytes_fused / graph_us / 1e3 / HBM_PEAK_GBS, 4)},
            "bytes_per_block": int(bytes_block),
            "block_us_wall": round(wall_us, 2), "block_us_kernels": round(kern_us, 2),
            "block_us_gemv_kernel": round(main_us, 2),
            "GBs_wall": round(bytes_block / wall_us / 1e3, 1), "GBs_kernels": round(bytes_block / kern_us / 1e3, 1),
            "frac_of_hbm_peak_wall": round(bytes_block / wall_us / 1e3 / HBM_PEAK_GBS, 4),
        }
    out["large_layer"] = large_layer(torch, peqa, cfg, stream)
    return out


def large_layer(torch, peqa, cfg, stream, reps=10):
    """What the matrix-vector kernel reaches when one launch is long enough to hide its ramp: a single
    32768 x 16384 layer of this workload's bit width (per-channel), T = 1, two rotating weight sets."""
    N, K, T, bits = 32768, 16384, 1, cfg["bits"]
    L = peqa.layout(N, K, bits, 0)
    g = torch.Generator(device="cuda")
    g.manual_seed(777)
    sets = [torch.randint(-2 ** 31, 2 ** 31 - 1, (peqa.packed_words(L),), generator=g, device="cuda", dtype=torch.int32)
            for _ in range(2)]
    s0 = torch.full((N, 1), 0.01, dtype=torch.float32, device="cuda")
    z0 = torch.full((N, 1), 7, dtype=torch.uint8, device="cuda")
    X = torch.randn((T, K), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    Y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    nb = peqa.workspace_bytes(L, T, peqa.PEQA_OP_FWD)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")

    def run():
        for pk in sets:
            peqa.linear_fwd(L, pk, s0, None, z0, X, T, Y, ws, nb, stream)

    for _ in range(2):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / (reps * len(sets)) * 1e6
    nbytes = N * K * bits / 8 + N * 9 + 2 * T * (K + N)
    return {"shape": "%dx%d, %d-bit per-channel, T=%d" % (N, K, bits, T), "bytes": int(nbytes), "us_wall": round(us, 2),
            "GBs_wall": round(nbytes / us / 1e3, 1), "frac_of_hbm_peak_wall": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)}


def kept_product(torch, peqa, layers, cfg, stream, steps):
    """The optional variant that keeps P = X (Q - z0)^T from the forward (per-channel layers): the same
    block step with peqa_linear_fwd_keep / peqa_linear_bwd_kept, which does 4 T N K flops per layer."""
    T = cfg["T"]
    fb = max(peqa.workspace_bytes(l.L, T, peqa.PEQA_OP_FWD_KEEP) for l in layers)
    bb = max(peqa.workspace_bytes(l.L, T, peqa.PEQA_OP_BWD_KEPT) for l in layers)
    nb = max(fb, bb)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    Ps = [torch.empty((T, l.N), dtype=torch.float32, device="cuda") for l in layers]

    def step(i):
        for l, P in zip(layers, Ps):
            peqa.linear_fwd_keep(l.L, l.packed, l.s0, l.ds, l.z0, l.X, T, l.Y, P, ws, nb, stream)
        for l, P in zip(reversed(layers), reversed(Ps)):
            peqa.linear_bwd_kept(l.L, l.packed, l.s0, l.ds, l.z0, P, l.dY, T, l.dX, l.dds, ws, nb, stream)
        for l in layers:
            peqa.scale_update(l.ds.numel(), l.ds, l.dds, l.m, l.v, l.s0, lr=1e-5, step=i, stream=stream)

    for i in range(3):
        step(1000 + i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(2000 + i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    flops = sum(4.0 * T * l.N * l.K for l in layers)
    return {"what": "same block step with the forward keeping fp32 P (4 T N bytes per layer) and the scale "
                    "gradient taken from it: 4 T N K flops per layer instead of 6 T N K; eager launches",
            "ms_per_step": round(dt * 1e3, 4), "tokens_per_s": round(T / dt, 1),
            "tflops_counted_4TNK": round(flops / dt / 1e12, 2),
            "kept_bytes": int(sum(P.numel() * 4 for P in Ps))}


def device_info(torch, peqa):
    """What the run saw of the device, and the denominators the fractions above use."""
    p = torch.cuda.get_device_properties(0)
    cus, clock_khz = peqa.device_info()
    return {"name": p.name, "compute_units": cus,
            "max_clock_mhz": round(clock_khz / 1e3),
            "hbm_bytes": p.total_memory,
            "mfma_peak_used": "2500 TFLOP/s dense bf16 (published; 256 CUs x 4096 flop/clk x 2.4 GHz = 2517)",
            "hbm_peak_used": "8000 GB/s (published)"}


def cpu_baseline(cfg, seconds):
    """The oracle as it stands, on a bounded sample: the first layer shape of the workload,
    forward + dX + scale gradient on a few token rows (rows are independent for Y and dX, and the
    scale gradient is a sum over rows), sized by a short calibration run."""
    import numpy as np
    from oracle import peqa_oracle as oracle
    from paper_2305_14152_amd import synth
    N, K, _ = cfg["layers"][0]
    W = synth.normal_f32(1, (N, K), cfg["w_std"])
    codes, s0, z0 = oracle.quantize(W, cfg["bits"], cfg["group"])

    def run(T):
        X = synth.normal_bf16(2, (T, K), 1.0)
        dY = synth.normal_bf16(3, (T, N), cfg["dy_std"])
        t0 = time.perf_counter()
        oracle.fwd(codes, s0, None, z0, X, cfg["group"])
        oracle.bwd(codes, s0, None, z0, X, dY, cfg["group"])
        return time.perf_counter() - t0

    # cost model t(T) = a + b T from two short runs (the oracle's second scale-gradient route has a
    # T-independent part), then one run sized to the time budget
    t8, t24 = run(8), run(24)
    b = max((t24 - t8) / 16.0, 1e-9)
    a = max(t8 - 8.0 * b, 0.0)
    T = int(max(32, min(cfg["T"], (seconds - a) / b)))
    dt = run(T)
    flops = 6.0 * T * N * K
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": "layer %dx%d, %d-bit, %d token rows: fwd + dX + scale gradient, %.1f s" % (N, K, cfg["bits"], T, dt),
            "tokens_per_s_block_extrapolated": None}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no cross-GPU step); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2305_14152_amd import peqa, synth
    peqa.lib()                                   # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = synth.CONFIGS[args.config]
    T, bits, group = cfg["T"], cfg["bits"], cfg["group"]

    layers = []
    li = 0
    for (N, K, count) in cfg["layers"]:
        for _ in range(count):
            layers.append(Layer(torch, peqa, N, K, bits, group, T, synth.seed_for(args.config, li, 0),
                                cfg["w_std"], cfg["dy_std"]))
            li += 1
    # layers that read one input in a decoder block: (q, k, v), o, (gate, up), down
    groups = shared_input_groups(cfg)
    for grp in groups:
        for j in grp[1:]:
            layers[j].X = layers[grp[0]].X
    # the layers the timed step runs: (q, k, v) and (gate, up) stacked along the output channels into one
    # layer each unless --separate
    block = layers
    if not args.separate:
        block = [layers[grp[0]] if len(grp) == 1 else stack_layers(torch, peqa, [layers[j] for j in grp], bits, group)
                 for grp in groups]
        groups_run = [[i] for i in range(len(block))]
    else:
        groups_run = groups
    ws_bytes = max(max(l.ws_fwd, l.ws_bwd) for l in layers + block)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    step_no = [0]

    # per-channel layers: the row sums of every distinct input are taken once per step (peqa_row_sums) and
    # handed to the forward of the layers that read it and to their backward
    share_sums = not group
    for grp in groups_run:
        rs = torch.empty((T, 2), dtype=torch.float32, device="cuda") if share_sums else None
        for j in grp:
            block[j].rs = rs

    def fwd_bwd(st):
        for grp in groups_run:                   # one forward call per shared input
            first = block[grp[0]]
            items = [(block[j].L, block[j].packed, block[j].s0, block[j].ds, block[j].z0, block[j].Y) for j in grp]
            if share_sums:
                peqa.row_sums(first.X, T, first.K, first.rs, st)
            peqa.linear_fwd_fused_rs(items, first.X, first.rs, T, ws, ws_bytes, st)
        for l in reversed(block):
            peqa.linear_bwd_rs(l.L, l.packed, l.s0, l.ds, l.z0, l.X, l.rs, l.dY, T, l.dX, l.dds, ws, ws_bytes, st)

    graph = [None]

    def step(use_graph=True):
        # forward and backward of the block's layers (launched one by one, or one HIP graph replayed with
        # --graph), then their scale updates (one launch), which carry the step number
        step_no[0] += 1
        if graph[0] is not None and use_graph:
            graph[0].replay()
        else:
            fwd_bwd(stream)
        peqa.scale_update_multi([(l.ds.numel(), l.ds, l.dds, l.m, l.v, l.s0) for l in block], lr=1e-5,
                                step=step_no[0], stream=stream)

    if args.pmc_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    step()
    torch.cuda.synchronize()
    if args.graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=torch.cuda.Stream()):
            fwd_bwd(torch.cuda.current_stream().cuda_stream)
        graph[0] = g
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    flops_step = synth.block_flops(args.config)
    tflops = flops_step / (dt / args.steps) / 1e12

    # per-kernel durations: the same steps again, every launch bracketed by HIP events
    launches_per_step = len(layers) * 12
    peqa.trace_begin(launches_per_step * args.steps + 16)
    for _ in range(args.steps):
        step(use_graph=False)
    torch.cuda.synchronize()
    trace = peqa.trace_end(16)
    # gemm_dw: the scale gradient of group-wise layers (contraction over tokens), same 2 T N K flops
    gemm_flops = {"gemm_y": 0.0, "gemm_dds": 0.0, "gemm_dx": 0.0, "gemm_dw": 0.0, "gemm_bwd": 0.0}
    for l in block:
        full = 2.0 * T * l.N * l.K * args.steps
        gemm_flops["gemm_y"] += full
        if group:
            for k in ("gemm_dds", "gemm_dx", "gemm_dw"):
                gemm_flops[k] += full
        else:
            # per-channel layers: the scale gradient and dX of one backward are one launch
            gemm_flops["gemm_bwd"] += 2.0 * full
    dom = max((k for k in gemm_flops if k in trace), key=lambda k: trace[k][1])
    # HBM bytes per launch of that kernel from the committed rocprofv3 --pmc summary (default workload only)
    traffic = None
    pmc_file = os.path.join(ROOT, "profiles", "gemm_llama7b_4bit_pc_hbm_traffic.txt")
    if args.config == 1 and os.path.exists(pmc_file):
        for line in open(pmc_file):
            if line.startswith("traffic_bytes_per_launch %s = " % dom):
                traffic = int(line.split("=")[1])
    dom_launches, dom_ms = trace[dom]
    achieved = gemm_flops[dom] / (dom_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                "avg_launch_us": round(dom_ms * 1e3 / dom_launches, 2), "launches": dom_launches}
    kernels = {k: {"launches": n, "avg_us": round(ms * 1e3 / n, 2),
                   "tflops": round(gemm_flops[k] / (ms * 1e-3) / 1e12, 1) if k in gemm_flops else None}
               for k, (n, ms) in trace.items()}

    small = small_batch(torch, peqa, layers, cfg, ws, ws_bytes, stream) if not args.no_small_batch else None

    kept = None
    if not args.no_kept_product and not group:
        kept = kept_product(torch, peqa, layers, cfg, stream, min(args.steps, 10))

    out = {
        "metric": "PEQA quantized-linear fwd+bwd TFLOP/s, LLaMA-7B shapes T=2048" if args.config == 1
                  else "PEQA quantized-linear fwd+bwd TFLOP/s, %s" % cfg["name"],
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: 7 linears of one decoder block, %d-bit %s, T=%d, fwd + dX + d_ds + AdamW"
                               % (cfg["name"], bits, "per-channel" if not group else "g%d" % group, T),
                   "layers_run": "7 separate layers" if args.separate else
                                 "q,k,v and gate,up each stacked along the output channels (same weights, same flops): "
                                 "%d layers of N = %s" % (len(block), [l.N for l in block])},
        "frac_of_bf16_mfma_peak": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "tokens_per_s": round(T / (dt / args.steps), 1),
        "flops_per_step": flops_step,
        "quantize_ms_total": round(sum(l.quantize_ms for l in layers), 3),
        "launch": ("hip graph of: " if args.graph else "direct launches: ") +
                  "%d forward calls (layers sharing an input in one peqa_linear_fwd_fused_rs, its row sums taken "
                  "once per step by peqa_row_sums and reused by the backward), %d backward calls; "
                  "then the %d scale updates in one direct launch" % (len(groups_run), len(block), len(block)),
        "kernels": kernels,
        "roofline": roofline,
        "device": device_info(torch, peqa),
    }
    if small is not None:
        out["small_batch"] = small
    if kept is not None:
        out["kept_product_variant"] = kept
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_seconds)
        out["cpu_baseline"].pop("tokens_per_s_block_extrapolated")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
