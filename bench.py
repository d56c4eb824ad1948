#!/usr/bin/env python3
"""Benchmark of the PEQA quantized-linear hot path on one MI355X.

One "step" = one training pass over the seven linears of a LLaMA-7B decoder block
(4-bit per-channel codes, T = 2048 tokens): forward Y, backward dX, scale gradient d_ds
and the AdamW scale update, all through the C-ABI library: peqa_block_fwd, peqa_block_bwd,
peqa_scale_update_multi.  Quantization is the method's one-time decomposition step and is done
(and timed) once before the loop.  The layers of the block that read one input (q, k, v; gate, up)
are passed stacked along their output channels as one item each, which is a property of the packed
layout, not another kernel (--separate passes the seven one by one).

Prints ONE JSON line: fwd+bwd TFLOP/s counting 6*T*N*K flops per layer (three dense
contractions: forward, dX, and the product recomputed for the scale gradient), with
  roofline          - the dominant kernel against the bf16 MFMA peak, timed with HIP events
  cpu_baseline      - the CPU oracle timed on a bounded sample of the same workload
  small_batch       - the deployment forward (T = 1 and 16) of the same block against the HBM peak
  small_batch_cfg4  - the same for the LLaMA-13B shapes, 3-bit, group size 128
                      (both rotate through more than 256 MB of distinct weights: every read is from HBM)
  other_configs     - the training step of the other workloads (3-bit T = 4096; LLaMA-65B shapes; 13B 3-bit g128)
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
CONTRACTIONS = ("gemm_multi_y", "gemm_multi_dds", "gemm_multi_dx", "gemm_y", "gemm_dds", "gemm_dx", "gemm_dw", "gemm_bwd")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="workload index (see synth.CONFIGS)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-small-batch", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--only-small-batch", action="store_true",
                    help="run only the T = 1 / 16 block forward of --config through peqa_block_fwd and print its "
                         "figures (for profiling that kernel alone)")
    ap.add_argument("--no-kept-product", action="store_true",
                    help="skip the secondary timing of the variant that keeps the forward's product")
    ap.add_argument("--separate", action="store_true",
                    help="pass q, k, v and gate, up as separate items (7 per block) instead of stacked along "
                         "their output channels (4 per block)")
    ap.add_argument("--graph", action="store_true",
                    help="replay a HIP graph of the forward and backward calls instead of launching them one by one")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three 256 MiB device copies, a kernel of known traffic against which "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


def block_shapes(cfg, separate):
    """(N, K, input index) of the items of one decoder block: q, k, v read input 0, o input 1, gate, up input 2,
    down input 3; layers that share an input are stacked along the output channels unless `separate`."""
    (n_a, k_a, _), (n_m, k_m, _), (n_d, k_d, _) = cfg["layers"]
    if separate:
        return [(n_a, k_a, 0)] * 3 + [(n_a, k_a, 1)] + [(n_m, k_m, 2)] * 2 + [(n_d, k_d, 3)]
    return [(3 * n_a, k_a, 0), (n_a, k_a, 1), (2 * n_m, k_m, 2), (n_d, k_d, 3)]


class Block:
    """The linears of one decoder block on the device: quantized by peqa_quantize from seeded random weights (one
    call per member layer, into its slice of the stacked arrays), with activations and gradients of the
    workload's distributions."""

    def __init__(self, torch, peqa, synth, config, separate, T=None, training=True):
        cfg = synth.CONFIGS[config]
        self.cfg, self.config = cfg, config
        self.bits, self.group = cfg["bits"], cfg["group"]
        self.T = T = T or cfg["T"]
        g = torch.Generator(device="cuda")
        g.manual_seed(synth.seed_for(config, 0, 0))
        shapes = block_shapes(cfg, separate)
        member_n = {0: cfg["layers"][0][0], 1: cfg["layers"][0][0], 2: cfg["layers"][1][0], 3: cfg["layers"][2][0]}
        self.layers, inputs = [], {}
        self.quantize_ms = 0.0
        for (N, K, xi) in shapes:
            L = peqa.layout(N, K, self.bits, self.group)
            G = L.groups
            d = dict(L=L, N=N, K=K, packed=torch.empty(peqa.packed_words(L), dtype=torch.int32, device="cuda"),
                     s0=torch.empty((N, G), dtype=torch.float32, device="cuda"),
                     z0=torch.empty((N, G), dtype=torch.uint8, device="cuda"))
            n_m = member_n[xi]
            Lm = peqa.layout(n_m, K, self.bits, self.group)
            wm = peqa.packed_words(Lm)
            for i in range(N // n_m):                         # member by member into slices of the stacked arrays
                W0 = torch.randn((n_m, K), generator=g, device="cuda", dtype=torch.float32) * cfg["w_std"]
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                peqa.quantize(Lm, W0, d["packed"][i * wm:(i + 1) * wm], d["s0"][i * n_m:(i + 1) * n_m],
                              d["z0"][i * n_m:(i + 1) * n_m])
                torch.cuda.synchronize()
                self.quantize_ms += (time.perf_counter() - t0) * 1e3
                del W0
            d["ds"] = torch.zeros((N, G), dtype=torch.float32, device="cuda")
            if xi not in inputs:
                X = torch.randn((T, K), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                inputs[xi] = (X, torch.empty((T, 2), dtype=torch.float32, device="cuda"))
            d["X"] = inputs[xi][0]
            d["Y"] = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
            if training:
                d["row_sums"] = inputs[xi][1] if not self.group else None
                d["dY"] = (torch.randn((T, N), generator=g, device="cuda", dtype=torch.float32) * cfg["dy_std"]).to(torch.bfloat16)
                d["dX"] = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
                d["d_ds"] = torch.empty((N, G), dtype=torch.float32, device="cuda")
                d["m"] = torch.zeros((N, G), dtype=torch.float32, device="cuda")
                d["v"] = torch.zeros((N, G), dtype=torch.float32, device="cuda")
            self.layers.append(d)
        self.items = peqa.block_items(self.layers)
        ops = (peqa.PEQA_OP_FWD, peqa.PEQA_OP_BWD) if training else (peqa.PEQA_OP_FWD,)
        self.ws_bytes = max(peqa.block_workspace_bytes(self.items, T, op) for op in ops)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.flops = sum(6.0 * T * d["N"] * d["K"] for d in self.layers)


def time_steps(torch, peqa, blk, steps, warmup, use_graph=False):
    """Times `steps` training steps of the block.  Returns seconds per step; the per-kernel trace of a few extra
    steps with every launch bracketed by HIP events, and their number; the trace of the dominant contraction
    kernel's launches inside the timed region, and that kernel's name."""
    stream = torch.cuda.current_stream().cuda_stream
    upd = [(d["ds"].numel(), d["ds"], d["d_ds"], d["m"], d["v"], d["s0"]) for d in blk.layers]
    T = blk.T
    step_no = [0]
    graph = [None]

    def fwd_bwd(st):
        peqa.block_fwd(blk.items, T, blk.ws, blk.ws_bytes, st)
        peqa.block_bwd(blk.items, T, blk.ws, blk.ws_bytes, st)

    def step(replay=True):
        step_no[0] += 1
        if graph[0] is not None and replay:
            graph[0].replay()
        else:
            fwd_bwd(stream)
        # the scale updates carry the step number: one direct launch for all items
        peqa.scale_update_multi(upd, lr=1e-5, step=step_no[0], stream=stream)

    step()
    torch.cuda.synchronize()
    if use_graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=torch.cuda.Stream()):
            fwd_bwd(torch.cuda.current_stream().cuda_stream)
        graph[0] = g
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # every launch bracketed by HIP events: the per-kernel table, and which contraction kernel dominates.  (Events
    # between all launches leave gaps in which the chip cools: kernels measure a few per cent shorter here than in
    # the timed region, where launches are back to back.)
    n_all = max(2, min(steps, 5))
    peqa.trace_begin(64 * n_all + 16)
    for _ in range(n_all):
        step(replay=False)
    torch.cuda.synchronize()
    trace_all = peqa.trace_end()
    dom = dominant_kernel(trace_all)
    # the timed region; only the dominant kernel's launches are bracketed by events (one pair per launch, every
    # other launch back to back as without tracing), which is where the roofline figure comes from
    if graph[0] is None:
        peqa.trace_begin(8 * steps + 16, prefix=dom)
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    trace_dom = peqa.trace_end() if graph[0] is None else {}
    return dt, trace_all, n_all, trace_dom, dom


def dominant_kernel(trace):
    """Name prefix of the contraction kernel with the most time; the three kinds of multi-contraction launch are one
    kernel (gemm_multi_kernel) and count together."""
    groups = {}
    for k, (n, ms) in trace.items():
        if k in CONTRACTIONS:
            key = "gemm_multi" if k.startswith("gemm_multi") else k
            groups[key] = groups.get(key, 0.0) + ms
    return max(groups, key=groups.get)


def kernel_table(blk, trace, steps):
    """Per-kernel averages; contraction kernels with the flops of their launches (2 T N K per contraction)."""
    contraction_flops = blk.flops / 3.0                        # every item once, per kind of contraction
    out = {}
    for k, (n, ms) in trace.items():
        e = {"launches_per_step": round(n / steps, 2), "avg_us": round(ms * 1e3 / n, 2)}
        if k in CONTRACTIONS:
            # the launches of one kind in one step together do one contraction per item (gemm_bwd: two)
            per_step_flops = contraction_flops * (2.0 if k == "gemm_bwd" else 1.0)
            e["tflops"] = round(per_step_flops * steps / (ms * 1e-3) / 1e12, 1)
        out[k] = e
    return out


def roofline_of(blk, trace_dom, dom, timed_steps):
    """The dominant contraction kernel: algorithmic flops of its launches / their HIP-event duration, both over
    the timed region (the two warm-up steps before it included)."""
    n = sum(v[0] for k, v in trace_dom.items() if k.startswith(dom))
    ms = sum(v[1] for k, v in trace_dom.items() if k.startswith(dom))
    kinds = [k for k in trace_dom if k.startswith(dom)]
    steps = timed_steps + 2
    # per step the launches of one kind do one contraction per item (gemm_bwd: two)
    flops = blk.flops / 3.0 * (2.0 if dom == "gemm_bwd" else 1.0) * len(kinds) * steps
    achieved = flops / (ms * 1e-3) / 1e12
    return {"bound": "mfma", "kernel": dom + ("_kernel: the forward, scale-gradient and dX launches of a step" if dom == "gemm_multi" else ""),
            "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
            "traffic_note": "not measured in this run; rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries of this "
                            "command are under profiles/ (see profiles/README.md)",
            "flops_per_launch": flops / n, "avg_launch_us": round(ms * 1e3 / n, 2),
            "launches_per_step": round(n / steps, 2),
            "timing": "HIP events on the launching stream around this kernel's launches only, inside the timed region"}


def small_batch(torch, peqa, synth, config, reps=20, per_layer=True):
    """Forward of one block at T = 1 and T = 16 through the matrix-vector path: all seven layers in one
    peqa_block_fwd call (one launch plus the sum of the sliced layers), and, for comparison, seven
    peqa_linear_fwd calls.  Algorithmic bytes per layer: packed codes + s0, ds (fp32) and z0 (uint8) per scale +
    X and Y (bf16).  Wall time per block on the stream, over > 256 MB of rotating weight sets."""
    cfg = synth.CONFIGS[config]
    bits = cfg["bits"]
    out = {"workload": "%s: forward of the 7 linears of one decoder block, %d-bit %s" % (
        cfg["name"], bits, "per-channel" if not cfg["group"] else "g%d" % cfg["group"]), "hbm_peak_GBs": HBM_PEAK_GBS}
    stream = torch.cuda.current_stream().cuda_stream
    for T in (1, 16):
        blk = Block(torch, peqa, synth, config, separate=True, T=T, training=False)
        block_packed = sum(d["packed"].numel() * 4 for d in blk.layers)
        nsets = max(2, -(-(300 << 20) // block_packed))        # > 256 MB of distinct weight bytes
        g = torch.Generator(device="cuda")
        g.manual_seed(12345)
        sets = [blk.items]
        packed_sets = [[d["packed"] for d in blk.layers]]
        for _ in range(nsets - 1):
            pk = [torch.randint(-2 ** 31, 2 ** 31 - 1, (d["packed"].numel(),), generator=g, device="cuda",
                                dtype=torch.int32) for d in blk.layers]
            packed_sets.append(pk)
            sets.append(peqa.block_items([dict(d, packed=p) for d, p in zip(blk.layers, pk)]))
        inputs = {id(d["X"]): d["K"] for d in blk.layers}
        nbytes = sum(d["N"] * d["K"] * bits / 8 + d["N"] * d["L"].groups * 9 + 2 * T * d["N"] for d in blk.layers) + \
            sum(2 * T * k for k in inputs.values())

        def run_block():
            for it in sets:
                peqa.block_fwd(it, T, blk.ws, blk.ws_bytes, stream)

        nb1 = max(peqa.workspace_bytes(d["L"], T, peqa.PEQA_OP_FWD) for d in blk.layers)
        ws1 = torch.empty(nb1, dtype=torch.uint8, device="cuda")

        def run_layers():
            for pk in packed_sets:
                for d, p in zip(blk.layers, pk):
                    peqa.linear_fwd(d["L"], p, d["s0"], d["ds"], d["z0"], d["X"], T, d["Y"], ws1, nb1, stream)

        res = {}
        for name, fn in (("block_call", run_block), ("per_layer_calls", run_layers))[:2 if per_layer else 1]:
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) / (reps * nsets) * 1e6
            res[name] = {"block_us_wall": round(us, 2), "GBs": round(nbytes / us / 1e3, 1),
                         "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)}
        peqa.trace_begin(4 * reps * nsets + 16)
        for _ in range(reps):
            run_block()
        torch.cuda.synchronize()
        tr = peqa.trace_end()
        res["block_call"]["kernels_avg_us"] = {k: round(ms * 1e3 / n, 2) for k, (n, ms) in tr.items()}
        res["bytes_per_block"] = int(nbytes)
        res["weight_sets"] = nsets
        out["T%d" % T] = res
        del blk, sets, packed_sets
    return out


def kept_product(torch, peqa, blk, steps):
    """The optional variant that keeps P = X (Q - z0)^T from the forward (per-channel layers): the same
    block step with peqa_linear_fwd_keep / peqa_linear_bwd_kept, which does 4 T N K flops per layer."""
    T = blk.T
    stream = torch.cuda.current_stream().cuda_stream
    layers = blk.layers
    nb = max(max(peqa.workspace_bytes(d["L"], T, peqa.PEQA_OP_FWD_KEEP), peqa.workspace_bytes(d["L"], T, peqa.PEQA_OP_BWD_KEPT))
             for d in layers)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    Ps = [torch.empty((T, d["N"]), dtype=torch.float32, device="cuda") for d in layers]
    upd = [(d["ds"].numel(), d["ds"], d["d_ds"], d["m"], d["v"], d["s0"]) for d in layers]

    def step(i):
        for d, P in zip(layers, Ps):
            peqa.linear_fwd_keep(d["L"], d["packed"], d["s0"], d["ds"], d["z0"], d["X"], T, d["Y"], P, ws, nb, stream)
        for d, P in zip(reversed(layers), reversed(Ps)):
            peqa.linear_bwd_kept(d["L"], d["packed"], d["s0"], d["ds"], d["z0"], P, d["dY"], T, d["dX"], d["d_ds"], ws, nb, stream)
        peqa.scale_update_multi(upd, lr=1e-5, step=i, stream=stream)

    for i in range(3):
        step(1000 + i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(2000 + i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    flops = sum(4.0 * T * d["N"] * d["K"] for d in layers)
    return {"what": "same block step with the forward keeping fp32 P (4 T N bytes per layer) and the scale "
                    "gradient taken from it: 4 T N K flops per layer instead of 6 T N K; per-layer calls",
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
            "sample": "layer %dx%d, %d-bit, %d token rows: fwd + dX + scale gradient, %.1f s" % (N, K, cfg["bits"], T, dt)}


def workload_name(cfg, T):
    return "%s: 7 linears of one decoder block, %d-bit %s, T=%d, fwd + dX + d_ds + AdamW" % (
        cfg["name"], cfg["bits"], "per-channel" if not cfg["group"] else "g%d" % cfg["group"], T)


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
    if args.only_small_batch:
        print(json.dumps({"small_batch": small_batch(torch, peqa, synth, args.config, per_layer=False)}))
        return

    if args.pmc_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    blk = Block(torch, peqa, synth, args.config, args.separate)
    dt, trace, n_all, trace_dom, dom = time_steps(torch, peqa, blk, args.steps, args.warmup, args.graph)
    tflops = blk.flops / dt / 1e12
    assert abs(blk.flops - synth.block_flops(args.config)) < 1e-6 * blk.flops

    out = {
        "metric": "PEQA quantized-linear fwd+bwd TFLOP/s, LLaMA-7B shapes T=2048" if args.config == 1
                  else "PEQA quantized-linear fwd+bwd TFLOP/s, %s" % cfg["name"],
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload_name(cfg, blk.T),
                   "layers_run": "7 separate items" if args.separate else
                                 "q,k,v and gate,up each stacked along the output channels (same weights, same flops): "
                                 "%d items of N = %s" % (len(blk.layers), [d["N"] for d in blk.layers])},
        "frac_of_bf16_mfma_peak": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "tokens_per_s": round(blk.T / dt, 1),
        "flops_per_step": blk.flops,
        "quantize_ms_total": round(blk.quantize_ms, 3),
        "launch": ("hip graph of: " if args.graph else "direct calls: ") +
                  "peqa_block_fwd, peqa_block_bwd (row sums of the inputs kept from the forward), then "
                  "peqa_scale_update_multi (one direct launch)",
        "kernels": kernel_table(blk, trace, n_all),
        "kernels_note": "from %d extra steps with every launch bracketed by HIP events (not part of the timed region)" % n_all,
        "roofline": roofline_of(blk, trace_dom, dom, args.steps) if trace_dom else None,
        "device": device_info(torch, peqa),
    }
    if not args.no_kept_product and not cfg["group"]:
        out["kept_product_variant"] = kept_product(torch, peqa, blk, min(args.steps, 10))
    del blk
    torch.cuda.empty_cache()

    if not args.no_small_batch:
        out["small_batch"] = small_batch(torch, peqa, synth, args.config)
        if args.config != 4:
            out["small_batch_cfg4"] = small_batch(torch, peqa, synth, 4)
        torch.cuda.empty_cache()

    if not args.no_other_configs and args.config == 1:
        others = {}
        for c in (2, 3, 4):
            b = Block(torch, peqa, synth, c, args.separate)
            steps = max(3, min(args.steps, 10))
            d, tr, n_all_c, tr_dom, dom_c = time_steps(torch, peqa, b, steps, 2)
            r = roofline_of(b, tr_dom, dom_c, steps)
            others["cfg%d" % c] = {"workload": workload_name(synth.CONFIGS[c], b.T), "ms_per_step": round(d * 1e3, 4),
                                   "tflops": round(b.flops / d / 1e12, 1),
                                   "frac_of_bf16_mfma_peak": round(b.flops / d / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                                   "tokens_per_s": round(b.T / d, 1), "steps": steps,
                                   "dominant_kernel": {k: r[k] for k in ("kernel", "achieved", "frac", "avg_launch_us")},
                                   "kernels": kernel_table(b, tr, n_all_c)}
            del b
            torch.cuda.empty_cache()
        out["other_configs"] = others

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
