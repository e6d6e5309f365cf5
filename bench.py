#!/usr/bin/env python3
"""Benchmark of the double-pruned 2:4 sparse linear layer on one MI355X.

One step = one pass of the whole hot path over the linear layers of one OPT-66B-shaped
transformer block (q, k, v, o: 9216 x 9216; fc1: 36864 x 9216; fc2: 9216 x 36864; 16384 tokens,
rank-128 adapters in the forward): for every layer slope_prune_rows, slope_double_prune (weights
are re-pruned from dense each step), slope_spmm_fwd with the adapter, slope_spmm_bwd_x and the
masked weight gradient (token-contiguous copies + slope_wgrad_masked_t; q, k and v share the copy of
their common input).  All inputs are synthetic (seeded Gaussians, generated on the device) and
resident in HBM before the clock starts.

Prints ONE JSON line.  value = effective TFLOP/s = 3 * 2 * b * d_in * d_out summed over the
layers (the dense-equivalent flops of fwd + dX + dW; adapter flops are not credited) divided by
the step time.  Details ride in the same line: per-call times, the dense bf16 GEMM comparison, the
ceilings measured by micro-benchmarks in the same run, the other layer sets of the benchmark
configurations (`other_configs`), the CPU-oracle baseline.

Other modes: --workload opt13b | opt2.7b | opt125m_fc1 (the same step on another layer set),
--workload opt66b_infer (forward at 1, 16, 128 tokens), --workload sweep (shape study: aspect
ratios at 2048 tokens and a token sweep at 9216 x 9216), --ceilings (the micro-benchmarks alone).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_DENSE_BF16 = 2500.0     # TFLOP/s, MI355X dense bf16 MFMA
PEAK_SPARSE_BF16 = 5000.0    # TFLOP/s dense-equivalent, structured-sparse bf16 MFMA
PEAK_HBM = 8000.0            # GB/s
NOMINAL_MHZ = 2400.0         # shader clock the published MFMA peaks assume

CALLS = ["prune_rows", "double_prune", "spmm_fwd", "spmm_bwd_x", "wgrad_masked"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="opt66b",
                    help="opt66b (headline) | opt13b | opt2.7b | opt125m_fc1 | opt66b_infer (forward at 1/16/128 tokens) "
                         "| sweep (shape study)")
    ap.add_argument("--ceilings", action="store_true", help="run only the micro-benchmarks of the chip's ceilings")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sclk", action="store_true", help="skip the shader-clock sampling loops (for profiling runs)")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other layer sets and the side measurements")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step (and the dense comparison) replayed from a captured HIP graph")
    return ap.parse_args()


def timed_ms(torch, fn, iters, warmup=2):
    """Average milliseconds of fn() over `iters` calls, by HIP events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def measure_ceilings(torch, sl, dev):
    """Register-resident MFMA loops and plain streams, in this run and under this run's power management.
    The MFMA loops run twice: on Gaussian operands (what a product sees) and on zeros (the pipe switches
    little, the clock stays higher), which is the spread the published peak hides."""
    nbytes = 1 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    head = sl.lib().slope_ceiling_min_bytes()
    buf[:head].view(torch.bfloat16).copy_(torch.randn(head // 2, generator=gen, device=dev, dtype=torch.float32))
    out = {}

    def rate(kind, iters, reps):
        work = [0.0]

        def fn():
            work[0] = sl.slope_ceiling(kind, buf, iters)
        ms = timed_ms(torch, fn, reps, warmup=1)
        return work[0] / (ms * 1e-3)

    out["sparse_bf16_tflops"] = rate(sl.SLOPE_CEILING_SPARSE_MFMA, 8000, 6) / 1e12
    out["dense_bf16_tflops"] = rate(sl.SLOPE_CEILING_DENSE_MFMA, 8000, 6) / 1e12
    out["sparse_bf16_tflops_32x32"] = rate(sl.SLOPE_CEILING_SPARSE_MFMA_32, 8000, 6) / 1e12
    out["dense_bf16_tflops_32x32"] = rate(sl.SLOPE_CEILING_DENSE_MFMA_32, 8000, 6) / 1e12
    buf[:head].zero_()
    out["sparse_bf16_tflops_zero_operands"] = rate(sl.SLOPE_CEILING_SPARSE_MFMA, 8000, 6) / 1e12
    out["dense_bf16_tflops_zero_operands"] = rate(sl.SLOPE_CEILING_DENSE_MFMA, 8000, 6) / 1e12
    out["hbm_read_gbs"] = rate(sl.SLOPE_CEILING_READ, 1, 10) / 1e9
    out["hbm_copy_gbs"] = rate(sl.SLOPE_CEILING_COPY, 1, 10) / 1e9
    out["how"] = ("slope_ceiling: register-resident loops of v_smfmac_f32_16x16x64_bf16 / v_mfma_f32_16x16x32_bf16 (and of "
                  "their 32 x 32 forms) on Gaussian operands, the same on zeros, a read-only stream and a copy over 1 GiB")
    del buf
    return out


def build_layers(torch, sl, inputs, dev, workload):
    spec = inputs.LAYER_SETS[workload]
    b, rank = spec["b"], spec["rank"]
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE + 3)

    def gauss(shape, std):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)

    # activations and output gradients are shared by layers of equal width (they are inputs only)
    acts, grads, layers = {}, {}, []
    for name, d_out, d_in in spec["layers"]:
        if d_in not in acts:
            acts[d_in] = gauss((b, d_in), inputs.STD["X"])
        if d_out not in grads:
            grads[d_out] = gauss((b, d_out), inputs.STD["dY"])
        lay = {"name": name, "d_out": d_out, "d_in": d_in, "X": acts[d_in], "dY": grads[d_out],
               "W": gauss((d_out, d_in), inputs.STD["W"])}
        lay["L"] = gauss((d_in, rank), inputs.STD["L"]) if rank else None
        lay["R"] = gauss((rank, d_out), inputs.STD["R"]) if rank else None
        nws = sl.slope_spmm_fwd_workspace_bytes(b, d_in, d_out, rank)
        lay["ws"] = torch.empty(nws, dtype=torch.uint8, device=dev) if nws else None
        lay["vals"] = torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=dev)
        lay["meta"] = torch.empty((d_out, d_in // 8), dtype=torch.uint8, device=dev)
        lay["vals_t"] = torch.empty((d_in, d_out // 2), dtype=torch.bfloat16, device=dev)
        lay["meta_t"] = torch.empty((d_in, d_out // 8), dtype=torch.uint8, device=dev)
        lay["Y"] = torch.empty((b, d_out), dtype=torch.bfloat16, device=dev)
        lay["dX"] = torch.empty((b, d_in), dtype=torch.bfloat16, device=dev)
        lay["G"] = torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=dev)
        # q, k and v of a transformer block read the same input: one token-contiguous copy serves all three
        lay["x_group"] = "qkv" if name in ("q", "k", "v") else name
        layers.append(lay)
    return spec, layers


def train(args, torch, sl, inputs, dev, workload, steps, warmup, full):
    """The timed step on one layer set.  full: also the side measurements of the headline run."""
    spec, layers = build_layers(torch, sl, inputs, dev, workload)
    b, rank = spec["b"], spec["rank"]
    # token-contiguous copies for the weight gradient: one buffer per input group, one for the output gradients
    xt = {}
    for lay in layers:
        if lay["x_group"] not in xt:
            xt[lay["x_group"]] = torch.empty(sl.slope_token_copy_bytes(b, lay["d_in"]), dtype=torch.uint8, device=dev)
    dyt = torch.empty(max(sl.slope_token_copy_bytes(b, l["d_out"]) for l in layers), dtype=torch.uint8, device=dev)
    use_t = all(l["d_in"] % 32 == 0 for l in layers)
    wg_ws = torch.empty(max(sl.slope_wgrad_workspace_bytes(b, l["d_in"], l["d_out"]) for l in layers),
                        dtype=torch.uint8, device=dev)
    # scratch of the product from prepared copies (partial sums of the tiles a last partial round would hold)
    t_need = max(sl.slope_workspace_bytes(sl.SLOPE_CALL_WGRAD_MASKED_T, b, l["d_in"], l["d_out"]) for l in layers)
    wg_t_ws = torch.empty(t_need, dtype=torch.uint8, device=dev) if t_need else None

    shared = {g for g in xt if sum(1 for l in layers if l["x_group"] == g) > 1}

    def wgrad(lay, fresh):
        if not use_t or lay["x_group"] not in shared:         # nothing to share: both copies and the product in one call
            sl.slope_wgrad_masked(lay["dY"], lay["X"], lay["meta"], out=lay["G"], workspace=wg_ws)
            return
        if fresh:
            sl.slope_transpose_tokens(lay["X"], out=xt[lay["x_group"]])
        sl.slope_transpose_tokens(lay["dY"], out=dyt)
        sl.slope_wgrad_masked_t(dyt, xt[lay["x_group"]], b, lay["meta"], out=lay["G"], workspace=wg_t_ws)

    def step(events=None):
        copied = set()
        for li, lay in enumerate(layers):
            ev = events[li] if events is not None else None
            if ev: ev[0].record()
            sl.slope_prune_rows(lay["W"], out=(lay["vals"], lay["meta"], None))
            if ev: ev[1].record()
            sl.slope_double_prune(lay["vals"], lay["meta"], out=(lay["vals_t"], lay["meta_t"], None))
            if ev: ev[2].record()
            sl.slope_spmm_fwd(lay["X"], lay["vals"], lay["meta"], lay["L"], lay["R"], out=lay["Y"],
                              workspace=lay["ws"])
            if ev: ev[3].record()
            sl.slope_spmm_bwd_x(lay["dY"], lay["vals_t"], lay["meta_t"], out=lay["dX"])
            if ev: ev[4].record()
            wgrad(lay, lay["x_group"] not in copied)
            copied.add(lay["x_group"])
            if ev: ev[5].record()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # HIP events on the stream the kernels run on (torch's current stream), one set per step
    all_events = [[[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in layers] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        step(all_events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    def graph_ms(fn):
        """fn captured into a HIP graph on a side stream and replayed `steps` times (ms per replay)."""
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                fn()
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - g0) * 1e3 / steps

    # small layer sets are bound by launch overhead on the host: their step is also timed as a graph replay
    want_graph = (args.graph and full) or ms_per_step < 1.0
    graph = {"ms_per_step": graph_ms(step)} if want_graph else None

    flops_layer = [2.0 * b * l["d_in"] * l["d_out"] for l in layers]
    total_flops = 3.0 * sum(flops_layer)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # per-call average durations (ms) from the events of the timed region
    per_call = {c: 0.0 for c in CALLS}
    for li, lay in enumerate(layers):
        for ci, c in enumerate(CALLS):
            ms = sum(all_events[s][li][ci].elapsed_time(all_events[s][li][ci + 1]) for s in range(steps))
            per_call[c] += ms / steps
    sum_f = sum(flops_layer)
    elems = sum(l["d_in"] * l["d_out"] for l in layers)
    n_launch = len(layers)
    kernels = {
        # dense contraction: 2 b d_in d_out flops per launch against the dense bf16 MFMA peak
        "wgrad_masked": {"bound": "mfma", "achieved": sum_f / (per_call["wgrad_masked"] * 1e-3) / 1e12,
                         "peak": PEAK_DENSE_BF16, "unit": "TFLOP/s",
                         "note": "token-contiguous copies included (one per distinct input, one per output gradient)"},
        # sparse contraction: credited dense-equivalent 2 b d_in d_out against the sparse bf16 peak
        "spmm_bwd_x": {"bound": "mfma", "achieved": sum_f / (per_call["spmm_bwd_x"] * 1e-3) / 1e12,
                       "peak": PEAK_SPARSE_BF16, "unit": "TFLOP/s"},
        "spmm_fwd": {"bound": "mfma", "achieved": sum_f / (per_call["spmm_fwd"] * 1e-3) / 1e12,
                     "peak": PEAK_SPARSE_BF16, "unit": "TFLOP/s", "note": "includes the adapter kernels"},
        # streams: 3.125 B (read 2, write 1 + 1/8) and 2.25 B per weight element
        "prune_rows": {"bound": "hbm", "achieved": 3.125 * elems / (per_call["prune_rows"] * 1e-3) / 1e9,
                       "peak": PEAK_HBM, "unit": "GB/s"},
        "double_prune": {"bound": "hbm", "achieved": 2.25 * elems / (per_call["double_prune"] * 1e-3) / 1e9,
                         "peak": PEAK_HBM, "unit": "GB/s"},
    }
    for name, k in kernels.items():
        k["frac"] = k["achieved"] / k["peak"]
        k["launches_per_step"] = n_launch
        k["avg_ms"] = per_call[name] / n_launch

    # dense bf16 GEMM at the same shapes (the library GEMM torch.matmul dispatches to): Y = X W^T,
    # dX = dY W, dW = dY^T X
    dense = None
    if not args.no_dense:
        def dense_step():
            for lay in layers:
                torch.matmul(lay["X"], lay["W"].t(), out=lay["Y"])
                torch.matmul(lay["dY"], lay["W"], out=lay["dX"])
                torch.matmul(lay["dY"].t(), lay["X"], out=lay["Wg"])
        for lay in layers:
            lay["Wg"] = torch.empty((lay["d_out"], lay["d_in"]), dtype=torch.bfloat16, device=dev)
        for _ in range(max(1, warmup)):
            dense_step()
        torch.cuda.synchronize()
        d0 = time.perf_counter()
        nd = max(3, steps // 2)
        for _ in range(nd):
            dense_step()
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - d0) * 1e3 / nd
        if graph is not None:
            graph["dense_ms_per_step"] = graph_ms(dense_step)
            graph["speedup_vs_dense"] = graph["dense_ms_per_step"] / graph["ms_per_step"]
        gemm_ms = per_call["spmm_fwd"] + per_call["spmm_bwd_x"] + per_call["wgrad_masked"]
        dense = {"ms_per_step": dense_ms, "tflops": total_flops / (dense_ms * 1e-3) / 1e12,
                 "speedup_products_only": dense_ms / gemm_ms, "speedup_with_reprune": dense_ms / ms_per_step,
                 "library": "torch.matmul (hipBLASLt/rocBLAS)"}
        for lay in layers:
            del lay["Wg"]

    res = {"workload": "%s linear layers of one block: %s; tokens %d; adapter rank %d; re-pruned from dense every step"
                       % (workload, ", ".join("%s %dx%d" % (n, o, i) for n, o, i in spec["layers"]), b, rank),
           "value": value, "ms_per_step": ms_per_step, "per_call_ms": per_call, "kernels": kernels, "dense_gemm": dense,
           "hip_graph": graph, "flops_per_launch": sum_f / n_launch, "layers": layers, "b": b, "rank": rank,
           "wg_ws": wg_ws, "elems": elems}
    if not full:
        return res

    # Optimizer-side packed streams (Alg. 1 lines 15-18), timed apart from the step: g = G / scale + decay * W^R
    # in W^R's packed layout, then both sparse copies take the new values (static masks).
    def optimizer_step():
        for lay in layers:
            sl.slope_sparse_add(lay["G"], lay["vals"], 1.0 / 1024.0, 0.01, out=lay["G"])
            sl.slope_update_sparse(lay["G"], lay["meta"], lay["vals"], lay["meta_t"], lay["vals_t"])
    opt_ms = timed_ms(torch, optimizer_step, 3, warmup=1)
    # bytes per weight element (a packed value array holds 1 B per weight): sparse_add reads two arrays and
    # writes one = 3; update copies one array (1 + 1), reads packed W^R (1.125) and the transposed metadata
    # (0.125) and writes the transposed values (1) = 4.25
    res["optimizer_side"] = {"ms_per_step": opt_ms, "achieved": 7.25 * elems / (opt_ms * 1e-3) / 1e9, "unit": "GB/s",
                             "peak": PEAK_HBM, "calls": "slope_sparse_add + slope_update_sparse per layer"}

    # Backward pass with adapters (chain rule of Eq. 11), timed apart from the step: the same step with
    # slope_spmm_bwd_x_adapter and slope_wgrad_adapter in place of the plain backward calls.
    res["adapter_backward"] = None
    if rank > 0:
        big_ws = torch.empty(max(sl.slope_wgrad_adapter_workspace_bytes(b, l["d_in"], l["d_out"], rank)
                                 for l in layers), dtype=torch.uint8, device=dev)
        for lay in layers:
            lay["dL"] = torch.empty((lay["d_in"], rank), dtype=torch.bfloat16, device=dev)
            lay["dR"] = torch.empty((rank, lay["d_out"]), dtype=torch.bfloat16, device=dev)

        def adapter_step():
            for lay in layers:
                sl.slope_spmm_bwd_x_adapter(lay["dY"], lay["vals_t"], lay["meta_t"], lay["L"], lay["R"],
                                            out=lay["dX"], workspace=lay["ws"])
                sl.slope_wgrad_adapter(lay["dY"], lay["X"], lay["meta"], lay["L"], lay["R"],
                                       out=(lay["G"], lay["dL"], lay["dR"]), workspace=big_ws)
        ab_ms = timed_ms(torch, adapter_step, 3, warmup=1)
        res["adapter_backward"] = {
            "ms_per_step": ab_ms, "plain_backward_ms": per_call["spmm_bwd_x"] + per_call["wgrad_masked"],
            "calls": "slope_spmm_bwd_x_adapter + slope_wgrad_adapter per layer",
            "note": "the headline step times the forward with adapters and the backward without them (the five "
                    "calls); this is the backward pass that also differentiates through the adapters"}
        del big_ws
    return res


def sclk_under_load(args, torch, sl, res):
    """Shader clock (outside the timed region): the published MFMA peaks assume 2.4 GHz, but the power
    management lowers the clock while MFMA-bound kernels run.  The driver's clock table in sysfs is sampled
    while one kind of call loops for about a second."""
    if args.no_sclk:
        return None
    layers, b = res["layers"], res["b"]
    big = max(layers, key=lambda l: l["d_in"] * l["d_out"])
    return {
        "idle": sample_sclk(torch, None),
        "slope_spmm_bwd_x": sample_sclk(torch, lambda: sl.slope_spmm_bwd_x(big["dY"], big["vals_t"], big["meta_t"],
                                                                         out=big["dX"])),
        "slope_wgrad_masked": sample_sclk(torch, lambda: sl.slope_wgrad_masked(big["dY"], big["X"], big["meta"],
                                                                             out=big["G"], workspace=res["wg_ws"])),
        "dense_gemm": None if args.no_dense else sample_sclk(torch, lambda: torch.matmul(big["X"], big["W"].t(),
                                                                                        out=big["Y"])),
    }


def compact(res):
    """What `other_configs` keeps of a layer set's run."""
    d = res["dense_gemm"]
    return {"workload": res["workload"], "ms_per_step": res["ms_per_step"], "tflops": res["value"],
            "frac_of_sparse_peak": res["value"] / PEAK_SPARSE_BF16,
            "speedup_vs_dense": None if d is None else d["speedup_with_reprune"],
            "speedup_products_only": None if d is None else d["speedup_products_only"],
            "per_call_ms": res["per_call_ms"], "hip_graph": res["hip_graph"]}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2405_16325_amd import binding as sl
    from paper_2405_16325_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    sl.lib()  # fails loudly if libslope.so has not been built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.ceilings:
        print(json.dumps({"metric": "ceilings measured by micro-benchmarks", "n_gpus": 1,
                          "published": {"sparse_bf16_tflops": PEAK_SPARSE_BF16, "dense_bf16_tflops": PEAK_DENSE_BF16,
                                        "hbm_gbs": PEAK_HBM},
                          "measured": measure_ceilings(torch, sl, dev)}))
        return
    if args.workload == "sweep":
        print(json.dumps(sweep(args, torch, sl, inputs, dev)))
        return
    if args.workload.endswith("_infer"):
        print(json.dumps(inference(args, torch, sl, inputs, dev, args.workload[:-len("_infer")], args.steps,
                                   args.warmup)))
        return

    res = train(args, torch, sl, inputs, dev, args.workload, args.steps, args.warmup, full=not args.no_others)
    value, kernels, per_call = res["value"], res["kernels"], res["per_call_ms"]
    # Dominant kernel = spmm_split_kernel (forward and input-gradient products; the largest share of GPU
    # time in the rocprofv3 trace).  A slope_spmm_bwd_x call is exactly one launch of it, so the
    # events around those calls time the kernel itself: achieved = credited (dense-equivalent) flops
    # per launch / average launch duration, against the structured-sparse bf16 peak.
    roofline = {"kernel": "spmm_split_kernel", "timed_on": "slope_spmm_bwd_x launches", "bound": "mfma",
                "achieved": kernels["spmm_bwd_x"]["achieved"], "peak": PEAK_SPARSE_BF16, "unit": "TFLOP/s",
                "frac": kernels["spmm_bwd_x"]["frac"], "avg_launch_ms": kernels["spmm_bwd_x"]["avg_ms"],
                "flops_per_launch": res["flops_per_launch"], "traffic": read_traffic("spmm_split_kernel")}
    sclk = sclk_under_load(args, torch, sl, res)
    if sclk and sclk["slope_spmm_bwd_x"]:
        roofline["sclk_mhz_under_load"] = sclk["slope_spmm_bwd_x"]
        roofline["frac_at_that_clock"] = roofline["frac"] * NOMINAL_MHZ / sclk["slope_spmm_bwd_x"]
    cpu = None
    if not args.no_cpu_baseline:
        layers = res["layers"]
        cpu = cpu_baseline(layers[-2] if len(layers) > 1 else layers[0], res["b"], res["rank"])
    workload, ms_per_step = res["workload"], res["ms_per_step"]
    optimizer, adapter_bwd, dense, graph = (res.get("optimizer_side"), res.get("adapter_backward"), res["dense_gemm"],
                                            res["hip_graph"])
    del res                                                   # frees the layer set before the next ones are built

    ceil = other = None
    if not args.no_others:
        ceil = measure_ceilings(torch, sl, dev)
        other = {}
        light_steps = max(3, args.steps // 2)
        for w in ("opt125m_fc1", "opt2.7b", "opt13b", "opt66b"):
            if w != args.workload:
                other[w] = compact(train(args, torch, sl, inputs, dev, w, light_steps * (20 if w == "opt125m_fc1" else 1),
                                         max(1, args.warmup), full=False))
        inf = inference(args, torch, sl, inputs, dev, "opt66b", max(10, args.steps), max(2, args.warmup))
        other["opt66b_infer"] = {"workload": inf["config"]["workload"], "GB/s_at_16_tokens": inf["value"],
                                 "speedup_vs_dense": inf["speedup_vs_dense"],
                                 "cases": [{k: c[k] for k in ("layer", "tokens", "ms", "GB/s", "dense_gemm_ms")}
                                           for c in inf["cases"]]}

    def ceiling(ps, pd):
        # fwd + dX on the sparse pipe, dW on the dense pipe: the most 3 F can be credited at is 3 / (2 / Ps + 1 / Pd)
        return 3.0 / (2.0 / ps + 1.0 / pd)

    out = {
        "metric": "effective TFLOP/s of 2:4 sparse linear fwd+bwd; speedup vs dense bf16 GEMM",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload},
        "frac_of_sparse_peak": value / PEAK_SPARSE_BF16,
        "frac_of_fwd_bwd_ceiling": {"published": value / ceiling(PEAK_SPARSE_BF16, PEAK_DENSE_BF16),
                                    "measured": None if ceil is None else
                                    value / ceiling(ceil["sparse_bf16_tflops"], ceil["dense_bf16_tflops"])},
        "measured_ceilings": ceil,
        "speedup_vs_dense": None if dense is None else dense["speedup_with_reprune"],
        "roofline": roofline, "kernels": kernels, "dense_gemm": dense, "cpu_baseline": cpu,
        "per_call_ms": per_call, "hip_graph": graph, "optimizer_side": optimizer, "adapter_backward": adapter_bwd,
        "sclk_mhz": sclk, "other_configs": other,
    }
    print(json.dumps(out))


def sweep(args, torch, sl, inputs, dev):
    """Shape study (Sec. 2.4, App. E; the axes of the paper's kernel-speedup figure): attention (d x d),
    upsample (4d x d) and downsample (d x 4d) layers at 2048 tokens, and a token sweep from the HBM-bound to the
    MFMA-bound regime at 9216 x 9216.  Per case: forward, input gradient and weight gradient in effective
    TFLOP/s and the speedup of each (and of the three together) over torch.matmul."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE + 9)

    def gauss(shape, std):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)

    shapes = []
    for d in (1024, 2048, 4096, 8192, 12288):
        shapes += [("attention", 2048, d, d), ("upsample", 2048, 4 * d, d), ("downsample", 2048, d, 4 * d)]
    for b in (1, 16, 64, 128, 256, 512, 1024, 4096, 8192, 16384):
        shapes.append(("tokens", b, 9216, 9216))
    cases = []
    for kind, b, d_out, d_in in shapes:
        X, W, dY = gauss((b, d_in), 1.0), gauss((d_out, d_in), 0.02), gauss((b, d_out), 1e-3)
        vals, meta, _ = sl.slope_prune_rows(W)
        vals_t, meta_t, _ = sl.slope_double_prune(vals, meta)
        Y = torch.empty((b, d_out), dtype=torch.bfloat16, device=dev)
        dX = torch.empty((b, d_in), dtype=torch.bfloat16, device=dev)
        G = torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=dev)
        Wg = torch.empty((d_out, d_in), dtype=torch.bfloat16, device=dev)
        nws = sl.slope_spmm_fwd_workspace_bytes(b, d_in, d_out, 0)
        ws = torch.empty(nws, dtype=torch.uint8, device=dev) if nws else None
        wws = torch.empty(sl.slope_wgrad_workspace_bytes(b, d_in, d_out), dtype=torch.uint8, device=dev)
        flops = 2.0 * b * d_in * d_out
        iters = int(min(200, max(5, 2e12 / flops)))
        ours = [timed_ms(torch, lambda: sl.slope_spmm_fwd(X, vals, meta, out=Y, workspace=ws), iters),
                timed_ms(torch, lambda: sl.slope_spmm_bwd_x(dY, vals_t, meta_t, out=dX), iters),
                timed_ms(torch, lambda: sl.slope_wgrad_masked(dY, X, meta, out=G, workspace=wws), iters)]
        lib = [timed_ms(torch, lambda: torch.matmul(X, W.t(), out=Y), iters),
               timed_ms(torch, lambda: torch.matmul(dY, W, out=dX), iters),
               timed_ms(torch, lambda: torch.matmul(dY.t(), X, out=Wg), iters)]
        cases.append({"kind": kind, "tokens": b, "d_out": d_out, "d_in": d_in,
                      "ms": {"fwd": ours[0], "dX": ours[1], "dW": ours[2]},
                      "tflops": {"fwd": flops / ours[0] / 1e9, "dX": flops / ours[1] / 1e9, "dW": flops / ours[2] / 1e9},
                      "speedup": {"fwd": lib[0] / ours[0], "dX": lib[1] / ours[1], "dW": lib[2] / ours[2],
                                  "all": sum(lib) / sum(ours)}})
        del X, W, dY, vals, meta, vals_t, meta_t, Y, dX, G, Wg, ws, wws
    big = [c for c in cases if c["kind"] != "tokens"]
    value = sum(c["speedup"]["all"] for c in big) / len(big)
    return {"metric": "speedup of the 2:4 sparse linear fwd + dX + dW over dense bf16 GEMM, mean over the aspect-ratio sweep",
            "value": value, "unit": "x", "n_gpus": 1, "steps": None, "warmup": 2, "ms_per_step": None,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "shape sweep: attention d x d, upsample 4d x d, downsample d x 4d at 2048 tokens for "
                                   "d = 1024 .. 12288; 9216 x 9216 at 1 .. 16384 tokens; no adapters; products only"},
            "roofline": None, "cpu_baseline": None, "cases": cases}


def inference(args, torch, sl, inputs, dev, workload, steps, warmup):
    """slope_spmm_fwd with adapters at inference batch sizes (1, 16, 128 tokens) on the fc1, fc2 and one
    attention projection of the layer set: a pass over the packed weight, reported as the HBM rate of the
    bytes the call has to move.  value = the rate at 16 tokens over the three layers."""
    spec = inputs.LAYER_SETS[workload]
    rank = spec["rank"]
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE + 5)

    def gauss(shape, std):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)

    picked = {}
    for name, d_out, d_in in spec["layers"]:
        picked[(d_out, d_in)] = name                      # one layer per distinct shape
    cases, tot_bytes, tot_ms, tot_dense_ms = [], {}, {}, {}
    for (d_out, d_in), name in picked.items():
        # enough copies of the weight that consecutive calls cannot be served from the 256 MB last-level cache
        copies = max(1, -(-600 * 2 ** 20 // int(1.125 * d_out * d_in)))
        packed, dense = [], []
        for _ in range(copies):
            W = gauss((d_out, d_in), inputs.STD["W"])
            vals, meta, _ = sl.slope_prune_rows(W)
            packed.append((vals, meta))
            dense.append(W)
        L = gauss((d_in, rank), inputs.STD["L"]) if rank else None
        R = gauss((rank, d_out), inputs.STD["R"]) if rank else None
        for b in (1, 16, 128):
            X = gauss((b, d_in), inputs.STD["X"])
            Y = torch.empty((b, d_out), dtype=torch.bfloat16, device=dev)
            nws = sl.slope_spmm_fwd_workspace_bytes(b, d_in, d_out, rank)
            ws = torch.empty(nws, dtype=torch.uint8, device=dev) if nws else None

            def ours(i):
                v, m_ = packed[i % copies]
                sl.slope_spmm_fwd(X, v, m_, L, R, out=Y, workspace=ws)

            def lib_dense(i):
                torch.matmul(X, dense[i % copies].t(), out=Y)

            def timed(fn):
                for i in range(max(2, warmup)):
                    fn(i)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                n_it = max(10, steps)
                e0.record()
                for i in range(n_it):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / n_it

            ms, dms = timed(ours), timed(lib_dense)
            warm_ms = timed(lambda i: ours(0))            # the same copy every call: served from the last-level cache
            # bytes the call has to move: packed weight, adapter factors, activations in and out
            nbytes = 1.125 * d_out * d_in + 2.0 * rank * (d_in + d_out) + 2.0 * b * (d_in + d_out)
            cases.append({"layer": name, "d_out": d_out, "d_in": d_in, "tokens": b, "ms": ms,
                          "GB/s": nbytes / ms / 1e6, "dense_gemm_ms": dms, "speedup_vs_dense": dms / ms,
                          "cache_warm_ms": warm_ms, "cache_warm_GB/s": nbytes / warm_ms / 1e6})
            tot_bytes[b] = tot_bytes.get(b, 0.0) + nbytes
            tot_ms[b] = tot_ms.get(b, 0.0) + ms
            tot_dense_ms[b] = tot_dense_ms.get(b, 0.0) + dms
        del packed, dense
    value = tot_bytes[16] / tot_ms[16] / 1e6
    return {
        "metric": "HBM rate of the 2:4 sparse linear forward (with adapters) at inference batch size",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": max(10, steps), "warmup": max(2, warmup),
        "ms_per_step": tot_ms[16], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s_infer forward at 16 tokens: %s; adapter rank %d; weights rotated past the last-level cache"
                               % (workload, ", ".join("%s %dx%d" % (n, o, i) for (o, i), n in picked.items()), rank)},
        "roofline": {"bound": "hbm", "achieved": value, "peak": PEAK_HBM, "unit": "GB/s", "frac": value / PEAK_HBM,
                     "traffic": None, "kernel": "spmm_stream_lds_kernel (+ the split-K X L kernels)"},
        "speedup_vs_dense": {str(b): tot_dense_ms[b] / tot_ms[b] for b in tot_ms},
        "cases": cases, "cpu_baseline": None,
    }


def read_traffic(kernel):
    """HBM-side bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE,
    calibrated against a plain copy), or None if the summary is absent."""
    path = os.path.join(ROOT, "profiles", "spmm_split_kernel_opt66b_pmc.txt")
    try:
        for line in open(path):
            t = line.split()
            if len(t) == 3 and t[0] == "traffic_bytes_per_launch" and t[1] == kernel:
                return float(t[2])
    except OSError:
        pass
    return None


def read_sclk_mhz():
    """Current shader clock (MHz) from the driver's sysfs table (the entry marked '*'), or None.  No child
    process is started: this runs in a process that has initialised the GPU."""
    import glob
    import re
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            for line in open(path):
                if "*" in line:
                    m = re.search(r"([0-9.]+)\s*[Mm][Hh]z", line)
                    if m:
                        return float(m.group(1))
        except OSError:
            continue
    return None


def sample_sclk(torch, fn, seconds=1.2):
    """Median shader clock (MHz) while fn loops (None: idle); None if it cannot be read."""
    import threading
    vals, stop = [], [False]

    def sampler():
        while not stop[0]:
            v = read_sclk_mhz()
            if v is not None:
                vals.append(v)
            time.sleep(0.05)
    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        if fn is None:
            time.sleep(0.05)
        else:
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
    stop[0] = True
    th.join()
    vals = sorted(vals[len(vals) // 3:])                 # drop the ramp at the start
    return vals[len(vals) // 2] if vals else None


def cpu_baseline(lay, b, rank):
    """The oracle, as it stands, on a bounded slice of one layer of the workload (host cores)."""
    import numpy as np
    from oracle import slope_oracle as so
    from paper_2405_16325_amd import binding as sl
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    rows, toks = min(8192, lay["d_out"]), min(1024, b)                # about 10 s of host work
    d_in = lay["d_in"]
    w = sl.bf16_to_host(lay["W"][:rows])
    x = sl.bf16_to_host(lay["X"][:toks])
    dy = sl.bf16_to_host(lay["dY"][:toks, :rows].contiguous())
    lb = sl.bf16_to_host(lay["L"]) if rank else None
    rb = sl.bf16_to_host(lay["R"][:, :rows].contiguous()) if rank else None
    t0 = time.perf_counter()
    vals, meta, _ = so.prune_rows_packed(w)
    mask_r = so.meta_to_mask(meta)
    mask_rc = so.double_prune(w, mask_r)
    so.pack_2to4(np.ascontiguousarray(w.T), np.ascontiguousarray(mask_rc.T))
    so.spmm_fwd(x, w, mask_r, lb, rb)
    so.spmm_bwd_x(dy, w, mask_rc)
    so.wgrad_masked(dy, x, meta)
    dt = time.perf_counter() - t0
    flops = 3.0 * 2.0 * toks * d_in * rows
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": dt,
            "sample": "%s layer slice: first %d of %d weight rows, first %d of %d tokens, d_in %d; prune, double "
                      "prune, fwd (+adapter), dX, dW in fp64 numpy" % (lay["name"], rows, lay["d_out"], toks, b, d_in)}


if __name__ == "__main__":
    main()
