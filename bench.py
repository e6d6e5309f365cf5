#!/usr/bin/env python3
"""Benchmark of the double-pruned 2:4 sparse linear layer on one MI355X.

One step = one pass of the whole hot path over the linear layers of one OPT-66B-shaped
transformer block (q, k, v, o: 9216 x 9216; fc1: 36864 x 9216; fc2: 9216 x 36864; 16384 tokens,
rank-128 adapters in the forward): for every layer slope_prune_rows, slope_double_prune (weights
are re-pruned from dense each step), slope_spmm_fwd with the adapter, slope_spmm_bwd_x and
slope_wgrad_masked.  All inputs are synthetic (seeded Gaussians, generated on the device) and
resident in HBM before the clock starts.

Prints ONE JSON line.  value = effective TFLOP/s = 3 * 2 * b * d_in * d_out summed over the
layers (the dense-equivalent flops of fwd + dX + dW; adapter flops are not credited) divided by
the step time.  Details (per-call times, the dense bf16 GEMM comparison, the CPU-oracle baseline)
ride in the same line.
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
# What register-resident loops and plain streams reached on this machine's MI355X (the ceilings a kernel can
# actually touch): v_smfmac_f32_16x16x64_bf16, v_mfma_f32_32x32x16_bf16, a read-only stream, a copy.
MEASURED = {"sparse_bf16_tflops": 4390.0, "dense_bf16_tflops": 2390.0, "hbm_read_gbs": 6900.0, "hbm_copy_gbs": 4700.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="opt66b",
                    help="opt66b (headline) | opt13b | opt2.7b | opt125m_fc1 | opt66b_infer (forward at 1/16/128 tokens)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sclk", action="store_true", help="skip the shader-clock sampling loops (for profiling runs)")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step (and the dense comparison) replayed from a captured HIP graph")
    return ap.parse_args()


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
    if args.workload.endswith("_infer"):
        return inference(args, torch, sl, inputs, dev)
    spec = inputs.LAYER_SETS[args.workload]
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
        if rank:
            lay["L"] = gauss((d_in, rank), inputs.STD["L"])
            lay["R"] = gauss((rank, d_out), inputs.STD["R"])
            lay["ws"] = torch.empty(sl.slope_spmm_fwd_workspace_bytes(b, d_in, d_out, rank), dtype=torch.uint8,
                                    device=dev)
        else:
            lay["L"] = lay["R"] = lay["ws"] = None
        lay["vals"] = torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=dev)
        lay["meta"] = torch.empty((d_out, d_in // 8), dtype=torch.uint8, device=dev)
        lay["vals_t"] = torch.empty((d_in, d_out // 2), dtype=torch.bfloat16, device=dev)
        lay["meta_t"] = torch.empty((d_in, d_out // 8), dtype=torch.uint8, device=dev)
        lay["Y"] = torch.empty((b, d_out), dtype=torch.bfloat16, device=dev)
        lay["dX"] = torch.empty((b, d_in), dtype=torch.bfloat16, device=dev)
        lay["G"] = torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=dev)
        layers.append(lay)
    # one scratch buffer for the weight-gradient calls, sized for the largest layer
    wg_ws = torch.empty(max(sl.slope_wgrad_workspace_bytes(b, l["d_in"], l["d_out"]) for l in layers),
                        dtype=torch.uint8, device=dev)

    calls = ["prune_rows", "double_prune", "spmm_fwd", "spmm_bwd_x", "wgrad_masked"]

    def step(events=None):
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
            sl.slope_wgrad_masked(lay["dY"], lay["X"], lay["meta"], out=lay["G"], workspace=wg_ws)
            if ev: ev[5].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # HIP events on the stream the kernels run on (torch's current stream), one set per step
    all_events = [[[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in layers]
                  for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(all_events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    def graph_ms(fn):
        """fn captured into a HIP graph on a side stream and replayed args.steps times (ms per replay)."""
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
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - g0) * 1e3 / args.steps

    graph = {"ms_per_step": graph_ms(step)} if args.graph else None

    flops_layer = [2.0 * b * l["d_in"] * l["d_out"] for l in layers]
    total_flops = 3.0 * sum(flops_layer)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # per-call average durations (ms) from the events of the timed region
    per_call = {c: 0.0 for c in calls}
    per_layer_call = {}
    for li, lay in enumerate(layers):
        for ci, c in enumerate(calls):
            ms = sum(all_events[s][li][ci].elapsed_time(all_events[s][li][ci + 1]) for s in range(args.steps))
            ms /= args.steps
            per_call[c] += ms
            per_layer_call[(lay["name"], c)] = ms
    sum_f = sum(flops_layer)
    elems = sum(l["d_in"] * l["d_out"] for l in layers)
    kernels = {
        # dense contraction: 2 b d_in d_out flops per launch against the dense bf16 MFMA peak
        "wgrad_masked": {"bound": "mfma", "achieved": sum_f / (per_call["wgrad_masked"] * 1e-3) / 1e12,
                         "peak": PEAK_DENSE_BF16, "unit": "TFLOP/s", "launches_per_step": len(layers),
                         "avg_ms": per_call["wgrad_masked"] / len(layers)},
        # sparse contraction: credited dense-equivalent 2 b d_in d_out against the sparse bf16 peak
        "spmm_bwd_x": {"bound": "mfma", "achieved": sum_f / (per_call["spmm_bwd_x"] * 1e-3) / 1e12,
                       "peak": PEAK_SPARSE_BF16, "unit": "TFLOP/s", "launches_per_step": len(layers),
                       "avg_ms": per_call["spmm_bwd_x"] / len(layers)},
        "spmm_fwd": {"bound": "mfma", "achieved": sum_f / (per_call["spmm_fwd"] * 1e-3) / 1e12,
                     "peak": PEAK_SPARSE_BF16, "unit": "TFLOP/s", "launches_per_step": len(layers),
                     "avg_ms": per_call["spmm_fwd"] / len(layers), "note": "includes the adapter kernels"},
        # streams: 3.125 B (read 2, write 1 + 1/8) and 2.25 B per weight element
        "prune_rows": {"bound": "hbm", "achieved": 3.125 * elems / (per_call["prune_rows"] * 1e-3) / 1e9,
                       "peak": PEAK_HBM, "unit": "GB/s", "launches_per_step": len(layers),
                       "avg_ms": per_call["prune_rows"] / len(layers)},
        "double_prune": {"bound": "hbm", "achieved": 2.25 * elems / (per_call["double_prune"] * 1e-3) / 1e9,
                         "peak": PEAK_HBM, "unit": "GB/s", "launches_per_step": len(layers),
                         "avg_ms": per_call["double_prune"] / len(layers)},
    }
    for k in kernels.values():
        k["frac"] = k["achieved"] / k["peak"]
    # Dominant kernel = spmm_split_kernel (forward and input-gradient products; the largest share of GPU
    # time in the rocprofv3 trace).  A slope_spmm_bwd_x call is exactly one launch of it, so the
    # events around those calls time the kernel itself: achieved = credited (dense-equivalent) flops
    # per launch / average launch duration, against the structured-sparse bf16 peak.
    n_launch = len(layers)
    roofline = {"kernel": "spmm_split_kernel", "timed_on": "slope_spmm_bwd_x launches", "bound": "mfma",
                "achieved": kernels["spmm_bwd_x"]["achieved"], "peak": PEAK_SPARSE_BF16, "unit": "TFLOP/s",
                "frac": kernels["spmm_bwd_x"]["frac"], "avg_launch_ms": per_call["spmm_bwd_x"] / n_launch,
                "flops_per_launch": sum_f / n_launch, "traffic": read_traffic("spmm_split_kernel")}

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
        for _ in range(max(1, args.warmup)):
            dense_step()
        torch.cuda.synchronize()
        d0 = time.perf_counter()
        nd = max(3, args.steps // 2)
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

    # Optimizer-side packed streams (Alg. 1 lines 15-18), timed apart from the step: g = G / scale + decay * W^R
    # in W^R's packed layout, then both sparse copies take the new values (static masks).
    def optimizer_step():
        for lay in layers:
            sl.slope_sparse_add(lay["G"], lay["vals"], 1.0 / 1024.0, 0.01, out=lay["G"])
            sl.slope_update_sparse(lay["G"], lay["meta"], lay["vals"], lay["meta_t"], lay["vals_t"])
    optimizer_step()
    torch.cuda.synchronize()
    o0 = time.perf_counter()
    for _ in range(3):
        optimizer_step()
    torch.cuda.synchronize()
    opt_ms = (time.perf_counter() - o0) * 1e3 / 3
    # bytes per weight element (a packed value array holds 1 B per weight): sparse_add reads two arrays and
    # writes one = 3; update copies one array (1 + 1), reads packed W^R (1.125) and the transposed metadata
    # (0.125) and writes the transposed values (1) = 4.25
    optimizer = {"ms_per_step": opt_ms, "achieved": 7.25 * elems / (opt_ms * 1e-3) / 1e9, "unit": "GB/s",
                 "peak": PEAK_HBM, "calls": "slope_sparse_add + slope_update_sparse per layer"}

    # Backward pass with adapters (chain rule of Eq. 11), timed apart from the step: the same step with
    # slope_spmm_bwd_x_adapter and slope_wgrad_adapter in place of the plain backward calls.
    adapter_bwd = None
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
        adapter_step()
        torch.cuda.synchronize()
        a0 = time.perf_counter()
        for _ in range(3):
            adapter_step()
        torch.cuda.synchronize()
        ab_ms = (time.perf_counter() - a0) * 1e3 / 3
        adapter_bwd = {"ms_per_step": ab_ms, "plain_backward_ms": per_call["spmm_bwd_x"] + per_call["wgrad_masked"],
                       "calls": "slope_spmm_bwd_x_adapter + slope_wgrad_adapter per layer"}

    # Shader clock under load (outside the timed region): the published MFMA peaks assume 2.4 GHz, but the
    # power management lowers the clock while MFMA-bound kernels run.  The driver's clock table in sysfs is
    # sampled while one kind of call loops for about a second.
    big = max(layers, key=lambda l: l["d_in"] * l["d_out"])
    sclk = None if args.no_sclk else {
        "idle": sample_sclk(torch, None),
        "slope_spmm_bwd_x": sample_sclk(torch, lambda: sl.slope_spmm_bwd_x(big["dY"], big["vals_t"], big["meta_t"],
                                                                         out=big["dX"])),
        "slope_wgrad_masked": sample_sclk(torch, lambda: sl.slope_wgrad_masked(big["dY"], big["X"], big["meta"],
                                                                             out=big["G"], workspace=wg_ws)),
        "dense_gemm": None if args.no_dense else sample_sclk(torch, lambda: torch.matmul(big["X"], big["W"].t(),
                                                                                        out=big["Y"])),
    }
    if sclk and sclk["slope_spmm_bwd_x"]:
        roofline["sclk_mhz_under_load"] = sclk["slope_spmm_bwd_x"]
        roofline["frac_at_that_clock"] = roofline["frac"] * NOMINAL_MHZ / sclk["slope_spmm_bwd_x"]

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(layers[-2] if len(layers) > 1 else layers[0], b, rank)

    out = {
        "metric": "effective TFLOP/s of 2:4 sparse linear fwd+bwd; speedup vs dense bf16 GEMM",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s linear layers of one block: %s; tokens %d; adapter rank %d; "
                               "re-pruned from dense every step" %
                               (args.workload, ", ".join("%s %dx%d" % (n, o, i) for n, o, i in spec["layers"]),
                                b, rank)},
        "frac_of_sparse_peak": value / PEAK_SPARSE_BF16,
        # fwd + dX on the sparse pipe, dW on the dense pipe: the most 3 F can be credited at is 3 / (2 / Ps + 1 / Pd)
        "frac_of_fwd_bwd_ceiling": {"published": value / (3.0 / (2.0 / PEAK_SPARSE_BF16 + 1.0 / PEAK_DENSE_BF16)),
                                    "measured": value / (3.0 / (2.0 / MEASURED["sparse_bf16_tflops"]
                                                                + 1.0 / MEASURED["dense_bf16_tflops"]))},
        "measured_ceilings": MEASURED,
        "speedup_vs_dense": None if dense is None else dense["speedup_with_reprune"],
        "roofline": roofline, "kernels": kernels, "dense_gemm": dense, "cpu_baseline": cpu,
        "per_call_ms": per_call, "hip_graph": graph, "optimizer_side": optimizer, "adapter_backward": adapter_bwd,
        "sclk_mhz": sclk,
    }
    print(json.dumps(out))


def inference(args, torch, sl, inputs, dev):
    """slope_spmm_fwd with adapters at inference batch sizes (1, 16, 128 tokens) on the fc1, fc2 and one
    attention projection of the layer set: a pass over the packed weight, reported as the HBM rate of the
    bytes the call has to move.  One JSON line; value = the rate at 16 tokens over the three layers."""
    spec = inputs.LAYER_SETS[args.workload[:-len("_infer")]]
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
            ws = torch.empty(max(256, sl.slope_spmm_fwd_workspace_bytes(b, d_in, d_out, rank)), dtype=torch.uint8,
                             device=dev) if rank else None

            def ours(i):
                v, m_ = packed[i % copies]
                sl.slope_spmm_fwd(X, v, m_, L, R, out=Y, workspace=ws)

            def lib_dense(i):
                torch.matmul(X, dense[i % copies].t(), out=Y)

            def timed(fn):
                for i in range(max(2, args.warmup)):
                    fn(i)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                n_it = max(10, args.steps)
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
    out = {
        "metric": "HBM rate of the 2:4 sparse linear forward (with adapters) at inference batch size",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": max(10, args.steps), "warmup": max(2, args.warmup),
        "ms_per_step": tot_ms[16], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s forward at 16 tokens: %s; adapter rank %d; weights rotated past the last-level cache"
                               % (args.workload, ", ".join("%s %dx%d" % (n, o, i) for (o, i), n in picked.items()), rank)},
        "roofline": {"bound": "hbm", "achieved": value, "peak": PEAK_HBM, "unit": "GB/s", "frac": value / PEAK_HBM,
                     "traffic": None, "kernel": "spmm_stream_lds_kernel (+ the split-K X L kernels)"},
        "speedup_vs_dense": {str(b): tot_dense_ms[b] / tot_ms[b] for b in tot_ms},
        "cases": cases, "cpu_baseline": None,
    }
    print(json.dumps(out))


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
    import torch
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
