#!/usr/bin/env python3
"""Benchmark of the DropIT hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
dropit_compress (min-k drop of the cached layer input) followed by
dropit_weight_grad (dW from the sparse cache), both through the C ABI.
Workload at N=1: ViT-B/16 FC1 input, batch 64 (x bf16 [12608, 768], gamma 0.9,
dY bf16 [12608, 3072]).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is whole-step throughput in dense-equivalent
dW TFLOP/s (the paper keeps the dense GEMM, Sec. 3.2, so flops are the dense
2*C_out*C_in*N_tok); the two halves of the metric are broken out under
"halves", each with its own roofline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

def measured_traffic(workload, kernel_prefix):
    """HBM bytes per launch of `kernel_prefix` on `workload`, from the table of rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE readings in profiles/hbm_traffic.md (each row names the summary file it was read from and the
    commit it was taken at; readings are scaled by what the same counter reads for a plain 256 MiB copy in the
    same run).  None for a kernel/workload pair that is not in the table."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.md")
    if not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 8 or cells[0] != workload or not cells[1].startswith(kernel_prefix):
            continue
        try:
            fetch_kib, fetch_factor, write_kib, write_factor = (float(cells[i]) for i in (2, 3, 4, 5))
        except ValueError:
            continue
        return {"bytes": int((fetch_kib * fetch_factor + write_kib * write_factor) * 1024),
                "fetch_bytes": int(fetch_kib * fetch_factor * 1024), "write_bytes": int(write_kib * write_factor * 1024),
                "source": cells[6], "commit": cells[7]}
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vitb_fc1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layout", choices=["nchw", "nhwc"], default="nchw",
                    help="convolution workloads only: run on channels-last tensors (x [N,H,W,C], dY [N,OH,OW,J], "
                         "dW [J,kh,kw,C]) through dropit_weight_grad_nhwc; the CPU baseline is skipped")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time the vendor library's dense weight gradient (torch.mm / conv2d_weight) on the "
                         "same shapes and inputs, reported as context under 'vendor_gemm'")
    ap.add_argument("--fc-recover", choices=["dense", "lds"], default="dense",
                    help="where the recover step of a bf16 fully-connected layer happens: a dense operand in the "
                         "workspace (default, the faster form) or inside the product, in LDS (dropit_set_fc_recover)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of ONE captured HIP graph of the step (one input copy) instead of eager calls: "
                         "what a launch-bound layer costs once the host's per-call work is out of the loop")
    ap.add_argument("--warm", action="store_true",
                    help="time with ONE input copy (x / dY then stay in the 256 MB Infinity Cache) instead of "
                         "rotating over > 600 MB of copies; the rotating (cold) figure is the default")
    return ap.parse_args()


def event_ms(events):
    return [events[i].elapsed_time(events[i + 1]) for i in range(len(events) - 1)]


def cpu_baseline(w, flops_per_step):
    """The oracle, as it stands, on this host's cores, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from dropit_inputs import make

    x, dy = make(w)
    k = oracle.keep_count(x.size, w.gamma)
    t0 = time.perf_counter()
    vals, idx = oracle.compress(x, k)
    t_compress = time.perf_counter() - t0
    xh = oracle.densify(vals, idx, x.shape)
    dyw = oracle.widen(dy)
    def run_rows(r0, r1):
        t0 = time.perf_counter()
        if w.conv is None:
            oracle.dw_fc(xh, dyw, r0, r1)
        else:
            oracle.dw_conv(xh, dyw, w.conv[0], w.conv[1], (w.conv[2],) * 2, (w.conv[3],) * 2, (1, 1), r0, r1)
        return time.perf_counter() - t0

    probe_rows = min(w.c_out, 2 * oracle.num_threads())
    t_probe = run_rows(0, probe_rows)
    # then as many output rows as fit in about ten seconds of CPU time (all of them if possible)
    rows = int(min(w.c_out, max(probe_rows, probe_rows * 10.0 / max(t_probe, 1e-6))))
    t_rows = run_rows(0, rows) if rows > probe_rows else t_probe
    t_step = t_compress + t_rows * (w.c_out / rows)
    return {
        "value": flops_per_step / t_step * 1e-12,
        "unit": "TFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "full-sort compress of the whole tensor (%.2f s) + fp64 dW for %d of %d output rows "
                  "(%.2f s), extrapolated to all rows" % (t_compress, rows, w.c_out, t_rows),
        "compress_GBps": (x.nbytes + k * (x.itemsize + 4)) / t_compress * 1e-9,
        "dw_GFLOPs": flops_per_step * (rows / w.c_out) / t_rows * 1e-9,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); multi-GPU runs are not part of it.",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2202_13808_amd as dropit
    from dropit_inputs import EXTRA_WORKLOADS, WORKLOADS, make

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    dropit.lib()  # fail loudly if the extension is not built
    dropit.set_fc_recover(1 if args.fc_recover == "lds" else 0)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = {**WORKLOADS, **EXTRA_WORKLOADS}[args.workload]
    xh, dyh = make(w)
    nhwc = args.layout == "nhwc"
    if nhwc and w.conv is None:
        print("bench.py: --layout nhwc is for the convolution workloads.", file=sys.stderr)
        sys.exit(2)
    x_shape, dw_shape = tuple(w.x_shape), tuple(w.dw_shape)
    if nhwc:
        xh = np.ascontiguousarray(xh.transpose(0, 2, 3, 1))
        dyh = np.ascontiguousarray(dyh.transpose(0, 2, 3, 1))
        x_shape = tuple(xh.shape)
        dw_shape = (w.c_out, w.conv[0], w.conv[1], w.x_shape[1])

    def dev_tensor(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(a).to(dev)

    copies = 1
    if not args.warm and not args.graph:
        per = xh.nbytes + dyh.nbytes
        copies = max(2, int(np.ceil(600e6 / per)))
    xs = [dev_tensor(xh) for _ in range(copies)]
    dys = [dev_tensor(dyh) for _ in range(copies)]
    conv = None if w.conv is None else (w.conv[0], w.conv[1], w.conv[2], w.conv[2], w.conv[3], w.conv[3], 1, 1)

    k = dropit.keep_count(w.numel, w.gamma)
    vals = torch.empty(k, dtype=xs[0].dtype, device=dev)
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    dW = torch.empty(dw_shape, dtype=torch.float32, device=dev)
    ws_c = torch.empty(dropit.compress_workspace_bytes(w.numel, xs[0].dtype), dtype=torch.uint8, device=dev)
    ws_g = torch.empty(max(1, dropit.weight_grad_workspace_bytes(x_shape, xs[0].dtype, k, w.c_out, conv,
                                                                       layout=args.layout)),
                       dtype=torch.uint8, device=dev)

    def step(i):
        x, dy = xs[i % copies], dys[i % copies]
        dropit.compress(x, w.gamma, vals=vals, idx=idx, workspace=ws_c)
        dropit.weight_grad(vals, idx, x_shape, dy, w.c_out, conv=conv, dW=dW, workspace=ws_g, layout=args.layout)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(0)
        for i in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if args.graph:
            graph.replay()
        else:
            step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    # beside it, outside the timed region that `value` comes from: the same steps on one input copy
    warm_ms_per_step = ms_per_step
    if copies > 1:
        for i in range(min(args.warmup, 5)):
            step(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(0)
        torch.cuda.synchronize()
        warm_ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3

    if args.copy_calibration:
        src = torch.full((256 << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- per-call and per-kernel durations with HIP events on the launch stream ----
    n_meas = min(args.steps, 50)
    ce = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(n_meas)]
    ge = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(n_meas)]
    for evs in ce + ge:                      # create the underlying handles
        for e in evs:
            e.record()
    torch.cuda.synchronize()
    # An event pair with nothing between them still reads a few microseconds (the marks are packets on
    # the queue).  That reading is measured on the same stream and taken out of every interval: with it
    # removed the per-kernel figures agree with a rocprofv3 kernel trace of the same run to about 1 %
    # (checked dispatch by dispatch: GEMM 53.5 us in the trace, 57.9 - 4.6 = 53.3 us here); left in,
    # every kernel would read 4-5 us long.
    # The marks must already be queued when the GPU reaches them, or the reading is the host's pace of
    # submitting them: a few milliseconds of kernels go in front.
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(65)]
    for i in range(max(8, int(3.0 / max(ms_per_step, 1e-3)))):
        step(i)
    for e in pe:
        e.record()
    torch.cuda.synchronize()
    event_overhead_ms = float(np.median(event_ms(pe)))
    n_c = n_g = 0
    for i in range(n_meas):
        x, dy = xs[i % copies], dys[i % copies]
        dropit.trace_events(ce[i])
        dropit.compress(x, w.gamma, vals=vals, idx=idx, workspace=ws_c)
        dropit.trace_events(ge[i])
        dropit.weight_grad(vals, idx, x_shape, dy, w.c_out, conv=conv, dW=dW, workspace=ws_g, layout=args.layout)
        dropit.trace_events(None)
    torch.cuda.synchronize()
    bf16 = w.dtype == "bf16"
    # marks recorded per compress call: before and after the one persistent select kernel
    n_c = 2
    path = dropit.weight_grad_path(x_shape, xs[0].dtype, k, w.c_out, conv, layout=args.layout)   # which kernels the library runs
    fc_mfma = path == "fc_mfma"
    fc_fused = path == "fc_fused"                          # token-block starts, pairs regrouped by tile, product, slice sum
    conv_gemm = path in ("conv_gemm", "conv_im2col")      # operand preparation, then the fully-connected GEMM
    conv_mfma = path == "conv_bands"
    conv_padded = conv_mfma and w.x_shape[3] % 8 != 0       # one more kernel: the zero-padded copy of dY
    mfma = fc_mfma or fc_fused or conv_mfma or conv_gemm
    # marks per call: prep, [pad,] gemm, reduce, end  |  zero+scatter, gemm, end
    fc_small = path == "fc_small"                          # one launch: recover in LDS + fp32 multiply-adds
    n_g = 5 if (conv_padded or fc_fused) else 4 if mfma else 2 if fc_small else 3
    c_ms = np.maximum(np.array([event_ms(e[:n_c]) for e in ce]) - event_overhead_ms, 0.0)   # [n_meas, n_c-1]
    g_ms = np.maximum(np.array([event_ms(e[:n_g]) for e in ge]) - event_overhead_ms, 0.0)
    c_med = np.median(c_ms, axis=0)
    g_med = np.median(g_ms, axis=0)
    c_names = ["select"]
    g_names = (["recover", "mfma_gemm", "splitk_reduce"] if fc_mfma else
               ["token_block_starts", "pairs_by_tile", "mfma_gemm_with_recover", "splitk_reduce"] if fc_fused else
               ["im2col_recover_and_dY_tokens", "mfma_gemm", "splitk_reduce"] if path == "conv_gemm" else
               ["im2col_rows_and_dY_tokens", "mfma_gemm", "splitk_reduce"] if conv_gemm else
               ["row_starts", "pad_dY", "mfma_conv", "partial_reduce"] if conv_padded else
               ["row_starts", "mfma_conv", "partial_reduce"] if conv_mfma else
               ["recover_and_fma_gemm"] if fc_small else ["zero_scatter", "fma_gemm"])
    compress_ms = float(c_med.sum())
    grad_ms = float(g_med.sum())

    esz = 2 if bf16 else 4
    compress_bytes = w.numel * esz + k * (esz + 4)           # read x once + write k (value, index) pairs
    flops = float(w.dense_flops)
    main_idx = 2 if (conv_padded or fc_fused) else 0 if fc_small else 1
    main_ms = float(np.mean(g_ms[:, main_idx]))
    dw_tflops_kernel = flops / (main_ms * 1e-3) * 1e-12
    hist_ms = float(np.mean(c_ms[:, 0]))
    hist_gbps = compress_bytes / (hist_ms * 1e-3) * 1e-9

    main_kernel = ("fc_dense_kernel" if (fc_mfma or conv_gemm or fc_fused) else "conv3x3_mfma_kernel" if conv_mfma else
                   "fc_small_kernel" if fc_small else "fc_fma_kernel")
    select_kernel = "select_small_kernel" if w.numel // (8 if bf16 else 4) <= 8 * 1024 else "select_fused_kernel"
    dw_traffic = measured_traffic(w.name + ("+lds" if fc_fused else ""), main_kernel)
    sel_traffic = measured_traffic(w.name, select_kernel)
    out = {
        "metric": "min-k compress GB/s (% HBM peak) + sparse-input dW TFLOP/s (% MFMA peak)",
        "value": flops / (ms_per_step * 1e-3) * 1e-12,
        "unit": "TFLOP/s (dense-equivalent dW flops per whole compress+dW step)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: x %s %s gamma=%.2f, dY %s, dW %s fp32%s" % (
            w.name + (" channels-last" if nhwc else "") + (" recover-in-LDS" if fc_fused else ""), w.dtype, list(x_shape), w.gamma, list(dyh.shape), list(dw_shape),
            " (cold: %d rotating input copies, %.0f MB)" % (copies, copies * (xh.nbytes + dyh.nbytes) / 1e6)
            if copies > 1 else " (inputs warm in Infinity Cache%s)" % (", replays of one captured graph" if args.graph else ""))},
        "warm": {"ms_per_step": warm_ms_per_step, "value": flops / (warm_ms_per_step * 1e-3) * 1e-12,
                 "note": "same steps on one input copy (x and dY stay in the 256 MB Infinity Cache)"},
        "event_overhead_ms": event_overhead_ms,
        "halves": {
            "compress_GBps": compress_bytes / (compress_ms * 1e-3) * 1e-9,
            "compress_pct_hbm_peak": 100.0 * compress_bytes / (compress_ms * 1e-3) * 1e-9 / HBM_PEAK_GBPS,
            "compress_ms": compress_ms,
            "compress_kernels_ms": dict(zip(c_names, [float(v) for v in c_med])),
            "dw_TFLOPs": flops / (grad_ms * 1e-3) * 1e-12,
            "dw_pct_mfma_peak": 100.0 * flops / (grad_ms * 1e-3) * 1e-12 / MFMA_BF16_PEAK_TFLOPS,
            "dw_ms": grad_ms,
            "dw_kernels_ms": dict(zip(g_names, [float(v) for v in g_med])),
        },
        "roofline": {
            "kernel": main_kernel,
            "bound": "mfma" if mfma else "alu",
            "achieved": dw_tflops_kernel,
            "peak": MFMA_BF16_PEAK_TFLOPS if mfma else 157.3,
            "unit": "TFLOP/s",
            "frac": dw_tflops_kernel / (MFMA_BF16_PEAK_TFLOPS if mfma else 157.3),
            "traffic": (dw_traffic or {}).get("bytes"),
            "traffic_source": dw_traffic,
            "avg_kernel_ms": main_ms,
        },
        "roofline_compress": {
            "kernel": select_kernel,
            "bound": "hbm",
            "achieved": hist_gbps,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": hist_gbps / HBM_PEAK_GBPS,
            "traffic": (sel_traffic or {}).get("bytes"),
            "traffic_source": sel_traffic,
            "avg_kernel_ms": hist_ms,
        },
    }
    if args.vendor_gemm and bf16:
        # Context, not part of the path: what the dense weight gradient of the same layer costs through the
        # vendor libraries torch calls (no dropping, no recover), same rotating inputs, events on the stream.
        def vendor(i):
            x, dy = xs[i % copies], dys[i % copies]
            if w.conv is None:
                return torch.mm(dy.reshape(-1, w.c_out).t(), x.reshape(-1, w.x_shape[-1]))
            if nhwc:       # the same tensors as channels-last views of NCHW shapes
                x, dy = x.permute(0, 3, 1, 2), dy.permute(0, 3, 1, 2)
            return torch.nn.grad.conv2d_weight(x, w.dw_shape, dy, stride=w.conv[2], padding=w.conv[3])
        for i in range(10):
            vendor(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(50):
            vendor(i)
        e1.record()
        torch.cuda.synchronize()
        v_ms = e0.elapsed_time(e1) / 50
        out["vendor_gemm"] = {"ms": v_ms, "TFLOPs": flops / (v_ms * 1e-3) * 1e-12,
                              "pct_mfma_peak": 100.0 * flops / (v_ms * 1e-3) * 1e-12 / MFMA_BF16_PEAK_TFLOPS,
                              "note": "dense dW of the same layer by torch (vendor GEMM / convolution library), "
                                      "bf16 output; this library's recover + GEMM + reduce take dw_ms"}
    if not args.no_cpu_baseline and not nhwc:
        out["cpu_baseline"] = cpu_baseline(w, flops)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
