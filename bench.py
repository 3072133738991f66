#!/usr/bin/env python3
"""Benchmark of the kernel-segregated transpose convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers all|none] [--no-cpu]

One step = one pass of the whole hot path on the headline workload (the
single-channel bandwidth-bound layer): weight pre-segregation, then the
segregated forward pass with its edge masking, through the C ABI, inputs
resident in HBM.  Prints ONE JSON line: whole-job useful GMAC/s, the roofline
of the dominant kernel (measured live with events on the launch stream), the
CPU oracle as a baseline, a per-layer table for the five benchmark layers (time, useful
GMAC/s, roofline fraction, speed-up over the zero-insert path), a table for the paper's
own shapes with padding factor 2 (Tables 1 and 3) at a batch that fills the chip, and Table 3's
four generator families on one input sample with the seconds the paper prints beside them.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MEASURED_TRAFFIC_BYTES = {}      # filled by measured_traffic() from profiles/hbm_traffic_pmc.txt


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--layers", default="all", choices=["all", "none"],
                    help="also time each of the five benchmark layers")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only", default=None,
                    help="time just one pass of one layer (profiling aid): cfg1..cfg5, a paper-shaped layer's name, or copy")
    ap.add_argument("--what", default="forward", choices=["forward", "backward_input", "backward_weight"],
                    help="with --only: which pass of the layer")
    return ap.parse_args()


class Resident:
    """A layer's operands in HBM, with `sets` rotating input/output buffers so that
    successive launches cannot be served from the last-level cache."""

    def __init__(self, layer, sets, torch, kst, wl):
        self.layer = layer
        x, w = wl.make_tensors(layer)
        self.host = (x, w)
        self.w = w.cuda()
        self.x = [x.cuda() if i == 0 else x.cuda().clone() for i in range(sets)]
        self.out = [torch.empty(layer.out_shape, dtype=torch.float32, device="cuda") for _ in range(sets)]
        dt = kst.KST_BF16 if layer.dtype == "bf16" else kst.KST_F32
        self.w_seg = torch.empty(kst.kst_segregated_elems(layer.Cin, layer.Cout, layer.n, dt),
                                 dtype=w.dtype, device="cuda")
        need = kst.kst_workspace_bytes(layer.B, layer.Cin, layer.Cout, layer.N, layer.n, dt, kst.KST_PATH_AUTO)
        self.ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda") if need else None
        self.sets = sets


def time_launches(torch, fn, iters, warmup):
    """Average milliseconds per call of fn(i), by events on the current stream."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(iters):
        fn(i)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def settle(torch, fn, seconds):
    """Untimed launches for about `seconds`: the first tens of milliseconds of work after an idle
    period run several per cent slower than the steady state, whatever the kernel."""
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(5):
            fn(i)
            i += 1
        torch.cuda.synchronize()


def launch_spread(torch, fn, iters, warmup):
    """(median, min) milliseconds of single calls of fn(i): one event between every two calls on
    the current stream (the events add a little to each call; the mean of time_launches has none)."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    ev[0].record()
    for i in range(iters):
        fn(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    d = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))
    return d[len(d) // 2], d[0]


def one_pass(layer, what, torch, kst, wl):
    """A launcher fn(i) for one pass of `layer` (pre-segregated weights, caller's workspace, three
    rotating buffer sets for the forward pass) and the buffers it needs, kept alive by the closure."""
    dt = {"f32": kst.KST_F32, "bf16": kst.KST_BF16, "f16": kst.KST_F16}[layer.dtype]
    x, w = wl.make_tensors(layer)
    xd = [x.cuda().clone() for _ in range(3)]
    wd = w.cuda()
    if what == "forward":
        outs = [torch.empty(layer.out_shape, dtype=torch.float32, device="cuda") for _ in range(3)]
        w_seg = kst.kst_segregate_weights(wd)
        need = kst.kst_workspace_bytes_padded(layer.B, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, dt)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        return lambda i: kst.kst_forward_seg_padded(xd[i % 3], w_seg, layer.Cout, layer.n, layer.P, out=outs[i % 3], ws=ws)
    g = torch.randn(layer.out_shape, dtype=torch.float32, device="cuda")
    if what == "backward_input":
        din = torch.empty(layer.in_shape, dtype=torch.float32, device="cuda")
        ws = torch.empty(max(kst.kst_backward_input_workspace_bytes(
            layer.B, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, dt), 16), dtype=torch.uint8, device="cuda")
        return lambda i: kst.kst_backward_input(g, wd, layer.N, layer.P, din=din, ws=ws)
    dw = torch.empty(layer.w_shape, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(kst.kst_backward_weight_workspace_bytes(
        layer.B, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, dt), 16), dtype=torch.uint8, device="cuda")
    return lambda i: kst.kst_backward_weight(xd[0], g, layer.n, layer.P, dw=dw, ws=ws)


def measured_traffic():
    """HBM bytes per forward launch of each layer, read from the committed counter summary
    (profiles/hbm_traffic_pmc.txt: table rows `layer | kernel | ... | HBM bytes | ...`; a layer's
    kernels add up).  Measurements of an earlier run of these kernels, quoted beside the live timing."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")
    out = {}
    try:
        with open(path) as f:
            for line in f:
                cells = [c.strip() for c in line.split("|")]
                if len(cells) >= 6 and cells[0].startswith(("cfg", "table")) and cells[4].isdigit():
                    out[cells[0]] = out.get(cells[0], 0) + int(cells[4])
    except OSError:
        pass
    return out


def roofline_for(layer, ms, metrics):
    """Roofline entry of the forward kernel of `layer` given its launch time."""
    direct = layer.Cout < 16 or layer.Cin < 8
    if direct:
        a = metrics.algorithmic_bytes(layer) / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(a, 1), "peak": metrics.HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(a / metrics.HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(layer.name)}
    peak = metrics.MFMA_PEAK_TFLOPS[layer.dtype]
    a = 2.0 * metrics.useful_macs(layer) / (ms * 1e-3) / 1e12
    return {"bound": "mfma", "achieved": round(a, 2), "peak": peak, "unit": "TFLOP/s",
            "frac": round(a / peak, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(layer.name)}


def paper_roofline(layer, fwd_ms, din_ms, dw_ms, metrics):
    """Roofline fractions of a paper-shaped layer's three passes.  Many-channel layers are priced
    against the fp32 matrix-core peak (each gradient does the forward's useful MACs once), the
    few-channel ones against HBM (the forward by its algorithmic bytes; the gradients read `g` and
    the other operand and write the gradient: the same byte count)."""
    macs = metrics.useful_macs(layer)
    many = layer.Cin >= 8 and layer.Cout >= 16
    # Few output channels fed by many input channels (the 128 -> 3 output layer of the generators):
    # 2 * useful MACs / algorithmic bytes = 22 flop/B, past the ridge of the vector ALUs
    # (157.3 TFLOP/s / 8 TB/s = 19.7 flop/B), and too narrow for the matrix cores with the output
    # channels down the MFMA rows (3 of 32): the gradients run on the vector ALUs and are priced
    # against the fp32 vector peak; the forward pass of a batch runs on the matrix cores with the
    # taps of all sub-kernels as rows (48 of 48), whose fp32 peak is the same 157.3 TFLOP/s.  The
    # HBM fraction is given beside it.
    alu = not many and 2.0 * macs / metrics.algorithmic_bytes(layer) > metrics.VALU_PEAK_TFLOPS * 1e12 / (metrics.HBM_PEAK_GBS * 1e9)
    out = {"bound": "mfma" if many else "alu" if alu else "hbm"}
    if alu:
        out["forward_bound"] = "mfma"
    for name, ms in (("forward", fwd_ms), ("backward_input", din_ms), ("backward_weight", dw_ms)):
        if many:
            out[name + "_frac"] = round(2.0 * macs / (ms * 1e-3) / 1e12 / metrics.MFMA_PEAK_TFLOPS["f32"], 4)
        elif alu:
            out[name + "_frac"] = round(2.0 * macs / (ms * 1e-3) / 1e12 / metrics.VALU_PEAK_TFLOPS, 4)
            out[name + "_hbm_frac"] = round(metrics.algorithmic_bytes(layer) / (ms * 1e-3) / 1e9 / metrics.HBM_PEAK_GBS, 4)
        else:
            out[name + "_frac"] = round(metrics.algorithmic_bytes(layer) / (ms * 1e-3) / 1e9 / metrics.HBM_PEAK_GBS, 4)
    return out


def cpu_baseline(layer, host, metrics, wl, budget_s=12.0):
    """The fp64 zero-insert oracle on the host cores, on a bounded sample of the workload: as many
    batch items as fit the budget, repeated until about budget_s seconds of work have been timed."""
    import oracle
    x, w = host
    x64, w64 = wl.to_f64(x), wl.to_f64(w)
    per_item = metrics.useful_macs(layer) / layer.B
    t0 = time.perf_counter()
    oracle.forward(x64[:1], w64)
    t1 = time.perf_counter() - t0
    items = int(max(1, min(layer.B, budget_s / max(t1, 1e-6))))
    reps, total = 0, 0.0
    while reps == 0 or (total < budget_s and reps < 1000):
        t0 = time.perf_counter()
        oracle.forward(x64[:items], w64)
        total += time.perf_counter() - t0
        reps += 1
    # the oracle shares its work over output channels only (one thread per plane of a batch item)
    used = max(1, min(oracle.threads(), layer.Cout))
    return {"value": round(per_item * items * reps / total / 1e9, 4), "unit": "GMAC/s", "cores": used,
            "kind": "oracle",
            "sample": "%d x (%d of %d batch items of %s), fp64 zero-insert + Eq. 1, %.1f s" % (
                reps, items, layer.B, layer.name, total)}


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (--gpus 1 only)")
    import torch

    from paper_2209_03704_amd import binding as kst
    from paper_2209_03704_amd import metrics
    from paper_2209_03704_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    kst.lib()   # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    MEASURED_TRAFFIC_BYTES.update(measured_traffic())

    def fwd_seg(r):
        L = r.layer
        return lambda i: kst.kst_forward_seg(r.x[i % r.sets], r.w_seg, L.Cout, L.n, out=r.out[i % r.sets], ws=r.ws)

    def whole_path(r):
        L = r.layer

        def step(i):
            kst.kst_segregate_weights(r.w, r.w_seg)
            kst.kst_forward_seg(r.x[i % r.sets], r.w_seg, L.Cout, L.n, out=r.out[i % r.sets], ws=r.ws)
        return step

    if args.only == "copy":
        # A plain device copy of known size (256 MiB read + 256 MiB written per launch): the
        # yardstick the HBM counters and the achievable bandwidth are scaled by.
        n = 64 * 1024 * 1024
        bufs = [(torch.empty(n, dtype=torch.float32, device="cuda").normal_(),
                 torch.empty(n, dtype=torch.float32, device="cuda")) for _ in range(3)]
        ms = time_launches(torch, lambda i: bufs[i % 3][1].copy_(bufs[i % 3][0]), args.steps, args.warmup)
        print(json.dumps({"kernel": "copy", "bytes_read": 4 * n, "bytes_written": 4 * n, "kernel_ms": ms,
                          "GB_per_s": round(8 * n / (ms * 1e-3) / 1e9, 1)}))
        return
    if args.only:
        layer = wl.layer_by_name(args.only)
        fn = one_pass(layer, args.what, torch, kst, wl)
        settle(torch, fn, 0.05)
        ms = time_launches(torch, fn, args.steps, args.warmup)
        line = {"layer": layer.name, "pass": args.what, "kernel_ms": ms}
        if args.what == "forward" and layer.P == 0:
            line["roofline"] = roofline_for(layer, ms, metrics)
        print(json.dumps(line))
        return

    # ---- headline: whole path on the bandwidth-bound single-channel layer ----------------
    head = wl.LAYERS[1]
    r = Resident(head, 3, torch, kst, wl)
    step = whole_path(r)
    # Let the clocks settle: the first ~10 ms of work after an idle period run several per cent
    # slower than the steady state, whatever the kernel.  Untimed, before the W warm-up steps.
    t_settle = time.perf_counter()
    i = 0
    while time.perf_counter() - t_settle < 0.25:
        for _ in range(50):
            step(i)
            i += 1
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = time_launches(torch, fwd_seg(r), args.steps, args.warmup)
    value = metrics.useful_macs(head) / (ms_per_step * 1e-3) / 1e9
    roof = roofline_for(head, kernel_ms, metrics)
    roof["kernel"] = "direct forward (kst_forward_seg)"
    roof["kernel_us"] = round(kernel_ms * 1e3, 2)

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(head, r.host, metrics, wl)
    del r
    torch.cuda.empty_cache()

    # ---- yardsticks: what the chip sustains with nothing in the way --------------------------
    yard = None
    if args.layers == "all":
        n = 64 * 1024 * 1024
        cb = [(torch.empty(n, dtype=torch.float32, device="cuda").normal_(),
               torch.empty(n, dtype=torch.float32, device="cuda")) for _ in range(3)]
        copy_ms = time_launches(torch, lambda i: kst.kst_yardstick_copy(cb[i % 3][0], cb[i % 3][1]), 30, 5)
        del cb
        torch.cuda.empty_cache()
        sink = torch.empty(kst.kst_yardstick_mfma_sink_elems(), dtype=torch.float32, device="cuda")
        f32_it, bf16_it = 2048, 4096
        f32_ms = time_launches(torch, lambda i: kst.kst_yardstick_mfma(kst.KST_F32, f32_it, sink), 30, 10)
        bf16_ms = time_launches(torch, lambda i: kst.kst_yardstick_mfma(kst.KST_BF16, bf16_it, sink), 30, 10)
        yard = {
            "copy_GB_per_s": round(8 * n / (copy_ms * 1e-3) / 1e9, 1),
            "mfma_TFLOP_per_s": {
                "f32": round(kst.kst_yardstick_mfma_flops(kst.KST_F32, f32_it) / (f32_ms * 1e-3) / 1e12, 1),
                "bf16": round(kst.kst_yardstick_mfma_flops(kst.KST_BF16, bf16_it) / (bf16_ms * 1e-3) / 1e12, 1)},
            "what": "256 MiB streaming copy (bytes read + written); loops of matrix-core instructions only, "
                    "two waves per SIMD on all CUs",
        }
        del sink

    def of_measured(layer, roof_l):
        if yard is None:
            return None
        if roof_l["bound"] == "hbm":
            return round(roof_l["achieved"] / yard["copy_GB_per_s"], 4)
        return round(roof_l["achieved"] / yard["mfma_TFLOP_per_s"][layer.dtype], 4)

    # ---- per-layer table ---------------------------------------------------------------------
    table = []
    if args.layers == "all":
        for layer in wl.LAYERS:
            r = Resident(layer, 3, torch, kst, wl)
            kst.kst_segregate_weights(r.w, r.w_seg)
            iters = max(5, min(args.steps, 30))
            settle(torch, fwd_seg(r), 0.05)
            ms = time_launches(torch, fwd_seg(r), iters, 3)
            med_ms, min_ms = launch_spread(torch, fwd_seg(r), 50, 5)
            seg_ms = time_launches(torch, lambda i: kst.kst_segregate_weights(r.w, r.w_seg), 10, 2)
            U = torch.empty((layer.B, layer.Cin, 2 * layer.N - 1, 2 * layer.N - 1), dtype=r.w.dtype, device="cuda")
            zi_ms = time_launches(
                torch, lambda i: kst.kst_forward_zero_insert(r.x[0], r.w, U=U, out=r.out[0]), 2, 1)
            # (settled again: the zero-insert launches above take tens of milliseconds each and leave the
            # clocks elsewhere; measured without it kst_forward read 5 % slower than the same two
            # launches through the caller's buffers, in isolation they are equal)
            unseg = lambda i: kst.kst_forward(r.x[i % r.sets], r.w, out=r.out[i % r.sets])
            settle(torch, unseg, 0.05)
            unseg_ms = time_launches(torch, unseg, iters, 5)
            parts_ms = time_launches(torch, whole_path(r), iters, 5)
            # the same layer with a bias and a ReLU applied at the stores
            bias = torch.zeros(layer.Cout, dtype=torch.float32, device="cuda")
            epi_ms = time_launches(torch, lambda i: kst.kst_forward_seg_epilogue(
                r.x[i % r.sets], r.w_seg, layer.Cout, layer.n, bias, kst.KST_ACT_RELU, 0, out=r.out[i % r.sets],
                ws=r.ws), iters, 3)
            roof_l = roofline_for(layer, ms, metrics)
            roof_l["frac_of_measured_yardstick"] = of_measured(layer, roof_l)
            table.append({
                "layer": layer.name,
                "shape": {"B": layer.B, "Cin": layer.Cin, "Cout": layer.Cout, "N": layer.N, "n": layer.n,
                          "dtype": layer.dtype},
                "forward_us": round(ms * 1e3, 2),
                "forward_us_median_of_50": round(med_ms * 1e3, 2),
                "forward_us_min_of_50": round(min_ms * 1e3, 2),
                "segregate_us": round(seg_ms * 1e3, 2),
                "forward_unsegregated_w_us": round(unseg_ms * 1e3, 2),              # kst_forward
                "segregate_then_forward_us": round(parts_ms * 1e3, 2),              # its two parts, caller's buffers
                "forward_bias_relu_us": round(epi_ms * 1e3, 2),                     # kst_forward_seg_epilogue
                "useful_GMAC_per_s": round(metrics.useful_macs(layer) / (ms * 1e-3) / 1e9, 1),
                "algorithmic_GB_per_s": round(metrics.algorithmic_bytes(layer) / (ms * 1e-3) / 1e9, 1),
                "hbm_frac": round(metrics.algorithmic_bytes(layer) / (ms * 1e-3) / 1e9 / metrics.HBM_PEAK_GBS, 4),
                "roofline": roof_l,
                "zero_insert_us": round(zi_ms * 1e3, 1),
                "speedup_vs_zero_insert": round(zi_ms / ms, 2),
                "algorithmic_mac_ratio": round(metrics.conventional_macs(layer) / metrics.useful_macs(layer), 3),
            })
            del r, U
            torch.cuda.empty_cache()

    # ---- the paper's own shapes (padding factor 2), framed-input entry point -------------------
    paper_table = []
    if args.layers == "all":
        for layer in wl.PAPER_LAYERS:
            x, w = wl.make_tensors(layer)
            xd = [x.cuda().clone() for _ in range(3)]
            outs = [torch.empty(layer.out_shape, dtype=torch.float32, device="cuda") for _ in range(3)]
            w_seg = kst.kst_segregate_weights(w.cuda())
            need = kst.kst_workspace_bytes_padded(layer.B, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, kst.KST_F32)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
            fwd_p = lambda i: kst.kst_forward_seg_padded(xd[i % 3], w_seg, layer.Cout, layer.n, layer.P,
                                                         out=outs[i % 3], ws=ws)
            settle(torch, fwd_p, 0.03)
            ms = time_launches(torch, fwd_p, 30, 5)
            # gradients of the same layer: g = d(loss)/d(out)
            g = torch.randn(layer.out_shape, dtype=torch.float32, device="cuda")
            wd = w.cuda()
            din = torch.empty((layer.B, layer.Cin, layer.N, layer.N), dtype=torch.float32, device="cuda")
            dw = torch.empty_like(wd)
            dt_code = kst.KST_F32
            ws_bi = torch.empty(max(kst.kst_backward_input_workspace_bytes(
                layer.B, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, dt_code), 16), dtype=torch.uint8, device="cuda")
            ws_bw = torch.empty(max(kst.kst_backward_weight_workspace_bytes(
                layer.B, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, dt_code), 16), dtype=torch.uint8, device="cuda")
            bi = lambda i: kst.kst_backward_input(g, wd, layer.N, layer.P, din=din, ws=ws_bi)
            bw = lambda i: kst.kst_backward_weight(xd[0], g, layer.n, layer.P, dw=dw, ws=ws_bw)
            settle(torch, bi, 0.03)
            bi_ms = time_launches(torch, bi, 10, 2)
            settle(torch, bw, 0.03)
            bw_ms = time_launches(torch, bw, 10, 2)
            del g, din, dw, ws_bi, ws_bw
            paper_table.append({
                "layer": layer.name,
                "shape": {"B": layer.B, "Cin": layer.Cin, "Cout": layer.Cout, "N": layer.N, "n": layer.n,
                          "P": layer.P, "M": layer.M, "dtype": layer.dtype},
                "forward_us": round(ms * 1e3, 2),
                "us_per_image": round(ms * 1e3 / layer.B, 3),
                "useful_GMAC_per_s": round(metrics.useful_macs(layer) / (ms * 1e-3) / 1e9, 1),
                "algorithmic_GB_per_s": round(metrics.algorithmic_bytes(layer) / (ms * 1e-3) / 1e9, 1),
                "algorithmic_mac_ratio": round(metrics.conventional_macs(layer) / metrics.useful_macs(layer), 3),
                "backward_input_us": round(bi_ms * 1e3, 1),
                "backward_weight_us": round(bw_ms * 1e3, 1),
                "roofline": paper_roofline(layer, ms, bi_ms, bw_ms, metrics),
            })
            del xd, outs, ws
            torch.cuda.empty_cache()

    # ---- Table 1's first rows: a whole class of 769 images per launch ----------------------------
    class_rows = []
    if args.layers == "all":
        for layer, paper_s in wl.table1_class_layers():
            x, w = wl.make_tensors(layer)
            xd = [x.cuda(), x.cuda().clone()]
            outs = [torch.empty(layer.out_shape, dtype=torch.float32, device="cuda") for _ in range(2)]
            w_seg = kst.kst_segregate_weights(w.cuda())
            need = kst.kst_workspace_bytes_padded(layer.B, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, kst.KST_F32)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
            fwd_c = lambda i: kst.kst_forward_seg_padded(xd[i % 2], w_seg, layer.Cout, layer.n, layer.P,
                                                         out=outs[i % 2], ws=ws)
            settle(torch, fwd_c, 0.03)
            ms = time_launches(torch, fwd_c, 20, 3)
            class_rows.append({
                "layer": layer.name,
                "shape": {"images": layer.B, "Cin": layer.Cin, "Cout": layer.Cout, "N": layer.N, "n": layer.n, "P": layer.P,
                          "M": layer.M},
                "forward_us": round(ms * 1e3, 1),
                "us_per_image": round(ms * 1e3 / layer.B, 3),
                "hbm_frac": round(metrics.algorithmic_bytes(layer) / (ms * 1e-3) / 1e9 / metrics.HBM_PEAK_GBS, 4),
                "paper_rtx2070_proposed_s": paper_s[1],
                "paper_rtx2070_conventional_s": paper_s[0],
                "paper_xeon_proposed_s": paper_s[3],
            })
            del xd, outs, ws, x
            torch.cuda.empty_cache()

    # ---- Table 3's generator layers on one input sample, as the paper times them ---------------
    one_sample = []
    if args.layers == "all":
        for model in wl.TABLE3_GENERATORS:
            rows, tot_seg, tot_whole, tot_paper = [], 0.0, 0.0, 0.0
            for layer, paper_s in wl.table3_layers(model, 1):
                x, w = wl.make_tensors(layer)
                xd, wd = x.cuda(), w.cuda()
                out = torch.empty(layer.out_shape, dtype=torch.float32, device="cuda")
                w_seg = kst.kst_segregate_weights(wd)
                need = kst.kst_workspace_bytes_padded(1, layer.Cin, layer.Cout, layer.N, layer.n, layer.P, kst.KST_F32)
                ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
                f_seg = lambda i: kst.kst_forward_seg_padded(xd, w_seg, layer.Cout, layer.n, layer.P, out=out, ws=ws)
                f_all = lambda i: kst.kst_forward_padded(xd, wd, layer.P, out=out)
                settle(torch, f_seg, 0.02)
                seg_ms = time_launches(torch, f_seg, 30, 5)
                whole_ms = time_launches(torch, f_all, 30, 5)
                # a sample reads every weight once: weights + maps are the bytes that must move
                bytes_min = 4 * (layer.Cin * layer.Cout * 16 + layer.Cin * layer.N ** 2 + layer.Cout * layer.M ** 2)
                rows.append({
                    "layer": layer.name,
                    "shape": {"Cin": layer.Cin, "Cout": layer.Cout, "N": layer.N, "M": layer.M},
                    "forward_seg_us": round(seg_ms * 1e3, 2),
                    "forward_unsegregated_w_us": round(whole_ms * 1e3, 2),
                    "hbm_frac": round(bytes_min / (seg_ms * 1e-3) / 1e9 / metrics.HBM_PEAK_GBS, 4),
                    "paper_rtx2070_proposed_us": round(paper_s[1] * 1e6, 1),
                    "paper_rtx2070_conventional_us": round(paper_s[0] * 1e6, 1),
                    "paper_xeon_proposed_us": round(paper_s[3] * 1e6, 1),
                })
                tot_seg += seg_ms
                tot_whole += whole_ms
                tot_paper += paper_s[1]
                del xd, wd, out, w_seg, ws
            torch.cuda.empty_cache()
            one_sample.append({"model": model, "layers": rows,
                               "total_forward_seg_us": round(tot_seg * 1e3, 1),
                               "total_forward_unsegregated_w_us": round(tot_whole * 1e3, 1),
                               "paper_rtx2070_proposed_total_us": round(tot_paper * 1e6, 1)})

    line = {
        "metric": "useful GMAC/s (segregated transpose convolution, whole path)",
        "value": round(value, 1),
        "unit": "GMAC/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": head.name, "B": head.B, "Cin": head.Cin, "Cout": head.Cout, "N": head.N,
                   "n": head.n, "out": list(head.out_shape),
                   "step": "kst_segregate_weights + kst_forward_seg, inputs resident in HBM, 3 rotating buffer sets"},
        "roofline": roof,
        "cpu_baseline": cpu,
        "yardsticks": yard,
        "layers": table,
        "paper_shaped_layers": paper_table,
        "table1_class_of_769_images": class_rows,
        "table3_one_sample": one_sample,
        "paper_context": "paper reports 3.7x (Xeon CPU) / 3.4x (RTX 2070) average speed-up over zero-insert; ideal 4x",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
