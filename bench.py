#!/usr/bin/env python3
"""Benchmark of the forward-convolution hot path on one MI355X.

A "step" is one pass of the whole path (validate, select variant, launch)
over the VGG-16-style 3x3 sweep at batch 16 (five layers, fp32, stride 1, SAME
padding), inputs and filters resident in HBM before the timed region.  The
metric is conv2d forward TFLOP/s with the direct-convolution flop count
2*N*P*Q*K*R*S*C (padded taps count as work).

Prints ONE JSON line.  Besides the contract's fields it carries
  roofline     -- the layer with the largest share of the step, from HIP events on the launch
                  stream: its flop rate against the MFMA peak of the element type, or, for a
                  layer whose flop per algorithmic byte lies under the ridge, its algorithmic
                  bytes per second against the HBM peak
  cpu_baseline -- the CPU oracle timed on a bounded sample of the same workload
  groups       -- every other configuration group (bf16 VGG sweep, VGG at batch 1, ResNet-style
                  layers at batch 32 in fp32 and bf16, the large-batch layer and its VALID /
                  stride-2 forms, the tiny case): per layer ms, TFLOP/s and the fraction of the
                  layer's own bound (the larger of flop / MFMA peak and algorithmic bytes / HBM
                  peak, over the measured time; cold caches where rotating buffers are feasible)
  ceilings     -- the reachable rates of this GPU measured in the same process (register-only
                  MFMA loop, LDS fragment reads, streaming copy); roofline.achievable_peak is
                  the one that belongs to the roofline's bound
  layers       -- per-layer times (context): back to back on one buffer set (`ms`: mean;
                  `median_ms`, `min_ms`: per launch, from an event between launches) and rotating
                  over more than 1 GiB of buffer sets (`cold_ms`, large layers only)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2516.6}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0

def measured_traffic():
    """HBM bytes per launch (all kernels of a call) per "dtype|layer|variant", as written by
    `python -m paper_1904_04174_amd.profile_summary --json` from two rocprofv3 --pmc runs
    (FETCH_SIZE, WRITE_SIZE, scaled on a copy of known size).  Not measurable inside this
    process; keyed by the variant as well, so that another selection reports null, not a wrong
    figure."""
    path = os.path.join(ROOT, "paper_1904_04174_amd", "measured_traffic.json")
    if not os.path.exists(path):
        return {}
    with open(path) as fh:
        return json.load(fh)


def layer_flops(B, p):
    g = B.conv2d_get_geometry(p)
    return (2.0 * p.batch * g.out_rows * g.out_cols * p.features *
            p.window_rows * p.window_cols * p.channels)


def layer_bytes(B, p):
    """Algorithmic bytes: input (its touched pixels) read once + filter read once + output
    written once."""
    g = B.conv2d_get_geometry(p)
    isz = 4 if p.in_dtype == B.F32 else 2
    osz = 4 if p.out_dtype == B.F32 else 2
    # a window that is no larger than the stride skips pixels: only the touched ones count
    rows = min(p.in_rows, g.out_rows * p.window_rows) if p.stride_rows >= p.window_rows else p.in_rows
    cols = min(p.in_cols, g.out_cols * p.window_cols) if p.stride_cols >= p.window_cols else p.in_cols
    return (isz * p.batch * rows * cols * p.channels +
            isz * p.window_rows * p.window_cols * p.channels * p.features +
            osz * p.batch * g.out_rows * g.out_cols * p.features)


def measure_ceilings():
    """{name: (value, unit)} from the ceilings helper library (register-only MFMA loops, LDS
    read loops, streaming copies), or None if it is not built."""
    import ctypes
    path = os.path.join(ROOT, "paper_1904_04174_amd", "libconv2d_ceilings.so")
    if not os.path.exists(path):
        return None

    class Record(ctypes.Structure):
        _fields_ = [("name", ctypes.c_char * 64), ("value", ctypes.c_double),
                    ("unit", ctypes.c_char * 16)]
    lib = ctypes.CDLL(path)
    buf = (Record * 64)()
    n = lib.conv2d_ceilings_measure(buf, 64)
    if n < 0:
        return None
    return {buf[i].name.decode(): (round(buf[i].value, 2), buf[i].unit.decode()) for i in range(n)}


# The configuration groups beside the headline sweep: (key, dtype, layer names).
def config_groups(wl):
    return [
        ("vgg_n16_bf16", "bf16", wl.VGG_N16),
        ("vgg_n1_f32", "f32", wl.VGG_N1),
        ("resnet_n32_f32", "f32", ["R7x7", "R1x1a", "R1x1b", "R3x3", "R1x1s2"]),
        ("resnet_n32_bf16", "bf16", ["R3x3", "R1x1a", "R1x1b", "R1x1s2"]),
        ("large_batch_f32", "f32", ["L-same", "L-valid", "L-s2"]),
        ("tiny_f32", "f32", ["T1"]),
    ]


def time_group(torch, B, wl, stream, dtype, names, reps=20):
    """Per layer of a group: mean ms of back-to-back calls of conv2d_forward's direct-sum
    selection (repack and reduce kernels included), a cold-cache ms where at most 64 rotating
    buffer sets exceed 1.25 GiB, TFLOP/s, and the fraction of the layer's own bound."""
    dev = torch.device("cuda:0")
    in_dtype = B.F32 if dtype == "f32" else B.BF16
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    handle = stream.cuda_stream
    rows = []
    for name in names:
        L = wl.ALL_LAYERS[name]
        x, f = wl.make_inputs(L)
        p = B.params_of_layer(L, in_dtype, B.F32)
        xd = torch.from_numpy(x).to(dev).to(tdt).contiguous()
        fd = torch.from_numpy(f).to(dev).to(tdt).contiguous()
        del x, f
        g = B.conv2d_get_geometry(p)
        out = torch.empty((p.batch, g.out_rows, g.out_cols, p.features), dtype=torch.float32,
                          device=dev)
        vid = B.conv2d_select_variant(p, B.SELECT_DIRECT_SUM_ONLY)
        ws_bytes = B.conv2d_workspace_size(p, vid)
        ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=dev)
        ws_ptr = ws.data_ptr() if ws_bytes else 0
        flops, nbytes = layer_flops(B, p), layer_bytes(B, p)

        def call(xp, op):
            rc = B.conv2d_forward_raw(p, xp, fd.data_ptr(), op, ws_ptr, ws_bytes, handle, vid)
            if rc:
                raise B.Conv2dError(rc, "conv2d_forward(%s)" % name)
        n = reps if flops > 2e9 else 10 * reps
        for _ in range(3):
            call(xd.data_ptr(), out.data_ptr())
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            call(xd.data_ptr(), out.data_ptr())
        e1.record(stream)
        stream.synchronize()
        ms = e0.elapsed_time(e1) / n
        cold_ms = None
        per_set = xd.numel() * xd.element_size() + out.numel() * 4
        sets = -(-(5 << 28) // per_set)
        if 2 <= sets <= 64:
            xs = [xd] + [xd.clone() for _ in range(sets - 1)]
            outs = [out] + [torch.empty_like(out) for _ in range(sets - 1)]
            torch.cuda.synchronize()
            for xx, oo in zip(xs, outs):
                call(xx.data_ptr(), oo.data_ptr())
            rounds = max(2, -(-n // sets))
            e0.record(stream)
            for _ in range(rounds):
                for xx, oo in zip(xs, outs):
                    call(xx.data_ptr(), oo.data_ptr())
            e1.record(stream)
            stream.synchronize()
            cold_ms = e0.elapsed_time(e1) / (rounds * sets)
            del xs, outs
        t_mfma = flops / (PEAK_TFLOPS[dtype] * 1e12) * 1e3
        t_hbm = nbytes / (PEAK_HBM_GBS * 1e9) * 1e3
        bound_ms = max(t_mfma, t_hbm)
        rows.append({"name": name, "variant": B.conv2d_variant_name(vid), "ms": round(ms, 5),
                     "cold_ms": None if cold_ms is None else round(cold_ms, 5),
                     "tflops": round(flops / (ms * 1e-3) / 1e12, 2),
                     "cold_tflops": None if cold_ms is None else
                     round(flops / (cold_ms * 1e-3) / 1e12, 2),
                     "alg_gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "cold_alg_gbs": None if cold_ms is None else
                     round(nbytes / (cold_ms * 1e-3) / 1e9, 1),
                     "bound": "mfma" if t_mfma >= t_hbm else "hbm",
                     "bound_ms": round(bound_ms, 5),
                     "frac_of_bound": round(bound_ms / ms, 4),
                     "frac_of_bound_cold": None if cold_ms is None else
                     round(bound_ms / cold_ms, 4)})
        del xd, fd, out, ws
    total_flops = sum(layer_flops(B, B.params_of_layer(wl.ALL_LAYERS[n_], in_dtype, B.F32))
                      for n_ in names)
    total_ms = sum(r["ms"] for r in rows)
    return {"dtype": dtype, "tflops": round(total_flops / (total_ms * 1e-3) / 1e12, 2),
            "ms": round(total_ms, 5),
            "note": "ms: back-to-back calls on one buffer set; cold_ms: rotating over more than "
                    "1.25 GiB of buffer sets (null where that takes more than 64 sets)",
            "layers": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32")
    ap.add_argument("--workload", choices=["vgg16", "resnet50"], default="vgg16",
                    help="vgg16: the five VGG-style 3x3 layers at batch 16 (the headline workload); "
                         "resnet50: the 26 distinct ResNet-50 convolution shapes (--batch 1, 4 or 32) "
                         "(the workload of the paper's Figure 1)")
    ap.add_argument("--algorithms", choices=["direct", "all"], default="direct",
                    help="direct: the selector's pick among the variants that sum the window "
                         "directly, so that the executed multiply-adds are the metric's (default); "
                         "all: also the Winograd variants, which execute 2.25x fewer and can "
                         "therefore exceed the MFMA peak in the metric's terms")
    ap.add_argument("--skip-all-algorithms-leg", action="store_true",
                    help="with --algorithms direct: do not also time the unrestricted selection "
                         "and the packed-filter leg (keeps a profile of the run to the headline's "
                         "kernels)")
    ap.add_argument("--batch", type=int, choices=[1, 4, 32], default=32,
                    help="batch size of the resnet50 workload (the paper's Figures 1-3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the per-layer timing that rotates over more than 1 GiB of distinct "
                         "input/output buffers (the cold-cache figures in `layers`)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="lower bound on the CPU oracle's timed work")
    ap.add_argument("--variant", default=None,
                    help="with --only: run this variant (by name) instead of the selector's pick")
    ap.add_argument("--only", default=None,
                    help="profile mode: launch only this layer (any name in workloads.LAYERS) "
                         "--steps times, plus one device-to-device copy of --copy-mb MiB as the "
                         "known-size reference for memory counters; prints no JSON")
    ap.add_argument("--copy-mb", type=int, default=256)
    ap.add_argument("--ceilings", action="store_true",
                    help="only measure this GPU's reachable rates (register-only MFMA loops, LDS "
                         "fragment reads, streaming copies) and print them, one per line")
    ap.add_argument("--no-groups", action="store_true",
                    help="skip the other configuration groups (the `groups` key)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); "
                 "use --gpus 1")

    import torch

    from paper_1904_04174_amd import binding as B
    from paper_1904_04174_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs the GPU")
    if args.ceilings:
        torch.cuda.init()
        torch.zeros(1, device="cuda:0")
        c = measure_ceilings()
        if c is None:
            sys.exit("bench.py --ceilings: libconv2d_ceilings.so is not built or failed")
        for k, (v, u) in c.items():
            print("%-48s %12.2f %s" % (k, v, u))
        return
    dev = torch.device("cuda:0")
    in_dtype = B.F32 if args.dtype == "f32" else B.BF16
    tdt = torch.float32 if args.dtype == "f32" else torch.bfloat16

    if args.only:
        names = [args.only]
    elif args.workload == "resnet50":
        names = list(wl.RESNET50_BY_BATCH[args.batch])
    else:
        names = wl.VGG_N16
    layers = []
    for name in names:
        L = wl.ALL_LAYERS[name]
        x, f = wl.make_inputs(L, dist="uniform")
        p = B.params_of_layer(L, in_dtype, B.F32)
        xd = torch.from_numpy(x).to(dev).to(tdt).contiguous()
        fd = torch.from_numpy(f).to(dev).to(tdt).contiguous()
        g = B.conv2d_get_geometry(p)
        out = torch.empty((p.batch, g.out_rows, g.out_cols, p.features), dtype=torch.float32,
                          device=dev)
        vid = B.conv2d_select_variant(
            p, B.SELECT_DIRECT_SUM_ONLY if args.algorithms == "direct" else 0)
        if args.only and args.variant:
            vid = B.variant_id_by_name(args.variant)
        ws_bytes = B.conv2d_workspace_size(p, vid)
        ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=dev)
        layers.append(dict(name=name, layer=L, p=p, x=xd, f=fd, out=out, ws=ws, ws_bytes=ws_bytes,
                           vid=vid, flops=layer_flops(B, p), bytes=layer_bytes(B, p),
                           variant=B.conv2d_variant_name(vid)))
        del x, f

    stream = torch.cuda.Stream(device=dev)
    handle = stream.cuda_stream

    def launch(l):
        rc = B.conv2d_forward_raw(l["p"], l["x"].data_ptr(), l["f"].data_ptr(),
                                  l["out"].data_ptr(), l["ws"].data_ptr() if l["ws_bytes"] else 0,
                                  l["ws_bytes"], handle, l["vid"])
        if rc:
            raise B.Conv2dError(rc, "conv2d_forward(%s)" % l["name"])

    def step():
        for l in layers:
            launch(l)

    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    stream.synchronize()
    torch.cuda.synchronize()

    if args.only:
        # profile mode: the layer's kernels, then a plain copy of known size
        for _ in range(args.steps):
            step()
        stream.synchronize()
        n = args.copy_mb * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        l = layers[0]
        print("profiled %s (%s): %.3f GFLOP, %.1f MB algorithmic; reference copy: %d MiB read + "
              "%d MiB written" % (l["name"], l["variant"], l["flops"] / 1e9, l["bytes"] / 1e6,
                                  args.copy_mb, args.copy_mb))
        return

    # ---- timed region: exactly --steps passes over the sweep
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / args.steps
    total_flops = sum(l["flops"] for l in layers)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-layer kernel time from HIP events recorded on the launch stream
    reps = max(10, args.steps)
    for l in layers:
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        launch(l)
        e0.record(stream)
        for _ in range(reps):
            launch(l)
        e1.record(stream)
        stream.synchronize()
        l["ms"] = e0.elapsed_time(e1) / reps
    # ---- per launch: an event between consecutive launches (20 of them, 200 for layers under
    # 0.1 ms); median and minimum of the intervals
    for l in layers:
        n = 200 if l["ms"] < 0.1 else 20
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        launch(l)
        for i in range(n):
            evs[i].record(stream)
            launch(l)
        evs[n].record(stream)
        stream.synchronize()
        times = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n))
        l["median_ms"], l["min_ms"] = times[n // 2], times[0]

    # ---- the same per-layer time with cold caches: the launches rotate over enough distinct
    # input/output buffers (over 1 GiB together) that no launch finds its tensors in the 256 MB
    # last-level cache; only for layers large enough to get there with at most 16 buffer sets
    for l in layers:
        l["cold_ms"] = None
        per_set = l["x"].numel() * l["x"].element_size() + l["out"].numel() * 4
        sets = -(-(5 << 28) // per_set)
        if args.no_cold or sets > 16:
            continue
        sets = max(sets, 2)
        xs = [l["x"]] + [l["x"].clone() for _ in range(sets - 1)]
        outs = [l["out"]] + [torch.empty_like(l["out"]) for _ in range(sets - 1)]
        ws_ptr = l["ws"].data_ptr() if l["ws_bytes"] else 0
        calls = [(l["p"], x.data_ptr(), l["f"].data_ptr(), o.data_ptr(), ws_ptr, l["ws_bytes"],
                  handle, l["vid"]) for x, o in zip(xs, outs)]
        torch.cuda.synchronize()
        rounds = max(2, -(-reps // sets))
        for c in calls:
            B.conv2d_forward_raw(*c)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(rounds):
            for c in calls:
                B.conv2d_forward_raw(*c)
        e1.record(stream)
        stream.synchronize()
        l["cold_ms"] = e0.elapsed_time(e1) / (rounds * sets)
        del xs, outs
    dom = max(layers, key=lambda l: l["ms"])
    peak = PEAK_TFLOPS[args.dtype]
    achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
    # the layer is bound by the matrix cores unless its flop per algorithmic byte lies under the
    # ridge of the two peaks (fp32: 19.7 flop/B, bf16: 315): then by HBM
    ridge = peak * 1e12 / (PEAK_HBM_GBS * 1e9)
    hbm_bound = dom["flops"] / dom["bytes"] < ridge
    if hbm_bound:
        achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        peak = PEAK_HBM_GBS
    roofline = {"bound": "hbm" if hbm_bound else "mfma", "achieved": round(achieved, 3),
                "peak": peak, "unit": "GB/s" if hbm_bound else "TFLOP/s",
                "frac": round(achieved / peak, 4),
                "traffic": measured_traffic().get(
                    "%s|%s|%s" % (args.dtype, dom["name"], dom["variant"]),
                    {}).get("hbm_bytes_per_launch"),
                "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled)",
                "algorithmic_bytes_per_launch": dom["bytes"],
                "kernel": dom["variant"], "layer": dom["name"],
                "kernel_ms": round(dom["ms"], 4),
                "algorithmic_gflop_per_launch": round(dom["flops"] / 1e9, 3)}

    def time_packed():
        """ms per step of the sweep with every layer's filter packed ahead of time for its
        current variant, and the ms per call of each layer."""
        calls = []
        keep = []
        for l in layers:
            packed = B.conv2d_pack_filter(l["p"], l["vid"], l["f"])
            keep.append(packed)
            ws_ptr = l["ws"].data_ptr() if l["ws_bytes"] else 0
            calls.append((l["p"], l["vid"], l["x"].data_ptr(), packed.data_ptr(), 0, 0,
                          l["out"].data_ptr(), ws_ptr, l["ws_bytes"], handle))

        def packed_step():
            for a in calls:
                rc = B.conv2d_forward_packed_raw(*a)
                if rc:
                    raise B.Conv2dError(rc, "conv2d_forward_packed")
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            packed_step()
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            packed_step()
        stream.synchronize()
        torch.cuda.synchronize()
        ms_sweep = 1e3 * (time.perf_counter() - t0) / args.steps
        # per layer, from HIP events on the launch stream (as for the ordinary calls)
        per_layer = []
        for a in calls:
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            B.conv2d_forward_packed_raw(*a)
            e0.record(stream)
            for _ in range(reps):
                B.conv2d_forward_packed_raw(*a)
            e1.record(stream)
            stream.synchronize()
            per_layer.append(e0.elapsed_time(e1) / reps)
        return ms_sweep, per_layer

    # ---- the same sweep with the unrestricted selection (Winograd variants allowed), reported
    # beside the headline value: they execute 2.25x fewer multiply-adds than the metric counts
    with_transforms = None
    if args.algorithms == "direct" and not args.skip_all_algorithms_leg:
        changed = False
        for l in layers:
            vid = B.conv2d_select_variant(l["p"], 0)
            l["direct_vid"], l["direct_variant"] = l["vid"], l["variant"]
            l["direct_ws"], l["direct_ws_bytes"] = l["ws"], l["ws_bytes"]
            if vid != l["vid"]:
                changed = True
                l["vid"], l["variant"] = vid, B.conv2d_variant_name(vid)
                l["ws_bytes"] = B.conv2d_workspace_size(l["p"], vid)
                l["ws"] = torch.empty(max(l["ws_bytes"], 1), dtype=torch.uint8, device=dev)
        if changed:
            for _ in range(args.warmup):
                step()
            stream.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step()
            stream.synchronize()
            torch.cuda.synchronize()
            ms_all = 1e3 * (time.perf_counter() - t0) / args.steps
            with_transforms = {
                "value": round(total_flops / (ms_all * 1e-3) / 1e12, 3), "unit": "TFLOP/s",
                "ms_per_step": round(ms_all, 4),
                "variants": {l["name"]: l["variant"] for l in layers
                             if l["variant"] != l["direct_variant"]},
                "note": "conv2d_forward's own selection; the Winograd variants execute 2.25x "
                        "fewer multiply-adds than the metric counts, so this is not a fraction "
                        "of the MFMA peak"}
            ms_all_packed, _ = time_packed()
            with_transforms["packed_filters_value"] = round(
                total_flops / (ms_all_packed * 1e-3) / 1e12, 3)
            with_transforms["packed_filters_ms_per_step"] = round(ms_all_packed, 4)
        for l in layers:
            l["vid"], l["variant"] = l["direct_vid"], l["direct_variant"]
            l["ws"], l["ws_bytes"] = l["direct_ws"], l["direct_ws_bytes"]

    # ---- the same sweep (direct-sum selection) with the filters packed ahead of time
    # (conv2d_pack_filter once, outside the timed region; conv2d_forward_packed in it): what an
    # inference loop with constant filters runs.  Reported beside the headline value, which packs
    # the filter inside every call.
    packed_leg = None
    if args.algorithms == "direct" and not args.skip_all_algorithms_leg:
        ms_packed, ms_layers = time_packed()
        packed_leg = {
            "value": round(total_flops / (ms_packed * 1e-3) / 1e12, 3), "unit": "TFLOP/s",
            "ms_per_step": round(ms_packed, 4),
            "layers": [{"name": l["name"], "ms": round(ms, 4),
                        "tflops": round(l["flops"] / (ms * 1e-3) / 1e12, 2),
                        "frac_of_mfma_peak": round(l["flops"] / (ms * 1e-3) / 1e12 /
                                                   PEAK_TFLOPS[args.dtype], 4)}
                       for l, ms in zip(layers, ms_layers)],
            "note": "filters packed once outside the timed region (conv2d_pack_filter), "
                    "conv2d_forward_packed inside it; the headline value repacks in every call"}

    # ---- this GPU's reachable rates, measured now (a second or two), and the other groups
    ceilings = None if args.skip_all_algorithms_leg else measure_ceilings()
    if ceilings:
        key = ({"f32": "mfma_f32_32x32x2 x4acc", "bf16": "mfma_bf16_16x16x32 x8acc"}[args.dtype]
               if not hbm_bound else "hbm_copy (read+write)")
        roofline["achievable_peak"] = ceilings[key][0]
        roofline["achievable_peak_source"] = key + " (measured in this run)"
        roofline["frac_of_achievable"] = round(roofline["achieved"] / ceilings[key][0], 4)
    groups = None
    if (args.workload == "vgg16" and args.dtype == "f32" and args.algorithms == "direct"
            and not args.no_groups and not args.skip_all_algorithms_leg):
        groups = {}
        for key, dt, group_names in config_groups(wl):
            groups[key] = time_group(torch, B, wl, stream, dt, group_names)

    result = {
        "metric": "conv2d forward TFLOP/s (2*N*P*Q*K*R*S*C / time)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": ({"workload": "VGG-16-style 3x3 sweep, stride 1, SAME, N=16: "
                                "(224,64,64) (112,128,128) (56,256,256) (28,512,512) (14,512,512); "
                                "NHWC/HWCF, uniform[-1,1]",
                    "batch": 16, "layers": names, "algorithms": args.algorithms}
                   if args.workload == "vgg16" else
                   {"workload": "the 26 distinct ResNet-50 convolution shapes (7x7 stem, 1x1 and "
                                "3x3 bottleneck layers, stride 1 and 2), SAME, N=%d; NHWC/HWCF, " % args.batch +
                                "uniform[-1,1]",
                    "batch": args.batch, "layers": names, "algorithms": args.algorithms}),
        "frac_of_mfma_peak": round(value / PEAK_TFLOPS[args.dtype], 4),
        "roofline": roofline,
        "all_algorithms": with_transforms,
        "packed_filters": packed_leg,
        "groups": groups,
        "ceilings": ({k: {"value": v, "unit": u} for k, (v, u) in ceilings.items()}
                     if ceilings else None),
        "layers": [{"name": l["name"], "variant": l["variant"], "ms": round(l["ms"], 4),
                    "tflops": round(l["flops"] / (l["ms"] * 1e-3) / 1e12, 2),
                    "median_ms": round(l["median_ms"], 4), "min_ms": round(l["min_ms"], 4),
                    "alg_gbs": round(l["bytes"] / (l["ms"] * 1e-3) / 1e9, 1),
                    "cold_ms": None if l["cold_ms"] is None else round(l["cold_ms"], 4),
                    "cold_alg_gbs": None if l["cold_ms"] is None else
                    round(l["bytes"] / (l["cold_ms"] * 1e-3) / 1e9, 1)} for l in layers],
    }

    if not args.no_cpu_baseline:
        import oracle
        cpu_in = []
        for l in layers:
            L = l["layer"]
            x, f = wl.make_inputs(L, dist="uniform")
            if args.dtype == "bf16":
                x, _ = wl.round_to_bf16(x)
                f, _ = wl.round_to_bf16(f)
            cpu_in.append((L, x, f))
        cpu_flops, cpu_s, passes = 0.0, 0.0, 0
        while cpu_s < args.cpu_seconds and passes < 64:
            for (L, x, f), l in zip(cpu_in, layers):
                t = time.perf_counter()
                oracle.forward_f32(x, f, (L.stride_rows, L.stride_cols), L.padding)
                cpu_s += time.perf_counter() - t
                cpu_flops += l["flops"]
            passes += 1
        result["cpu_baseline"] = {
            "value": round(cpu_flops / cpu_s / 1e12, 5), "unit": "TFLOP/s",
            "cores": oracle.max_threads(), "kind": "oracle",
            "sample": "%d passes of the oracle over the same %d layers at full batch, "
                      "%.1f GFLOP in %.2f s" % (passes, len(layers), cpu_flops / 1e9, cpu_s)}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
