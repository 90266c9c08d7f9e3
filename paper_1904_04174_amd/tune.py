"""Per-device tuning of the variant selector.

The paper (section 3) tunes the choice of algorithm and of its parameters by
hand for each target device and names an automated search as future work.
This script is that search for one device: it times every variant that
supports a layer, through the C ABI's forced-variant entry point, for every
named layer in `workloads.LAYERS` and the ResNet-50 shapes at batch 1, 4 and 32 (fp32 and bf16;
of `LAYERS` only `workloads.BF16_LAYERS` in bf16),
and writes the winners as a table that the selector compiles in
(`csrc/tuned_table.inc`).  Shapes that are not in the table fall back to the
selector's cost model.

    python -m paper_1904_04174_amd.tune --out paper_1904_04174_amd/csrc/tuned_table.inc

Needs the GPU.  Rebuild the library afterwards.
"""
import argparse
import sys

from . import binding as B
from . import workloads as wl

SPLIT_PENALTY = 1.03   # a split-reduction variant must win by 3 % to be chosen (it needs scratch)
WINOGRAD_MARGIN = 1.05  # a Winograd variant must win by 5 % (its workspace is several inputs large)
MAX_WORKSPACE = 1 << 30


def time_variant(torch, layer, in_dtype, variant_id, iters, warmup=2):
    """Milliseconds per call of one forced variant on random data of the layer's shape."""
    tdt = torch.float32 if in_dtype == B.F32 else torch.bfloat16
    x = (torch.rand((layer.batch, layer.in_rows, layer.in_cols, layer.channels), device="cuda")
         * 2 - 1).to(tdt)
    f = (torch.rand((layer.window_rows, layer.window_cols, layer.channels, layer.features),
                    device="cuda") * 2 - 1).to(tdt)
    p = B.params_of_layer(layer, in_dtype, B.F32)
    need = B.conv2d_workspace_size(p, variant_id)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    out = B.conv2d_forward(p, x, f, workspace=ws, variant_id=variant_id)
    # pointer-level calls in the timed loop: the checks of the tensor-level wrapper cost more
    # host time than a small layer takes on the GPU
    stream = torch.cuda.current_stream().cuda_stream
    args = (p, x.data_ptr(), f.data_ptr(), out.data_ptr(), ws.data_ptr() if need else 0, need,
            stream, variant_id)
    for _ in range(warmup):
        B.conv2d_forward_raw(*args)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        B.conv2d_forward_raw(*args)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def candidates(params):
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    def elementwise(n):
        return "scalar" in n or n.endswith("_e") or "_e_" in n
    # (the zero-padded-channel variants and the window-row gather kernel run exactly where the
    # vector tiles cannot: they do not count as "vector tiles can run")
    vec_ok = any(B.conv2d_variant_supports(params, v) for v, n in enumerate(names)
                 if n != "direct" and not elementwise(n)
                 and not n.startswith(("padc_", "rowgather_")))
    for v, n in enumerate(names):
        if n == "direct" or not B.conv2d_variant_supports(params, v):
            continue
        if elementwise(n) and vec_ok:
            continue   # element-wise tiles only where the vector tiles cannot run
        if B.conv2d_workspace_size(params, v) > MAX_WORKSPACE:
            continue
        yield v, n


def tune_layer(torch, layer, in_dtype, repeats=2):
    p = B.params_of_layer(layer, in_dtype, B.F32)
    iters = 5 if layer.batch >= 64 else (10 if layer.batch >= 16 else (30 if layer.batch > 4 else 60))
    rows = []
    for v, n in candidates(p):
        ms = min(time_variant(torch, layer, in_dtype, v, iters) for _ in range(repeats))
        rows.append((ms * (SPLIT_PENALTY if n.endswith("_splitk") else 1.0), ms, n))
    rows.sort()
    return rows


FAMILIES = (
    ("register-staged implicit GEMM", lambda n: n.startswith("igemm_") and not n.startswith(
        ("igemm_dma_", "igemm_patch_"))),
    ("direct-to-LDS implicit GEMM", lambda n: n.startswith(("igemm_dma_", "padc_"))),
    ("LDS-resident patch", lambda n: n.startswith("igemm_patch_")),
    ("Winograd F(2x2,3x3), transform passes", lambda n: n.startswith("winograd2x2_") and "_lds_" not in n),
    ("Winograd F(2x2,3x3), one launch", lambda n: n.startswith("winograd2x2_lds_")),
    ("window-row gather", lambda n: n.startswith("rowgather_")),
    ("1x1 streaming", lambda n: n.startswith("conv1x1_")),
    ("3x3, filter in registers", lambda n: n.startswith("conv3x3_")),
)


def family_report(results):
    """Markdown table: per layer the best time of each kernel family (the per-layer algorithm
    comparison of the paper's Figure 1, for this library's families)."""
    lines = ["dtype | layer | GFLOP | " + " | ".join(f for f, _ in FAMILIES) + " | best variant",
             "---|---|---|" + "---|" * len(FAMILIES) + "---"]
    for dt, name, gflop, rows in results:
        cells = []
        for _, pred in FAMILIES:
            mine = [ms for _, ms, n in rows if pred(n)]
            cells.append("%.1f us (%.1f TFLOP/s)" % (min(mine) * 1e3, gflop / min(mine))
                         if mine else "-")
        best = min(rows, key=lambda r: r[1])
        lines.append("%s | %s | %.2f | %s | %s" % (dt, name, gflop, " | ".join(cells), best[2]))
    return "\n".join(lines) + "\n"


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--out", required=True, help="path of the table to write")
    ap.add_argument("--report", default=None,
                    help="also write a markdown table of the best time per kernel family and layer")
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        sys.exit("tune.py needs the GPU")
    rn50 = [name for n in wl.RESNET50_BATCHES for name in wl.RESNET50_BY_BATCH[n]]
    f32 = list(wl.LAYERS) + rn50
    bf16 = list(wl.BF16_LAYERS) + rn50
    lines = [
        "// Winners of `python -m paper_1904_04174_amd.tune` on one MI355X: the fastest variant",
        "// per named layer (milliseconds per call in the comment).  Columns: bf16 input?,",
        "// N, H, W, C, K, R, S, stride rows, stride cols, padding, variant name.  A shape whose",
        "// fastest variant is a Winograd one has that row first, then its best direct-sum variant.",
    ]
    seen = set()
    results = []
    for in_dtype, names in ((B.F32, f32), (B.BF16, bf16)):
        for name in names:
            L = wl.ALL_LAYERS[name]
            key = (in_dtype,) + tuple(L[1:11])   # the same shape under two names is tuned once
            if key in seen:
                continue
            seen.add(key)
            rows = tune_layer(torch, L, in_dtype)
            if not rows:
                continue
            g = B.conv2d_get_geometry(B.params_of_layer(L, in_dtype, B.F32))
            gflop = 2e-9 * L.batch * g.out_rows * g.out_cols * L.features * L.window_rows * \
                L.window_cols * L.channels
            results.append(("bf16" if in_dtype == B.BF16 else "f32", name, gflop, rows))
            # the best variant overall goes first if it is a transform (Winograd) variant and
            # wins by the margin; the best direct-sum variant always gets a row
            direct = [r for r in rows if not r[2].startswith("winograd")]
            chosen = []
            if rows[0][2].startswith("winograd") and (
                    not direct or rows[0][0] * WINOGRAD_MARGIN < direct[0][0]):
                chosen.append(rows[0])
            if direct:
                chosen.append(direct[0])
            for _, ms, best in chosen:
                print("%-5s %-10s %-46s %9.4f ms" % (
                    "bf16" if in_dtype == B.BF16 else "f32", name, best, ms), flush=True)
                lines.append('{%d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, "%s"},  // %s %.4f ms'
                             % (1 if in_dtype == B.BF16 else 0, L.batch, L.in_rows, L.in_cols,
                                L.channels, L.features, L.window_rows, L.window_cols,
                                L.stride_rows, L.stride_cols, L.padding, best, name, ms))
    with open(args.out, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("wrote", args.out)
    if args.report:
        with open(args.report, "w") as fh:
            fh.write(family_report(results))
        print("wrote", args.report)


if __name__ == "__main__":
    main()
