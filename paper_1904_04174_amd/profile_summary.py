"""Summary of rocprofv3 counter runs of `bench.py --only LAYER` (the profile step).

The counter runs themselves are plain rocprofv3 commands (printed by `--print-commands`), one
run per counter set and layer, each into `DIR/<layer>_<dtype>_<algorithms>/`, its standard
output into `DIR/<layer>_<dtype>_<algorithms>_<first counter>.log`:

    python -m paper_1904_04174_amd.profile_summary --print-commands V112-N16:f32 V56-N16:bf16 ...

`bench.py --only` launches the layer's kernels and then one device-to-device copy of known
size; that copy calibrates the memory counters (FETCH_SIZE and WRITE_SIZE count in units that
differ from KiB by a constant factor).  This script reads the CSV files that rocprofv3 wrote
and produces

  * a markdown table per layer and kernel (HBM bytes read and written, GPU cycles, MFMA busy
    fraction): `--md FILE`
  * the HBM bytes per launch of each layer's kernels, keyed by element type, layer and variant,
    as JSON: `--json FILE` (bench.py reads `paper_1904_04174_amd/measured_traffic.json` for
    its `roofline.traffic` field, so that figure is never typed by hand)

    python -m paper_1904_04174_amd.profile_summary --dir gpurun_out/prof \\
        --md profiles/counters_per_layer.md --json paper_1904_04174_amd/measured_traffic.json

`--stats DIR` prints the per-kernel table of a `rocprofv3 --kernel-trace --stats` run.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

COUNTER_SETS = (
    "FETCH_SIZE",
    "WRITE_SIZE",
    "SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES GRBM_GUI_ACTIVE SQ_INSTS_MFMA "
    "SQ_INSTS_VALU_MFMA_MOPS_F32 SQ_INSTS_VALU_MFMA_MOPS_BF16",
)
COPY_MIB = 256

# kernels of the library by a substring of their name, in launch order
KINDS = (
    ("filter_transform", "filter_transform"), ("input_transform", "input_transform"),
    ("filter_transform", "winograd_lds_pack_kernel"), ("convolution", "winograd_lds_kernel"),
    ("pad_channels", "pad_channels"), ("repack", "repack_filter_kernel"),
    ("convolution", "igemm_dma_kernel"), ("convolution", "igemm_patch_kernel"),
    ("convolution", "igemm_kernel"), ("convolution", "conv1x1_kernel"),
    ("convolution", "conv3x3_regfilter_kernel"),
    ("convolution", "row_gather_kernel"), ("convolution", "direct_kernel"),
    ("tail_reduce", "tail_reduce_kernel"), ("split_reduce", "split_reduce_kernel"),
    ("output_transform", "output_transform"), ("max_pool", "max_pool_2x2_kernel"),
)


def kind_of(kernel_name):
    for kind, key in KINDS:
        if key in kernel_name:
            return kind
    return None


def commands(specs, out_dir):
    lines = ["cd /tmp && export TMPDIR=/tmp && cd <repository root>"]
    for spec in specs:
        parts = spec.split(":")
        layer, dtype = parts[0], parts[1]
        alg = parts[2] if len(parts) > 2 else "direct"
        d = "%s/%s_%s_%s" % (out_dir, layer, dtype, alg)
        for cs in COUNTER_SETS:
            tag = cs.split()[0]
            lines.append(
                "rocprofv3 --pmc %s --output-format csv -d %s -o %s -- python3 bench.py --only %s "
                "--dtype %s --algorithms %s --steps 3 --warmup 1 > %s_%s.log 2>&1"
                % (cs, d, tag, layer, dtype, alg, d, tag))
    return lines


def read_layer(layer_dir):
    """{kind: {counter: last value}}, {kind: kernel name}, copy kernel's {counter: value}."""
    vals = collections.defaultdict(dict)
    names = {}
    copy = {}
    for fn in sorted(glob.glob(os.path.join(layer_dir, "**", "*counter_collection.csv"),
                               recursive=True)):
        for r in csv.DictReader(open(fn)):
            k = r["Kernel_Name"]
            kind = kind_of(k)
            value = float(r["Counter_Value"])
            if kind is not None:
                vals[kind][r["Counter_Name"]] = value     # the last launch of the run
                names[kind] = k
            elif "copy" in k.lower() or "elementwise" in k.lower():
                copy[r["Counter_Name"]] = max(copy.get(r["Counter_Name"], 0.0), value)
    return vals, names, copy


def variant_of(layer_dir):
    """The variant name that bench.py --only printed into the run's log."""
    for log in sorted(glob.glob(layer_dir + "_*.log")):
        m = re.search(r"profiled \S+ \(([^)]+)\)", open(log, errors="replace").read())
        if m:
            return m.group(1)
    return None


def tile_label(kernel_name):
    """`kernel Tile<...>` without namespaces, return type and argument list."""
    m = re.search(r"(\w+_kernel)", kernel_name)
    name = m.group(1) if m else kernel_name.split("(")[0][-60:]
    i = kernel_name.find("Tile<")
    if i < 0:
        return name
    return "%s %s" % (name, kernel_name[i:kernel_name.find(">", i) + 1])


def kernel_stats(stats_dir):
    """Markdown table of a `rocprofv3 --kernel-trace --stats` run (its *_kernel_stats.csv)."""
    lines = ["kernel | calls | average us | min us | max us | % of GPU time", "---|---|---|---|---|---"]
    for fn in sorted(glob.glob(os.path.join(stats_dir, "**", "*kernel_stats.csv"), recursive=True)):
        for r in csv.DictReader(open(fn)):
            name = r["Name"]
            # (kernels of other libraries: their name without return type and arguments)
            label = tile_label(name) if "conv2d::" in name else re.sub(
                r"^void ", "", name).replace("(anonymous namespace)::", "").split("(")[0][:70]
            lines.append("%s | %s | %.1f | %.1f | %.1f | %.2f" % (
                label.replace("|", "/"), r["Calls"], float(r["AverageNs"]) / 1e3,
                float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    return "\n".join(lines) + "\n"


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--print-commands", nargs="+", metavar="LAYER:DTYPE[:ALGORITHMS]")
    ap.add_argument("--dir", default="gpurun_out/prof")
    ap.add_argument("--md")
    ap.add_argument("--json")
    ap.add_argument("--stats", metavar="DIR",
                    help="print the kernel table of a `rocprofv3 --kernel-trace --stats "
                         "--output-format csv -d DIR` run instead")
    args = ap.parse_args(argv)
    if args.stats:
        sys.stdout.write(kernel_stats(args.stats))
        return
    if args.print_commands:
        print("\n".join(commands(args.print_commands, args.dir)))
        return
    rows, table = [], {}
    for layer_dir in sorted(glob.glob(os.path.join(args.dir, "*_*_*"))):
        if not os.path.isdir(layer_dir):
            continue
        base = os.path.basename(layer_dir)
        try:
            layer, dtype, alg = base.rsplit("_", 2)
        except ValueError:
            continue
        vals, names, copy = read_layer(layer_dir)
        if not vals:
            continue
        # calibration on the copy of known size: KiB read / FETCH_SIZE, KiB written / WRITE_SIZE
        kib = COPY_MIB * 1024.0
        f_scale = kib / copy["FETCH_SIZE"] if copy.get("FETCH_SIZE") else 2.0
        w_scale = kib / copy["WRITE_SIZE"] if copy.get("WRITE_SIZE") else 1.0
        total = 0.0
        for kind in dict.fromkeys(k for k, _ in KINDS):
            if kind not in vals:
                continue
            c = vals[kind]
            fetch_mb = c.get("FETCH_SIZE", 0.0) * f_scale * 1024 / 1e6
            write_mb = c.get("WRITE_SIZE", 0.0) * w_scale * 1024 / 1e6
            total += fetch_mb + write_mb
            cycles = c.get("GRBM_GUI_ACTIVE", 0.0) / 8
            busy = (c.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / (cycles * 1024)) if cycles else 0.0
            label = tile_label(names[kind]) if kind == "convolution" else kind
            rows.append("%s %s (%s) | %s | %.0f | %.1f | %.0f | %.1f | %.0f | %s" % (
                layer, dtype, alg, label, c.get("FETCH_SIZE", 0.0), fetch_mb,
                c.get("WRITE_SIZE", 0.0), write_mb, cycles, ("%.2f" % busy) if busy > 0.005 else "-"))
        variant = variant_of(layer_dir)
        if variant and alg == "direct":
            table["%s|%s|%s" % (dtype, layer, variant)] = {
                "hbm_bytes_per_launch": round(total * 1e6),
                "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4),
                "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on `bench.py --only %s --dtype "
                          "%s`, all kernels of the call, scaled on a %d MiB copy" % (
                              layer, dtype, COPY_MIB)}
    header = [
        "layer dtype (selection) | kernel | FETCH_SIZE raw | HBM read MB | WRITE_SIZE raw | "
        "HBM written MB | GPU cycles / 8 XCDs | MFMA busy",
        "---|---|---|---|---|---|---|---"]
    text = "\n".join(header + rows) + "\n"
    if args.md:
        with open(args.md, "w") as fh:
            fh.write(text)
    else:
        sys.stdout.write(text)
    if args.json:
        with open(args.json, "w") as fh:
            json.dump(table, fh, indent=1, sort_keys=True)
            fh.write("\n")


if __name__ == "__main__":
    main()
