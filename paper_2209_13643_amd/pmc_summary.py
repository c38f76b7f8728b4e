"""Counter summary of the configs[1] leg: `python -m paper_2209_13643_amd.pmc_summary FETCH.csv WRITE.csv`.

Input: the `*_counter_collection.csv` files of two rocprofv3 runs of `python3 bench.py --only-config1`, one with
`--pmc FETCH_SIZE`, one with `--pmc WRITE_SIZE` (values in KiB per dispatch).  Each counter is scaled by what it
reads for the plain copy kernel of that step, whose size is known (the wire copy of the masked operands of the
Beaver conv: both parties' x - a and w - b words), and averaged per kernel and grid.  Prints a markdown summary
(kept under profiles/) that carries a digest of the HIP sources; bench.py quotes the GEMM row as `roofline.traffic`
only while that digest matches the sources it runs.
"""
from __future__ import annotations

import collections
import csv
import hashlib
import os
import sys

from . import synth

CSRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")


def sources_digest() -> str:
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(name.encode()); h.update(f.read())
    return h.hexdigest()[:16]


def clean(name):
    return name.replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0]


def dispatches(path, counter):
    """[(dispatch id, kernel, grid, KiB)] in dispatch order; library kernels of torch are left out."""
    rows = []
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            name = r["Kernel_Name"]
            if "at::native" in name or name.startswith("Cijk") or "rocclr" in name:
                continue
            rows.append((int(r["Dispatch_Id"]), clean(name), int(r["Grid_Size"]), float(r["Counter_Value"])))
    rows.sort()
    return rows


def per_kernel(rows):
    """Ordered {(kernel, grid): mean KiB per dispatch}."""
    groups = collections.OrderedDict()
    for _, name, grid, v in rows:
        groups.setdefault((name, grid), []).append(v)
    return collections.OrderedDict((k, sum(v) / len(v)) for k, v in groups.items())


def is_relu(name):
    return name.startswith(("k_relu_stage", "k_relu_msb_stage", "k_wire_words", "k_wire_bytes"))


def relu_calls(rows):
    """KiB per secure-ReLU call by chain and exchange: a call is a maximal run of stage and wire dispatches (the
    conv call's kernels separate the runs; the chunks of a call follow each other), the chain shows in the stage
    kernels' name, the exchange in their last template argument."""
    out = collections.defaultdict(list)
    run = []
    for r in list(rows) + [(0, "end", 0, 0.0)]:
        if is_relu(r[1]):
            run.append(r)
            continue
        if run:
            stages = [q[1] for q in run if "stage<" in q[1]]
            if stages:
                chain = "sign-only" if any("msb" in q for q in stages) else "whole words"
                put = any(q.rstrip(">").endswith("true") for q in stages)
                out[(chain, "remote store" if put else "copy")].append(sum(q[3] for q in run))
            run = []
    return {k: sum(v) / len(v) for k, v in out.items()}


def gemm_launches(rows):
    """{form of the Beaver call: [value per two-party GEMM launch]} for rows of (id, kernel, grid, value) in dispatch
    order.  The form is read off the call's own kernels before the launch: the remote-store folded call recodes with
    k_recode_rows alone; the other forms use one k_recode_mixed launch whose grid grows with the number of plane
    sets (prepared call: e; folded call with the copy exchange: x_0 + e_1 and e; plain call: six sets)."""
    biggest = max((r[2] for r in rows if r[1].startswith("k_limb_gemm")), default=0)
    groups = collections.OrderedDict()
    prologue = []
    for r in rows:
        if is_relu(r[1]):
            prologue = []
        elif r[1].startswith("k_limb_gemm"):
            if r[2] == biggest and prologue:
                mixed = [g for n, g in prologue if n.startswith("k_recode_mixed")]
                rows_only = not mixed and any(n.startswith("k_recode_rows") for n, _ in prologue)
                if mixed or rows_only:
                    groups.setdefault(("rows", 0) if rows_only else ("mixed", mixed[-1]), []).append(r[3])
            prologue = []
        else:
            prologue.append((r[1], r[2]))
    out = collections.OrderedDict()
    if ("rows", 0) in groups:
        out["folded prepared call (three products)"] = groups[("rows", 0)]
    mixed = sorted(k for k in groups if k[0] == "mixed")
    names = ["prepared call (four products)", "folded prepared call with the copy exchange (three products)", "plain call (four products)"]
    for i, k in enumerate(mixed):
        out[names[i] if len(mixed) == 3 else f"call whose recoding launch has grid {k[1]}"] = groups[k]
    return out


def gemm_calls(rows):
    """Mean KiB per two-party GEMM launch by the form of the Beaver call."""
    return collections.OrderedDict((k, sum(v) / len(v)) for k, v in gemm_launches(rows).items())


def main(argv):
    if len(argv) != 2:
        print(__doc__, file=sys.stderr)
        return 2
    frows, wrows = dispatches(argv[0], "FETCH_SIZE"), dispatches(argv[1], "WRITE_SIZE")
    fetch, write = per_kernel(frows), per_kernel(wrows)
    L = synth.config_vgg_block().layers[0]
    copy_kib = 2 * 8 * (L.B * L.H * L.W * L.Cin + L.KH * L.KW * L.Cin * L.Cout) / 1024      # read once, written once
    ck = [k for k in fetch if k[0].startswith("k_copy_multi")]
    if not ck:
        print("no k_copy_multi dispatch in the counter file: cannot calibrate", file=sys.stderr)
        return 1
    ck = max(ck, key=lambda k: fetch[k])                 # the plain Beaver conv's exchange (the largest copy)
    fscale, wscale = copy_kib / fetch[ck], copy_kib / write[ck]
    print("# HBM traffic counters: configs[1] leg of bench.py\n")
    print(f"sources sha256/16: {sources_digest()}\n")
    print("Commands (one counter per run; from /tmp with TMPDIR=/tmp), then this summary:\n")
    print("    rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/pmc_fetch -o f -- python3 bench.py --only-config1 --steps 3 --warmup 1")
    print("    rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/pmc_write -o w -- python3 bench.py --only-config1 --steps 3 --warmup 1")
    print("    python3 -m paper_2209_13643_amd.pmc_summary <f_counter_collection.csv> <w_counter_collection.csv>\n")
    print(f"Calibration on the plain copy kernel {ck[0]} (the wire copy of the plain call's masked operands: {copy_kib:.0f} KiB in, the same "
          f"out, per launch): FETCH_SIZE reads {fetch[ck]:.1f} KiB -> scale x{fscale:.3f}; WRITE_SIZE reads {write[ck]:.1f} KiB -> scale x{wscale:.3f}.\n")
    print("Per launch, after scaling (MiB; mean over the launches of that kernel and grid in the run):\n")
    print("| kernel | grid | fetch MiB | write MiB |\n|---|---:|---:|---:|")
    for k in fetch:
        print(f"| {k[0]} | {k[1]} | {fetch[k] * fscale / 1024:.1f} | {write.get(k, 0.0) * wscale / 1024:.1f} |")
    gf, gw = gemm_calls(frows), gemm_calls(wrows)
    if gf:
        print("\nThe two-party GEMM launch by the form of the Beaver call (MiB per launch):\n")
        print("| call | fetch MiB | write MiB |\n|---|---:|---:|")
        for name in gf:
            print(f"| k_limb_gemm in the {name} | {gf[name] * fscale / 1024:.1f} | {gw.get(name, 0.0) * wscale / 1024:.1f} |")
    n = L.B * L.Ho * L.Wo * L.Cout
    fr, wr = relu_calls(frows), relu_calls(wrows)
    print()
    for key in sorted(fr):
        if key in wr:
            fb, wb = fr[key] * fscale * 1024, wr[key] * wscale * 1024
            print(f"Secure ReLU, {key[0]}, exchange by {key[1]}, all kernels of one call (both parties + wire), {n} elements: "
                  f"fetch {fb / 1e6:.0f} MB + write {wb / 1e6:.0f} MB = {(fb + wb) / n:.0f} bytes per element.\n")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
