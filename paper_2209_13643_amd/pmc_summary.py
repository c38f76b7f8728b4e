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
            name = name.split("(")[0].replace("void ", "").replace("(anonymous namespace)::", "")
            rows.append((int(r["Dispatch_Id"]), name, int(r["Grid_Size"]), float(r["Counter_Value"])))
    rows.sort()
    return rows


def per_kernel(rows):
    """Ordered {(kernel, grid): mean KiB per dispatch}."""
    groups = collections.OrderedDict()
    for _, name, grid, v in rows:
        groups.setdefault((name, grid), []).append(v)
    return collections.OrderedDict((k, sum(v) / len(v)) for k, v in groups.items())


def relu_call_kib(rows, n, auto_chunk=1 << 20):
    """KiB per secure-ReLU call, whole-word chain and sign-only chain: every stage and wire dispatch of the chain's
    leg summed, divided by the number of calls (dispatches of the chain's last stage / chunks per call).  The legs
    run one after the other, so a wire copy belongs to the chain whose stage kernels surround it."""
    chunks = max(1, (n + auto_chunk // 2) // auto_chunk)
    first_msb = next((i for i, r in enumerate(rows) if "k_relu_msb_stage" in r[1]), len(rows))
    if first_msb < len(rows) and first_msb > 0 and "k_wire" in rows[first_msb - 1][1]:
        first_msb -= 1                                   # the A2B mask copy that opens the first sign-only call
    out = {}
    for chain, lo, hi, stage in (("relu", 0, first_msb, "k_relu_stage<9"), ("relu_msb", first_msb, len(rows), "k_relu_msb_stage<9")):
        part = [r for r in rows[lo:hi] if "k_relu" in r[1] or "k_wire" in r[1]]
        calls = sum(1 for r in part if r[1].startswith(stage)) / chunks
        if calls > 0:
            out[chain] = sum(r[3] for r in part) / calls
    return out


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
    ck = max(ck, key=lambda k: fetch[k])                 # the Beaver conv's exchange (the largest copy)
    fscale, wscale = copy_kib / fetch[ck], copy_kib / write[ck]
    print("# HBM traffic counters: configs[1] leg of bench.py\n")
    print(f"sources sha256/16: {sources_digest()}\n")
    print("Commands (one counter per run; from /tmp with TMPDIR=/tmp), then this summary:\n")
    print("    rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/pmc_fetch -o f -- python3 bench.py --only-config1 --steps 3 --warmup 1")
    print("    rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/pmc_write -o w -- python3 bench.py --only-config1 --steps 3 --warmup 1")
    print("    python3 -m paper_2209_13643_amd.pmc_summary <f_counter_collection.csv> <w_counter_collection.csv>\n")
    print(f"Calibration on the plain copy kernel {ck[0]} (the wire copy of the masked operands: {copy_kib:.0f} KiB in, the same out, "
          f"per launch): FETCH_SIZE reads {fetch[ck]:.1f} KiB -> scale x{fscale:.3f}; WRITE_SIZE reads {write[ck]:.1f} KiB -> scale x{wscale:.3f}.\n")
    print("Per launch, after scaling (MiB):\n")
    print("| kernel | grid | fetch MiB | write MiB |\n|---|---:|---:|---:|")
    for k in fetch:
        print(f"| {k[0]} | {k[1]} | {fetch[k] * fscale / 1024:.1f} | {write.get(k, 0.0) * wscale / 1024:.1f} |")
    n = L.B * L.Ho * L.Wo * L.Cout
    fr, wr = relu_call_kib(frows, n), relu_call_kib(wrows, n)
    print()
    for chain, label in (("relu", "Secure ReLU on whole words (mpc_relu)"), ("relu_msb", "Sign-only packed chain (mpc_relu_msb)")):
        if chain in fr and chain in wr:
            fb, wb = fr[chain] * fscale * 1024, wr[chain] * wscale * 1024
            print(f"{label}, all kernels of one call (both parties + wire), {n} elements: fetch {fb / 1e6:.0f} MB + write {wb / 1e6:.0f} MB "
                  f"= {(fb + wb) / n:.0f} bytes per element.\n")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
