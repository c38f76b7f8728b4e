#!/usr/bin/env python3
"""Benchmark of the secure-layer hot path on one MI355X.

A step is one pass of the whole online path over one batch of the VGG16-style
CIFAR conv block (batch 64, 128x16x16 input, 3x3 conv 128->128, i.e. the Beaver
GEMM [16384 x 1152] x [1152 x 128] over Z_2^64 with truncation, then secure
ReLU on its 2 097 152 outputs).  All shares, triples and ReLU material are
dealt on the device before the timed region (synthetic stand-ins for the
paper's models: only shapes and value distributions matter to this path).

Prints one JSON line.  `value` is secure MACs/s of the Beaver convolution call
(mask, exchange, digit recoding, int8-MFMA GEMM, truncation); the secure ReLU
rate and the whole-step time are reported beside it.  `roofline` describes the
digit-plane GEMM kernel against the int8 MFMA peak, `roofline_relu` the ReLU
chain against HBM bandwidth, `value_prepared_planes` the convolution call when
the digit planes of the triple and of the opened weight mask were recoded ahead
of time (mpc_conv2d_prepared), `roofline_relu_msb` the same ReLU evaluated on the
sign's carry chain only with bit-packed triples (mpc_relu_msb, timed on its own
after the steps); `three_party` the same conv block, masked rescale and ReLU with
three simulated parties (Alg. 1 / Alg. 2 for N = 3), timed on its own;
`cpu_baseline` is the CPU oracle timed on this
box's host cores on the same workload (a reported baseline, not a target).
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

INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_OPS_PER_SECURE_MAC = 288          # 2 parties x 2 ring GEMMs x 36 digit products x 2 ops
RELU_BYTES_PER_ELEMENT = 86 * 8 + 2 + 216 * 8 + 137 * 8   # compulsory + openings + carried state, both parties
# the sign-only packed chain (mpc_relu_msb), same three classes: 31.72 W + 2 B, 71.25 W + 8 B, 41.56 W + 6 B
RELU_MSB_BYTES_PER_ELEMENT = (31.71875 + 71.25 + 41.5625) * 8 + 16


RELU3_BYTES_PER_ELEMENT = 966 * 8 + 33      # three parties: 141 W + 3 B, 606 W + 21 B, 219 W + 9 B (same three classes)
RELU3_MSB_BYTES_PER_ELEMENT = 2961          # three parties, sign-only chain: 59.6 W + 3 B, 226.0 W + 21 B, 80.3 W + 9 B


def three_party_leg(lane, L, steps, warmup):
    """The step's three calls with three simulated parties, each timed by its own region / the host clock."""
    import statistics

    import torch
    from paper_2209_13643_amd import dealer, mpc, synth

    dev = lane.device
    g = dealer.gen(synth.BASE_SEED + 31, dev)
    d = dealer.conv_layer3(lane, g, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, L.x_std, L.w_std)
    M, K, N = L.gemm_mkn
    n = M * N
    mat = dealer.relu3_material(g, n, dev)
    z = tuple(torch.empty_like(d["c"][0]) for _ in range(3))
    y = tuple(torch.empty_like(d["c"][0]) for _ in range(3))

    def step():
        lane.conv2d3(d["x"], d["w"], d["a"], d["b"], d["c"], L.pad, L.stride, out=z)
        lane.truncate3(z, d["r"], d["rt"])               # in place
        lane.relu3(z, mat, out=y)

    for _ in range(warmup):
        step()
    lane.sync(); torch.cuda.synchronize()
    lane.set_profiling(True); lane.profile_reset()
    for _ in range(steps):
        step()
    lane.sync(); torch.cuda.synchronize()
    lane.set_profiling(False)
    lin = statistics.median(lane.profile_samples(mpc.PROF_LINEAR))
    gemm = sum(lane.profile_samples(mpc.PROF_GEMM_KERNEL)) / steps          # two launches per call
    relu = statistics.median(lane.profile_samples(mpc.PROF_RELU))
    # properties that hold for every element: product, rescale band, ReLU
    zz = lane.conv2d3(d["x"], d["w"], d["a"], d["b"], d["c"], L.pad, L.stride)      # the product before the rescale
    lane.sync()
    rz = zz[0] + zz[1] + zz[2]; rt = z[0] + z[1] + z[2]; ry = y[0] + y[1] + y[2]
    dlt = rt - (rz >> 16)
    assert int(dlt.min()) >= 0 and int(dlt.max()) <= 1, "three-party rescale left the floor + {0, 1} band"
    assert torch.equal(ry, torch.clamp(rt, min=0)), "three-party ReLU output does not reconstruct to max(t, 0)"
    ref = torch.nn.functional.conv2d((d["X"][:2].double() / 65536).permute(0, 3, 1, 2),
                                     (d["W"].double() / 65536).permute(3, 2, 0, 1), padding=L.pad, stride=L.stride)
    err = (rt[:2].double() / 65536 - ref.permute(0, 2, 3, 1)).abs().max().item()
    assert err <= 2.0 ** -12, f"three-party decoded conv output off by {err}"
    # the same ReLU on the sign's carry chain only (packed material)
    del mat
    matp = dealer.relu3_material(g, n, dev, packed=True)
    y2 = tuple(torch.empty_like(v) for v in y)
    for _ in range(warmup):
        lane.relu3(z, matp, out=y2, packed=True)
    lane.sync(); lane.set_profiling(True); lane.profile_reset()
    for _ in range(steps):
        lane.relu3(z, matp, out=y2, packed=True)
    lane.sync(); lane.set_profiling(False)
    msb = statistics.median(lane.profile_samples(mpc.PROF_RELU))
    assert torch.equal(y2[0] + y2[1] + y2[2], ry), "three-party sign-only ReLU reconstructs differently"
    macs = M * K * N
    return {"parties": 3, "ms_beaver_conv_call": lin, "value": macs / (lin * 1e-3), "unit": "secure MACs/s",
            "ms_gemm_kernels": gemm, "gemm_frac_of_int8_peak": 432 * macs / (gemm * 1e-3) / 1e12 / INT8_PEAK_TOPS,
            "ms_relu_call": relu, "relu_value": n / (relu * 1e-3),
            "relu_bytes_per_element": RELU3_BYTES_PER_ELEMENT,
            "relu_frac_of_hbm_peak": RELU3_BYTES_PER_ELEMENT * n / (relu * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "ms_relu_msb_call": msb, "relu_msb_value": n / (msb * 1e-3),
            "relu_msb_bytes_per_element": RELU3_MSB_BYTES_PER_ELEMENT,
            "relu_msb_frac_of_hbm_peak": RELU3_MSB_BYTES_PER_ELEMENT * n / (msb * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "max_abs_err_vs_float64": err}


def cpu_baseline(layer, budget_s=12.0):
    """The oracle as it stands, on the host cores, on the same conv block."""
    import numpy as np
    import oracle
    from paper_2209_13643_amd import synth

    rng = synth.rng_for(1, 7)
    B = 16                                              # a quarter of the batch per repetition
    X = synth.normal_fixed(rng, (B, layer.H, layer.W, layer.Cin), layer.x_std)
    Wt = synth.normal_fixed(rng, (layer.KH, layer.KW, layer.Cin, layer.Cout), layer.w_std)
    xs, ws = synth.share_additive(rng, X), synth.share_additive(rng, Wt)
    a, b, c = synth.deal_product_triple(rng, X.shape, Wt.shape,
                                        lambda A, Bf: oracle.ring_conv2d(A, Bf, layer.pad, layer.stride))
    n = B * layer.Ho * layer.Wo * layer.Cout
    mat = synth.deal_relu_material(rng, n)
    macs = B * layer.Ho * layer.Wo * layer.KH * layer.KW * layer.Cin * layer.Cout
    t_lin = t_relu = 0.0
    reps = 0
    t_start = time.perf_counter()
    while reps < 1 or (time.perf_counter() - t_start) < budget_s:
        t0 = time.perf_counter()
        z = oracle.truncate(oracle.beaver_conv2d(xs, ws, a, b, c, layer.pad, layer.stride), 16)
        t1 = time.perf_counter()
        oracle.relu(z, mat)
        t2 = time.perf_counter()
        t_lin += t1 - t0; t_relu += t2 - t1; reps += 1
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next(l.split(":", 1)[1].strip() for l in f if l.startswith("model name"))
    except (OSError, StopIteration):
        pass
    return {"value": macs * reps / t_lin, "unit": "secure MACs/s", "cores": oracle.n_threads(), "cpu": cpu_model,
            "kind": "oracle",
            "relu_value": n * reps / t_relu, "relu_unit": "secure ReLU elems/s",
            "sample": f"{reps} x (batch {B} of 64 of the same conv block: Alg. 1 with five direct ring "
                      f"convolutions + truncation, then ReLU on {n} elements), {t_lin + t_relu:.1f} s of CPU work"}


def cpu_baseline_all_configs():
    """The oracle on a bounded sample of every layer of the five workloads (rows of a dense layer,
    images of a convolution; at most 2^18 ReLU elements): secure MACs/s and ReLU elements/s per layer.
    Only with --cpu-all-configs: it adds about a minute of CPU work."""
    import numpy as np
    import oracle
    from paper_2209_13643_amd import synth

    out = []
    for make in synth.CONFIGS:
        wl = make()
        rng = synth.rng_for(wl.index, 8)
        for L in wl.layers:
            if isinstance(L, synth.Conv):
                Bs = max(1, min(L.B, (1 << 28) // max(1, L.Ho * L.Wo * L.KH * L.KW * L.Cin * L.Cout)))
                xs = tuple(synth.rand_words(rng, (Bs, L.H, L.W, L.Cin)) for _ in range(2))
                ws = tuple(synth.rand_words(rng, (L.KH, L.KW, L.Cin, L.Cout)) for _ in range(2))
                cs = tuple(synth.rand_words(rng, (Bs, L.Ho, L.Wo, L.Cout)) for _ in range(2))
                t0 = time.perf_counter()
                z = oracle.truncate(oracle.beaver_conv2d(xs, ws, xs, ws, cs, L.pad, L.stride), 16)
                dt = time.perf_counter() - t0
                macs = Bs * L.Ho * L.Wo * L.KH * L.KW * L.Cin * L.Cout
                sample = f"{Bs} of {L.B} images"
            else:
                Ms = max(1, min(L.M, (1 << 28) // max(1, L.K * L.N)))
                xs = tuple(synth.rand_words(rng, (Ms, L.K)) for _ in range(2))
                ws = tuple(synth.rand_words(rng, (L.K, L.N)) for _ in range(2))
                cs = tuple(synth.rand_words(rng, (Ms, L.N)) for _ in range(2))
                t0 = time.perf_counter()
                z = oracle.truncate(oracle.beaver_matmul(xs, ws, xs, ws, cs), 16)
                dt = time.perf_counter() - t0
                macs = Ms * L.K * L.N
                sample = f"{Ms} of {L.M} rows" + (f", 1 of {L.batch} batch items" if L.batch > 1 else "")
            row = {"config": wl.index, "layer": L.name, "secure_macs_per_s": macs / dt, "sample": sample}
            if L.relu:
                n = min(z[0].size, 1 << 18)
                zz = (z[0].reshape(-1)[:n], z[1].reshape(-1)[:n])
                mat = synth.deal_relu_material(rng, n)
                t0 = time.perf_counter()
                oracle.relu(zz, mat)
                row["relu_elems_per_s"] = n / (time.perf_counter() - t0)
            out.append(row)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-three-party", action="store_true", help="skip the three-party leg (same workload, N = 3)")
    ap.add_argument("--cpu-all-configs", action="store_true",
                    help="also time the oracle on a sample of every layer of all five workloads")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build simulates both parties on a single MI355X and has no "
              "multi-GPU path (run with --gpus 1).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2209_13643_amd import dealer, mpc, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    wl = synth.config_vgg_block()
    L = wl.layers[0]
    M, K, N = L.gemm_mkn
    n = M * N
    lane = mpc.Lane(0)
    lane.use_single_queue()      # one in-order queue per lane: no cross-stream event latency inside a call
    dev = lane.device
    g = dealer.gen(synth.BASE_SEED + wl.index, dev)
    d = dealer.conv_layer(lane, g, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, L.x_std, L.w_std)
    mat = dealer.relu_material(g, n, dev)
    z = tuple(torch.empty((L.B, L.Ho, L.Wo, L.Cout), dtype=torch.int64, device=dev) for _ in range(2))
    y = tuple(torch.empty_like(z[0]) for _ in range(2))
    torch.cuda.synchronize()

    def step():
        lane.conv2d(d["x"], d["w"], d["a"], d["b"], d["c"], L.pad, L.stride, out=z)      # Alg. 1 / Eq. 3 + truncation
        lane.relu(z, mat, out=y)                                                            # Alg. 2 + Sec. 4.2

    for _ in range(args.warmup):
        step()
    lane.sync(); torch.cuda.synchronize()
    lane.set_profiling(True); lane.profile_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    lane.sync(); torch.cuda.synchronize()
    t1 = time.perf_counter()
    lane.set_profiling(False)
    ms_step = (t1 - t0) * 1e3 / args.steps
    gemm_ms, gemm_n = lane.profile(mpc.PROF_GEMM_KERNEL)
    lin_ms, lin_n = lane.profile(mpc.PROF_LINEAR)
    relu_ms, relu_n = lane.profile(mpc.PROF_RELU)
    gemm_ms /= gemm_n; lin_ms /= lin_n; relu_ms /= relu_n
    import statistics
    spread = {}
    for key, which in (("gemm_kernel", mpc.PROF_GEMM_KERNEL), ("beaver_conv_call", mpc.PROF_LINEAR), ("relu_call", mpc.PROF_RELU)):
        smp = lane.profile_samples(which)
        spread[key] = {"median_ms": statistics.median(smp), "min_ms": min(smp), "max_ms": max(smp), "n": len(smp)}

    # sanity on the result of the last step: ReLU of the reconstructed conv output, exactly
    rec_z = (z[0] + z[1]); rec_y = (y[0] + y[1])
    assert torch.equal(rec_y, torch.clamp(rec_z, min=0)), "secure ReLU output does not reconstruct to max(z, 0)"
    ref = torch.nn.functional.conv2d((d["X"].double() / 65536).permute(0, 3, 1, 2)[:2],
                                     (d["W"].double() / 65536).permute(3, 2, 0, 1), padding=L.pad).permute(0, 2, 3, 1)
    err = (rec_z[:2].double() / 65536 - ref).abs().max().item()
    assert err <= 2.0 ** -12, f"decoded conv output off by {err}"

    # the sign-only packed chain on the same conv output, timed on its own
    mat_p = dealer.relu_material(g, n, dev, packed=True)
    y2 = tuple(torch.empty_like(z[0]) for _ in range(2))
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        lane.relu(z, mat_p, out=y2, packed=True)
    lane.sync()
    lane.set_profiling(True); lane.profile_reset()
    for _ in range(args.steps):
        lane.relu(z, mat_p, out=y2, packed=True)
    lane.sync(); torch.cuda.synchronize()
    lane.set_profiling(False)
    msb_ms, msb_n = lane.profile(mpc.PROF_RELU)
    msb_ms /= msb_n
    smp = lane.profile_samples(mpc.PROF_RELU)
    spread["relu_msb_call"] = {"median_ms": statistics.median(smp), "min_ms": min(smp), "max_ms": max(smp), "n": len(smp)}
    assert torch.equal(y2[0] + y2[1], torch.clamp(rec_z, min=0)), "mpc_relu_msb output does not reconstruct to max(z, 0)"
    msb_gbs = RELU_MSB_BYTES_PER_ELEMENT * n / (msb_ms * 1e-3) / 1e9

    # the Beaver convolution with the input-independent operands' digit planes recoded ahead of time
    right, left = lane.prepare_conv2d(d["a"], d["b"], d["f_public"], L.pad, L.stride)
    for _ in range(args.warmup):
        lane.conv2d_prepared(d["x"], d["a"], d["c"], right, left, L.KH, L.KW, L.pad, L.stride, out=y2)
    lane.sync()
    lane.set_profiling(True); lane.profile_reset()
    for _ in range(args.steps):
        lane.conv2d_prepared(d["x"], d["a"], d["c"], right, left, L.KH, L.KW, L.pad, L.stride, out=y2)
    lane.sync(); torch.cuda.synchronize()
    lane.set_profiling(False)
    prep_ms, prep_n = lane.profile(mpc.PROF_LINEAR)
    prep_ms /= prep_n
    assert torch.equal(y2[0], z[0]) and torch.equal(y2[1], z[1]), "prepared-plane convolution differs from the plain call"

    macs = M * K * N
    gemm_tops = INT8_OPS_PER_SECURE_MAC * macs / (gemm_ms * 1e-3) / 1e12
    relu_gbs = RELU_BYTES_PER_ELEMENT * n / (relu_ms * 1e-3) / 1e9
    out = {
        "metric": "secure Z_2^64 MACs/s (Beaver GEMM) + secure ReLU elems/s, 1 GPU, online",
        "value": macs / (lin_ms * 1e-3), "unit": "secure MACs/s",
        "relu_value": n / (relu_ms * 1e-3), "relu_unit": "secure ReLU elems/s",
        "relu_msb_value": n / (msb_ms * 1e-3),
        "value_prepared_planes": M * K * N / (prep_ms * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64 ring (int8 digits, int32 accumulate)",
        "data": "synthetic",
        "config": {"workload": "configs[1] vgg16-cifar-conv-block: batch 64, 128x16x16, conv3x3 128->128 pad 1 "
                               "= Beaver GEMM [16384x1152]x[1152x128] + truncation + secure ReLU on 2097152 elements",
                   "parties": 2, "frac_bits": 16, "n_chunks": 1, "relu_chunks": "auto (about 2^20 elements each)", "lane": "single in-order queue",
                   "ms_beaver_conv_call": lin_ms, "ms_gemm_kernel": gemm_ms, "ms_relu_call": relu_ms,
                   "ms_relu_msb_call": msb_ms, "ms_beaver_conv_call_prepared_planes": prep_ms, "region_times": spread,
                   "max_abs_err_vs_float64": err},
        "roofline": {"kernel": "k_limb_gemm<2,2,true> (both parties, [e|a_i] x [b_i';f], fused add-c + truncation)",
                     "bound": "mfma", "achieved": gemm_tops, "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": gemm_tops / INT8_PEAK_TOPS,
                     "traffic": {"fetch_bytes": 135.0 * 2 ** 20, "write_bytes": 32.0 * 2 ** 20,
                                 "algorithmic_bytes": (100.6 + 32.0) * 2 ** 20,
                                 "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, calibrated on a copy kernel "
                                           "(profiles/bench_vgg_block_hbm_traffic.md)"},
                     "note": "288 int8 ops per secure MAC; power-limited attainable rate with random int8 operands "
                             "measured on this chip with a back-to-back MFMA loop is about 3070 TOP/s"},
        "roofline_relu": {"kernel": "secure ReLU chain: k_relu_stage<0..9> (both parties per launch) + k_wire_words / k_wire_bytes",
                          "bound": "hbm", "achieved": relu_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": relu_gbs / HBM_PEAK_GBS,
                          "traffic": {"bytes_per_element": 3388, "source": "rocprofv3 --pmc, same summary"},
                          "bytes_per_element": RELU_BYTES_PER_ELEMENT},
        "roofline_relu_msb": {"kernel": "sign-only packed ReLU chain: k_relu_msb_stage<0..9> + k_wire_words / k_wire_bytes",
                              "bound": "hbm", "achieved": msb_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": msb_gbs / HBM_PEAK_GBS,
                              "traffic": {"bytes_per_element": 1164, "source": "rocprofv3 --pmc, same summary"},
                              "bytes_per_element": RELU_MSB_BYTES_PER_ELEMENT},
    }
    if not args.no_three_party:
        out["three_party"] = three_party_leg(lane, L, args.steps, args.warmup)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L)
        if args.cpu_all_configs:
            out["cpu_baseline"]["per_layer"] = cpu_baseline_all_configs()
    lane.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
