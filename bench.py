#!/usr/bin/env python3
"""Benchmark of the secure-layer hot path on one MI355X.

A step is one forward pass of the whole online path over one batch of the
largest single-GPU workload, configs[4]: the VGG16-shaped CIFAR network (13
conv3x3 layers 64..512 channels with 2x2 max-pooling, FC 512-512-10), batch 128
as four micro-batches of 32 on four lanes (the inter-batch pipeline of Sec. 4.3):
per layer the Beaver convolution of Alg. 1 / Eq. 3 (mask, exchange, digit
recoding, int8-MFMA ring GEMM, truncation), the secure ReLU of Alg. 2 / Sec. 4.2
on whole words and the max-pool by two conversions.  All shares, triples and
ReLU material are dealt on the device before the timed region (synthetic
stand-ins for the paper's models: only shapes and value distributions matter to
this path); every output tensor is allocated before it too.

Prints one JSON line.  `value` is secure MACs/s of the whole job (all Beaver
products of the batch over the step's wall time, ReLU and pooling included in
that time), `relu_value` the secure comparisons (ReLU elements + max-pool
comparisons) per second over the same wall time.  Beside them:
  `pipeline`     serial vs four-lane wall time in the default mode and in the
                 best mode (sign-only packed ReLU, prepared planes, pooled layers
                 as ReLU(maxpool), remote-store exchange, recorded graphs);
  `per_kind`     the serial pass split into its Beaver-call, ReLU-call and
                 max-pool regions (HIP events), with each kind's own rate;
  `configs`      all five workloads, per config: summed Beaver-call time, secure
                 MACs/s, call-level and kernel-level fraction of the int8 peak,
                 ReLU rate and HBM fraction (per layer with --layers);
  `roofline`     the secure GEMM of configs[1] (the launch the committed
                 rocprofv3 summaries cover): call-level fraction as `frac`, the
                 bare kernel's beside it;
  `roofline_relu`, `roofline_relu_msb`  the ReLU chains against HBM bandwidth;
  `three_party`  configs[1] with three simulated parties;
  `cpu_baseline` the CPU oracle on this machine's host cores on a sample of the
                 same network (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_OPS_PER_SECURE_MAC = 288          # 2 parties x 2 ring GEMMs x 36 digit products x 2 ops
RELU_BYTES_PER_ELEMENT = 86 * 8 + 2 + 216 * 8 + 137 * 8   # compulsory + openings + carried state, both parties
RELU_COMPULSORY_BYTES = 86 * 8 + 2                        # x, y, r, 12 AND triples, B2A pair, select triple: DRAM-compulsory
# the sign-only packed chain (mpc_relu_msb), same three classes: 31.72 W + 2 B, 71.25 W + 8 B, 41.56 W + 6 B
RELU_MSB_BYTES_PER_ELEMENT = (31.71875 + 71.25 + 41.5625) * 8 + 16
RELU_MSB_COMPULSORY_BYTES = 31.71875 * 8 + 2
RELU3_BYTES_PER_ELEMENT = 966 * 8 + 33      # three parties: 141 W + 3 B, 606 W + 21 B, 219 W + 9 B (same three classes)
RELU3_MSB_BYTES_PER_ELEMENT = 2961          # three parties, sign-only chain: 59.6 W + 3 B, 226.0 W + 21 B, 80.3 W + 9 B

N_MB, MICRO_BATCH = 4, 32


def sources_digest() -> str:
    """sha256 over the HIP sources: a profile summary taken from other kernels is not quoted."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2209_13643_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(name.encode()); h.update(f.read())
    return h.hexdigest()[:16]


def read_pmc_summary(path):
    """HBM traffic per launch of the GEMM kernel from a counter summary written by
    `python -m paper_2209_13643_amd.pmc_summary` (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by a
    copy kernel of known size).  Returns None unless the summary was taken from the sources as they are now."""
    try:
        with open(path) as f:
            text = f.read()
    except OSError:
        return None
    m = re.search(r"sources sha256/16: ([0-9a-f]{16})", text)
    rows = re.findall(r"k_limb_gemm[^|\n]*\|\s*(\d+)\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|", text)
    if not m or not rows or m.group(1) != sources_digest():
        return None
    grid, fetch, write = max(rows, key=lambda r: int(r[0]))       # the two-party launch of the Beaver call
    out = {"fetch_bytes": float(fetch) * 2 ** 20, "write_bytes": float(write) * 2 ** 20,
           "source": os.path.relpath(path, ROOT), "measured_in_this_run": False}
    for key, label in (("relu_bytes_per_element", "Secure ReLU on whole words"), ("relu_msb_bytes_per_element", "Sign-only packed chain")):
        r = re.search(re.escape(label) + r"[^\n]*= (\d+) bytes per element", text)
        if r:
            out[key] = int(r.group(1))
    return out


class Net:
    """configs[4] on four lanes in one mode: lanes, material, inputs and preallocated outputs."""

    def __init__(self, seed, packed_relu=False, prepared=False, pool_first=False, exchange="copy"):
        import torch
        from paper_2209_13643_amd import dealer, mpc, pipeline, synth
        self.pipeline, self.torch = pipeline, torch
        self.layers = synth.config_vgg16_pipeline(MICRO_BATCH).layers
        self.lanes = [mpc.Lane(0) for _ in range(N_MB)]
        for ln in self.lanes:
            ln.use_single_queue(); ln.set_exchange(exchange)
        dev = self.lanes[0].device
        g = dealer.gen(seed, dev)
        self.weights = pipeline.deal_weights(g, self.layers, dev)
        self.states, self.xs, self.X, self.outs = [], [], [], []
        for m in range(N_MB):
            st = pipeline.deal_microbatch(self.lanes[m], g, self.layers, self.weights, packed_relu=packed_relu,
                                          pool_first=pool_first)
            X = dealer.normal_fixed(g, (MICRO_BATCH, 32, 32, 3), 1.0, dev)
            self.states.append(st); self.X.append(X); self.xs.append(dealer.share(g, X))
            torch.cuda.synchronize()
            pipeline.preopen_weights(self.lanes[m], st)          # Alg. 3: weight masks travel ahead of the inputs
            if prepared:
                pipeline.prepare_layers(self.lanes[m], self.layers, st)
            self.outs.append(pipeline.alloc_outputs(self.lanes[m], self.layers, st))
        # serial runs put every micro-batch on lane 0: its outputs are reused from step to step as well
        torch.cuda.synchronize()

    def step_pipelined(self):
        return self.pipeline.forward_pipelined(self.lanes, self.layers, self.states, self.xs, [], outs_per_mb=self.outs)

    def step_serial(self):
        return [self.pipeline.forward(self.lanes[0], self.layers, self.states[m], self.xs[m], [], outs=self.outs[m])
                for m in range(N_MB)]

    def sync(self):
        for ln in self.lanes:
            ln.sync()
        self.torch.cuda.synchronize()

    def timed(self, fn, steps, warmup):
        for _ in range(warmup):
            fn()
        self.sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        self.sync()
        return (time.perf_counter() - t0) * 1e3 / steps

    def graphs(self):
        """One recorded graph per lane (the whole micro-batch forward), replayed on its lane."""
        gs = []
        for m, ln in enumerate(self.lanes):
            with ln.capture() as cap:
                self.pipeline.forward(ln, self.layers, self.states[m], self.xs[m], [], outs=self.outs[m])
            gs.append(cap.graph)
        return gs

    def close(self):
        for ln in self.lanes:
            ln.close()


def check_network(net, torch):
    """Properties of the last step that hold for every element: the logits of every micro-batch reconstruct to the
    plain fixed-point network on the reconstructed input to within the accumulated rescale error."""
    from paper_2209_13643_amd import synth
    F = torch.nn.functional
    worst = 0.0
    for m in range(N_MB):
        out = net.outs[m][-1]["z"]
        got = (out[0] + out[1]).double() / 65536
        x = (net.X[m].double() / 65536).permute(0, 3, 1, 2)
        for L, (W, _) in zip(net.layers, net.weights):
            w = W.double() / 65536
            if isinstance(L, synth.Conv):
                x = F.conv2d(x, w.permute(3, 2, 0, 1), padding=L.pad, stride=L.stride)
                x = torch.floor(x * 65536) / 65536
                if L.relu: x = torch.clamp(x, min=0)
                if L.pool: x = F.max_pool2d(x, 2)
            else:
                x = x.permute(0, 2, 3, 1).reshape(x.shape[0], -1) if x.dim() == 4 else x
                x = torch.floor((x @ w) * 65536) / 65536
                if L.relu: x = torch.clamp(x, min=0)
        worst = max(worst, (got - x).abs().max().item())
    # 16 layers, each off by at most one unit in the last place before the next layer amplifies it
    assert worst <= 2.0 ** -8, f"logits differ from the plain fixed-point network by {worst}"
    return worst


def pipeline_legs(args, torch):
    """The timed steps (default mode), the serial pass and its per-kind split, and the best mode."""
    from paper_2209_13643_amd import bench_configs, mpc, synth
    seed = synth.BASE_SEED + 4
    net = Net(seed)
    layers = net.layers
    macs = sum(bench_configs.layer_macs(L) for L in layers) * N_MB
    relu_el = pool_cmp = 0
    for L in layers:
        n_out = (L.B * L.Ho * L.Wo * L.Cout) if isinstance(L, synth.Conv) else L.M * L.N
        if L.relu: relu_el += n_out * N_MB
        if isinstance(L, synth.Conv) and L.pool: pool_cmp += 3 * (n_out // 4) * N_MB
    # ---- the timed region: exactly `steps` pipelined steps between two synchronisations
    ms_step = net.timed(net.step_pipelined, args.steps, args.warmup)
    err = check_network(net, torch)
    ms_serial = net.timed(net.step_serial, max(2, args.steps // 2), 2)
    # ---- serial pass with timing regions: which kind of call takes the time
    lane = net.lanes[0]
    lane.set_profiling(True); lane.profile_reset()
    reps = 3
    for _ in range(reps):
        net.step_serial()
    net.sync(); lane.set_profiling(False)
    lin = sum(lane.profile_samples(mpc.PROF_LINEAR)) / reps
    gem = sum(lane.profile_samples(mpc.PROF_GEMM_KERNEL)) / reps
    rel = sum(lane.profile_samples(mpc.PROF_RELU)) / reps
    lane.profile_reset()
    gs = net.graphs()
    ms_graphs = net.timed(lambda: [g.launch(ln) for g, ln in zip(gs, net.lanes)], args.steps, 3)
    del gs
    net.close(); del net
    torch.cuda.empty_cache()
    out = {
        "ms_per_step": ms_step, "macs": macs, "relu_elements": relu_el, "pool_comparisons": pool_cmp, "err": err,
        "pipeline": {"default_mode": {"relu": "whole-word (mpc_relu)", "exchange": "copy kernels", "planes": "recoded in the call",
                                      "serial_ms": ms_serial, "four_lanes_ms": ms_step,
                                      "four_lanes_recorded_graphs_ms": ms_graphs,
                                      "speedup_four_lanes": ms_serial / ms_step,
                                      "speedup_recorded_graphs": ms_serial / ms_graphs,
                                      "images_per_s_serial": N_MB * MICRO_BATCH / ms_serial * 1e3,
                                      "images_per_s_four_lanes": N_MB * MICRO_BATCH / ms_step * 1e3,
                                      "images_per_s_recorded_graphs": N_MB * MICRO_BATCH / ms_graphs * 1e3}},
        "per_kind": {"source": "serial pass, HIP-event regions of the library, batch 128",
                     "ms_beaver_calls": lin, "ms_gemm_kernels": gem, "ms_relu_calls": rel,
                     "ms_maxpool_and_gaps": ms_serial - lin - rel,
                     "beaver_macs_per_s": macs / (lin * 1e-3), "relu_elems_per_s": relu_el / (rel * 1e-3),
                     "beaver_call_frac_of_int8_peak": INT8_OPS_PER_SECURE_MAC * macs / (lin * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                     "gemm_kernel_frac_of_int8_peak": INT8_OPS_PER_SECURE_MAC * macs / (gem * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                     "relu_frac_of_hbm_peak": RELU_BYTES_PER_ELEMENT * relu_el / (rel * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if not args.no_best_mode:
        net = Net(seed, packed_relu=True, prepared=True, pool_first=True, exchange="put")
        b_pipe = net.timed(net.step_pipelined, args.steps, 3)
        err_b = check_network(net, torch)
        b_serial = net.timed(net.step_serial, max(2, args.steps // 2), 2)
        gs = net.graphs()
        b_graphs = net.timed(lambda: [g.launch(ln) for g, ln in zip(gs, net.lanes)], args.steps, 3)
        del gs
        net.close(); del net
        torch.cuda.empty_cache()
        out["pipeline"]["best_mode"] = {
            "relu": "sign-only packed chain (mpc_relu_msb), pooled layers as ReLU(maxpool(z))",
            "exchange": "remote store", "planes": "prepared (input-independent operands recoded ahead of time)",
            "serial_ms": b_serial, "four_lanes_ms": b_pipe, "four_lanes_recorded_graphs_ms": b_graphs,
            "speedup_four_lanes": b_serial / b_pipe, "speedup_recorded_graphs": b_serial / b_graphs,
            "images_per_s_four_lanes": N_MB * MICRO_BATCH / b_pipe * 1e3,
            "images_per_s_recorded_graphs": N_MB * MICRO_BATCH / b_graphs * 1e3, "max_abs_err_logits": err_b}
    return out


def per_config_table(args):
    """All five workloads layer by layer (HIP-event regions, 10 repetitions after 5 warm-up), summed per config."""
    from paper_2209_13643_amd import bench_configs, synth
    table = []
    for idx in range(len(synth.CONFIGS)):
        name, rows = bench_configs.bench_layers(idx, reps=10)
        macs = sum(bench_configs.layer_macs(L) for L in synth.CONFIGS[idx]().layers)
        call = sum(r["call_ms"] for r in rows); kern = sum(r["kernel_ms"] for r in rows); prep = sum(r["prepared_call_ms"] for r in rows)
        e = {"config": idx, "name": name, "secure_macs": macs, "ms_beaver_calls": call, "ms_beaver_calls_prepared_planes": prep,
             "ms_gemm_kernels": kern, "secure_macs_per_s": macs / (call * 1e-3),
             "call_frac_of_int8_peak": INT8_OPS_PER_SECURE_MAC * macs / (call * 1e-3) / 1e12 / INT8_PEAK_TOPS,
             "prepared_call_frac_of_int8_peak": INT8_OPS_PER_SECURE_MAC * macs / (prep * 1e-3) / 1e12 / INT8_PEAK_TOPS,
             "kernel_frac_of_int8_peak": INT8_OPS_PER_SECURE_MAC * macs / (kern * 1e-3) / 1e12 / INT8_PEAK_TOPS}
        rl = [r for r in rows if "relu_ms" in r]
        if rl:
            n = sum(r["relu_n"] for r in rl); t = sum(r["relu_ms"] for r in rl); tm = sum(r["msb_ms"] for r in rl)
            e.update(relu_elements=n, ms_relu_calls=t, relu_elems_per_s=n / (t * 1e-3),
                     relu_frac_of_hbm_peak=RELU_BYTES_PER_ELEMENT * n / (t * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     ms_relu_msb_calls=tm, relu_msb_elems_per_s=n / (tm * 1e-3),
                     relu_msb_frac_of_hbm_peak=RELU_MSB_BYTES_PER_ELEMENT * n / (tm * 1e-3) / 1e9 / HBM_PEAK_GBS)
        if args.layers:
            e["layers"] = [{k: (round(v, 6) if isinstance(v, float) else v) for k, v in r.items()} for r in rows]
        table.append(e)
    return table


def config1_leg(steps, warmup, pmc_summary):
    """configs[1] alone (VGG16-style conv block: Beaver conv [16384x1152]x[1152x128] + truncation, secure ReLU on its
    2 097 152 outputs): the step whose kernels the committed rocprofv3 summaries cover (`bench.py --only-config1`).
    Returns the three roofline objects and the leg's times."""
    import torch
    from paper_2209_13643_amd import bench_configs, dealer, mpc, synth

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

    def timed(fn):
        for _ in range(warmup):
            fn()
        lane.sync(); torch.cuda.synchronize()
        lane.set_profiling(True); lane.profile_reset()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        lane.sync(); torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        lane.set_profiling(False)
        reg = {}
        for key, which in (("gemm_kernel", mpc.PROF_GEMM_KERNEL), ("beaver_conv_call", mpc.PROF_LINEAR), ("relu_call", mpc.PROF_RELU)):
            smp = lane.profile_samples(which)
            if smp:
                reg[key] = {"mean_ms": sum(smp) / len(smp), "median_ms": statistics.median(smp), "min_ms": min(smp),
                            "max_ms": max(smp), "n": len(smp)}
        return ms, reg

    ms_step, reg = timed(step)
    gemm_ms, lin_ms, relu_ms = (reg[k]["mean_ms"] for k in ("gemm_kernel", "beaver_conv_call", "relu_call"))
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
    _, r2 = timed(lambda: lane.relu(z, mat_p, out=y2, packed=True))
    msb_ms = r2["relu_call"]["mean_ms"]; reg["relu_msb_call"] = r2["relu_call"]
    assert torch.equal(y2[0] + y2[1], torch.clamp(rec_z, min=0)), "mpc_relu_msb output does not reconstruct to max(z, 0)"
    # the Beaver convolution with the input-independent operands' digit planes recoded ahead of time
    right, left = lane.prepare_conv2d(d["a"], d["b"], d["f_public"], L.pad, L.stride)
    _, r3 = timed(lambda: lane.conv2d_prepared(d["x"], d["a"], d["c"], right, left, L.KH, L.KW, L.pad, L.stride, out=y2))
    prep_ms = r3["beaver_conv_call"]["mean_ms"]; reg["beaver_conv_call_prepared_planes"] = r3["beaver_conv_call"]
    assert torch.equal(y2[0], z[0]) and torch.equal(y2[1], z[1]), "prepared-plane convolution differs from the plain call"
    lane.close()

    macs = M * K * N
    tops = lambda ms: INT8_OPS_PER_SECURE_MAC * macs / (ms * 1e-3) / 1e12
    pmc = read_pmc_summary(pmc_summary)
    traffic = relu_traffic = msb_traffic = None
    if pmc is not None:
        src = {"source": pmc["source"], "measured_in_this_run": False}
        traffic = {"fetch_bytes": pmc["fetch_bytes"], "write_bytes": pmc["write_bytes"],
                   "algorithmic_bytes": bench_configs.gemm_algorithmic_bytes(L), **src}
        if "relu_bytes_per_element" in pmc: relu_traffic = {"bytes_per_element": pmc["relu_bytes_per_element"], **src}
        if "relu_msb_bytes_per_element" in pmc: msb_traffic = {"bytes_per_element": pmc["relu_msb_bytes_per_element"], **src}
    relu_gbs = RELU_BYTES_PER_ELEMENT * n / (relu_ms * 1e-3) / 1e9
    msb_gbs = RELU_MSB_BYTES_PER_ELEMENT * n / (msb_ms * 1e-3) / 1e9
    return {
        "times": {"workload": "configs[1] vgg16-cifar-conv-block: batch 64, 128x16x16, conv3x3 128->128 pad 1 = Beaver GEMM "
                              f"[{M}x{K}]x[{K}x{N}] + truncation + secure ReLU on {n} elements",
                  "ms_step": ms_step, "ms_beaver_conv_call": lin_ms, "ms_gemm_kernel": gemm_ms, "ms_relu_call": relu_ms,
                  "ms_relu_msb_call": msb_ms, "ms_beaver_conv_call_prepared_planes": prep_ms,
                  "secure_macs_per_s": macs / (lin_ms * 1e-3), "secure_macs_per_s_prepared_planes": macs / (prep_ms * 1e-3),
                  "relu_elems_per_s": n / (relu_ms * 1e-3), "relu_msb_elems_per_s": n / (msb_ms * 1e-3),
                  "region_times": reg, "max_abs_err_vs_float64": err},
        "roofline": {
            "kernel": "secure GEMM: k_limb_gemm<2,2,true> (both parties, [e|a_i] x [b_i';f], fused add-c + truncation) inside the "
                      "Beaver conv call (mask, exchange, digit recoding, GEMM)",
            "workload": f"configs[1] conv3x3 as [{M}x{K}]x[{K}x{N}]",
            "bound": "mfma", "achieved": tops(lin_ms), "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": tops(lin_ms) / INT8_PEAK_TOPS,
            "level": "call: 288 int8 ops per secure MAC over the whole Beaver conv call (HIP events around the call's launches)",
            "kernel_only": {"achieved": tops(gemm_ms), "frac": tops(gemm_ms) / INT8_PEAK_TOPS, "ms": gemm_ms,
                            "level": "HIP events around the GEMM launch alone"},
            "prepared_planes_call": {"achieved": tops(prep_ms), "frac": tops(prep_ms) / INT8_PEAK_TOPS, "ms": prep_ms},
            "ms_call": lin_ms, "traffic": traffic,
            "note": "power-limited attainable rate with random int8 operands measured on this chip with a back-to-back "
                    "MFMA loop is about 3070 TOP/s"},
        "roofline_relu": {
            "kernel": "secure ReLU chain: k_relu_stage<0..9> (both parties per launch) + k_wire_words / k_wire_bytes",
            "workload": f"configs[1], {n} elements", "bound": "hbm", "achieved": relu_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": relu_gbs / HBM_PEAK_GBS, "bytes_per_element": RELU_BYTES_PER_ELEMENT, "ms_call": relu_ms,
            "dram_compulsory": {"bytes_per_element": RELU_COMPULSORY_BYTES,
                                "frac": RELU_COMPULSORY_BYTES * n / (relu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                "note": "inputs, outputs and offline material only: the exchanged words and the state carried from "
                                        "round to round are served by the 256 MB last-level cache when a chunk fits it"},
            "traffic": relu_traffic},
        "roofline_relu_msb": {
            "kernel": "sign-only packed ReLU chain: k_relu_msb_stage<0..9> + k_wire_words / k_wire_bytes",
            "workload": f"configs[1], {n} elements", "bound": "hbm", "achieved": msb_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": msb_gbs / HBM_PEAK_GBS, "bytes_per_element": RELU_MSB_BYTES_PER_ELEMENT, "ms_call": msb_ms,
            "dram_compulsory": {"bytes_per_element": RELU_MSB_COMPULSORY_BYTES,
                                "frac": RELU_MSB_COMPULSORY_BYTES * n / (msb_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "traffic": msb_traffic},
    }


def three_party_leg(steps, warmup):
    """configs[1]'s three calls with three simulated parties, each timed by its own region."""
    import torch
    from paper_2209_13643_amd import dealer, mpc, synth

    L = synth.config_vgg_block().layers[0]
    lane = mpc.Lane(0); lane.use_single_queue()
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
    lane.close()
    macs = M * K * N
    return {"parties": 3, "workload": "configs[1]", "ms_beaver_conv_call": lin, "value": macs / (lin * 1e-3), "unit": "secure MACs/s",
            "ms_gemm_kernels": gemm, "gemm_frac_of_int8_peak": 432 * macs / (gemm * 1e-3) / 1e12 / INT8_PEAK_TOPS,
            "call_frac_of_int8_peak": 432 * macs / (lin * 1e-3) / 1e12 / INT8_PEAK_TOPS,
            "ms_relu_call": relu, "relu_value": n / (relu * 1e-3),
            "relu_bytes_per_element": RELU3_BYTES_PER_ELEMENT,
            "relu_frac_of_hbm_peak": RELU3_BYTES_PER_ELEMENT * n / (relu * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "ms_relu_msb_call": msb, "relu_msb_value": n / (msb * 1e-3),
            "relu_msb_bytes_per_element": RELU3_MSB_BYTES_PER_ELEMENT,
            "relu_msb_frac_of_hbm_peak": RELU3_MSB_BYTES_PER_ELEMENT * n / (msb * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "max_abs_err_vs_float64": err}


def cpu_baseline(budget_s=15.0, images=2):
    """The oracle as it stands, on the host cores: the same network, layer by layer (Alg. 1 with five direct
    ring convolutions, truncation, ReLU, max-pool), on a few images per repetition."""
    import oracle
    from paper_2209_13643_amd import synth

    layers = synth.config_vgg16_pipeline(images).layers
    rng = synth.rng_for(4, 7)
    mats = []
    for L in layers:                      # material of every layer, dealt once (untimed, as on the GPU)
        conv = isinstance(L, synth.Conv)
        xshape = (L.B, L.H, L.W, L.Cin) if conv else (L.M, L.K)
        wshape = (L.KH, L.KW, L.Cin, L.Cout) if conv else (L.K, L.N)
        Wt = synth.normal_fixed(rng, wshape, L.w_std)
        prod = (lambda A, Bf, L=L: oracle.ring_conv2d(A, Bf, L.pad, L.stride)) if conv else oracle.ring_matmul
        a, b, c = synth.deal_product_triple(rng, xshape, wshape, prod)
        n_out = (L.B * L.Ho * L.Wo * L.Cout) if conv else L.M * L.N
        m = dict(w=synth.share_additive(rng, Wt), a=a, b=b, c=c, relu=None, p1=None, p2=None)
        if L.relu: m["relu"] = synth.deal_relu_material(rng, n_out)
        if conv and L.pool:
            m["p1"] = synth.deal_relu_material(rng, n_out // 2); m["p2"] = synth.deal_relu_material(rng, n_out // 4)
        mats.append(m)
    X = synth.normal_fixed(rng, (images, 32, 32, 3), 1.0)
    x0 = synth.share_additive(rng, X)
    macs = relu_el = 0
    for L in layers:
        conv = isinstance(L, synth.Conv)
        macs += (L.B * L.Ho * L.Wo * L.KH * L.KW * L.Cin * L.Cout) if conv else L.M * L.K * L.N
        n_out = (L.B * L.Ho * L.Wo * L.Cout) if conv else L.M * L.N
        if L.relu: relu_el += n_out
        if conv and L.pool: relu_el += 3 * (n_out // 4)
    t_lin = t_non = 0.0
    reps = 0
    t_start = time.perf_counter()
    while reps < 1 or (time.perf_counter() - t_start) < budget_s:
        x = x0
        for L, m in zip(layers, mats):
            t0 = time.perf_counter()
            if isinstance(L, synth.Conv):
                xs = (x[0].reshape(L.B, L.H, L.W, L.Cin), x[1].reshape(L.B, L.H, L.W, L.Cin))
                z = oracle.truncate(oracle.beaver_conv2d(xs, m["w"], m["a"], m["b"], m["c"], L.pad, L.stride), 16)
            else:
                xs = (x[0].reshape(L.M, L.K), x[1].reshape(L.M, L.K))
                z = oracle.truncate(oracle.beaver_matmul(xs, m["w"], m["a"], m["b"], m["c"]), 16)
            t1 = time.perf_counter()
            if m["relu"] is not None: z = oracle.relu(z, m["relu"]).y
            if m["p1"] is not None: z = oracle.maxpool2x2(z, m["p1"], m["p2"])
            t2 = time.perf_counter()
            t_lin += t1 - t0; t_non += t2 - t1
            x = z
        reps += 1
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next(l.split(":", 1)[1].strip() for l in f if l.startswith("model name"))
    except (OSError, StopIteration):
        pass
    total = t_lin + t_non
    return {"value": macs * reps / total, "unit": "secure MACs/s", "cores": oracle.n_threads(), "cpu": cpu_model,
            "kind": "oracle", "relu_value": relu_el * reps / total, "relu_unit": "secure comparisons/s",
            "images_per_s": images * reps / total,
            "beaver_macs_per_s_linear_time_only": macs * reps / t_lin, "relu_elems_per_s_nonlinear_time_only": relu_el * reps / t_non,
            "sample": f"{reps} x ({images} of the step's 128 images through the whole network: Alg. 1 with five direct ring "
                      f"convolutions + truncation, ReLU and max-pool per layer), {total:.1f} s of CPU work; rates are over the "
                      f"whole pass like the GPU's `value`"}


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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-three-party", action="store_true", help="skip the three-party leg (configs[1], N = 3)")
    ap.add_argument("--no-per-config", action="store_true", help="skip the table of all five workloads (and the rooflines taken from it)")
    ap.add_argument("--no-best-mode", action="store_true", help="skip the best-mode pipeline leg")
    ap.add_argument("--layers", action="store_true", help="per-layer rows inside `configs`")
    ap.add_argument("--only-config1", action="store_true",
                    help="run only the configs[1] leg (conv block + ReLU) and print its rooflines: the command the rocprofv3 summaries are taken with")
    ap.add_argument("--cpu-all-configs", action="store_true",
                    help="also time the oracle on a sample of every layer of all five workloads")
    ap.add_argument("--pmc-summary", default=os.path.join(ROOT, "profiles", "gemm_vgg_block_hbm_traffic.md"),
                    help="counter summary to quote as roofline.traffic (ignored unless taken from the current sources)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build simulates both parties on a single MI355X and has no "
              "multi-GPU path (run with --gpus 1).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2209_13643_amd import bench_configs, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)

    if args.only_config1:
        # the configs[1] leg alone, for rocprofv3 runs: same code, same kernels, same roofline objects
        c1 = config1_leg(args.steps, args.warmup, args.pmc_summary)
        print(json.dumps({"mode": "configs[1] leg only", "steps": args.steps, "warmup": args.warmup, **c1}))
        return

    legs = pipeline_legs(args, torch)
    ms_step = legs["ms_per_step"]
    out = {
        "metric": "secure Z_2^64 MACs/s (Beaver GEMM) + secure ReLU elems/s, 1 GPU, online",
        "value": legs["macs"] / (ms_step * 1e-3), "unit": "secure MACs/s",
        "relu_value": (legs["relu_elements"] + legs["pool_comparisons"]) / (ms_step * 1e-3),
        "relu_unit": "secure comparisons/s (ReLU elements + max-pool comparisons)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64 ring (int8 digits, int32 accumulate)",
        "data": "synthetic",
        "config": {"workload": "configs[4] vgg16-cifar inter-batch pipeline: 32x32x3 input, 13 conv3x3 layers 64..512 channels with "
                               "2x2 max-pooling, FC 512-512-10, batch 128 = 4 micro-batches of 32 on four lanes; per layer Beaver "
                               "conv / matmul + truncation, whole-word secure ReLU, max-pool by two conversions",
                   "parties": 2, "frac_bits": 16, "lanes": N_MB, "lane": "single in-order queue each", "relu_chunks": "auto (about 2^20 elements each)",
                   "secure_macs_per_step": legs["macs"], "relu_elements_per_step": legs["relu_elements"],
                   "maxpool_comparisons_per_step": legs["pool_comparisons"], "images_per_s": N_MB * MICRO_BATCH / ms_step * 1e3,
                   "max_abs_err_logits_vs_plain_fixed_point": legs["err"]},
        "pipeline": legs["pipeline"], "per_kind": legs["per_kind"],
    }
    if not args.no_per_config:
        out["configs"] = per_config_table(args)
    c1 = config1_leg(args.steps, args.warmup, args.pmc_summary)
    out["config1_step"] = c1["times"]
    for k in ("roofline", "roofline_relu", "roofline_relu_msb"):
        out[k] = c1[k]
    if not args.no_three_party:
        out["three_party"] = three_party_leg(max(5, args.steps // 2), args.warmup)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
        if args.cpu_all_configs:
            out["cpu_baseline"]["per_layer"] = cpu_baseline_all_configs()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
