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
# the same chain with the exchange by remote store (no copy kernels; a level stage recomputes its own masked words from
# the carried state and stores them to the peer only; so do the first and the B2A stage, whose own words the next stage
# re-forms from x, r, P and from x, ra and the opened bit), per party in words: A2B copy 2, first 8, level-0 stage 18,
# levels 1..4 22 each, level 5 18, sign 7, B2A 6, select 8 = 155 W, plus 9 bytes (sign bit, random bit, masked bits)
RELU_PUT_BYTES_PER_ELEMENT = 2 * (155 * 8 + 9)
RELU_COMPULSORY_BYTES = 86 * 8 + 2                        # x, y, r, 12 AND triples, B2A pair, select triple: DRAM-compulsory
# the sign-only packed chain (mpc_relu_msb), same three classes: 31.72 W + 2 B, 71.25 W + 8 B, 41.56 W + 6 B
RELU_MSB_BYTES_PER_ELEMENT = (31.71875 + 71.25 + 41.5625) * 8 + 16
# remote store: one of the four traversals of every opened word less, and the first and the B2A stage store their
# masked words (2 W each per party) to the peer only (the select stage reads two bytes more instead)
RELU_MSB_PUT_BYTES_PER_ELEMENT = RELU_MSB_BYTES_PER_ELEMENT - 71.25 * 8 / 4 - 2 * 4 * 8 + 2 * 2
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
    forms = dict((k, (float(f), float(w))) for k, f, w in
                 re.findall(r"k_limb_gemm in the ([a-z ]+call) \([a-z ]+\)\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|", text))
    if not m or "folded prepared call" not in forms or m.group(1) != sources_digest():
        return None
    out = {"fetch_bytes": forms["folded prepared call"][0] * 2 ** 20, "write_bytes": forms["folded prepared call"][1] * 2 ** 20,
           "source": os.path.relpath(path, ROOT), "measured_in_this_run": False}
    if "plain call" in forms:
        out["four_product_launch"] = {"fetch_bytes": forms["plain call"][0] * 2 ** 20, "write_bytes": forms["plain call"][1] * 2 ** 20}
    for key, label in (("relu_bytes_per_element", "whole words, exchange by copy"), ("relu_put_bytes_per_element", "whole words, exchange by remote store"),
                       ("relu_msb_bytes_per_element", "sign-only, exchange by copy"), ("relu_msb_put_bytes_per_element", "sign-only, exchange by remote store")):
        r = re.search(re.escape(label) + r"[^\n]*= (\d+) bytes per element", text)
        if r:
            out[key] = int(r.group(1))
    return out


class Net:
    """configs[4] on four lanes in one mode: lanes, material, inputs and preallocated outputs."""

    def __init__(self, seed, packed_relu=False, prepared=False, fold=False, pool_first=False, exchange="copy"):
        import torch
        from paper_2209_13643_amd import dealer, mpc, pipeline, synth
        self.pipeline, self.torch = pipeline, torch
        self.layers = synth.config_vgg16_pipeline(MICRO_BATCH).layers
        self.lanes = [mpc.Lane(0, single_queue=True) for _ in range(N_MB)]
        for ln in self.lanes:
            ln.set_exchange(exchange)
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
                pipeline.prepare_layers(self.lanes[m], self.layers, st, fold=fold)
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
        self.pipeline.share_cache(self.lanes)           # the graphs run four at a time
        for m, ln in enumerate(self.lanes):
            with ln.capture() as cap:
                self.pipeline.forward(ln, self.layers, self.states[m], self.xs[m], [], outs=self.outs[m])
            gs.append(cap.graph)
        self.pipeline.share_cache(self.lanes, False)
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


def run_mode(seed, args, torch, with_kinds=False, **mode):
    """configs[4] in one mode: four lanes eager (the timed step when `with_kinds`), serial on one lane, and one
    recorded graph per lane; optionally the serial pass split by kind of call (HIP-event regions)."""
    from paper_2209_13643_amd import mpc
    net = Net(seed, **mode)
    ms_pipe = net.timed(net.step_pipelined, args.steps, args.warmup)
    err = check_network(net, torch)
    ms_serial = net.timed(net.step_serial, max(2, args.steps // 2), 2)
    res = {"serial_ms": ms_serial, "four_lanes_ms": ms_pipe, "max_abs_err_logits": err}
    if with_kinds:
        lane = net.lanes[0]
        lane.set_profiling(True); lane.profile_reset()
        reps = 3
        for _ in range(reps):
            net.step_serial()
        net.sync(); lane.set_profiling(False)
        res["kinds"] = tuple(sum(lane.profile_samples(w)) / reps for w in (mpc.PROF_LINEAR, mpc.PROF_GEMM_KERNEL, mpc.PROF_RELU))
        lane.profile_reset()
    gs = net.graphs()
    ms_graphs = net.timed(lambda: [g.launch(ln) for g, ln in zip(gs, net.lanes)], args.steps, 3)
    del gs
    net.close(); del net
    torch.cuda.empty_cache()
    res.update(four_lanes_recorded_graphs_ms=ms_graphs, speedup_four_lanes=ms_serial / ms_pipe,
               speedup_recorded_graphs=ms_serial / ms_graphs,
               images_per_s_serial=N_MB * MICRO_BATCH / ms_serial * 1e3,
               images_per_s_four_lanes=N_MB * MICRO_BATCH / ms_pipe * 1e3,
               images_per_s_recorded_graphs=N_MB * MICRO_BATCH / ms_graphs * 1e3)
    return res


def pipeline_legs(args, torch):
    """The timed steps (the step's mode), its serial pass split by kind, and the other modes beside it."""
    from paper_2209_13643_amd import bench_configs, synth
    seed = synth.BASE_SEED + 4
    layers = synth.config_vgg16_pipeline(MICRO_BATCH).layers
    macs = sum(bench_configs.layer_macs(L) for L in layers) * N_MB
    relu_el = pool_cmp = 0
    for L in layers:
        n_out = (L.B * L.Ho * L.Wo * L.Cout) if isinstance(L, synth.Conv) else L.M * L.N
        if L.relu: relu_el += n_out * N_MB
        if isinstance(L, synth.Conv) and L.pool: pool_cmp += 3 * (n_out // 4) * N_MB
    # ---- the timed region: exactly `steps` four-lane steps between two synchronisations
    step = run_mode(seed, args, torch, with_kinds=True, prepared=True, fold=True, exchange="put")
    lin, gem, rel = step.pop("kinds")
    ms_step, ms_serial = step["four_lanes_ms"], step["serial_ms"]
    step = {"relu": "whole words (mpc_relu: the full 64-bit adder of Sec. 4.2)", "exchange": "remote store into the peer's receive buffer",
            "planes": "prepared: weight masks opened ahead (Alg. 3), triples' digit planes and party 0's folded addend formed offline",
            "network": "as written (ReLU, then max-pool)", **step}
    out = {
        "ms_per_step": ms_step, "macs": macs, "relu_elements": relu_el, "pool_comparisons": pool_cmp, "err": step["max_abs_err_logits"],
        "pipeline": {"step_mode": step},
        "per_kind": {"source": "serial pass of the step's mode, HIP-event regions of the library, batch 128",
                     "ms_beaver_calls": lin, "ms_gemm_kernels": gem, "ms_relu_calls": rel,
                     "ms_maxpool_and_gaps": ms_serial - lin - rel,
                     "beaver_macs_per_s": macs / (lin * 1e-3), "relu_elems_per_s": relu_el / (rel * 1e-3),
                     "beaver_call_frac_of_int8_peak": INT8_OPS_PER_SECURE_MAC * macs / (lin * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                     "gemm_kernel_frac_of_int8_peak": INT8_OPS_PER_SECURE_MAC * macs / (gem * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                     "relu_frac_of_hbm_peak": RELU_PUT_BYTES_PER_ELEMENT * relu_el / (rel * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "relu_bytes_per_element": RELU_PUT_BYTES_PER_ELEMENT,
                     "note": "the four-lane pipeline hides MFMA-bound GEMM time behind the HBM-bound ReLU, pooling and recoding "
                             "of other micro-batches: its floor is the larger of the two sums, here the HBM-bound one"},
    }
    if not args.no_other_modes:
        r = run_mode(seed, args, torch)
        out["pipeline"]["copy_exchange_planes_in_call"] = {
            "relu": "whole words (mpc_relu)", "exchange": "copy kernels on the wire queue", "planes": "recoded inside every call (mpc_conv2d with f_public)",
            "network": "as written", **r}
        r = run_mode(seed, args, torch, packed_relu=True, prepared=True, fold=True, pool_first=True, exchange="put")
        out["pipeline"]["best_mode"] = {
            "relu": "sign-only packed chain (mpc_relu_msb: the adder evaluated where bit 63 depends on it)",
            "exchange": "remote store", "planes": "prepared and folded", "network": "pooled layers as ReLU(maxpool(z))", **r}
    return out


def per_config_table(args):
    """All five workloads layer by layer (HIP-event regions, 10 repetitions after 5 warm-up), summed per config."""
    from paper_2209_13643_amd import bench_configs, synth
    table = []
    for idx in range(len(synth.CONFIGS)):
        name, rows = bench_configs.bench_layers(idx, reps=10)
        macs = sum(bench_configs.layer_macs(L) for L in synth.CONFIGS[idx]().layers)
        call = sum(r["call_ms"] for r in rows); kern = sum(r["kernel_ms"] for r in rows)
        # products of two activations (per-head attention) run the folded call that opens f online
        fold = sum(r["folded_call_ms"] for r in rows)
        fkern = sum(r["folded_kernel_ms"] for r in rows)
        f = lambda ms: INT8_OPS_PER_SECURE_MAC * macs / (ms * 1e-3) / 1e12 / INT8_PEAK_TOPS
        e = {"config": idx, "name": name, "secure_macs": macs,
             "folded_prepared_calls": {"ms_beaver_calls": fold, "ms_gemm_kernels": fkern, "secure_macs_per_s": macs / (fold * 1e-3),
                                       "call_frac_of_int8_peak": f(fold), "kernel_frac_of_int8_peak": f(fkern),
                                       "call_frac_of_hbm_peak": sum(r["folded_call_bytes"] for r in rows) / (fold * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                       "executed_int8_ops_per_secure_mac": 216,
                                       "note": "three ring products per call, party 0's addend c_0 - a_0 b_0 and the planes of the "
                                               "triple's a, b from the offline phase; layers whose right operand is a weight also "
                                               "keep the planes of f; products of two activations (per-head attention) open f in "
                                               "the call; remote-store exchange throughout"},
             "plain_calls_remote_store": {"ms_beaver_calls": sum(r["call_put_ms"] for r in rows), "ms_gemm_kernels": sum(r["kernel_put_ms"] for r in rows),
                                          "secure_macs_per_s": macs / (sum(r["call_put_ms"] for r in rows) * 1e-3),
                                          "call_frac_of_int8_peak": f(sum(r["call_put_ms"] for r in rows)),
                                          "kernel_frac_of_int8_peak": f(sum(r["kernel_put_ms"] for r in rows)),
                                          "executed_int8_ops_per_secure_mac": 288},
             "plain_calls": {"ms_beaver_calls": call, "ms_gemm_kernels": kern, "secure_macs_per_s": macs / (call * 1e-3),
                             "call_frac_of_int8_peak": f(call), "kernel_frac_of_int8_peak": f(kern),
                             "executed_int8_ops_per_secure_mac": 288}}
        if idx > 0:
            # wall clock of back-to-back layers (no ReLU between): one call per layer, and the better of one call and two
            # row chunks on two lanes (Alg. 3's overlap inside a layer; the runner picks per layer)
            ov = bench_configs.bench_config_overlap(idx)
            one = sum(r["one_call_ms"] for r in ov); best = sum(min(r["one_call_ms"], r["two_chunks_ms"]) for r in ov)
            e["folded_calls_back_to_back_wall_clock"] = {
                "ms_one_call_per_layer": one, "call_frac_of_int8_peak_one_call": f(one),
                "ms_best_of_one_call_and_two_chunks_on_two_lanes": best, "call_frac_of_int8_peak_best": f(best),
                "layers_faster_as_two_chunks": [r["layer"] for r in ov if r["two_chunks_ms"] < r["one_call_ms"]]}
        rl = [r for r in rows if "relu_ms" in r]
        if rl:
            n = sum(r["relu_n"] for r in rl)
            t = {k: sum(r[k] for r in rl) for k in ("relu_ms", "relu_put_ms", "msb_ms", "msb_put_ms")}
            h = lambda bpe, ms: bpe * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
            e["relu"] = {"elements": n,
                         "whole_words_remote_store": {"ms": t["relu_put_ms"], "elems_per_s": n / (t["relu_put_ms"] * 1e-3),
                                                      "frac_of_hbm_peak": h(RELU_PUT_BYTES_PER_ELEMENT, t["relu_put_ms"])},
                         "whole_words_copy": {"ms": t["relu_ms"], "elems_per_s": n / (t["relu_ms"] * 1e-3),
                                              "frac_of_hbm_peak": h(RELU_BYTES_PER_ELEMENT, t["relu_ms"])},
                         "sign_only_remote_store": {"ms": t["msb_put_ms"], "elems_per_s": n / (t["msb_put_ms"] * 1e-3),
                                                    "frac_of_hbm_peak": h(RELU_MSB_PUT_BYTES_PER_ELEMENT, t["msb_put_ms"])},
                         "sign_only_copy": {"ms": t["msb_ms"], "elems_per_s": n / (t["msb_ms"] * 1e-3),
                                            "frac_of_hbm_peak": h(RELU_MSB_BYTES_PER_ELEMENT, t["msb_ms"])}}
        if args.layers:
            e["layers"] = [{k: (round(v, 6) if isinstance(v, float) else v) for k, v in r.items()} for r in rows]
        table.append(e)
    return table


def config1_leg(steps, warmup, pmc_summary):
    """configs[1] alone (VGG16-style conv block: Beaver conv [16384x1152]x[1152x128] + truncation, secure ReLU on its
    2 097 152 outputs): the step whose kernels the committed rocprofv3 summaries cover (`bench.py --only-config1`).
    Three sequences, each conv call followed by its ReLU as in a network (the chip is power-limited: a GEMM
    that follows a memory-bound phase runs at a higher clock than one in a back-to-back series of GEMMs):
      step mode   folded prepared conv call + whole-word ReLU with the remote-store exchange;
      plain       mpc_conv2d (planes recoded in the call, four ring products) + ReLU with the copy exchange;
      sign-only   the folded call + mpc_relu_msb.
    Returns the roofline objects and the leg's times."""
    import torch
    from paper_2209_13643_amd import bench_configs, dealer, mpc, synth

    wl = synth.config_vgg_block()
    L = wl.layers[0]
    M, K, N = L.gemm_mkn
    n = M * N
    lane = mpc.Lane(0, single_queue=True)      # one in-order queue per lane: no cross-stream event latency inside a call
    dev = lane.device
    g = dealer.gen(synth.BASE_SEED + wl.index, dev)
    d = dealer.conv_layer(lane, g, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, L.x_std, L.w_std)
    mat = dealer.relu_material(g, n, dev)
    mat_p = dealer.relu_material(g, n, dev, packed=True)
    z = tuple(torch.empty((L.B, L.Ho, L.Wo, L.Cout), dtype=torch.int64, device=dev) for _ in range(2))
    zf = tuple(torch.empty_like(z[0]) for _ in range(2))
    y = tuple(torch.empty_like(z[0]) for _ in range(2))
    y2 = tuple(torch.empty_like(z[0]) for _ in range(2))
    # offline: planes of the triple and of the opened weight mask, party 0's folded addend
    right, left = lane.prepare_conv2d(d["a"], d["b"], d["f_public"], L.pad, L.stride)
    cf = (lane.fold_conv2d(d["a"], d["b"], d["c"], L.pad, L.stride), d["c"][1])
    lane.sync(); torch.cuda.synchronize()

    def conv_folded():
        lane.conv2d_prepared(d["x"], d["a"], cf, right, left, L.KH, L.KW, L.pad, L.stride, out=zf,
                             flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)                    # Alg. 1 / Eq. 3 + truncation

    def conv_prepared():
        lane.conv2d_prepared(d["x"], d["a"], d["c"], right, left, L.KH, L.KW, L.pad, L.stride, out=zf)

    def conv_plain():
        lane.conv2d(d["x"], d["w"], d["a"], d["b"], d["c"], L.pad, L.stride, out=z)

    def timed(fn, exchange):
        lane.set_exchange(exchange)
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
        reg = {"ms_step": ms}
        for key, which in (("gemm_kernel", mpc.PROF_GEMM_KERNEL), ("beaver_conv_call", mpc.PROF_LINEAR), ("relu_call", mpc.PROF_RELU)):
            smp = lane.profile_samples(which)
            if smp:
                reg[key] = {"mean_ms": sum(smp) / len(smp), "median_ms": statistics.median(smp), "min_ms": min(smp),
                            "max_ms": max(smp), "n": len(smp)}
        return reg

    seq = {
        "step_mode": timed(lambda: (conv_folded(), lane.relu(zf, mat, out=y)), "put"),
        "plain_call_copy_exchange": timed(lambda: (conv_plain(), lane.relu(z, mat, out=y2)), "copy"),
        "prepared_call_unfolded": timed(lambda: (conv_prepared(), lane.relu(zf, mat, out=y2)), "put"),
        "sign_only_relu": timed(lambda: (conv_folded(), lane.relu(zf, mat_p, out=y2, packed=True)), "put"),
        "sign_only_relu_copy_exchange": timed(lambda: (conv_folded(), lane.relu(zf, mat_p, out=y2, packed=True)), "copy"),
    }
    # Alg. 3's overlap inside the layer: the batch cut into two image chunks, each a complete folded call, on two lanes
    # (one chunk's HBM-bound mask / exchange / recoding under the other's MFMA-bound GEMM).  Wall clock of back-to-back
    # layers without the ReLU between, the one-call layer timed the same way beside it.
    from paper_2209_13643_amd import pipeline
    lanes2 = [mpc.Lane(0, single_queue=True), mpc.Lane(0, single_queue=True)]
    for ln in lanes2:
        ln.set_exchange("put")
    chunked = pipeline.ChunkedLinear(lanes2, L, pipeline.LayerState(w=d["w"], a=d["a"], b=d["b"], c=d["c"], f_public=d["f_public"]), n_chunks=2)
    zc = tuple(torch.empty_like(z[0]) for _ in range(2))

    def wall(fn, sync_lanes):
        for _ in range(warmup):
            fn()
        for ln in sync_lanes:
            ln.sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        for ln in sync_lanes:
            ln.sync()
        return (time.perf_counter() - t0) * 1e3 / steps

    lane.set_exchange("put")
    # the chip's clock under a series of GEMMs depends on what ran just before: alternate the two forms and take medians
    ones, twos = [], []
    for _ in range(5):
        ones.append(wall(conv_folded, [lane]))
        twos.append(wall(lambda: chunked(d["x"], zc), lanes2))
    one_ms, two_ms = statistics.median(ones), statistics.median(twos)
    assert torch.equal(zc[0], zf[0]) and torch.equal(zc[1], zf[1]), "the layer as two image chunks differs from the one-call layer"
    for ln in lanes2:
        ln.close()
    chunk_leg = {"what": "configs[1] conv layer as two image chunks (32 + 32) on two lanes, each chunk a folded prepared call; wall clock "
                         "of back-to-back layers, no ReLU between; same output words as the one-call layer",
                 "ms_one_call": one_ms, "ms_two_chunks_two_lanes": two_ms, "speedup": one_ms / two_ms,
                 "call_frac_of_int8_peak_one_call": INT8_OPS_PER_SECURE_MAC * M * K * N / (one_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                 "call_frac_of_int8_peak_two_chunks": INT8_OPS_PER_SECURE_MAC * M * K * N / (two_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS}
    # what the matrix cores sustain on register-resident operands in the GEMM's instruction order, measured now (the
    # chip is power-limited: uniformly random digits, which is what shares are, hold a lower clock than constant operands)
    zero_tops, rand_tops = lane.mfma_rate(False, 2000, 30) / 1e12, lane.mfma_rate(True, 2000, 30) / 1e12
    kern_exec = INT8_OPS_PER_SECURE_MAC * 0.75 * M * K * N / (seq["step_mode"]["gemm_kernel"]["mean_ms"] * 1e-3) / 1e12
    ceiling = {"what": "mpc_mfma_rate: 72 v_mfma_i32_32x32x32_i8 per K step on register operands, one wave per SIMD, no memory "
                       "traffic, 30 launches of 2000 steps",
               "zero_operands_tops": zero_tops, "random_operands_tops": rand_tops,
               "gemm_launch_executed_tops": kern_exec, "gemm_launch_frac_of_random_operand_ceiling": kern_exec / rand_tops}
    # sanity on the results of the last steps: same shares from all three conv calls, ReLU of the reconstructed output exactly
    assert torch.equal(z[0], zf[0]) and torch.equal(z[1], zf[1]), "folded / prepared convolution differs from the plain call"
    rec_z = z[0] + z[1]
    assert torch.equal(y[0] + y[1], torch.clamp(rec_z, min=0)), "secure ReLU output does not reconstruct to max(z, 0)"
    assert torch.equal(y2[0] + y2[1], torch.clamp(rec_z, min=0)), "mpc_relu_msb output does not reconstruct to max(z, 0)"
    ref = torch.nn.functional.conv2d((d["X"].double() / 65536).permute(0, 3, 1, 2)[:2],
                                     (d["W"].double() / 65536).permute(3, 2, 0, 1), padding=L.pad).permute(0, 2, 3, 1)
    err = (rec_z[:2].double() / 65536 - ref).abs().max().item()
    assert err <= 2.0 ** -12, f"decoded conv output off by {err}"
    lane.close()

    macs = M * K * N
    tops = lambda ms: INT8_OPS_PER_SECURE_MAC * macs / (ms * 1e-3) / 1e12
    lvl = lambda r: {"achieved": tops(r["mean_ms"]), "frac": tops(r["mean_ms"]) / INT8_PEAK_TOPS, "ms": r["mean_ms"]}
    sm, pl, pu = seq["step_mode"], seq["plain_call_copy_exchange"], seq["prepared_call_unfolded"]
    pmc = read_pmc_summary(pmc_summary)
    traffic = traffic4 = None
    rt = {}
    if pmc is not None:
        src = {"source": pmc["source"], "measured_in_this_run": False}
        # algorithmic bytes of the folded launch: party 0 reads one left and one right plane set instead of two each
        alg4 = bench_configs.gemm_algorithmic_bytes(L)
        act, wts = L.B * L.H * L.W * L.Cin, L.KH * L.KW * L.Cin * L.Cout
        traffic = {"fetch_bytes": pmc["fetch_bytes"], "write_bytes": pmc["write_bytes"], "algorithmic_bytes": alg4 - 8 * (act + wts), **src}
        if "four_product_launch" in pmc:
            traffic4 = {**pmc["four_product_launch"], "algorithmic_bytes": alg4, **src}
        for key in ("relu_bytes_per_element", "relu_put_bytes_per_element", "relu_msb_bytes_per_element", "relu_msb_put_bytes_per_element"):
            if key in pmc:
                rt[key] = {"bytes_per_element": pmc[key], **src}
    gbs = lambda bpe, ms: bpe * n / (ms * 1e-3) / 1e9
    relu_ms, relu_copy_ms = sm["relu_call"]["mean_ms"], pl["relu_call"]["mean_ms"]
    msb_ms, msb_copy_ms = seq["sign_only_relu"]["relu_call"]["mean_ms"], seq["sign_only_relu_copy_exchange"]["relu_call"]["mean_ms"]
    call = lvl(sm["beaver_conv_call"])
    return {
        "times": {"workload": "configs[1] vgg16-cifar-conv-block: batch 64, 128x16x16, conv3x3 128->128 pad 1 = Beaver GEMM "
                              f"[{M}x{K}]x[{K}x{N}] + truncation + secure ReLU on {n} elements",
                  "ms_step": sm["ms_step"], "ms_beaver_conv_call": sm["beaver_conv_call"]["mean_ms"],
                  "ms_gemm_kernel": sm["gemm_kernel"]["mean_ms"], "ms_relu_call": relu_ms,
                  "secure_macs_per_s": macs / (sm["beaver_conv_call"]["mean_ms"] * 1e-3), "relu_elems_per_s": n / (relu_ms * 1e-3),
                  "plain_call_copy_exchange": {"ms_step": pl["ms_step"], "ms_beaver_conv_call": pl["beaver_conv_call"]["mean_ms"],
                                               "ms_gemm_kernel": pl["gemm_kernel"]["mean_ms"], "ms_relu_call": relu_copy_ms,
                                               "secure_macs_per_s": macs / (pl["beaver_conv_call"]["mean_ms"] * 1e-3),
                                               "relu_elems_per_s": n / (relu_copy_ms * 1e-3)},
                  "ms_relu_msb_call": msb_ms, "relu_msb_elems_per_s": n / (msb_ms * 1e-3),
                  "ms_relu_msb_call_copy_exchange": msb_copy_ms,
                  "overlap_inside_the_layer": chunk_leg,
                  "region_times": seq, "max_abs_err_vs_float64": err},
        "roofline": {
            "kernel": "secure GEMM: k_limb_gemm<2,2,true> (party 0: [x_0 + e_1] x [b_0 + f]; party 1: [e | a_1] x [b_1 ; f]; fused "
                      "addend + truncation) inside the folded prepared Beaver conv call (mask + remote-store exchange, digit recoding, GEMM)",
            "workload": f"configs[1] conv3x3 as [{M}x{K}]x[{K}x{N}]",
            "bound": "mfma", "achieved": call["achieved"], "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": call["frac"],
            "level": "call: 288 useful int8 ops per secure MAC (2 parties x 2 ring products x 36 digit products x 2, the frozen "
                     "accounting) over the whole Beaver conv call, HIP events around the call's launches",
            "executed_int8_ops_per_secure_mac": 216,
            "frac_executed_ops": call["frac"] * 0.75,
            "executed_note": "the folded call contracts three ring products online instead of four (party 0's a_0*b_0 moved to the "
                             "offline phase): `frac` counts the useful 288 ops, `frac_executed_ops` the 216 the matrix cores execute",
            "ms_call": call["ms"],
            "kernel_only": {**lvl(sm["gemm_kernel"]), "frac_executed_ops": lvl(sm["gemm_kernel"])["frac"] * 0.75,
                            "level": "HIP events around the GEMM launch alone"},
            "prepared_call_unfolded": {"call": lvl(pu["beaver_conv_call"]), "kernel_only": lvl(pu["gemm_kernel"]),
                                       "note": "prepared planes, four ring products (executed = useful ops)"},
            "plain_call": {"call": lvl(pl["beaver_conv_call"]), "kernel_only": lvl(pl["gemm_kernel"]),
                           "note": "mpc_conv2d: every digit plane recoded inside the call, copy exchange, four ring products",
                           "traffic": traffic4},
            "traffic": traffic,
            "measured_ceiling": ceiling},
        "roofline_relu": {
            "kernel": "secure ReLU chain on whole words, exchange by remote store: k_relu_stage<0..9, put> (both parties per launch) "
                      "+ k_wire_words<1> for the A2B masks",
            "workload": f"configs[1], {n} elements", "bound": "hbm", "achieved": gbs(RELU_PUT_BYTES_PER_ELEMENT, relu_ms),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs(RELU_PUT_BYTES_PER_ELEMENT, relu_ms) / HBM_PEAK_GBS,
            "bytes_per_element": RELU_PUT_BYTES_PER_ELEMENT, "ms_call": relu_ms, "elems_per_s": n / (relu_ms * 1e-3),
            "copy_exchange": {"kernel": "k_relu_stage<0..9> + k_wire_words / k_wire_bytes", "bytes_per_element": RELU_BYTES_PER_ELEMENT,
                              "ms_call": relu_copy_ms, "elems_per_s": n / (relu_copy_ms * 1e-3),
                              "achieved": gbs(RELU_BYTES_PER_ELEMENT, relu_copy_ms),
                              "frac": gbs(RELU_BYTES_PER_ELEMENT, relu_copy_ms) / HBM_PEAK_GBS, "traffic": rt.get("relu_bytes_per_element")},
            "dram_compulsory": {"bytes_per_element": RELU_COMPULSORY_BYTES,
                                "frac": gbs(RELU_COMPULSORY_BYTES, relu_ms) / HBM_PEAK_GBS,
                                "note": "inputs, outputs and offline material only: the exchanged words and the state carried from "
                                        "round to round are served by the 256 MB last-level cache when a chunk fits it"},
            "traffic": rt.get("relu_put_bytes_per_element")},
        "roofline_relu_msb": {
            "kernel": "sign-only packed ReLU chain, exchange by remote store: k_relu_msb_stage<0..9, put>",
            "workload": f"configs[1], {n} elements", "bound": "hbm", "achieved": gbs(RELU_MSB_PUT_BYTES_PER_ELEMENT, msb_ms),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs(RELU_MSB_PUT_BYTES_PER_ELEMENT, msb_ms) / HBM_PEAK_GBS,
            "bytes_per_element": RELU_MSB_PUT_BYTES_PER_ELEMENT, "ms_call": msb_ms, "elems_per_s": n / (msb_ms * 1e-3),
            "copy_exchange": {"bytes_per_element": RELU_MSB_BYTES_PER_ELEMENT, "ms_call": msb_copy_ms,
                              "elems_per_s": n / (msb_copy_ms * 1e-3), "achieved": gbs(RELU_MSB_BYTES_PER_ELEMENT, msb_copy_ms),
                              "frac": gbs(RELU_MSB_BYTES_PER_ELEMENT, msb_copy_ms) / HBM_PEAK_GBS, "traffic": rt.get("relu_msb_bytes_per_element")},
            "dram_compulsory": {"bytes_per_element": RELU_MSB_COMPULSORY_BYTES,
                                "frac": gbs(RELU_MSB_COMPULSORY_BYTES, msb_ms) / HBM_PEAK_GBS},
            "traffic": rt.get("relu_msb_put_bytes_per_element")},
    }


def three_party_leg(steps, warmup):
    """configs[1]'s three calls with three simulated parties, each timed by its own region."""
    import torch
    from paper_2209_13643_amd import dealer, mpc, synth

    L = synth.config_vgg_block().layers[0]
    lane = mpc.Lane(0, single_queue=True)
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


def cpu_baseline(budget_s=15.0, images=8):
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
    ap.add_argument("--no-other-modes", action="store_true", help="skip the pipeline legs beside the step's own mode")
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
                   "parties": 2, "frac_bits": 16, "lanes": N_MB, "lane": "single in-order queue each", "relu_chunks": "auto: 2^20 elements on one lane, 2^20 / lanes = 2^18 on the four concurrent lanes (their share of the last-level cache)",
                   "mode": legs["pipeline"]["step_mode"]["relu"] + "; exchange: " + legs["pipeline"]["step_mode"]["exchange"] + "; planes: " + legs["pipeline"]["step_mode"]["planes"],
                   "secure_macs_per_step": legs["macs"], "relu_elements_per_step": legs["relu_elements"],
                   "maxpool_comparisons_per_step": legs["pool_comparisons"], "images_per_s": N_MB * MICRO_BATCH / ms_step * 1e3,
                   "max_abs_err_logits_vs_plain_fixed_point": legs["err"]},
        "pipeline": legs["pipeline"], "per_kind": legs["per_kind"],
    }
    if not args.no_per_config:
        out["configs"] = per_config_table(args)
    c1 = config1_leg(args.steps, args.warmup, args.pmc_summary)
    out["config1_step"] = c1["times"]
    out["value_definition"] = {
        "value": "whole job: all secure MACs of the configs[4] batch over the wall time of the step (ReLU and pooling included)",
        "earlier_lines": "quoted the Beaver conv call of configs[1] alone (its secure MACs over the call's own time, plain call)",
        "that_quantity_now": {"plain_call": c1["times"]["plain_call_copy_exchange"]["secure_macs_per_s"],
                              "folded_prepared_call": c1["times"]["secure_macs_per_s"], "unit": "secure MACs/s"}}
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
