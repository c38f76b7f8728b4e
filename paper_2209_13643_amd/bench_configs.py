"""Per-config measurements on one MI355X: `python -m paper_2209_13643_amd.bench_configs [indices]`.

For every workload of `synth.CONFIGS` the secure layers are dealt on the device,
run a few times on a single-queue lane, and reported per layer: Beaver GEMM call
time, secure MACs/s, int8-MFMA fraction of the GEMM kernel, secure ReLU elems/s
and HBM fraction.  Config 4 (VGG16 on CIFAR shapes, batch 128 as 4 micro-batches
of 32) is additionally timed serial vs inter-batch pipelined (Sec. 4.3).
"""
from __future__ import annotations

import json
import sys
import time

import torch

from . import dealer, mpc, pipeline, synth

INT8_PEAK = 5.0e15
HBM_PEAK = 8.0e12
RELU_BYTES = 3514
RELU_MSB_BYTES = 1172.25      # the sign-only packed chain
RELU_PUT_BYTES = 2 * (155 * 8 + 9)            # whole words, exchange by remote store (bench.py derives it)
RELU_MSB_PUT_BYTES = RELU_MSB_BYTES - 71.25 * 8 / 4 - 2 * 4 * 8 + 2 * 2


def layer_macs(L):
    if isinstance(L, synth.Conv):
        M, K, N = L.gemm_mkn
        return M * K * N
    return L.M * L.K * L.N * max(L.batch, 1)


def gemm_algorithmic_bytes(L) -> int:
    """Both parties: read the digit planes of e and a_i (un-expanded activation for a conv), of
    f and b_i', the addend c_i; write z_i.  One byte per digit, eight digits per ring word."""
    if isinstance(L, synth.Conv):
        act, wts, out = L.B * L.H * L.W * L.Cin, L.KH * L.KW * L.Cin * L.Cout, L.B * L.Ho * L.Wo * L.Cout
    else:
        b = max(L.batch, 1)
        act, wts, out = b * L.M * L.K, b * L.K * L.N, b * L.M * L.N
    return 2 * 8 * (2 * act + 2 * wts + 2 * out)


def folded_call_algorithmic_bytes(L) -> int:
    """The folded call with the remote-store exchange, every word counted once per pass that has to touch it.  Activation
    (8-byte words): mask and send e_0 (read x_0, a_0; write e_0), party 1's recode (read x_1, a_1, e_0; write e_1 and the
    planes of e), party 0's recode (read x_0, e_1; write the planes of x_0 + e_1) = 11 passes, and the same 11 over the
    right operand when it is a share too (per-head attention).  GEMM launch: the planes of x_0 + e_1, e, a_1 (3 x
    activation) and of b_0 + f, b_1, f (3 x right operand), the addends c_i and the outputs z_i."""
    if isinstance(L, synth.Conv):
        act, wts, out, shared_right = L.B * L.H * L.W * L.Cin, L.KH * L.KW * L.Cin * L.Cout, L.B * L.Ho * L.Wo * L.Cout, False
    else:
        b = max(L.batch, 1)
        act, wts, out, shared_right = b * L.M * L.K, b * L.K * L.N, b * L.M * L.N, L.batch > 1
    return 8 * (14 * act + (14 if shared_right else 3) * wts + 4 * out)


def bench_layers(idx: int, reps: int = 20, workload=None):
    wl = workload if workload is not None else synth.CONFIGS[idx]()
    lane = mpc.Lane(0, single_queue=True)
    dev = lane.device
    g = dealer.gen(synth.BASE_SEED + idx, dev)
    rows = []
    for L in wl.layers:
        if isinstance(L, synth.Conv):
            d = dealer.conv_layer(lane, g, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, L.x_std, L.w_std)
            run = lambda: lane.conv2d(d["x"], d["w"], d["a"], d["b"], d["c"], L.pad, L.stride, out=z)
            n_out = L.B * L.Ho * L.Wo * L.Cout
            z = tuple(torch.empty((L.B, L.Ho, L.Wo, L.Cout), dtype=torch.int64, device=dev) for _ in range(2))
            shape = "x".join(map(str, L.gemm_mkn))
        else:
            d = dealer.matmul_layer(lane, g, L.M, L.K, L.N, L.x_std, L.w_std, batch=L.batch if L.batch > 1 else None)
            run = lambda: lane.beaver_matmul(d["x"], d["w"], d["a"], d["b"], d["c"], out=z)
            n_out = L.M * L.N * max(L.batch, 1)
            z = (torch.empty_like(d["c"][0]), torch.empty_like(d["c"][1]))
            shape = f"{L.M}x{L.K}x{L.N}" + (f" x{L.batch}" if L.batch > 1 else "")
        # the same layer as a folded prepared call: input-independent operands recoded ahead of time, party 0's
        # addend c_0 - a_0 b_0 formed offline (three ring products online instead of four)
        if isinstance(L, synth.Conv):
            right, left = lane.prepare_conv2d(d["a"], d["b"], d["f_public"], L.pad, L.stride)
            cf = (lane.fold_conv2d(d["a"], d["b"], d["c"], L.pad, L.stride), d["c"][1])
            run_prep = lambda: lane.conv2d_prepared(d["x"], d["a"], cf, right, left, L.KH, L.KW, L.pad, L.stride, out=z,
                                                    flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
        elif L.batch > 1:
            # per-head attention products multiply two activations: f opens in the call, a_1's and b_1's planes and
            # the folded addend still come from the offline phase
            right, left = lane.prepare_matmul(d["a"], d["b"], None)
            cf = (lane.fold_matmul(d["a"], d["b"], d["c"]), d["c"][1])
            run_prep = lambda: lane.beaver_matmul_folded(d["x"], d["w"], d["a"], d["b"], cf, right, left, out=z)
        else:
            right, left = lane.prepare_matmul(d["a"], d["b"], d["f_public"])
            cf = (lane.fold_matmul(d["a"], d["b"], d["c"]), d["c"][1])
            run_prep = lambda: lane.beaver_matmul_prepared(d["x"], d["a"], cf, right, left, out=z,
                                                           flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
        mat = dealer.relu_material(g, n_out, dev) if L.relu else None
        y = (torch.empty_like(z[0]), torch.empty_like(z[1])) if L.relu else None
        # both variants are timed in the same sequence (linear call, then the layer's ReLU): the chip is
        # power-limited, and a GEMM that follows a memory-bound phase runs at a higher clock than one in a
        # back-to-back series of GEMMs
        lane.set_exchange("put")
        for _ in range(5):
            run_prep()
            if mat: lane.relu(z, mat, out=y)
        lane.sync(); lane.set_profiling(True); lane.profile_reset()
        for _ in range(reps):
            run_prep()
            if mat: lane.relu(z, mat, out=y)
        lane.sync(); lane.set_profiling(False)
        prep_ms, prep_n = lane.profile(mpc.PROF_LINEAR); fk, fkn = lane.profile(mpc.PROF_GEMM_KERNEL)
        prep_ms /= prep_n; fk /= fkn
        put_ms = None
        if mat:
            rl, rn = lane.profile(mpc.PROF_RELU); put_ms = rl / rn
        del right, left, cf
        # the plain call in the same exchange mode (what a product of two activations runs as in that mode)
        for _ in range(5):
            run()
            if mat: lane.relu(z, mat, out=y)
        lane.sync(); lane.set_profiling(True); lane.profile_reset()
        for _ in range(reps):
            run()
            if mat: lane.relu(z, mat, out=y)
        lane.sync(); lane.set_profiling(False)
        pp_ms, pp_n = lane.profile(mpc.PROF_LINEAR); pk, pkn = lane.profile(mpc.PROF_GEMM_KERNEL)
        pp_ms /= pp_n; pk /= pkn
        lane.set_exchange("copy")
        for _ in range(5):
            run()
            if mat: lane.relu(z, mat, out=y)
        lane.sync(); lane.set_profiling(True); lane.profile_reset()
        for _ in range(reps):
            run()
            if mat: lane.relu(z, mat, out=y)
        lane.sync(); lane.set_profiling(False)
        gk, gn = lane.profile(mpc.PROF_GEMM_KERNEL); lin, ln = lane.profile(mpc.PROF_LINEAR)
        macs = layer_macs(L)
        # activation_product: both operands are shares (per-head attention); its folded call opens f online
        row = dict(layer=L.name, gemm=shape, repeat=L.repeat, activation_product=(not isinstance(L, synth.Conv)) and L.batch > 1,
                   call_ms=lin / ln, kernel_ms=gk / gn,
                   kernel_min_ms=min(lane.profile_samples(mpc.PROF_GEMM_KERNEL)),
                   folded_call_ms=prep_ms, folded_kernel_ms=fk, call_put_ms=pp_ms, kernel_put_ms=pk,
                   secure_macs_per_s=macs / (lin / ln * 1e-3), folded_secure_macs_per_s=macs / (prep_ms * 1e-3),
                   mfma_frac=288 * macs / (gk / gn * 1e-3) / INT8_PEAK, folded_mfma_frac=288 * macs / (fk * 1e-3) / INT8_PEAK,
                   gemm_hbm_frac=gemm_algorithmic_bytes(L) / (gk / gn * 1e-3) / HBM_PEAK,
                   folded_call_bytes=folded_call_algorithmic_bytes(L),
                   folded_call_hbm_frac=folded_call_algorithmic_bytes(L) / (prep_ms * 1e-3) / HBM_PEAK)
        if mat:
            rl, rn = lane.profile(mpc.PROF_RELU)
            row.update(relu_n=n_out, relu_ms=rl / rn, relu_elems_per_s=n_out / (rl / rn * 1e-3),
                       hbm_frac=RELU_BYTES * n_out / (rl / rn * 1e-3) / HBM_PEAK,
                       relu_put_ms=put_ms, relu_put_elems_per_s=n_out / (put_ms * 1e-3),
                       put_hbm_frac=RELU_PUT_BYTES * n_out / (put_ms * 1e-3) / HBM_PEAK)
            # the same ReLU on the sign's carry chain only, packed material
            del mat
            mat = dealer.relu_material(g, n_out, dev, packed=True)
            for ex, key in (("copy", "msb"), ("put", "msb_put")):
                lane.set_exchange(ex)
                for _ in range(5):
                    lane.relu(z, mat, out=y, packed=True)
                lane.sync(); lane.set_profiling(True); lane.profile_reset()
                for _ in range(reps):
                    lane.relu(z, mat, out=y, packed=True)
                lane.sync(); lane.set_profiling(False)
                rl, rn = lane.profile(mpc.PROF_RELU)
                bpe = RELU_MSB_BYTES if ex == "copy" else RELU_MSB_PUT_BYTES
                row.update({f"{key}_ms": rl / rn, f"{key}_elems_per_s": n_out / (rl / rn * 1e-3),
                            f"{key}_hbm_frac": bpe * n_out / (rl / rn * 1e-3) / HBM_PEAK})
            lane.set_exchange("copy")
        rows.append(row)
        del d, mat, z, y
        torch.cuda.empty_cache()
    lane.close()
    return wl.name, rows


def bench_backward(idx: int, reps: int = 5):
    """Per layer: the two gradient products (weight / activation masks opened in the forward
    pass reused) and the ReLU backward, timed with host clocks around a synchronised lane."""
    wl = synth.CONFIGS[idx]()
    lane = mpc.Lane(0, single_queue=True)
    dev = lane.device
    g = dealer.gen(synth.BASE_SEED + 50 + idx, dev)

    def timed(fn):
        for _ in range(2):
            fn()
        lane.sync(); t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        lane.sync()
        return (time.perf_counter() - t0) / reps

    rows = []
    for L in wl.layers:
        macs = layer_macs(L)
        if isinstance(L, synth.Conv):
            f = dealer.conv_layer(lane, g, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, L.x_std, L.w_std)
            b = dealer.conv_backward(lane, g, f, L.pad, L.stride)
            n_out = L.B * L.Ho * L.Wo * L.Cout
            gx = tuple(torch.empty_like(f["x"][0]) for _ in range(2)); gw = tuple(torch.empty_like(f["w"][0]) for _ in range(2))
            t_x = timed(lambda: lane.conv2d_grad_x(b["g"], None, b["gx"]["a"], b["gx"]["b"], b["gx"]["c"], L.pad, L.stride,
                                                   f_public=b["gx"]["f_public"], out=gx)) if "gx" in b else float("nan")
            t_w = timed(lambda: lane.conv2d_grad_w(None, b["g"], b["gw"]["a"], b["gw"]["b"], b["gw"]["c"], L.pad, L.stride,
                                                   e_public=b["gw"]["e_public"], out=gw))
            shape = "x".join(map(str, L.gemm_mkn))
        else:
            f = dealer.matmul_layer(lane, g, L.M, L.K, L.N, L.x_std, L.w_std, batch=L.batch if L.batch > 1 else None)
            b = dealer.matmul_backward(lane, g, f)
            n_out = L.M * L.N * max(L.batch, 1)
            gx = tuple(torch.empty_like(f["x"][0]) for _ in range(2)); gw = tuple(torch.empty_like(f["w"][0]) for _ in range(2))
            t_x = timed(lambda: lane.beaver_matmul(b["g"], None, b["gx"]["a"], b["gx"]["b"], b["gx"]["c"],
                                                   f_public=b["gx"]["f_public"], flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_Y, out=gx))
            t_w = timed(lambda: lane.beaver_matmul(f["x"], b["g"], b["gw"]["a"], b["gw"]["b"], b["gw"]["c"],
                                                   flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_X, out=gw))
            shape = f"{L.M}x{L.K}x{L.N}" + (f" x{L.batch}" if L.batch > 1 else "")
        row = dict(layer=L.name, gemm=shape, grad_x_ms=t_x * 1e3, grad_w_ms=t_w * 1e3,
                   grad_x_macs_per_s=macs / t_x, grad_w_macs_per_s=macs / t_w)
        if L.relu:
            ta, tb, tc = dealer.mul_triple(g, n_out, dev)
            sa = dealer.share(g, torch.randint(0, 2, (n_out,), generator=g, device=dev, dtype=torch.int64))
            gr = tuple(torch.empty(n_out, dtype=torch.int64, device=dev) for _ in range(2))
            gflat = (b["g"][0].view(-1), b["g"][1].view(-1))
            torch.cuda.synchronize()
            t_r = timed(lambda: lane.relu_backward(gflat, sa, ta, tb, tc, out=gr))
            row.update(relu_bwd_ms=t_r * 1e3, relu_bwd_elems_per_s=n_out / t_r)
        rows.append(row)
        del f, b, gx, gw
        torch.cuda.empty_cache()
    lane.close()
    return wl.name, rows


def bench_training(n_mb: int = 4, micro_batch: int = 32, reps: int = 3, packed_relu: bool = True):
    """Config 4 as a training step: forward with tape, backward, SGD update, per micro-batch;
    serial on one lane vs one lane per micro-batch."""
    wl = synth.config_vgg16_pipeline(micro_batch)
    layers = wl.layers
    lanes = [mpc.Lane(0, single_queue=True) for _ in range(n_mb)]
    dev = lanes[0].device
    g = dealer.gen(synth.BASE_SEED + 70, dev)
    weights = pipeline.deal_weights(g, layers, dev)
    states, bstates, xs, gouts = [], [], [], []
    for m in range(n_mb):
        states.append(pipeline.deal_microbatch(lanes[m], g, layers, weights, packed_relu=packed_relu))
        bstates.append(pipeline.deal_backward(lanes[m], g, layers, states[m]))
        xs.append(dealer.share(g, dealer.normal_fixed(g, (micro_batch, 32, 32, 3), 1.0, dev)))
        gouts.append(dealer.share(g, dealer.normal_fixed(g, (micro_batch, 10), 0.1, dev)))
    torch.cuda.synchronize()
    res = {}
    for mode in ("serial", "pipelined"):
        best = None
        for _ in range(reps + 1):
            keep = []
            torch.cuda.synchronize(); t0 = time.perf_counter()
            for m in range(n_mb):
                ln = lanes[0] if mode == "serial" else lanes[m]
                out, tape = pipeline.forward_train(ln, layers, states[m], xs[m], keep)
                pipeline.backward(ln, layers, states[m], bstates[m], tape, gouts[m], keep)
            for ln in lanes:
                ln.sync()
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
            del keep
        res[mode] = dict(ms=best * 1e3, images_per_s=n_mb * micro_batch / best)
    # the same step recorded once per lane and replayed
    graphs, pins = [], []
    for m in range(n_mb):
        pin = []
        with lanes[m].capture() as cap:
            out, tape = pipeline.forward_train(lanes[m], layers, states[m], xs[m], pin)
            pipeline.backward(lanes[m], layers, states[m], bstates[m], tape, gouts[m], pin)
        graphs.append(cap.graph); pins.append((pin, tape))
    best = None
    for _ in range(reps + 1):
        torch.cuda.synchronize(); t0 = time.perf_counter()
        for m in range(n_mb):
            graphs[m].launch(lanes[m])
        for ln in lanes:
            ln.sync()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    res["graphs"] = dict(ms=best * 1e3, images_per_s=n_mb * micro_batch / best)
    for ln in lanes:
        ln.close()
    return res


def bench_training3(n_mb: int = 4, micro_batch: int = 32, reps: int = 3, packed_relu: bool = True):
    """bench_training's step (forward with tape + backward, no update) with three simulated parties."""
    wl = synth.config_vgg16_pipeline(micro_batch)
    layers = wl.layers
    lanes = [mpc.Lane(0, single_queue=True) for _ in range(n_mb)]
    dev = lanes[0].device
    g = dealer.gen(synth.BASE_SEED + 71, dev)
    weights = pipeline.deal_weights3(g, layers, dev)
    states, bstates, xs, gouts = [], [], [], []
    for m in range(n_mb):
        states.append(pipeline.deal_microbatch3(lanes[m], g, layers, weights, packed_relu=packed_relu))
        bstates.append(pipeline.deal_backward3(lanes[m], g, layers, states[m]))
        xs.append(dealer.share3(g, dealer.normal_fixed(g, (micro_batch, 32, 32, 3), 1.0, dev)))
        gouts.append(dealer.share3(g, dealer.normal_fixed(g, (micro_batch, 10), 0.1, dev)))
        torch.cuda.synchronize()
        pipeline.preopen_weights3(lanes[m], states[m])
    res = {}
    for mode in ("serial", "pipelined"):
        best = None
        for _ in range(reps + 1):
            keep = []
            torch.cuda.synchronize(); t0 = time.perf_counter()
            for m in range(n_mb):
                ln = lanes[0] if mode == "serial" else lanes[m]
                out, tape = pipeline.forward_train3(ln, layers, states[m], xs[m], keep)
                pipeline.backward3(ln, layers, states[m], bstates[m], tape, gouts[m], keep)
            for ln in lanes:
                ln.sync()
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
            del keep
        res[mode] = dict(ms=best * 1e3, images_per_s=n_mb * micro_batch / best)
    for ln in lanes:
        ln.close()
    return res


def bench_graph(reps: int = 50, pool_first: bool = False, exchange: str = "copy"):
    """Eager issue vs replay of a captured HIP graph: the tiny secure layer (configs[0]) and one
    VGG16-CIFAR micro-batch forward (sign-only packed ReLU, prepared planes).
    pool_first: pooled layers run as ReLU(maxpool(z)) (same function, fewer conversions)."""
    res = {}
    lane = mpc.Lane(0, single_queue=True); lane.set_exchange(exchange)
    dev = lane.device
    g = dealer.gen(synth.BASE_SEED + 90, dev)
    L = synth.config_tiny().layers[0]
    d = dealer.matmul_layer(lane, g, L.M, L.K, L.N, L.x_std, L.w_std)
    mat = dealer.relu_material(g, L.M * L.N, dev)
    z = (torch.empty_like(d["c"][0]), torch.empty_like(d["c"][1])); y = (torch.empty_like(z[0]), torch.empty_like(z[1]))

    def tiny():
        lane.beaver_matmul(d["x"], d["w"], d["a"], d["b"], d["c"], out=z)
        lane.relu(z, mat, out=y)

    def timed(fn, n):
        for _ in range(5):
            fn()
        lane.sync(); t0 = time.perf_counter()
        for _ in range(n):
            fn()
        lane.sync()
        return (time.perf_counter() - t0) / n * 1e3

    res["tiny_eager_ms"] = timed(tiny, 4 * reps)
    with lane.capture() as cap:
        tiny()
    res["tiny_graph_ms"] = timed(lambda: cap.graph.launch(lane), 4 * reps)

    wl = synth.config_vgg16_pipeline(32)
    weights = pipeline.deal_weights(g, wl.layers, dev)
    states = pipeline.deal_microbatch(lane, g, wl.layers, weights, packed_relu=True, pool_first=pool_first)
    pipeline.prepare_layers(lane, wl.layers, states, fold=True)
    x = dealer.share(g, dealer.normal_fixed(g, (32, 32, 32, 3), 1.0, dev))
    torch.cuda.synchronize()
    keep = []
    def eager():
        keep.clear()          # the previous pass's tensors go back to torch's allocator: no device allocation in the timed loop
        pipeline.forward(lane, wl.layers, states, x, keep)
    res["vgg16_eager_ms"] = timed(eager, reps // 5)
    keep.clear()
    kept = []
    with lane.capture() as cap2:
        out = pipeline.forward(lane, wl.layers, states, x, kept)        # `kept` pins every tensor the replay touches
    res["vgg16_graph_ms"] = timed(lambda: cap2.graph.launch(lane), reps // 5)
    lane.sync()
    eager = pipeline.forward(lane, wl.layers, states, x, keep); lane.sync()
    assert torch.equal(eager[0], out[0]) and torch.equal(eager[1], out[1]), "graph replay differs from eager forward"
    # inter-batch pipeline with one recorded graph per micro-batch lane
    lanes = [lane] + [mpc.Lane(0, single_queue=True) for _ in range(3)]
    graphs, pins = [cap2.graph], [kept]
    for ln in lanes[1:]:
        ln.set_exchange(exchange)
        st = pipeline.deal_microbatch(ln, g, wl.layers, weights, packed_relu=True, pool_first=pool_first)
        pipeline.prepare_layers(ln, wl.layers, st, fold=True)
        xm = dealer.share(g, dealer.normal_fixed(g, (32, 32, 32, 3), 1.0, dev))
        torch.cuda.synchronize()
        warm = []; pipeline.forward(ln, wl.layers, st, xm, warm); ln.sync(); del warm
        pin = []
        with ln.capture() as cp:
            pipeline.forward(ln, wl.layers, st, xm, pin)
        graphs.append(cp.graph); pins.append((pin, st, xm))
    def replay_all():
        for gr, ln in zip(graphs, lanes):
            gr.launch(ln)
    for _ in range(3):
        replay_all()
    for ln in lanes:
        ln.sync()
    t0 = time.perf_counter()
    for _ in range(reps // 5):
        replay_all()
    for ln in lanes:
        ln.sync()
    res["vgg16_4lanes_graph_ms"] = (time.perf_counter() - t0) / (reps // 5) * 1e3
    for ln in lanes:
        ln.close()
    return res


def bench_pipeline(n_mb: int = 4, micro_batch: int = 32, reps: int = 3, packed_relu: bool = False, prepared: bool = False,
                   pool_first: bool = False, exchange: str = "copy"):
    """Config 4: serial (one lane, micro-batches one after the other) vs pipelined (one lane each)."""
    wl = synth.config_vgg16_pipeline(micro_batch)
    layers = wl.layers
    lanes = [mpc.Lane(0, single_queue=True) for _ in range(n_mb)]
    for ln in lanes:
        ln.set_exchange(exchange)
    dev = lanes[0].device
    g = dealer.gen(synth.BASE_SEED + wl.index, dev)
    weights = pipeline.deal_weights(g, layers, dev)
    states, xs = [], []
    for m in range(n_mb):
        states.append(pipeline.deal_microbatch(lanes[m], g, layers, weights, packed_relu=packed_relu, pool_first=pool_first))
        X = dealer.normal_fixed(g, (micro_batch, 32, 32, 3), 1.0, dev)
        xs.append(dealer.share(g, X))
        torch.cuda.synchronize()
        pipeline.preopen_weights(lanes[m], states[m])
        if prepared:
            pipeline.prepare_layers(lanes[m], layers, states[m], fold=True)
    res = {}
    for mode in ("serial", "pipelined"):
        best = None
        for _ in range(reps + 1):
            keep = []
            torch.cuda.synchronize(); t0 = time.perf_counter()
            if mode == "serial":
                for m in range(n_mb):
                    pipeline.forward(lanes[0], layers, states[m], xs[m], keep)
                lanes[0].sync()
            else:
                pipeline.forward_pipelined(lanes, layers, states, xs, keep)
                for ln in lanes:
                    ln.sync()
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
            del keep
        res[mode] = dict(ms=best * 1e3, images_per_s=n_mb * micro_batch / best)
    res["macs_per_image"] = sum(layer_macs(L) for L in layers) // micro_batch
    for ln in lanes:
        ln.close()
    return res


def sweep_tiles(n: int = 2097152, reps: int = 10):
    """Tile-count ablation of the inner-layer pipeline (Alg. 4; Sec. 4.2 "the number of tiles")
    on one secure ReLU: the Alg. 4 order on three streams, and the chunk-major order on one queue."""
    dev = torch.device("cuda", 0)
    g = dealer.gen(synth.BASE_SEED + 100, dev)
    x = dealer.share(g, dealer.normal_fixed(g, (n,), 1.0, dev))
    mats = {False: dealer.relu_material(g, n, dev), True: dealer.relu_material(g, n, dev, packed=True)}
    y = (torch.empty_like(x[0]), torch.empty_like(x[1]))
    torch.cuda.synchronize()
    for packed in (False, True):
        for mode in ("three streams (Alg. 4 order)", "one queue (chunk-major)", "one queue, remote-store exchange"):
            lane = mpc.Lane(0)
            if mode.startswith("one"):
                lane.use_single_queue()
            if "remote-store" in mode:
                lane.set_exchange("put")
            for tiles in (1, 2, 4, 8, 16, 32):
                for _ in range(3):
                    lane.relu(x, mats[packed], n_chunks=tiles, out=y, packed=packed)
                lane.sync(); t0 = time.perf_counter()
                for _ in range(reps):
                    lane.relu(x, mats[packed], n_chunks=tiles, out=y, packed=packed)
                lane.sync(); dt = (time.perf_counter() - t0) / reps
                print(f"  {'sign-only packed' if packed else 'whole-word':16s} {mode:30s} tiles={tiles:2d}: "
                      f"{dt * 1e3:7.3f} ms  {n / dt / 1e9:5.2f} G elems/s", flush=True)
            lane.close()
    # small inputs: the fixed cost per launch dominates; remote-store exchange halves the launches
    for packed in (False, True):
        for ns in (50176, 200704, 802816):
            line = f"  {'sign-only packed' if packed else 'whole-word':16s} n={ns:7d}:"
            for ex in ("copy", "put"):
                lane = mpc.Lane(0, single_queue=True); lane.set_exchange(ex)
                xs = (x[0][:ns], x[1][:ns]); ys = (y[0][:ns], y[1][:ns])
                ms = dealer.relu_material(g, ns, dev, packed=packed)
                for _ in range(3):
                    lane.relu(xs, ms, out=ys, packed=packed)
                lane.sync(); t0 = time.perf_counter()
                for _ in range(20):
                    lane.relu(xs, ms, out=ys, packed=packed)
                lane.sync(); dt = (time.perf_counter() - t0) / 20
                line += f"  {'copy kernels' if ex == 'copy' else 'remote store'} {dt * 1e3:6.3f} ms"
                lane.close()
            print(line, flush=True)
    # the listing's prefix tree as the carry network (same rounds and bytes as Kogge-Stone)
    lane = mpc.Lane(0, single_queue=True); lane.set_adder("tree")
    for _ in range(3):
        lane.relu(x, mats[False], n_chunks=2, out=y)
    lane.sync(); t0 = time.perf_counter()
    for _ in range(reps):
        lane.relu(x, mats[False], n_chunks=2, out=y)
    lane.sync(); dt = (time.perf_counter() - t0) / reps
    print(f"  {'whole-word, tree':16s} {'one queue (chunk-major)':30s} tiles= 2: {dt * 1e3:7.3f} ms  {n / dt / 1e9:5.2f} G elems/s", flush=True)
    lane.close()


def bench_three_parties(reps: int = 20):
    """configs[1] with three simulated parties: Beaver conv, masked rescale, secure ReLU.

    Algorithmic bytes of the three-party ReLU per element, all parties, by the rules of the two-party
    accounting (W = 8 B): compulsory I/O + material 3 * (x, y, r0, r1, 39 triple words, ra, ma, mb, mc) =
    141 W + 3 B; openings: 28 words per party broadcast (written once, then per peer copied = read + write,
    and read: 7 traversals) and 2 A2B masks per party to one peer each (3 traversals) = 3 * 202 = 606 W + 21 B;
    carried state per party S, W, P written and read (6), G (12), own masked words read again (28), a and b
    of every triple read again (26), x again (1) = 3 * 73 = 219 W + 9 B  =>  966 W + 33 B = 7761 B.

    Sign-only chain (mpc_relu3_msb), same rules.  Per party a triple component is 2 + 2 * 31/32 + 1/64 =
    3.953 words and the broadcast words are 2 + 2 + 4 * 31/32 + 2/64 + 2 = 9.906: material and I/O
    8 + 3 * 3.953 = 19.86 W + 1 B; openings 7 * 9.906 + 6 = 75.34 W + 7 B; carried state S, W, P (6), kept G
    bits (2 * 63/64), own masked words again (9.906), a and b again (7.906), x again (1) = 26.78 W + 3 B
    =>  3 * 121.98 W + 33 B = 2961 B."""
    wl = synth.CONFIGS[1](); L = wl.layers[0]
    lane = mpc.Lane(0, single_queue=True)
    dev = lane.device
    g = dealer.gen(synth.BASE_SEED + 31, dev)
    d = dealer.conv_layer3(lane, g, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, L.x_std, L.w_std)
    M, K, N = L.gemm_mkn
    n = M * N
    mat = dealer.relu3_material(g, n, dev)
    z = tuple(torch.empty_like(d["c"][0]) for _ in range(3))
    y = tuple(torch.empty_like(d["c"][0]) for _ in range(3))

    def conv():
        return lane.conv2d3(d["x"], d["w"], d["a"], d["b"], d["c"], L.pad, L.stride, out=z)

    def timed(fn, which):
        for _ in range(5):
            fn()
        lane.sync(); lane.set_profiling(True); lane.profile_reset()
        for _ in range(reps):
            fn()
        lane.sync()
        s = sorted(lane.profile_samples(which)); k = sorted(lane.profile_samples(mpc.PROF_GEMM_KERNEL))
        lane.set_profiling(False)
        return s[len(s) // 2], s[0], (sum(k) / reps if k else 0.0)

    conv_med, conv_min, gemm_ms = timed(conv, mpc.PROF_LINEAR)
    relu_med, relu_min, _ = timed(lambda: lane.relu3(z, mat, out=y), mpc.PROF_RELU)
    y_whole = tuple(v.clone() for v in y)
    del mat
    matp = dealer.relu3_material(g, n, dev, packed=True)
    msb_med, msb_min, _ = timed(lambda: lane.relu3(z, matp, out=y, packed=True), mpc.PROF_RELU)
    lane.sync()
    # other material, same function: the reconstructed outputs agree
    assert torch.equal(y[0] + y[1] + y[2], y_whole[0] + y_whole[1] + y_whole[2]), "sign-only chain reconstructs differently"
    del matp
    # the rescale has no region of its own: wall clock around back-to-back calls
    t = tuple(v.clone() for v in z)
    for _ in range(5):
        lane.truncate3(t, d["r"], d["rt"])
    lane.sync(); t0 = time.perf_counter()
    for _ in range(reps):
        lane.truncate3(t, d["r"], d["rt"])
    lane.sync(); trunc_ms = (time.perf_counter() - t0) / reps * 1e3
    lane.close()
    macs = M * K * N
    relu_bytes = 966 * 8 + 33
    msb_bytes = 2961
    return dict(gemm=f"{M}x{K}x{N}", conv_ms=conv_med, conv_min_ms=conv_min, gemm_kernels_ms=gemm_ms,
                secure_macs_per_s=macs / conv_med * 1e3, mfma_frac=432 * macs / (gemm_ms * 1e-3) / 5.0e15,
                trunc_ms=trunc_ms, relu_n=n, relu_ms=relu_med, relu_min_ms=relu_min,
                relu_elems_per_s=n / relu_med * 1e3, relu_bytes_per_element=relu_bytes,
                relu_hbm_frac=relu_bytes * n / (relu_med * 1e-3) / 8.0e12,
                msb_ms=msb_med, msb_min_ms=msb_min, msb_elems_per_s=n / msb_med * 1e3, msb_bytes_per_element=msb_bytes,
                msb_hbm_frac=msb_bytes * n / (msb_med * 1e-3) / 8.0e12)


def bench_pipeline3(n_mb: int = 4, micro_batch: int = 32, reps: int = 3, packed_relu: bool = False, pool_first: bool = False,
                    prepared: bool = False, exchange: str = "copy"):
    """Config 4's network with three parties: serial on one lane vs one lane per micro-batch."""
    wl = synth.config_vgg16_pipeline(micro_batch)
    layers = wl.layers
    lanes = [mpc.Lane(0, single_queue=True) for _ in range(n_mb)]
    dev = lanes[0].device
    g = dealer.gen(synth.BASE_SEED + 34, dev)
    weights = pipeline.deal_weights3(g, layers, dev)
    states, xs = [], []
    for m in range(n_mb):
        states.append(pipeline.deal_microbatch3(lanes[m], g, layers, weights, packed_relu=packed_relu, pool_first=pool_first))
        xs.append(dealer.share3(g, dealer.normal_fixed(g, (micro_batch, 32, 32, 3), 1.0, dev)))
        torch.cuda.synchronize()
        lanes[m].set_exchange(exchange)
        pipeline.preopen_weights3(lanes[m], states[m])
        if prepared:
            pipeline.prepare_layers3(lanes[m], layers, states[m])
    res = {}
    for mode in ("serial", "pipelined"):
        best = None
        for _ in range(reps + 1):
            keep = []
            for ln in lanes:
                ln.sync()
            t0 = time.perf_counter()
            if mode == "serial":
                for m in range(n_mb):
                    pipeline.forward3(lanes[0], layers, states[m], xs[m], keep)
                lanes[0].sync()
            else:
                pipeline.forward_pipelined3(lanes, layers, states, xs, keep)
                for ln in lanes:
                    ln.sync()
            ms = (time.perf_counter() - t0) * 1e3
            best = ms if best is None or ms < best else best
            del keep
        res[mode] = dict(ms=best, images_per_s=n_mb * micro_batch / best * 1e3)
    for ln in lanes:
        ln.close()
    return res


def bench_hbm_copy(reps: int = 20):
    """Attainable streaming rate of this device: a plain device-to-device copy (torch's copy kernel) at
    footprints inside and far beyond the 256 MB last-level cache.  Context for the HBM fractions of the
    ReLU chains, which are quoted against the nominal 8 TB/s."""
    dev = torch.device("cuda", 0)
    rows = []
    for mib in (32, 128, 512, 2048):
        n = mib * (1 << 20) // 8
        src = torch.ones(n, dtype=torch.int64, device=dev); dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            dst.copy_(src)
        e1.record(); torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        rows.append((mib, ms, 2 * n * 8 / (ms * 1e-3) / 1e12))
        del src, dst
    return rows


def bench_config_overlap(idx, reps=10):
    """Every linear layer of a workload as back-to-back folded calls, wall clock: one call per layer, and the better of
    one call and two row chunks on two lanes (pipeline.ChunkedLinear).  Products of two shares (batched, per-head) are
    already many independent products and run as one mpc_beaver_matmul_folded call in both columns."""
    rows = []
    for L in synth.CONFIGS[idx]().layers:
        if not isinstance(L, synth.Conv) and L.batch > 1:
            lane = mpc.Lane(0, single_queue=True); lane.set_exchange("put")
            g = dealer.gen(synth.BASE_SEED + 90 + idx, lane.device)
            d = dealer.matmul_layer(lane, g, L.M, L.K, L.N, L.x_std, L.w_std, batch=L.batch)
            right, left = lane.prepare_matmul(d["a"], d["b"], None)
            cf = (lane.fold_matmul(d["a"], d["b"], d["c"]), d["c"][1])
            z = (torch.empty_like(d["c"][0]), torch.empty_like(d["c"][1]))
            ts = []
            for _ in range(3):
                for _ in range(3):
                    lane.beaver_matmul_folded(d["x"], d["w"], d["a"], d["b"], cf, right, left, out=z)
                lane.sync(); t0 = time.perf_counter()
                for _ in range(reps):
                    lane.beaver_matmul_folded(d["x"], d["w"], d["a"], d["b"], cf, right, left, out=z)
                lane.sync(); ts.append((time.perf_counter() - t0) * 1e3 / reps)
            lane.close()
            one_ms = two_ms = sorted(ts)[1]
        else:
            one_ms, two_ms, same = bench_chunks(L, 2, 2, reps=reps, rounds=3)
            if not same:
                raise RuntimeError(f"{L.name}: the layer as two chunks differs from the one-call layer")
        rows.append(dict(layer=L.name, macs=layer_macs(L), one_call_ms=one_ms, two_chunks_ms=two_ms))
    return rows


def bench_chunks(L, n_chunks=2, n_lanes=2, reps=20, seed=78, rounds=5):
    """One layer as a single folded prepared call and as row chunks on lanes (pipeline.ChunkedLinear): wall clock of
    back-to-back layers, remote-store exchange; the outputs must be the same words."""
    from . import pipeline
    lanes = [mpc.Lane(0, single_queue=True) for _ in range(n_lanes)]
    for ln in lanes:
        ln.set_exchange("put")
    l0 = lanes[0]
    g = dealer.gen(seed, l0.device)
    conv = isinstance(L, synth.Conv)
    if conv:
        d = dealer.conv_layer(l0, g, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, L.x_std, L.w_std)
        right, left = l0.prepare_conv2d(d["a"], d["b"], d["f_public"], L.pad, L.stride)
        cf = (l0.fold_conv2d(d["a"], d["b"], d["c"], L.pad, L.stride), d["c"][1])
    else:
        d = dealer.matmul_layer(l0, g, L.M, L.K, L.N, L.x_std, L.w_std)
        right, left = l0.prepare_matmul(d["a"], d["b"], d["f_public"])
        cf = (l0.fold_matmul(d["a"], d["b"], d["c"]), d["c"][1])
    z = (torch.empty_like(d["c"][0]), torch.empty_like(d["c"][1]))
    zc = (torch.empty_like(z[0]), torch.empty_like(z[1]))
    F = mpc.MPC_TRUNCATE | mpc.MPC_FOLDED
    one = (lambda: l0.conv2d_prepared(d["x"], d["a"], cf, right, left, L.KH, L.KW, L.pad, L.stride, out=z, flags=F)) if conv else \
          (lambda: l0.beaver_matmul_prepared(d["x"], d["a"], cf, right, left, out=z, flags=F))
    chunked = pipeline.ChunkedLinear(lanes, L, pipeline.LayerState(w=d["w"], a=d["a"], b=d["b"], c=d["c"], f_public=d["f_public"]),
                                     n_chunks=n_chunks)

    def wall(fn, sync):
        for _ in range(5):
            fn()
        for ln in sync:
            ln.sync()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        for ln in sync:
            ln.sync()
        return (time.perf_counter() - t0) * 1e3 / reps

    # the chip's clock under a series of GEMMs depends on what ran just before: alternate the two forms, take medians
    ones, manys = [], []
    for _ in range(rounds):
        ones.append(wall(one, [l0]))
        manys.append(wall(lambda: chunked(d["x"], zc), lanes))
    one_ms, many_ms = sorted(ones)[rounds // 2], sorted(manys)[rounds // 2]
    same = torch.equal(z[0], zc[0]) and torch.equal(z[1], zc[1])
    for ln in lanes:
        ln.close()
    return one_ms, many_ms, same


def main(argv):
    if argv and argv[0] == "mfma":
        # the matrix cores' sustained int8 rate on register-resident operands (mpc_mfma_rate)
        lane = mpc.Lane(0, single_queue=True)
        print("== int8 MFMA rate on register operands (72 x v_mfma_i32_32x32x32_i8 per step, one wave per SIMD, no memory traffic)")
        for rnd in (False, True, False, True):
            for iters, launches in ((2000, 10), (2000, 50)):
                r = lane.mfma_rate(rnd, iters, launches)
                print(f"  {'uniformly random digits' if rnd else 'all-zero operands      '}  {launches:3d} launches x {iters} steps: "
                      f"{r / 1e15:.3f} POP/s = {100 * r / INT8_PEAK:.1f}% of 5.0 POP/s", flush=True)
        lane.close()
        return
    if argv and argv[0] == "chunks":
        # Alg. 3's overlap inside a layer: row chunks as complete calls on two lanes
        todo = [(1, None), (3, ("qkv", "out", "ffn1", "ffn2")), (4, ("conv2", "conv4", "conv6", "conv9"))]
        for idx, names in todo:
            wl = synth.CONFIGS[idx]()
            print(f"== config {idx}: {wl.name}")
            for L in wl.layers:
                if names is not None and L.name not in names:
                    continue
                shape = "x".join(map(str, L.gemm_mkn)) if isinstance(L, synth.Conv) else f"{L.M}x{L.K}x{L.N}"
                macs = layer_macs(L)
                line = f"  {L.name:8s} {shape:20s}"
                for nch, nl in ((2, 2), (4, 2), (4, 4)):
                    one_ms, many_ms, same = bench_chunks(L, nch, nl)
                    if nch == 2:
                        line += f" one call {one_ms:7.3f} ms ({100 * 288 * macs / (one_ms * 1e-3) / INT8_PEAK:4.1f}%)"
                    line += (f" | {nch} chunks on {nl} lanes {many_ms:7.3f} ms ({100 * 288 * macs / (many_ms * 1e-3) / INT8_PEAK:4.1f}%)"
                             f"{'' if same else ' DIFFERENT WORDS'}")
                print(line, flush=True)
        return
    if argv and argv[0] == "sweep":
        print("== tile-count sweep, secure ReLU on 2097152 elements")
        sweep_tiles()
        return
    if argv and argv[0] == "pipeline":
        # config 4's inter-batch pipeline alone (sign-only packed ReLU, prepared planes): the run a kernel trace is taken of
        p = bench_pipeline(packed_relu=True, prepared=True)
        print(f"  inter-batch pipeline, batch 128 = 4 x 32, sign-only packed ReLU, prepared planes: "
              f"serial {p['serial']['ms']:.2f} ms ({p['serial']['images_per_s']:.0f} img/s), "
              f"pipelined {p['pipelined']['ms']:.2f} ms ({p['pipelined']['images_per_s']:.0f} img/s)", flush=True)
        return
    if argv and argv[0] == "hbm":
        print("== device-to-device copy (read + write counted), repeated on the same buffers")
        for mib, ms, tbs in bench_hbm_copy():
            print(f"  {mib:5d} MiB source + {mib:5d} MiB destination: {ms * 1e3:8.1f} us  {tbs:5.2f} TB/s = {100 * tbs / 8.0:4.1f}% of 8 TB/s", flush=True)
        return
    if argv and argv[0] == "relu3":
        # the three-party ReLU alone, both chains (the command the per-kernel profile is taken with)
        n = int(argv[1]) if len(argv) > 1 else 2097152
        lane = mpc.Lane(0, single_queue=True)
        g = dealer.gen(synth.BASE_SEED + 33, lane.device)
        x = dealer.share3(g, dealer.normal_fixed(g, (n,), 1.0, lane.device))
        y = tuple(torch.empty_like(v) for v in x)
        for packed in (False, True):
            mat = dealer.relu3_material(g, n, lane.device, packed=packed)
            for ex in ("copy", "put"):
                lane.set_exchange(ex)
                for _ in range(3):
                    lane.relu3(x, mat, out=y, packed=packed)
                lane.sync(); t0 = time.perf_counter()
                for _ in range(20):
                    lane.relu3(x, mat, out=y, packed=packed)
                lane.sync(); ms = (time.perf_counter() - t0) / 20 * 1e3
                print(f"  three-party ReLU, {n} elements, {'sign-only packed' if packed else 'whole-word'} chain"
                      f"{', exchange by remote store' if ex == 'put' else ''}: {ms:.3f} ms ({n / ms / 1e6:.2f} G elems/s)", flush=True)
            del mat
        lane.close()
        return
    if argv and argv[0] == "parties3":
        r = bench_three_parties()
        print("== configs[1] with three simulated parties (432 int8 ops per secure MAC: 3 parties x 2 ring products x 36 x 2)")
        print(f"  conv3x3 {r['gemm']}: call {r['conv_ms']:.3f} ms (min {r['conv_min_ms']:.3f}), {r['secure_macs_per_s'] / 1e12:.2f} T secure MAC/s; "
              f"GEMM launches {r['gemm_kernels_ms']:.3f} ms = {100 * r['mfma_frac']:.1f}% of 5.0 POP/s")
        print(f"  masked rescale of {r['relu_n']} words: {r['trunc_ms']:.3f} ms (host clock around back-to-back calls)")
        print(f"  secure ReLU, {r['relu_n']} elements: {r['relu_ms']:.3f} ms (min {r['relu_min_ms']:.3f}), {r['relu_elems_per_s'] / 1e9:.2f} G elems/s; "
              f"{r['relu_bytes_per_element']} B per element -> {100 * r['relu_hbm_frac']:.1f}% of 8 TB/s", flush=True)
        print(f"  the same ReLU on the sign's carry chain only: {r['msb_ms']:.3f} ms (min {r['msb_min_ms']:.3f}), {r['msb_elems_per_s'] / 1e9:.2f} G elems/s; "
              f"{r['msb_bytes_per_element']} B per element -> {100 * r['msb_hbm_frac']:.1f}% of 8 TB/s", flush=True)
        for packed, pf, prep, ex in ((False, False, False, "copy"), (False, False, True, "put"), (True, False, False, "copy"),
                                     (True, True, False, "copy"), (True, True, True, "put")):
            p = bench_pipeline3(packed_relu=packed, pool_first=pf, prepared=prep, exchange=ex)
            print(f"  VGG16-CIFAR forward with three parties, batch 128 = 4 x 32 ({'sign-only packed' if packed else 'whole-word'} ReLU"
                  f"{', pooled layers as ReLU(maxpool(z))' if pf else ''}{', prepared planes' if prep else ''}"
                  f"{', ReLU exchange by remote store' if ex == 'put' else ''}, weight masks opened ahead): "
                  f"serial {p['serial']['ms']:.2f} ms ({p['serial']['images_per_s']:.0f} img/s), "
                  f"one lane per micro-batch {p['pipelined']['ms']:.2f} ms ({p['pipelined']['images_per_s']:.0f} img/s)", flush=True)
        for packed in (False, True):
            p = bench_training3(packed_relu=packed)
            print(f"  VGG16-CIFAR training step (forward + backward) with three parties, batch 128 = 4 x 32 "
                  f"({'sign-only packed' if packed else 'whole-word'} ReLU): serial {p['serial']['ms']:.2f} ms ({p['serial']['images_per_s']:.0f} img/s), "
                  f"one lane per micro-batch {p['pipelined']['ms']:.2f} ms ({p['pipelined']['images_per_s']:.0f} img/s)", flush=True)
        return
    if argv and argv[0] == "backward":
        for idx in ([int(a) for a in argv[1:]] or [1, 2, 3]):
            name, rows = bench_backward(idx)
            print(f"== backward products, config {idx}: {name}")
            for r in rows:
                line = (f"  {r['layer']:10s} {r['gemm']:22s} grad_x {r['grad_x_ms']:8.3f} ms {r['grad_x_macs_per_s'] / 1e12:6.2f} T MAC/s"
                        f"  | grad_w {r['grad_w_ms']:8.3f} ms {r['grad_w_macs_per_s'] / 1e12:6.2f} T MAC/s")
                if "relu_bwd_ms" in r:
                    line += f"  | relu bwd {r['relu_bwd_ms']:7.3f} ms {r['relu_bwd_elems_per_s'] / 1e9:6.2f} G elems/s"
                print(line, flush=True)
        return
    if argv and argv[0] == "paper":
        # the layer shapes of the models the paper evaluates (Sec. 5.2), forward pass
        for make in synth.PAPER_MODELS:
            wl = make()
            name, rows = bench_layers(wl.index, workload=wl)
            print(f"== {name}")
            tot_lin = tot_relu = tot_msb = tot_prep = 0.0
            for r in rows:
                line = (f"  {r['layer']:16s} x{r['repeat']:<2d} {r['gemm']:22s} call {r['call_ms']:8.3f} ms "
                        f"{r['secure_macs_per_s'] / 1e12:6.2f} T MAC/s  folded {r['folded_call_ms']:7.3f} ms  mfma {100 * r['mfma_frac']:5.1f}%")
                tot_lin += r['call_ms'] * r['repeat']; tot_prep += r['folded_call_ms'] * r['repeat']
                if "relu_ms" in r:
                    line += (f"  | relu {r['relu_n']:9d} el {r['relu_ms']:7.3f} ms hbm {100 * r['hbm_frac']:5.1f}%"
                             f"  | sign-only {r['msb_ms']:7.3f} ms hbm {100 * r['msb_hbm_frac']:5.1f}%")
                    tot_relu += r['relu_ms'] * r['repeat']; tot_msb += r['msb_ms'] * r['repeat']
                print(line, flush=True)
            print(f"  sum over layers (x multiplicity): linear {tot_lin:.2f} ms ({tot_prep:.2f} ms as folded prepared calls), ReLU {tot_relu:.2f} ms whole-word / "
                  f"{tot_msb:.2f} ms sign-only", flush=True)
        return
    if argv and argv[0] == "graph":
        r = bench_graph()
        print(f"  configs[0] secure layer (matmul + ReLU): eager {r['tiny_eager_ms']:.4f} ms, graph replay {r['tiny_graph_ms']:.4f} ms")
        print(f"  VGG16-CIFAR forward, 32 images (packed ReLU, prepared planes): eager {r['vgg16_eager_ms']:.3f} ms, "
              f"graph replay {r['vgg16_graph_ms']:.3f} ms; batch 128 = 4 x 32 as four recorded graphs on four lanes: "
              f"{r['vgg16_4lanes_graph_ms']:.2f} ms ({128 / r['vgg16_4lanes_graph_ms'] * 1e3:.0f} img/s)", flush=True)
        for pf, ex in ((False, "put"), (True, "put")):
            r = bench_graph(pool_first=pf, exchange=ex)
            print(f"  exchange by remote store{', pooled layers as ReLU(maxpool(z))' if pf else ''}: eager {r['vgg16_eager_ms']:.3f} ms, "
                  f"graph replay {r['vgg16_graph_ms']:.3f} ms; four recorded graphs on four lanes: "
                  f"{r['vgg16_4lanes_graph_ms']:.2f} ms ({128 / r['vgg16_4lanes_graph_ms'] * 1e3:.0f} img/s)", flush=True)
        r = bench_graph(pool_first=True)
        print(f"  the same with pooled layers as ReLU(maxpool(z)): eager {r['vgg16_eager_ms']:.3f} ms, "
              f"graph replay {r['vgg16_graph_ms']:.3f} ms; four recorded graphs on four lanes: "
              f"{r['vgg16_4lanes_graph_ms']:.2f} ms ({128 / r['vgg16_4lanes_graph_ms'] * 1e3:.0f} img/s)", flush=True)
        return
    if argv and argv[0] == "train":
        for packed in (False, True):
            p = bench_training(packed_relu=packed)
            print(f"  VGG16-CIFAR training step (forward + backward), batch 128 = 4 x 32, "
                  f"{'sign-only packed' if packed else 'whole-word'} ReLU: serial {p['serial']['ms']:.2f} ms "
                  f"({p['serial']['images_per_s']:.0f} img/s), one lane per micro-batch {p['pipelined']['ms']:.2f} ms "
                  f"({p['pipelined']['images_per_s']:.0f} img/s), as four recorded graphs {p['graphs']['ms']:.2f} ms "
                  f"({p['graphs']['images_per_s']:.0f} img/s)", flush=True)
        return
    which = [int(a) for a in argv] if argv else list(range(len(synth.CONFIGS)))
    for idx in which:
        name, rows = bench_layers(idx)
        print(f"== config {idx}: {name}")
        tot = dict(lin=0.0, relu=0.0, msb=0.0)
        for r in rows:
            # both roofs of the GEMM kernel; '*' marks the one that binds (the larger fraction)
            mf, hf = 100 * r['mfma_frac'], 100 * r['gemm_hbm_frac']
            line = (f"  {r['layer']:10s} {r['gemm']:22s} call {r['call_ms']:8.3f} ms  {r['secure_macs_per_s'] / 1e12:6.2f} T MAC/s"
                    f"  kernel {r['kernel_ms']:7.3f} ms  mfma {mf:5.1f}%{'*' if mf >= hf else ' '} hbm {hf:5.1f}%{'*' if hf > mf else ' '}"
                    f"  | folded call {r['folded_call_ms']:7.3f} ms {r['folded_secure_macs_per_s'] / 1e12:6.2f} T MAC/s kernel {r['folded_kernel_ms']:7.3f} ms {100 * r['folded_mfma_frac']:5.1f}%"
                    f" call: mfma {100 * 288 * r['folded_secure_macs_per_s'] / INT8_PEAK:5.1f}% hbm {100 * r['folded_call_hbm_frac']:5.1f}%")
            tot['lin'] += r['call_ms']; tot['prep'] = tot.get('prep', 0.0) + r['folded_call_ms']
            if r['activation_product']:
                line += f"  (both operands shared: f opens in the call; plain call with the remote-store exchange {r['call_put_ms']:.3f} ms)"
            if "relu_ms" in r:
                tot['relu'] += r['relu_ms']; tot['msb'] += r['msb_ms']
                tot['put'] = tot.get('put', 0.0) + r['relu_put_ms']; tot['msb_put'] = tot.get('msb_put', 0.0) + r['msb_put_ms']
                line += (f"  | relu {r['relu_n']:9d} el copy {r['relu_ms']:7.3f} ms {r['relu_elems_per_s'] / 1e9:5.2f} G/s {100 * r['hbm_frac']:5.1f}%"
                         f" put {r['relu_put_ms']:7.3f} ms {r['relu_put_elems_per_s'] / 1e9:5.2f} G/s {100 * r['put_hbm_frac']:5.1f}%")
                line += (f"  | sign-only copy {r['msb_ms']:7.3f} ms {r['msb_elems_per_s'] / 1e9:5.2f} G/s {100 * r['msb_hbm_frac']:5.1f}%"
                         f" put {r['msb_put_ms']:7.3f} ms {r['msb_put_elems_per_s'] / 1e9:5.2f} G/s {100 * r['msb_put_hbm_frac']:5.1f}%")
            print(line, flush=True)
        print(f"  totals: linear calls {tot['lin']:.3f} ms ({tot['prep']:.3f} ms as folded calls), ReLU whole-word {tot['relu']:.3f} ms copy / "
              f"{tot.get('put', 0.0):.3f} ms put, sign-only {tot['msb']:.3f} ms copy / {tot.get('msb_put', 0.0):.3f} ms put", flush=True)
        if idx == 4:
            for packed, prepared, pool_first, ex in ((False, False, False, "copy"), (True, False, False, "copy"), (True, True, False, "copy"),
                                                     (True, True, True, "copy"), (True, True, True, "put")):
                p = bench_pipeline(packed_relu=packed, prepared=prepared, pool_first=pool_first, exchange=ex)
                print(f"  inter-batch pipeline, batch 128 = 4 x 32, {'sign-only packed' if packed else 'whole-word'} ReLU"
                      f"{', folded prepared planes' if prepared else ''}{', pooled layers as ReLU(maxpool(z))' if pool_first else ''}"
                      f"{', exchange by remote store' if ex == 'put' else ''}: "
                      f"serial {p['serial']['ms']:.2f} ms ({p['serial']['images_per_s']:.0f} img/s), "
                      f"pipelined {p['pipelined']['ms']:.2f} ms ({p['pipelined']['images_per_s']:.0f} img/s)", flush=True)
        print(json.dumps({"config": idx, "layers": rows}), file=sys.stderr)


if __name__ == "__main__":
    main(sys.argv[1:])
