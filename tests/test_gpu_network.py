"""Whole-network parity and pipeline invariance on the GPU: a VGG16-shaped
CIFAR network (13 conv 3x3 layers with 2x2 max-pooling, three dense layers)
at a small batch, every layer's output shares against the oracle; the
inter-batch pipeline, pre-opened weight masks, the Alg. 3 ordering and chunked
exchanges must not change a single bit (Sec. 5.10)."""
import numpy as np
import pytest

import oracle
from helpers import (deal_backward_host, deal_backward_host3, deal_network_host, deal_network_host3, oracle_forward,
                     oracle_forward3, oracle_train_step, oracle_train_step3, rec)
from paper_2209_13643_amd import synth

pytestmark = pytest.mark.gpu
U64 = np.uint64


@pytest.fixture(scope="module")
def mods():
    from paper_2209_13643_amd import mpc, pipeline
    return mpc, pipeline


@pytest.fixture(scope="module")
def dealt():
    """Two micro-batches of two images through the full VGG16-CIFAR layer list."""
    base = synth.config_vgg16_pipeline(micro_batch=2)
    layers = base.layers
    rng = synth.rng_for(base.index, 11)
    mbs, weights = [], None
    for m in range(2):
        states, weights = deal_network_host(rng, layers, weights)
        X = synth.normal_fixed(rng, (2, 32, 32, 3), 1.0)
        xs = synth.share_additive(rng, X)
        mbs.append(dict(states=states, X=X, x=xs, want=oracle_forward(layers, states, xs)))
    return layers, mbs


def to_state(mpc, pipeline, st, pack_lane=None):
    """Upload one layer's host-dealt state; with `pack_lane` the ReLU / pool triples are
    packed on the device for the sign-only chain."""
    dv = lambda p: (mpc.to_device(p[0]), mpc.to_device(p[1]))
    def mat(m):
        if m is None:
            return None
        md = mpc.material_to_device(m)
        return pack_lane.pack_material(md) if pack_lane is not None else md
    return pipeline.LayerState(w=dv(st["w"]), a=dv(st["a"]), b=dv(st["b"]), c=dv(st["c"]),
                               relu=mat(st["relu"]), pool1=mat(st["pool1"]), pool2=mat(st["pool2"]),
                               packed=pack_lane is not None, pool_first=st.get("pool_first", False))


def check(mpc, got_pair, want_pair, what):
    for i in range(2):
        g = mpc.to_host(got_pair[i]).reshape(want_pair[i].shape)
        assert np.array_equal(g, want_pair[i]), f"{what}: party {i} differs in {(g != want_pair[i]).sum()} elements"


@pytest.mark.parametrize("packed_relu", [False, True], ids=["whole-word-relu", "sign-only-packed-relu"])
def test_vgg16_every_layer_matches_oracle(mods, dealt, packed_relu):
    mpc, pipeline = mods
    layers, mbs = dealt
    print(f"vgg16 per-layer parity, packed_relu={packed_relu}", flush=True)
    lane = mpc.Lane(0); lane.use_single_queue()
    mb = mbs[0]
    states = [to_state(mpc, pipeline, st, lane if packed_relu else None) for st in mb["states"]]
    x = (mpc.to_device(mb["x"][0]), mpc.to_device(mb["x"][1]))
    keep = []
    for li, (L, st) in enumerate(zip(layers, states)):
        x = pipeline.run_layer(lane, L, st, x, keep)
        lane.sync()
        check(mpc, x, mb["want"][li], f"layer {li} ({L.name})")
    # decoded logits close to a float64 run of the same quantised network
    logits = oracle.decode(rec((mpc.to_host(x[0]), mpc.to_host(x[1]))))
    assert logits.shape == (2, 10) and np.isfinite(logits).all()
    lane.close()


@pytest.mark.parametrize("packed_relu", [False, True], ids=["whole-word-relu", "sign-only-packed-relu"])
def test_pooled_layers_as_relu_of_maxpool(mods, dealt, packed_relu):
    """max and ReLU commute, so a layer with both may pool first and convert a quarter of the elements.
    The oracle run in that order reconstructs to the very values of the usual order at every layer
    (both are exact on the truncated product), and the device run matches it share for share."""
    mpc, pipeline = mods
    layers, mbs = dealt
    print(f"vgg16 with pooled layers as ReLU(maxpool(z)), packed_relu={packed_relu}", flush=True)
    mb = mbs[0]
    rng = synth.rng_for(4, 12)
    weights = [(st["W"], st["w"]) for st in mb["states"]]
    host, _ = deal_network_host(rng, layers, weights, pool_first=True)
    assert sum(st["pool_first"] for st in host) == 5
    want = oracle_forward(layers, host, mb["x"])
    # truncation noise differs with the triples (one unit in the last place per product), so the two
    # orders are compared on one layer's own input: same z, then both orders of the nonlinear part
    L, st, st0 = layers[1], host[1], mb["states"][1]
    z = want[0]
    zc = oracle.truncate(oracle.beaver_conv2d(z, st["w"], st["a"], st["b"], st["c"], L.pad, L.stride), 16)
    usual = oracle.maxpool2x2(oracle.relu(zc, st0["relu"]).y, st0["pool1"], st0["pool2"])
    assert np.array_equal(rec(usual), rec(want[1]))
    lane = mpc.Lane(0); lane.use_single_queue()
    states = [to_state(mpc, pipeline, s, lane if packed_relu else None) for s in host]
    x = (mpc.to_device(mb["x"][0]), mpc.to_device(mb["x"][1]))
    keep = []
    for li, (L, s) in enumerate(zip(layers, states)):
        x = pipeline.run_layer(lane, L, s, x, keep)
        lane.sync()
        check(mpc, x, want[li], f"layer {li} ({L.name}), pool first")
    lane.close()


@pytest.mark.parametrize("mode", ["serial-3stream", "pipelined", "pipelined-preopened", "pipelined-two-phase-chunked",
                                  "pipelined-packed-relu", "pipelined-prepared-planes", "pipelined-folded-preallocated",
                                  "pipelined-packed-relu-remote-store"])
def test_pipeline_invariance(mods, dealt, mode):
    mpc, pipeline = mods
    layers, mbs = dealt
    print(f"pipeline invariance: {mode}", flush=True)
    lanes = [mpc.Lane(0) for _ in mbs]
    if mode != "serial-3stream":
        for ln in lanes:
            ln.use_single_queue()
    pk = lanes[0] if mode.startswith("pipelined-packed-relu") else None
    if mode.endswith("remote-store"):
        for ln in lanes:
            ln.set_exchange("put")
    states = [[to_state(mpc, pipeline, st, pk) for st in mb["states"]] for mb in mbs]
    xs = [(mpc.to_device(mb["x"][0]), mpc.to_device(mb["x"][1])) for mb in mbs]
    kw = {}
    if mode in ("pipelined-preopened", "pipelined-two-phase-chunked"):
        for ln, sts in zip(lanes, states):
            pipeline.preopen_weights(ln, sts)
    if mode == "pipelined-prepared-planes":
        for ln, sts in zip(lanes, states):
            pipeline.prepare_layers(ln, layers, sts)
    outs_pre = None
    if mode == "pipelined-folded-preallocated":
        # prepared planes with party 0's addend folded, every output tensor allocated ahead of the pass
        for ln, sts in zip(lanes, states):
            pipeline.prepare_layers(ln, layers, sts, fold=True)
        outs_pre = [pipeline.alloc_outputs(ln, layers, sts) for ln, sts in zip(lanes, states)]
        kw = dict(outs_per_mb=outs_pre)
    if mode == "pipelined-two-phase-chunked":
        kw = dict(n_chunks=3, relu_chunks=3, flags=mpc.MPC_TRUNCATE | mpc.MPC_TWO_PHASE)
    keep = []
    if mode == "serial-3stream":
        outs = [pipeline.forward(lanes[m], layers, states[m], xs[m], keep) for m in range(len(mbs))]
    else:
        outs = pipeline.forward_pipelined(lanes, layers, states, xs, keep, **kw)
    for ln in lanes:
        ln.sync()
    for m, mb in enumerate(mbs):
        check(mpc, outs[m], mb["want"][-1], f"micro-batch {m} logits ({mode})")
    for ln in lanes:
        ln.close()


def test_whole_network_as_a_recorded_graph(mods, dealt):
    """The VGG16 forward of one micro-batch recorded into a HIP graph and replayed on both
    micro-batches' inputs (copied into the recorded input buffers): logits as in the oracle run."""
    import torch
    mpc, pipeline = mods
    layers, mbs = dealt
    print("whole network as a graph", flush=True)
    lane = mpc.Lane(0); lane.use_single_queue()
    # both micro-batches share weights but not triples: record micro-batch 0's states, replay it twice
    # (second time after other eager work), then check against its oracle logits
    mb = mbs[0]
    states = [to_state(mpc, pipeline, st, lane) for st in mb["states"]]
    pipeline.prepare_layers(lane, layers, states)
    x = (mpc.to_device(mb["x"][0]), mpc.to_device(mb["x"][1]))
    warm = []; pipeline.forward(lane, layers, states, x, warm); lane.sync(); del warm
    pin = []
    with lane.capture() as cap:
        out = pipeline.forward(lane, layers, states, x, pin)
    for rep in range(2):
        for t in out:
            t.zero_()
        torch.cuda.synchronize()
        cap.graph.launch(lane); lane.sync()
        check(mpc, out, mb["want"][-1], f"logits of graph replay {rep}")
        between = lane.add(x, x); lane.sync()                  # eager work between the replays
        assert torch.equal(between[0], x[0] + x[0])
    cap.graph.close(); lane.close()


@pytest.mark.parametrize("queues", ["three-streams", "single-queue"])
def test_interlinear_lookahead_across_layers(mods, dealt, queues):
    """Alg. 3 across layers: each weight mask is opened one layer ahead on a second lane and the
    compute lane waits for it on the device (mpc_ctx_wait); logits as in the oracle run."""
    mpc, pipeline = mods
    layers, mbs = dealt
    print(f"inter-linear look-ahead, {queues}", flush=True)
    lane, wlane = mpc.Lane(0), mpc.Lane(0)
    if queues == "single-queue":
        lane.use_single_queue(); wlane.use_single_queue()
    mb = mbs[1]
    states = [to_state(mpc, pipeline, st) for st in mb["states"]]
    keep = []
    out = pipeline.forward_interlinear(lane, wlane, layers, states, (mpc.to_device(mb["x"][0]), mpc.to_device(mb["x"][1])), keep)
    lane.sync(); wlane.sync()
    check(mpc, out, mb["want"][-1], "logits with one-layer-ahead weight masks")
    assert all(st.f_public is not None for st in states)
    lane.close(); wlane.close()


@pytest.mark.parametrize("packed_relu", [False, True], ids=["whole-word-relu", "sign-only-packed-relu"])
def test_vgg16_training_step_matches_oracle(mods, dealt, packed_relu):
    """Forward with the tape, backward through max-pool, ReLU, conv and dense layers, then
    an SGD step: logits, every layer's weight-gradient shares and the updated weight
    shares against the oracle run of the same step (Sec. 5.3)."""
    mpc, pipeline = mods
    layers, mbs = dealt
    print(f"vgg16 training step, packed_relu={packed_relu}", flush=True)
    mb = mbs[0]
    rng = synth.rng_for(4, 12)
    bhost = deal_backward_host(rng, layers, mb["states"])
    Gout = synth.normal_fixed(rng, (2, 10), 0.5)
    gout = synth.share_additive(rng, Gout)
    want_out, want_grads = oracle_train_step(layers, mb["states"], bhost, mb["x"], gout)
    check_pair = lambda got, want, what: check(mpc, got, want, what)

    lane = mpc.Lane(0); lane.use_single_queue()
    dv = lambda p: (mpc.to_device(p[0]), mpc.to_device(p[1]))
    states = [to_state(mpc, pipeline, st, lane if packed_relu else None) for st in mb["states"]]
    bstates = []
    for st, bs in zip(states, bhost):
        trip = lambda t: None if t is None else tuple(dv(q) for q in t)
        bstates.append(pipeline.BackwardState(
            gx=None if bs["gx"] is None else dict(a=dv(bs["gx"]["a"]), b=st.b, c=dv(bs["gx"]["c"])),
            gw=dict(a=st.a, b=dv(bs["gw"]["b"]), c=dv(bs["gw"]["c"])),
            relu_t=trip(bs["relu_t"]), pool_t1=trip(bs["pool_t1"]), pool_t2=trip(bs["pool_t2"])))
    keep = []
    out, tape = pipeline.forward_train(lane, layers, states, dv(mb["x"]), keep)
    grads = pipeline.backward(lane, layers, states, bstates, tape, dv(gout), keep)
    lane.sync()
    check_pair(out, want_out, "logits")
    for li, L in enumerate(layers):
        check_pair(grads[li], want_grads[li], f"weight gradient of layer {li} ({L.name})")
    # SGD step with learning rate 2^-6
    pipeline.sgd_step(lane, states, grads, 6)
    lane.sync()
    for li, (L, st) in enumerate(zip(layers, mb["states"])):
        step = oracle.truncate(want_grads[li], 6)
        want_w = (st["w"][0] - step[0].reshape(st["w"][0].shape), st["w"][1] - step[1].reshape(st["w"][1].shape))
        check_pair(states[li].w, want_w, f"updated weights of layer {li} ({L.name})")
    lane.close()


def test_strided_network_training_step(mods):
    """A small network with a strided 3x3 convolution, a strided 1x1 shortcut-like convolution,
    a pooled layer and a dense head: forward, backward and the weight gradients against the oracle."""
    mpc, pipeline = mods
    print("strided network training step", flush=True)
    B = 3
    layers = [synth.Conv("c1", B, 12, 12, 3, 8, 3, 3, 1, 2, 1.0, synth.he_std(27), True, False),
              synth.Conv("c2", B, 6, 6, 8, 8, 1, 1, 0, 2, 1.0, synth.he_std(8), True, False),
              synth.Conv("c3", B, 3, 3, 8, 16, 3, 3, 1, 1, 1.0, synth.he_std(72), True, False),
              synth.Conv("c4", B, 3, 3, 16, 16, 3, 3, 1, 1, 1.0, synth.he_std(144), True, False)]
    layers.append(synth.Gemm("fc", B, 3 * 3 * 16, 10, 1.0, synth.he_std(144)))
    rng = synth.rng_for(9, 1)
    states, _ = deal_network_host(rng, layers)
    bhost = deal_backward_host(rng, layers, states)
    X = synth.normal_fixed(rng, (B, 12, 12, 3), 1.0); xs = synth.share_additive(rng, X)
    gout = synth.share_additive(rng, synth.normal_fixed(rng, (B, 10), 0.5))
    want_out, want_grads = oracle_train_step(layers, states, bhost, xs, gout)
    lane = mpc.Lane(0); lane.use_single_queue()
    dv = lambda p: (mpc.to_device(p[0]), mpc.to_device(p[1]))
    dstates = [to_state(mpc, pipeline, st) for st in states]
    bstates = []
    for st, bs in zip(dstates, bhost):
        trip = lambda t: None if t is None else tuple(dv(q) for q in t)
        bstates.append(pipeline.BackwardState(
            gx=None if bs["gx"] is None else dict(a=dv(bs["gx"]["a"]), b=st.b, c=dv(bs["gx"]["c"])),
            gw=dict(a=st.a, b=dv(bs["gw"]["b"]), c=dv(bs["gw"]["c"])),
            relu_t=trip(bs["relu_t"]), pool_t1=trip(bs["pool_t1"]), pool_t2=trip(bs["pool_t2"])))
    keep = []
    out, tape = pipeline.forward_train(lane, layers, dstates, dv(xs), keep)
    grads = pipeline.backward(lane, layers, dstates, bstates, tape, dv(gout), keep)
    lane.sync()
    check(mpc, out, want_out, "logits")
    for li, L in enumerate(layers):
        check(mpc, grads[li], want_grads[li], f"weight gradient of layer {li} ({L.name})")
    lane.close()


@pytest.mark.parametrize("packed_relu", [False, True], ids=["whole-word-relu", "sign-only-packed-relu"])
def test_vgg16_with_three_parties(mods, packed_relu):
    """The whole VGG16-CIFAR layer list with three simulated parties (Sec. 5.6): every layer's three
    output shares against the oracle, then two micro-batches on two lanes in layer-major order and with
    the weight masks opened ahead of time: not a bit may change."""
    mpc, pipeline = mods
    packer = mpc.Lane(0)
    base = synth.config_vgg16_pipeline(micro_batch=2)
    layers = base.layers
    rng = synth.rng_for(base.index, 13)
    mbs, weights = [], None
    for m in range(2):
        states, weights = deal_network_host3(rng, layers, weights)
        X = synth.normal_fixed(rng, (2, 32, 32, 3), 1.0)
        xs = synth.share_additive3(rng, X)
        mbs.append(dict(states=states, X=X, x=xs, want=oracle_forward3(layers, states, xs)))
    d3 = lambda t: tuple(mpc.to_device(v) for v in t)
    def m3(m):
        if m is None:
            return None
        md = mpc.material_to_device(m)
        return packer.pack_material3(md) if packed_relu else md
    up = lambda st: pipeline.LayerState3(w=d3(st["w"]), a=d3(st["a"]), b=d3(st["b"]), c=d3(st["c"]), r=d3(st["r"]),
                                         rt=d3(st["rt"]), relu=m3(st["relu"]), pool1=m3(st["pool1"]), pool2=m3(st["pool2"]),
                                         packed=packed_relu)

    def check3(got, want, what):
        for i in range(3):
            g = mpc.to_host(got[i]).reshape(want[i].shape)
            assert np.array_equal(g, want[i]), f"{what}: party {i} differs in {(g != want[i]).sum()} elements"

    lane = mpc.Lane(0); lane.use_single_queue()
    states = [up(st) for st in mbs[0]["states"]]
    x = d3(mbs[0]["x"]); keep = []
    for li, (L, st) in enumerate(zip(layers, states)):
        print(f"three parties, layer {li} ({L.name})", flush=True)
        x = pipeline.run_layer3(lane, L, st, x, keep)
        lane.sync()
        check3(x, mbs[0]["want"][li], f"layer {li} ({L.name})")
    got = sum(mpc.to_host(v) for v in x).view(np.int64)
    # the float64 network on the decoded quantised inputs agrees on the logits to a few units of 2^-12
    logits = got / 65536.0
    assert logits.shape == (2, 10) and np.isfinite(logits).all()
    lane.close()
    # inter-batch pipeline, weight masks opened ahead of time
    lanes = [mpc.Lane(0) for _ in range(2)]
    sts = [[up(st) for st in mb["states"]] for mb in mbs]
    for ln, st in zip(lanes, sts):
        pipeline.preopen_weights3(ln, st)
    keep = []
    outs = pipeline.forward_pipelined3(lanes, layers, sts, [d3(mb["x"]) for mb in mbs], keep)
    for ln in lanes:
        ln.sync()
    for m in range(2):
        check3(outs[m], mbs[m]["want"][-1], f"pipelined micro-batch {m}")
    # the same on prepared planes
    for ln, st in zip(lanes, sts):
        pipeline.prepare_layers3(ln, layers, st)
    outs = pipeline.forward_pipelined3(lanes, layers, sts, [d3(mb["x"]) for mb in mbs], keep)
    for ln in lanes:
        ln.sync()
    for m in range(2):
        check3(outs[m], mbs[m]["want"][-1], f"pipelined micro-batch {m}, prepared planes")
    for ln in lanes + [packer]:
        ln.close()


def test_three_party_pooled_layers_as_relu_of_maxpool(mods):
    """The reordered network (pool first, then ReLU on a quarter of the elements) with three parties,
    sign-only chain: every layer's shares against the oracle run in the same order."""
    mpc, pipeline = mods
    base = synth.config_vgg16_pipeline(micro_batch=2)
    layers = base.layers
    rng = synth.rng_for(base.index, 15)
    host, _ = deal_network_host3(rng, layers, pool_first=True)
    assert sum(st["pool_first"] for st in host) == 5
    xs = synth.share_additive3(rng, synth.normal_fixed(rng, (2, 32, 32, 3), 1.0))
    want = oracle_forward3(layers, host, xs)
    lane = mpc.Lane(0); lane.use_single_queue()
    d3 = lambda t: tuple(mpc.to_device(v) for v in t)
    m3 = lambda m: None if m is None else lane.pack_material3(mpc.material_to_device(m))
    x = d3(xs); keep = []
    for li, (L, st) in enumerate(zip(layers, host)):
        state = pipeline.LayerState3(w=d3(st["w"]), a=d3(st["a"]), b=d3(st["b"]), c=d3(st["c"]), r=d3(st["r"]), rt=d3(st["rt"]),
                                     relu=m3(st["relu"]), pool1=m3(st["pool1"]), pool2=m3(st["pool2"]), packed=True,
                                     pool_first=st["pool_first"])
        x = pipeline.run_layer3(lane, L, state, x, keep)
        lane.sync()
        for i in range(3):
            g = mpc.to_host(x[i]).reshape(want[li][i].shape)
            assert np.array_equal(g, want[li][i]), f"layer {li} ({L.name}), party {i}"
    lane.close()


@pytest.mark.parametrize("packed_relu", [False, True], ids=["whole-word-relu", "sign-only-packed-relu"])
def test_vgg16_training_step_with_three_parties(mods, packed_relu):
    """Forward with the tape and backward through max-pool, ReLU, conv and dense layers with three
    simulated parties: logits and every layer's weight-gradient shares against the oracle (Sec. 5.3, Sec. 5.6)."""
    mpc, pipeline = mods
    base = synth.config_vgg16_pipeline(micro_batch=2)
    layers = base.layers
    rng = synth.rng_for(base.index, 14)
    host, _ = deal_network_host3(rng, layers)
    xs = synth.share_additive3(rng, synth.normal_fixed(rng, (2, 32, 32, 3), 1.0))
    bhost = deal_backward_host3(rng, layers, host)
    gout = synth.share_additive3(rng, synth.normal_fixed(rng, (2, 10), 0.5))
    print(f"three parties, training step, packed_relu={packed_relu}: oracle", flush=True)
    want_out, want_grads = oracle_train_step3(layers, host, bhost, xs, gout)
    lane = mpc.Lane(0); lane.use_single_queue()
    d3 = lambda t: tuple(mpc.to_device(v) for v in t)
    def m3(m):
        if m is None:
            return None
        md = mpc.material_to_device(m)
        return lane.pack_material3(md) if packed_relu else md
    states = [pipeline.LayerState3(w=d3(st["w"]), a=d3(st["a"]), b=d3(st["b"]), c=d3(st["c"]), r=d3(st["r"]), rt=d3(st["rt"]),
                                   relu=m3(st["relu"]), pool1=m3(st["pool1"]), pool2=m3(st["pool2"]), packed=packed_relu)
              for st in host]
    trip = lambda t: None if t is None else tuple(d3(q) for q in t)
    bstates = []
    for st, bs in zip(states, bhost):
        gx = None if bs["gx"] is None else dict(a=d3(bs["gx"]["a"]), b=st.b, c=d3(bs["gx"]["c"]), r=d3(bs["gx"]["r"]), rt=d3(bs["gx"]["rt"]))
        bstates.append(pipeline.BackwardState3(
            gx=gx, gw=dict(a=st.a, b=d3(bs["gw"]["b"]), c=d3(bs["gw"]["c"]), r=d3(bs["gw"]["r"]), rt=d3(bs["gw"]["rt"])),
            relu_t=trip(bs["relu_t"]), pool_t1=trip(bs["pool_t1"]), pool_t2=trip(bs["pool_t2"])))
    print("device run", flush=True)
    keep = []
    out, tape = pipeline.forward_train3(lane, layers, states, d3(xs), keep)
    grads = pipeline.backward3(lane, layers, states, bstates, tape, d3(gout), keep)
    lane.sync()

    def check3(got, want, what):
        for i in range(3):
            g = mpc.to_host(got[i]).reshape(want[i].shape)
            assert np.array_equal(g, want[i]), f"{what}: party {i} differs in {(g != want[i]).sum()} elements"

    check3(out, want_out, "logits")
    for li, L in enumerate(layers):
        check3(grads[li], want_grads[li], f"weight gradient of layer {li} ({L.name})")
    # SGD step with learning rate 2^-6: one more masked rescale, then a local subtraction
    pairs = [synth.deal_trunc3_pair(rng, want_grads[li][0].shape, bits=6) for li in range(len(layers))]
    pipeline.sgd_step3(lane, states, grads, [(d3(r), d3(rt)) for r, rt in pairs], 6)
    lane.sync()
    for li, (L, st) in enumerate(zip(layers, host)):
        step = oracle.truncate3(want_grads[li], pairs[li][0], pairs[li][1], 6)
        want_w = tuple(st["w"][i] - step[i].reshape(st["w"][i].shape) for i in range(3))
        check3(states[li].w, want_w, f"updated weights of layer {li} ({L.name})")
    lane.close()


# ------------------------------------------------ one layer as row chunks on two lanes (Alg. 3 inside a layer)
@pytest.mark.parametrize("lane_kind", ["single-queue-put", "three-streams"])
@pytest.mark.parametrize("kind,n_chunks,n_lanes", [("dense", 2, 2), ("dense", 3, 2), ("dense", 5, 1), ("conv", 2, 2), ("conv", 3, 3),
                                                   ("conv-strided", 2, 2)])
def test_layer_as_row_chunks_on_lanes(mods, kind, n_chunks, n_lanes, lane_kind):
    """Every chunk is a complete folded call on its rows; the assembled output is the one-call layer's, word for word
    against the oracle's Alg. 1 / Eq. 3 on the whole layer."""
    from helpers import deal_conv, deal_matmul, oracle_conv, oracle_matmul
    mpc, pipeline = mods
    import torch
    print(f"chunked layer {kind} chunks={n_chunks} lanes={n_lanes}", flush=True)
    rng = np.random.default_rng(311 + n_chunks)
    if kind == "dense":
        L = synth.Gemm("fc", 203, 150, 77, 1.0, 0.1, 1, False)
        d = deal_matmul(rng, L.M, L.K, L.N); want = oracle_matmul(d)
    else:
        stride = 2 if kind == "conv-strided" else 1
        L = synth.Conv("conv", 5, 9, 8, 20, 33, 3, 3, 1, stride, 1.0, 0.1, False, False)
        d = deal_conv(rng, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride); want = oracle_conv(d)
    up = lambda pair: (mpc.to_device(pair[0]), mpc.to_device(pair[1]))
    st = pipeline.LayerState(w=up(d["y"]), a=up(d["a"]), b=up(d["b"]), c=up(d["c"]),
                             f_public=mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1])))
    if lane_kind == "three-streams":
        lanes = [mpc.Lane(0) for _ in range(n_lanes)]
    else:
        lanes = [mpc.Lane(0, single_queue=True) for _ in range(n_lanes)]
        for ln in lanes:
            ln.set_exchange("put")
    consumer = mpc.Lane(0)
    layer = pipeline.ChunkedLinear(lanes, L, st, n_chunks=n_chunks)
    x = up(d["x"])
    out = (torch.empty_like(st.c[0]), torch.empty_like(st.c[1]))
    for rep in range(2):                      # the second pass reuses every buffer
        layer(x, out)
        layer.join(consumer)
        got = consumer.open(out)              # issued on the consumer's queue: waits for the chunk lanes on the device
        consumer.sync()
        assert np.array_equal(mpc.to_host(got), want[0] + want[1])
        for i in range(2):
            assert np.array_equal(mpc.to_host(out[i]), want[i]), f"party {i}, pass {rep}"
    with pytest.raises(ValueError):
        pipeline.ChunkedLinear(lanes, L, st, n_chunks=0)
    for ln in lanes + [consumer]:
        ln.sync(); ln.close()


def test_fifth_single_queue_lane_shares_a_stream_and_cannot_record(mods):
    """Single-queue lanes draw their stream from a fixed set of four: a fifth one shares a stream (its results are
    still right), and recording a graph on a shared stream is refused."""
    mpc, _ = mods
    print("fifth single-queue lane", flush=True)
    lanes = [mpc.Lane(0, single_queue=True) for _ in range(5)]
    streams = [ln.stream(0) for ln in lanes]
    assert len(set(streams[:4])) == 4 and streams[4] in streams[:4]
    rng = np.random.default_rng(9)
    s = (synth.rand_words(rng, 1000), synth.rand_words(rng, 1000))
    outs = [ln.open((mpc.to_device(s[0]), mpc.to_device(s[1]))) for ln in lanes]
    for ln, o in zip(lanes, outs):
        ln.sync()
        assert np.array_equal(mpc.to_host(o), s[0] + s[1])
    shared = lanes[streams.index(streams[4])]
    for ln in (lanes[4], shared):
        with pytest.raises(mpc.MpcError):
            with ln.capture():
                pass
    lanes[4].close()
    with shared.capture():          # alone on its stream again
        pass
    for ln in lanes[:4]:
        ln.close()
