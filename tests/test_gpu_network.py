"""Whole-network parity and pipeline invariance on the GPU: a VGG16-shaped
CIFAR network (13 conv 3x3 layers with 2x2 max-pooling, three dense layers)
at a small batch, every layer's output shares against the oracle; the
inter-batch pipeline, pre-opened weight masks, the Alg. 3 ordering and chunked
exchanges must not change a single bit (Sec. 5.10)."""
import numpy as np
import pytest

import oracle
from helpers import deal_network_host, oracle_forward, rec
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
                               packed=pack_lane is not None)


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
        x = pipeline.run_layer(lane, L, st, x)
        keep.extend(pipeline.run_layer.last_intermediates)
        lane.sync()
        check(mpc, x, mb["want"][li], f"layer {li} ({L.name})")
    # decoded logits close to a float64 run of the same quantised network
    logits = oracle.decode(rec((mpc.to_host(x[0]), mpc.to_host(x[1]))))
    assert logits.shape == (2, 10) and np.isfinite(logits).all()
    lane.close()


@pytest.mark.parametrize("mode", ["serial-3stream", "pipelined", "pipelined-preopened", "pipelined-two-phase-chunked",
                                  "pipelined-packed-relu"])
def test_pipeline_invariance(mods, dealt, mode):
    mpc, pipeline = mods
    layers, mbs = dealt
    print(f"pipeline invariance: {mode}", flush=True)
    lanes = [mpc.Lane(0) for _ in mbs]
    if mode != "serial-3stream":
        for ln in lanes:
            ln.use_single_queue()
    pk = lanes[0] if mode == "pipelined-packed-relu" else None
    states = [[to_state(mpc, pipeline, st, pk) for st in mb["states"]] for mb in mbs]
    xs = [(mpc.to_device(mb["x"][0]), mpc.to_device(mb["x"][1])) for mb in mbs]
    kw = {}
    if mode in ("pipelined-preopened", "pipelined-two-phase-chunked"):
        for ln, sts in zip(lanes, states):
            pipeline.preopen_weights(ln, sts)
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
