"""GPU parity at the hard layer shapes of the models the paper evaluates (Sec. 5.2: ResNet-50 and VGG16 at ImageNet
size, a Transformer encoder with H = 1024): every share of every party, full tensors, bit for bit against the oracle.
Inputs are synthetic (fixed-point N(0, 1) activations, He-normal / N(0, 0.02) weights, uniform triples), batch 1 or 2
so that the oracle's plain loops finish in seconds; only the shapes are the models'.

  conv 7x7 / stride 2 / pad 3, 3 -> 64 channels on 224x224 (ResNet-50's first layer): 49 filter taps, one
      16-channel block of which 3 channels are real, strided windows over the padding;
  conv 1x1 / stride 2, 256 -> 512 channels on 56x56 (ResNet-50's first down-sampling shortcut);
  dense 25088 -> 4096 at 2 rows (VGG16's first classifier layer): a 25088-deep contraction cut into the largest
      number of slices the launcher uses, two-row output tiles;
  dense [4096 x 1024] x [1024 x 3072] (the H = 1024 encoder's QKV projection at batch 8 x sequence 512).

Each layer runs as the plain call and as the folded prepared call."""
import functools

import numpy as np
import pytest

import oracle
from helpers import deal_conv, deal_matmul, oracle_conv, oracle_matmul
from paper_2209_13643_amd import synth

pytestmark = pytest.mark.gpu
TOL = 2.0 ** -12


@pytest.fixture(scope="module")
def mpc():
    from paper_2209_13643_amd import mpc as m
    return m


@pytest.fixture(params=["single-queue", "three-streams"])
def lane(mpc, request):
    ln = mpc.Lane(0)
    if request.param == "single-queue":
        ln.use_single_queue()
    yield ln
    ln.sync()
    ln.close()


def dev(mpc, pair):
    return (mpc.to_device(pair[0]), mpc.to_device(pair[1]))


def same(mpc, lane, got, want, what):
    lane.sync()
    for i in range(2):
        g = mpc.to_host(got[i]).reshape(want[i].shape)
        if not np.array_equal(g, want[i]):
            bad = np.argwhere(g != want[i])
            raise AssertionError(f"{what}: party {i} differs at {len(bad)} of {g.size} words, first {bad[0]}")


def decoded_close(want, X, Wt, ref):
    """Decoded product within 2^-12 of float64 on the decoded inputs wherever the local rescale did not wrap."""
    t = (want[0] + want[1])
    err = np.abs(oracle.decode(t) - ref)
    wrapped = err > 1.0          # a wrap is off by about 2^48 / 2^16: unmistakable
    assert wrapped.mean() < 1e-3
    assert err[~wrapped].max() <= TOL, err[~wrapped].max()


def run_conv_both_ways(mpc, lane, d, KH, KW, what):
    want = oracle_conv(d)
    x, y, a, b, c = (dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c"))
    z = lane.conv2d(x, y, a, b, c, d["pad"], d["stride"])
    same(mpc, lane, z, want, what + ", plain call")
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    right, left = lane.prepare_conv2d(a, b, f_public, d["pad"], d["stride"])
    c0f = lane.fold_conv2d(a, b, c, d["pad"], d["stride"])
    z = lane.conv2d_prepared(x, a, (c0f, c[1]), right, left, KH, KW, d["pad"], d["stride"],
                             flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
    same(mpc, lane, z, want, what + ", folded prepared call")
    return want


def test_resnet_first_layer_7x7_stride2_pad3_three_channels(mpc, lane):
    print("paper shape: conv 7x7 s2 p3, 3 -> 64, 224x224, batch 1", flush=True)
    rng = np.random.default_rng(701)
    d = deal_conv(rng, 1, 224, 224, 3, 64, 7, 7, 3, 2, x_std=1.0, w_std=synth.he_std(49 * 3))
    want = run_conv_both_ways(mpc, lane, d, 7, 7, "conv 7x7/2")
    assert want[0].shape == (1, 112, 112, 64)
    import torch
    ref = torch.nn.functional.conv2d(torch.from_numpy(oracle.decode(d["X"])).permute(0, 3, 1, 2),
                                     torch.from_numpy(oracle.decode(d["Y"])).permute(3, 2, 0, 1), padding=3, stride=2)
    decoded_close(want, d["X"], d["Y"], ref.permute(0, 2, 3, 1).numpy())


def test_resnet_downsample_1x1_stride2(mpc, lane):
    print("paper shape: conv 1x1 s2, 256 -> 512, 56x56, batch 2", flush=True)
    rng = np.random.default_rng(702)
    d = deal_conv(rng, 2, 56, 56, 256, 512, 1, 1, 0, 2, x_std=1.0, w_std=synth.he_std(256))
    want = run_conv_both_ways(mpc, lane, d, 1, 1, "conv 1x1/2")
    assert want[0].shape == (2, 28, 28, 512)


@functools.lru_cache(maxsize=1)
def dealt_classifier():
    """Dealt once for both lane modes: the 25088 x 4096 weight, its shares and triple are 0.8 GB each."""
    M, K, N = 2, 25088, 4096
    d = deal_matmul(np.random.default_rng(703), M, K, N, x_std=1.0, w_std=synth.he_std(K))
    return d, oracle_matmul(d)


def test_vgg16_classifier_25088_deep_at_two_rows(mpc, lane):
    print("paper shape: dense 25088 -> 4096, 2 rows", flush=True)
    M, K, N = 2, 25088, 4096
    d, want = dealt_classifier()
    print("  dealt", flush=True)
    # the contraction is sliced as finely as the launcher goes (more than 30 slices of the two-party launch)
    lib = mpc.lib()
    assert lib.mpc_matmul_workspace_bytes(M, K, N, 1) > 30 * 2 * M * N * 8, "fewer than 30 slices of partial products"
    x, y, a, b, c = (dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c"))
    z = lane.beaver_matmul(x, y, a, b, c)
    same(mpc, lane, z, want, "dense 25088x4096, plain call")
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    right, left = lane.prepare_matmul(a, b, f_public)
    c0f = lane.fold_matmul(a, b, c)
    z = lane.beaver_matmul_prepared(x, a, (c0f, c[1]), right, left, flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
    same(mpc, lane, z, want, "dense 25088x4096, folded prepared call")
    decoded_close(want, d["X"], d["Y"], oracle.decode(d["X"]) @ oracle.decode(d["Y"]))


def test_transformer_h1024_qkv_projection(mpc):
    print("paper shape: dense [4096 x 1024] x [1024 x 3072]", flush=True)
    lane = mpc.Lane(0); lane.use_single_queue()
    rng = np.random.default_rng(704)
    M, K, N = 4096, 1024, 3072
    d = deal_matmul(rng, M, K, N, x_std=1.0, w_std=0.02)
    want = oracle_matmul(d)
    x, y, a, b, c = (dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c"))
    z = lane.beaver_matmul(x, y, a, b, c)
    same(mpc, lane, z, want, "qkv H=1024, plain call")
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    right, left = lane.prepare_matmul(a, b, f_public)
    c0f = lane.fold_matmul(a, b, c)
    z = lane.beaver_matmul_prepared(x, a, (c0f, c[1]), right, left, n_chunks=4, flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
    same(mpc, lane, z, want, "qkv H=1024, folded prepared call")
    decoded_close(want, d["X"], d["Y"], oracle.decode(d["X"]) @ oracle.decode(d["Y"]))
    lane.close()
