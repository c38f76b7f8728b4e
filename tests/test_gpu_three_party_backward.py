"""GPU parity of the three-party backward calls (Sec. 4.1 and Sec. 5.3 with N = 3) against the
CPU oracle: gradient products of dense and convolution layers, the element-wise product, and
the backward of ReLU and max-pool with the sign shares of the forward conversions."""
import numpy as np
import pytest

import oracle
from paper_2209_13643_amd import synth

pytestmark = pytest.mark.gpu
U64 = np.uint64


@pytest.fixture(scope="module")
def mpc():
    from paper_2209_13643_amd import mpc as m
    return m


@pytest.fixture(params=["three-streams", "single-queue", "single-queue-put"])
def lane(mpc, request):
    ln = mpc.Lane(0)
    if request.param != "three-streams":
        ln.use_single_queue()
    if request.param == "single-queue-put":
        ln.set_exchange("put")
    yield ln
    ln.sync()
    ln.close()


def dev3(mpc, tri):
    return tuple(mpc.to_device(v) for v in tri)


def host3(mpc, lane, tri):
    lane.sync()
    return tuple(mpc.to_host(v) for v in tri)


def rec3(t):
    return np.asarray(t[0], dtype=U64) + np.asarray(t[1], dtype=U64) + np.asarray(t[2], dtype=U64)


def same3(got, want, what):
    for i in range(3):
        g = np.asarray(got[i]).reshape(np.shape(want[i]))
        assert np.array_equal(g, want[i]), f"{what}: party {i} differs in {(g != want[i]).sum()} of {g.size} words"


# ------------------------------------------------------------------ dense layers
def test_dense_layer_gradients_three_parties(mpc, lane):
    """grad_w = x^T g and grad_x = g w^T through the transposed-operand flags, then the masked rescale."""
    rng = np.random.default_rng(610)
    M, K, N = 70, 130, 36
    X = synth.normal_fixed(rng, (M, K), 1.0); Wt = synth.normal_fixed(rng, (K, N), 0.1); G = synth.normal_fixed(rng, (M, N), 0.5)
    xs, ws, gs = (synth.share_additive3(rng, v) for v in (X, Wt, G))
    # grad_w: left operand x stored [M][K] read transposed
    fw = lambda x, g: oracle.ring_matmul(np.ascontiguousarray(x.T), g)
    a, b, c = synth.deal_product_triple3(rng, X.shape, G.shape, fw)
    want = oracle.beaver_bilinear3(fw, xs, gs, a, b, c)
    gw = lane.beaver_matmul3(dev3(mpc, xs), dev3(mpc, gs), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c), flags=mpc.MPC_TRANS_X)
    same3(host3(mpc, lane, gw), want, "dense grad_w")
    r, rt = synth.deal_trunc3_pair(rng, (K, N))
    same3(host3(mpc, lane, lane.truncate3(gw, dev3(mpc, r), dev3(mpc, rt))), oracle.truncate3(want, r, rt), "dense grad_w rescaled")
    # grad_x: right operand w stored [K][N] read transposed
    fx = lambda g, w: oracle.ring_matmul(g, np.ascontiguousarray(w.T))
    a, b, c = synth.deal_product_triple3(rng, G.shape, Wt.shape, fx)
    want = oracle.beaver_bilinear3(fx, gs, ws, a, b, c)
    gx = lane.beaver_matmul3(dev3(mpc, gs), dev3(mpc, ws), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c), flags=mpc.MPC_TRANS_Y)
    same3(host3(mpc, lane, gx), want, "dense grad_x")
    ref = oracle.decode(G) @ oracle.decode(Wt).T
    r, rt = synth.deal_trunc3_pair(rng, (M, K))
    t = host3(mpc, lane, lane.truncate3(gx, dev3(mpc, r), dev3(mpc, rt)))
    assert np.abs(oracle.decode(rec3(t)) - ref).max() <= 2.0 ** -12


# ----------------------------------------------------------------- conv layers
GRAD_CASES = [  # B,H,W,Cin,Cout,KH,KW,pad,stride
    (1, 3, 3, 1, 1, 3, 3, 1, 1), (2, 5, 4, 3, 2, 3, 3, 1, 1), (1, 6, 6, 5, 7, 3, 3, 0, 1), (2, 4, 4, 5, 4, 1, 1, 0, 1),
    (2, 8, 8, 16, 32, 3, 3, 1, 1), (1, 9, 7, 20, 33, 3, 3, 2, 1), (2, 16, 16, 64, 48, 3, 3, 1, 1),
    (1, 7, 5, 2, 2, 3, 3, 1, 2), (1, 6, 6, 2, 3, 3, 3, 0, 2), (2, 6, 6, 3, 5, 5, 5, 2, 1)]


def deal_grad3(rng, case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, pad, stride)
    X = synth.normal_fixed(rng, (B, H, W, Cin), 1.0); Wt = synth.normal_fixed(rng, (KH, KW, Cin, Cout), 0.1)
    G = synth.normal_fixed(rng, (B, Ho, Wo, Cout), 0.5)
    return X, Wt, G, tuple(synth.share_additive3(rng, v) for v in (X, Wt, G))


@pytest.mark.parametrize("case", GRAD_CASES + [(2, 9, 9, 4, 6, 3, 3, 1, 3), (2, 12, 10, 8, 8, 3, 3, 1, 2)])
@pytest.mark.parametrize("preopened", [False, True])
def test_conv3_grad_x(mpc, lane, case, preopened):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print(f"conv3 grad_x {case} preopened={preopened}", flush=True)
    rng = np.random.default_rng(sum(case) + 600)
    X, Wt, G, (xs, ws, gs) = deal_grad3(rng, case)
    fx = lambda g, w: oracle.ring_conv2d_grad_x(g, w, X.shape, pad, stride)
    a, b, c = synth.deal_product_triple3(rng, G.shape, Wt.shape, fx)
    want = oracle.beaver_bilinear3(fx, gs, ws, a, b, c)
    f_public = mpc.to_device(sum((ws[i] - b[i] for i in range(1, 3)), ws[0] - b[0])) if preopened else None
    gx = lane.conv2d3_grad_x(dev3(mpc, gs), None if preopened else dev3(mpc, ws), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c),
                             pad, stride, f_public=f_public)
    same3(host3(mpc, lane, gx), want, "conv3 grad_x")
    assert np.array_equal(rec3(want), fx(G, Wt))


@pytest.mark.parametrize("case", GRAD_CASES)
def test_conv3_grad_w(mpc, lane, case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print(f"conv3 grad_w {case}", flush=True)
    rng = np.random.default_rng(sum(case) + 601)
    X, Wt, G, (xs, ws, gs) = deal_grad3(rng, case)
    fw = lambda x, g: oracle.ring_conv2d_grad_w(x, g, KH, KW, pad, stride)
    a, b, c = synth.deal_product_triple3(rng, X.shape, G.shape, fw)
    want = oracle.beaver_bilinear3(fw, xs, gs, a, b, c)
    gw = lane.conv2d3_grad_w(dev3(mpc, xs), dev3(mpc, gs), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c), pad, stride)
    same3(host3(mpc, lane, gw), want, "conv3 grad_w")


def test_conv3_grad_w_with_a_contraction_longer_than_one_exact_pass(mpc, lane):
    """16384 output pixels: the contraction is cut into slices that are exact in int32 and added in 64 bits."""
    case = (16, 32, 32, 4, 8, 3, 3, 1, 1)
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(612)
    X, Wt, G, (xs, ws, gs) = deal_grad3(rng, case)
    fw = lambda x, g: oracle.ring_conv2d_grad_w(x, g, KH, KW, pad, stride)
    a, b, c = synth.deal_product_triple3(rng, X.shape, G.shape, fw)
    want = oracle.beaver_bilinear3(fw, xs, gs, a, b, c)
    gw = lane.conv2d3_grad_w(dev3(mpc, xs), dev3(mpc, gs), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c), pad, stride)
    same3(host3(mpc, lane, gw), want, "conv3 grad_w, long contraction")


# ----------------------------------------------------------- non-linear layers
@pytest.mark.parametrize("n", [1, 2, 1000, 70001])
def test_mul3(mpc, lane, n):
    rng = np.random.default_rng(620 + n)
    X, Y = synth.rand_words(rng, n), synth.rand_words(rng, n)
    xs, ys = synth.share_additive3(rng, X), synth.share_additive3(rng, Y)
    a, b, c = synth.deal_product_triple3(rng, (n,), (n,), lambda p, q: p * q)
    want = oracle.beaver_mul3(xs, ys, a, b, c)
    z = lane.mul3(dev3(mpc, xs), dev3(mpc, ys), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c))
    got = host3(mpc, lane, z)
    same3(got, want, "mul3")
    assert np.array_equal(rec3(got), X * Y)


@pytest.mark.parametrize("n", [3, 4097, 50000])
@pytest.mark.parametrize("packed", [False, True])
def test_relu3_forward_then_backward(mpc, lane, n, packed):
    """Forward conversion on the GPU, its sign shares fed to the backward product."""
    print(f"relu3 backward n={n} packed={packed}", flush=True)
    rng = np.random.default_rng(630 + n)
    X = synth.normal_fixed(rng, (n,), 1.0); X[:3] = np.array([0, 1, -1], dtype=np.int64).view(U64)
    G = synth.normal_fixed(rng, (n,), 0.5)
    xs, gs = synth.share_additive3(rng, X), synth.share_additive3(rng, G)
    mat = synth.deal_relu3_material(rng, n)
    a, b, c = synth.deal_product_triple3(rng, (n,), (n,), lambda p, q: p * q)
    fwd = oracle.relu3(xs, mat)
    want = oracle.relu_backward3(gs, fwd.s_arith, a, b, c)
    md = mpc.material_to_device(mat)
    if packed:
        md = lane.pack_material3(md)
    y, sb, sa = lane.relu3(dev3(mpc, xs), md, want_sign=True, packed=packed)
    gx = lane.relu3_backward(dev3(mpc, gs), sa, dev3(mpc, a), dev3(mpc, b), dev3(mpc, c))
    got = host3(mpc, lane, gx)
    same3(got, want, "relu3 backward")
    assert np.array_equal(rec3(got), np.where(oracle.to_signed(X) >= 0, G, U64(0)))


@pytest.mark.parametrize("shape", [(1, 2, 2, 1), (2, 6, 4, 3), (3, 8, 8, 16), (2, 16, 16, 64)])
@pytest.mark.parametrize("packed", [False, True])
def test_maxpool3_forward_signs_then_backward(mpc, lane, shape, packed):
    print(f"maxpool3 backward {shape} packed={packed}", flush=True)
    B, H, W, C = shape
    rng = np.random.default_rng(sum(shape) + 640)
    X = rng.integers(-(1 << 30), 1 << 30, size=shape).astype(np.int64)
    n_out = B * (H // 2) * (W // 2) * C
    G = synth.normal_fixed(rng, (B, H // 2, W // 2, C), 0.5)
    xs, gs = synth.share_additive3(rng, X.view(U64)), synth.share_additive3(rng, G)
    m1, m2 = synth.deal_relu3_material(rng, 2 * n_out), synth.deal_relu3_material(rng, n_out)
    mul = lambda p, q: p * q
    t1 = synth.deal_product_triple3(rng, (2 * n_out,), (2 * n_out,), mul)
    t2 = synth.deal_product_triple3(rng, (n_out,), (n_out,), mul)
    want_y, ws1, ws2 = oracle.maxpool2x2_3(xs, m1, m2, want_signs=True)
    want_gx = oracle.maxpool2x2_backward3(gs, ws1, ws2, t1, t2, shape)
    d1, d2 = mpc.material_to_device(m1), mpc.material_to_device(m2)
    if packed:
        d1, d2 = lane.pack_material3(d1), lane.pack_material3(d2)
    y, s1, s2 = lane.maxpool3(dev3(mpc, xs), d1, d2, packed=packed, want_signs=True)
    gx = lane.maxpool3_backward(dev3(mpc, gs), s1, s2, [dev3(mpc, t) for t in t1], [dev3(mpc, t) for t in t2], shape)
    same3(host3(mpc, lane, y), want_y, "maxpool3 forward")
    same3(host3(mpc, lane, s1), ws1, "level-1 sign shares")
    same3(host3(mpc, lane, s2), ws2, "level-2 sign shares")
    same3(host3(mpc, lane, gx), want_gx, "maxpool3 backward")


def test_three_party_backward_argument_errors(mpc, lane):
    rng = np.random.default_rng(650)
    n = 16
    t = [dev3(mpc, v) for v in synth.deal_product_triple3(rng, (n,), (n,), lambda p, q: p * q)]
    x = dev3(mpc, synth.share_additive3(rng, synth.rand_words(rng, n)))
    lib = mpc.lib()
    assert lib.mpc_mul3_workspace_bytes(0) == 0 and lib.mpc_maxpool3_backward_workspace_bytes(1, 3, 2, 1) == 0
    with pytest.raises(mpc.MpcError):
        lane.maxpool3_backward(x, x, x, t, t, (1, 3, 2, 1))                    # odd height
    # square filters only, padding at most KH - 1 for the input gradient
    assert lib.mpc_conv2d3_grad_x_workspace_bytes(1, 8, 8, 2, 2, 3, 1, 0, 1) == 0
    assert lib.mpc_conv2d3_grad_x_workspace_bytes(1, 8, 8, 2, 2, 3, 3, 3, 1) == 0
    lane.sync()
