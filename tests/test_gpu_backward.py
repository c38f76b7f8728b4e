"""GPU parity of the backward-pass products (Sec. 4.1, 4.2, 5.3): dense-layer
gradients through transposed operands, conv gradients w.r.t. input and filter,
element-wise Alg. 1 and the ReLU backward, each against the CPU oracle on the
same seeded shares and triples, bit for bit."""
import numpy as np
import pytest

import oracle
from helpers import rec
from paper_2209_13643_amd import synth

pytestmark = pytest.mark.gpu
U64 = np.uint64
T = np.ascontiguousarray


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
        ln.set_exchange("put")          # ReLU rounds exchange by remote store instead of copy kernels
    yield ln
    ln.sync()
    ln.close()


def dev(mpc, pair):
    return (mpc.to_device(pair[0]), mpc.to_device(pair[1]))


def host(mpc, lane, pair):
    lane.sync()
    return (mpc.to_host(pair[0]), mpc.to_host(pair[1]))


def assert_shares_equal(got, want, what=""):
    for i in range(2):
        g = np.asarray(got[i]).reshape(np.shape(want[i]))
        if not np.array_equal(g, want[i]):
            bad = np.argwhere(g != want[i])
            raise AssertionError(f"{what}: party {i} differs at {len(bad)} of {g.size} elements, first {bad[0]}")


def tr(pair):
    """Transposed storage of a pair of (possibly batched) matrices."""
    return tuple(T(np.swapaxes(p, -1, -2)) for p in pair)


# ------------------------------------------------------------- dense layers
@pytest.mark.parametrize("shape", [(5, 7, 3), (64, 256, 128), (130, 70, 200), (33, 1000, 17)])
@pytest.mark.parametrize("trans", ["x", "y", "xy"])
def test_matmul_transposed_operands(mpc, lane, shape, trans):
    M, K, N = shape
    print(f"matmul trans={trans} {shape}", flush=True)
    rng = np.random.default_rng(M + K + N + len(trans))
    xs = synth.share_additive(rng, synth.normal_fixed(rng, (M, K), 1.0))
    ys = synth.share_additive(rng, synth.normal_fixed(rng, (K, N), 0.1))
    a, b, c = synth.deal_product_triple(rng, (M, K), (K, N), oracle.ring_matmul)
    want = oracle.truncate(oracle.beaver_matmul(xs, ys, a, b, c), 16)
    flags = mpc.MPC_TRUNCATE | (mpc.MPC_TRANS_X if "x" in trans else 0) | (mpc.MPC_TRANS_Y if "y" in trans else 0)
    xd, ad = (tr(xs), tr(a)) if "x" in trans else (xs, a)
    yd, bd = (tr(ys), tr(b)) if "y" in trans else (ys, b)
    z = lane.beaver_matmul(dev(mpc, xd), dev(mpc, yd), dev(mpc, ad), dev(mpc, bd), dev(mpc, c), flags=flags)
    assert_shares_equal(host(mpc, lane, z), want, "transposed matmul")


def test_dense_layer_gradients(mpc, lane):
    """grad_w = x^T g and grad_x = g w^T from the tensors as the forward pass stored them,
    the weight mask of the forward pass reused (f_public)."""
    M, K, N = 96, 200, 72
    print("dense gradients", flush=True)
    rng = np.random.default_rng(11)
    X = synth.normal_fixed(rng, (M, K), 1.0); Wt = synth.normal_fixed(rng, (K, N), 0.1)
    G = synth.normal_fixed(rng, (M, N), 0.5)
    xs, ws, gs = (synth.share_additive(rng, v) for v in (X, Wt, G))
    # grad_w [K x N] = x^T [K x M] . g [M x N]
    a, b, c = synth.deal_product_triple(rng, (K, M), (M, N), oracle.ring_matmul)
    want = oracle.truncate(oracle.beaver_matmul(tr(xs), gs, a, b, c), 16)
    gw = lane.beaver_matmul(dev(mpc, xs), dev(mpc, gs), dev(mpc, tr(a)), dev(mpc, b), dev(mpc, c),
                            flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_X)
    assert_shares_equal(host(mpc, lane, gw), want, "grad_w")
    assert np.abs(oracle.decode(rec(want)) - oracle.decode(X).T @ oracle.decode(G)).max() < 2.0 ** -12 * M
    # grad_x [M x K] = g [M x N] . w^T [N x K]; w - b was opened in the forward pass with mask b_w
    a, bw_t, c = synth.deal_product_triple(rng, (M, N), (N, K), oracle.ring_matmul)
    bw = tr(bw_t)                                               # the mask in w's own layout [K][N]
    f_public = (ws[0] - bw[0]) + (ws[1] - bw[1])
    want = oracle.truncate(oracle.beaver_matmul(gs, tr(ws), a, bw_t, c), 16)
    gx = lane.beaver_matmul(dev(mpc, gs), None, dev(mpc, a), dev(mpc, bw), dev(mpc, c),
                            f_public=mpc.to_device(f_public), flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_Y)
    assert_shares_equal(host(mpc, lane, gx), want, "grad_x")


@pytest.mark.parametrize("shape", [(8, 40000, 8), (24, 16400, 40), (1280, 20000, 1024)])
def test_contraction_longer_than_one_exact_pass(mpc, lane, shape):
    """K beyond the int32-exact length of one pass: the contraction is cut into
    slices (also when there are plenty of output tiles) and still exact."""
    M, K, N = shape
    print(f"long contraction {shape}", flush=True)
    rng = np.random.default_rng(K)
    L = synth.rand_words(rng, (M, K)); R = synth.rand_words(rng, (K, N))
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    assert np.array_equal(mpc.to_host(Z), oracle.ring_matmul(L, R))
    if M * N <= 1024:
        xs, ys = synth.share_additive(rng, L), synth.share_additive(rng, R)
        a, b, c = synth.deal_product_triple(rng, (M, K), (K, N), oracle.ring_matmul)
        z = lane.beaver_matmul(dev(mpc, xs), dev(mpc, ys), dev(mpc, a), dev(mpc, b), dev(mpc, c), flags=0)
        assert_shares_equal(host(mpc, lane, z), oracle.beaver_matmul(xs, ys, a, b, c), "long beaver matmul")


def test_beaver_long_contraction_many_tiles(mpc):
    M, K, N = 1280, 20000, 1024
    print(f"long beaver contraction {M}x{K}x{N}", flush=True)
    lane = mpc.Lane(0); lane.use_single_queue()
    rng = np.random.default_rng(4)
    xs = synth.share_additive(rng, synth.normal_fixed(rng, (M, K), 1.0))
    ys = synth.share_additive(rng, synth.normal_fixed(rng, (K, N), 0.05))
    a, b, c = synth.deal_product_triple(rng, (M, K), (K, N), oracle.ring_matmul)
    z = lane.beaver_matmul(dev(mpc, xs), dev(mpc, ys), dev(mpc, a), dev(mpc, b), dev(mpc, c))
    assert_shares_equal(host(mpc, lane, z), oracle.truncate(oracle.beaver_matmul(xs, ys, a, b, c), 16), "long beaver")
    lane.close()


# --------------------------------------------------------------- conv layers
GRAD_CASES = [  # B,H,W,Cin,Cout,KH,KW,pad,stride
    (1, 3, 3, 1, 1, 3, 3, 1, 1), (2, 5, 4, 3, 2, 3, 3, 1, 1), (1, 6, 6, 5, 7, 3, 3, 0, 1), (2, 4, 4, 5, 4, 1, 1, 0, 1),
    (2, 8, 8, 16, 32, 3, 3, 1, 1), (1, 9, 7, 20, 33, 3, 3, 2, 1), (2, 16, 16, 64, 48, 3, 3, 1, 1),
    (1, 7, 5, 2, 2, 3, 3, 1, 2), (1, 6, 6, 2, 3, 3, 3, 0, 2), (2, 6, 6, 3, 5, 5, 5, 2, 1)]


def deal_grad(rng, case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, pad, stride)
    X = synth.normal_fixed(rng, (B, H, W, Cin), 1.0); Wt = synth.normal_fixed(rng, (KH, KW, Cin, Cout), 0.1)
    G = synth.normal_fixed(rng, (B, Ho, Wo, Cout), 0.5)
    return X, Wt, G, tuple(synth.share_additive(rng, v) for v in (X, Wt, G))


@pytest.mark.parametrize("case", GRAD_CASES + [(2, 9, 9, 4, 6, 3, 3, 1, 3), (1, 8, 8, 16, 16, 1, 1, 0, 2), (2, 12, 10, 8, 8, 3, 3, 1, 2)])
@pytest.mark.parametrize("preopened", [False, True])
def test_conv_grad_x(mpc, lane, case, preopened):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print(f"conv grad_x {case} preopened={preopened}", flush=True)
    rng = np.random.default_rng(sum(case))
    X, Wt, G, (xs, ws, gs) = deal_grad(rng, case)
    fx = lambda g, w: oracle.ring_conv2d_grad_x(g, w, X.shape, pad, stride)
    a, b, c = synth.deal_product_triple(rng, G.shape, Wt.shape, fx)
    want = oracle.truncate(oracle.beaver_bilinear(fx, gs, ws, a, b, c), 16)
    f_public = mpc.to_device((ws[0] - b[0]) + (ws[1] - b[1])) if preopened else None
    gx = lane.conv2d_grad_x(dev(mpc, gs), None if preopened else dev(mpc, ws), dev(mpc, a), dev(mpc, b), dev(mpc, c),
                            pad, stride, f_public=f_public)
    assert_shares_equal(host(mpc, lane, gx), want, "conv grad_x")


@pytest.mark.parametrize("case", GRAD_CASES)
@pytest.mark.parametrize("preopened", [False, True])
def test_conv_grad_w(mpc, lane, case, preopened):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print(f"conv grad_w {case} preopened={preopened}", flush=True)
    rng = np.random.default_rng(sum(case) + 1)
    X, Wt, G, (xs, ws, gs) = deal_grad(rng, case)
    fw = lambda x, g: oracle.ring_conv2d_grad_w(x, g, KH, KW, pad, stride)
    a, b, c = synth.deal_product_triple(rng, X.shape, G.shape, fw)
    want = oracle.truncate(oracle.beaver_bilinear(fw, xs, gs, a, b, c), 16)
    e_public = mpc.to_device((xs[0] - a[0]) + (xs[1] - a[1])) if preopened else None
    gw = lane.conv2d_grad_w(None if preopened else dev(mpc, xs), dev(mpc, gs), dev(mpc, a), dev(mpc, b), dev(mpc, c),
                            pad, stride, e_public=e_public)
    assert_shares_equal(host(mpc, lane, gw), want, "conv grad_w")


def test_conv_gradients_float64_agreement(mpc, lane):
    """Decoded gradients against autograd in float64 on the decoded operands."""
    import torch
    case = (2, 8, 8, 16, 32, 3, 3, 1, 1)
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print("conv gradients vs float64", flush=True)
    rng = np.random.default_rng(9)
    X, Wt, G, (xs, ws, gs) = deal_grad(rng, case)
    xt = torch.from_numpy(oracle.decode(X)).permute(0, 3, 1, 2).requires_grad_()
    wt = torch.from_numpy(oracle.decode(Wt)).permute(3, 2, 0, 1).requires_grad_()
    torch.nn.functional.conv2d(xt, wt, padding=pad).backward(torch.from_numpy(oracle.decode(G)).permute(0, 3, 1, 2))
    fx = lambda g, w: oracle.ring_conv2d_grad_x(g, w, X.shape, pad, stride)
    fw = lambda x, g: oracle.ring_conv2d_grad_w(x, g, KH, KW, pad, stride)
    a, b, c = synth.deal_product_triple(rng, G.shape, Wt.shape, fx)
    gx = host(mpc, lane, lane.conv2d_grad_x(dev(mpc, gs), dev(mpc, ws), dev(mpc, a), dev(mpc, b), dev(mpc, c), pad))
    a, b, c = synth.deal_product_triple(rng, X.shape, G.shape, fw)
    gw = host(mpc, lane, lane.conv2d_grad_w(dev(mpc, xs), dev(mpc, gs), dev(mpc, a), dev(mpc, b), dev(mpc, c), pad, stride))
    assert np.abs(oracle.decode(rec(gx)) - xt.grad.permute(0, 2, 3, 1).numpy()).max() <= 2.0 ** -12
    assert np.abs(oracle.decode(rec(gw)).reshape(KH, KW, Cin, Cout) - wt.grad.permute(2, 3, 1, 0).numpy()).max() <= 2.0 ** -12


# ----------------------------------------------------------- non-linear layers
@pytest.mark.parametrize("n", [1, 2, 1000, 70001])
@pytest.mark.parametrize("trunc", [False, True])
def test_mul(mpc, lane, n, trunc):
    print(f"mul n={n} trunc={trunc}", flush=True)
    rng = np.random.default_rng(n + trunc)
    X = synth.normal_fixed(rng, (n,), 1.0) if trunc else synth.rand_words(rng, n)
    Y = synth.normal_fixed(rng, (n,), 1.0) if trunc else synth.rand_words(rng, n)
    xs, ys = synth.share_additive(rng, X), synth.share_additive(rng, Y)
    a, b, c = synth.deal_product_triple(rng, (n,), (n,), lambda p, q: p * q)
    want = oracle.beaver_mul(xs, ys, a, b, c)
    if trunc:
        want = oracle.truncate(want, 16)
    z = lane.mul(dev(mpc, xs), dev(mpc, ys), dev(mpc, a), dev(mpc, b), dev(mpc, c), flags=mpc.MPC_TRUNCATE if trunc else 0)
    assert_shares_equal(host(mpc, lane, z), want, "mul")


@pytest.mark.parametrize("n", [3, 4097, 50000])
@pytest.mark.parametrize("packed", [False, True])
def test_relu_forward_then_backward(mpc, lane, n, packed):
    """Forward conversion on the GPU, its sign shares fed to the backward product."""
    print(f"relu backward n={n} packed={packed}", flush=True)
    rng = np.random.default_rng(n)
    X = synth.normal_fixed(rng, (n,), 1.0); X[:3] = np.array([0, 1, -1], dtype=np.int64).view(U64)
    G = synth.normal_fixed(rng, (n,), 0.5)
    xs, gs = synth.share_additive(rng, X), synth.share_additive(rng, G)
    mat = synth.deal_relu_material(rng, n)
    a, b, c = synth.deal_product_triple(rng, (n,), (n,), lambda p, q: p * q)
    fwd = oracle.relu(xs, mat)
    want = oracle.relu_backward(gs, fwd.s_arith, a, b, c)
    md = mpc.material_to_device(mat)
    if packed:
        md = lane.pack_material(md)
    y, sb, sa = lane.relu(dev(mpc, xs), md, want_sign=True, packed=packed)
    gx = lane.relu_backward(dev(mpc, gs), sa, dev(mpc, a), dev(mpc, b), dev(mpc, c))
    got = host(mpc, lane, gx)
    assert_shares_equal(got, want, "relu backward")
    assert np.array_equal(rec(got), np.where(oracle.to_signed(X) >= 0, G, U64(0)))


@pytest.mark.parametrize("shape", [(1, 2, 2, 1), (2, 6, 4, 3), (3, 8, 8, 16), (2, 16, 16, 64)])
@pytest.mark.parametrize("packed", [False, True])
def test_maxpool_forward_signs_then_backward(mpc, lane, shape, packed):
    print(f"maxpool backward {shape} packed={packed}", flush=True)
    B, H, W, C = shape
    rng = np.random.default_rng(sum(shape))
    X = rng.integers(-(1 << 30), 1 << 30, size=shape).astype(np.int64)
    n_out = B * (H // 2) * (W // 2) * C
    G = synth.normal_fixed(rng, (B, H // 2, W // 2, C), 0.5)
    xs, gs = synth.share_additive(rng, X.view(U64)), synth.share_additive(rng, G)
    m1, m2 = synth.deal_relu_material(rng, 2 * n_out), synth.deal_relu_material(rng, n_out)
    mul = lambda p, q: p * q
    t1 = synth.deal_product_triple(rng, (2 * n_out,), (2 * n_out,), mul)
    t2 = synth.deal_product_triple(rng, (n_out,), (n_out,), mul)
    want_y, ws1, ws2 = oracle.maxpool2x2(xs, m1, m2, want_signs=True)
    want_gx = oracle.maxpool2x2_backward(gs, ws1, ws2, t1, t2, shape)
    d1, d2 = mpc.material_to_device(m1), mpc.material_to_device(m2)
    if packed:
        d1, d2 = lane.pack_material(d1), lane.pack_material(d2)
    y, s1, s2 = lane.maxpool2x2(dev(mpc, xs), d1, d2, packed=packed, want_signs=True)
    gx = lane.maxpool2x2_backward(dev(mpc, gs), s1, s2, [dev(mpc, t) for t in t1], [dev(mpc, t) for t in t2], shape)
    lane.sync()
    assert_shares_equal(host(mpc, lane, y), want_y, "maxpool forward")
    assert_shares_equal(host(mpc, lane, s1), ws1, "level-1 sign shares")
    assert_shares_equal(host(mpc, lane, s2), ws2, "level-2 sign shares")
    assert_shares_equal(host(mpc, lane, gx), want_gx, "maxpool backward")


def test_backward_argument_errors(mpc, lane):
    print("backward argument errors", flush=True)
    import torch
    L = mpc.lib()
    t = torch.zeros(4096, dtype=torch.int64, device=lane.device)
    sh = mpc._share((t, t))
    lane.reserve(1 << 20)
    h = lane._h
    # non-square filters have no input-gradient path; stride 0 is no stride
    assert L.mpc_conv2d_grad_x(h, sh, sh, sh, sh, sh, sh, 1, 8, 8, 2, 2, 3, 1, 0, 1, None, 1, 0) == -1
    assert L.mpc_conv2d_grad_x(h, sh, sh, sh, sh, sh, sh, 1, 8, 8, 2, 2, 3, 3, 1, 0, None, 1, 0) == -1
    assert L.mpc_conv2d_grad_w(h, sh, sh, sh, sh, sh, sh, 1, 8, 8, 2, 2, 3, 3, 1, 0, None, 1, 0) == -1
    assert L.mpc_conv2d_grad_w(h, mpc._share(None), sh, sh, sh, sh, sh, 1, 8, 8, 2, 2, 3, 3, 1, 1, None, 1, 0) == -1
    assert L.mpc_mul(h, sh, sh, sh, sh, sh, sh, 0, 0) == -1
    assert L.mpc_mul(h, sh, sh, sh, sh, sh, sh, 16, 2) == -1
    small = mpc.Lane(0); small.reserve(256)
    assert L.mpc_mul(small._h, sh, sh, sh, sh, sh, sh, 4096, 0) == -2
    small.close()
    assert L.mpc_conv2d_grad_x_workspace_bytes(1, 8, 8, 2, 2, 3, 3, 1, 2) > L.mpc_conv2d_grad_x_workspace_bytes(1, 8, 8, 2, 2, 3, 3, 1, 1)
    assert L.mpc_mul_workspace_bytes(0) == 0
