"""Pins for the CPU oracle: everything here runs without a GPU and compares the
oracle with something other than itself - Python big-int arithmetic, numpy /
torch library routines, closed forms, exhaustive enumeration.

Citations are to the paper's sections / algorithms / equations."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2209_13643_amd import synth

U64 = np.uint64
MOD = 1 << 64


def rec(pair):
    return np.asarray(pair[0], dtype=U64) + np.asarray(pair[1], dtype=U64)


def big_matmul(L, R):
    """Python big-int matrix product reduced mod 2^64 at the end."""
    L = [[int(v) for v in row] for row in L]
    R = [[int(v) for v in row] for row in R]
    return np.array([[sum(L[m][k] * R[k][n] for k in range(len(R))) % MOD
                      for n in range(len(R[0]))] for m in range(len(L))], dtype=U64)


def deal_matmul(rng, M, K, N, x=None, y=None):
    X = synth.rand_words(rng, (M, K)) if x is None else x
    Y = synth.rand_words(rng, (K, N)) if y is None else y
    xs, ys = synth.share_additive(rng, X), synth.share_additive(rng, Y)
    a, b, c = synth.deal_product_triple(rng, (M, K), (K, N), lambda A, B: A @ B)
    return X, Y, xs, ys, a, b, c


# ------------------------------------------------------------ Alg. 1 on matrices
@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 2), (3, 1, 4), (5, 7, 3)])
def test_ring_matmul_vs_bigint(shape):
    M, K, N = shape
    rng = np.random.default_rng(1)
    L, R = synth.rand_words(rng, (M, K)), synth.rand_words(rng, (K, N))
    assert np.array_equal(oracle.ring_matmul(L, R), big_matmul(L, R))


def test_ring_matmul_not_transposed():
    # a non-square, non-symmetric case with a known answer: [1 2 3] * [[1],[10],[100]]
    L = np.array([[1, 2, 3]], dtype=U64); R = np.array([[1], [10], [100]], dtype=U64)
    assert oracle.ring_matmul(L, R).tolist() == [[321]]
    # wrap-around: (2^63) * 2 = 0, (2^64 - 1)^2 = 1
    L = np.array([[1 << 63, MOD - 1]], dtype=U64); R = np.array([[2], [MOD - 1]], dtype=U64)
    assert oracle.ring_matmul(L, R).tolist() == [[1]]


@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 2), (3, 1, 4), (17, 33, 9), (64, 256, 128)])
def test_beaver_matmul_reconstructs_product(shape):
    """Sec. 3.2: the sum of the [z_i] is X*Y."""
    M, K, N = shape
    rng = np.random.default_rng(10 + M)
    X, Y, xs, ys, a, b, c = deal_matmul(rng, M, K, N)
    z, e, f = oracle.beaver_matmul(xs, ys, a, b, c, want_open=True)
    want = big_matmul(X, Y) if M * K * N <= 5000 else X @ Y
    assert np.array_equal(rec(z), want)
    assert np.array_equal(e, X - rec(a))      # Delta = X - A
    assert np.array_equal(f, Y - rec(b))      # epsilon = Y - B
    # the shares themselves are masked: neither equals the product on its own
    assert not np.array_equal(z[0], want) and not np.array_equal(z[1], want)


def test_beaver_matmul_independent_of_triple_and_masks():
    rng = np.random.default_rng(3)
    X, Y = synth.rand_words(rng, (6, 5)), synth.rand_words(rng, (5, 4))
    outs = []
    for _ in range(3):
        _, _, xs, ys, a, b, c = deal_matmul(rng, 6, 5, 4, X, Y)
        outs.append(rec(oracle.beaver_matmul(xs, ys, a, b, c)))
    assert all(np.array_equal(o, outs[0]) for o in outs)


def test_beaver_matmul_zero_triple_degenerates_to_plain_product():
    """A = B = C = 0: e = X, f = Y, party 0 ends with X*Y, party 1 with 0."""
    rng = np.random.default_rng(4)
    X, Y = synth.rand_words(rng, (4, 6)), synth.rand_words(rng, (6, 3))
    xs, ys = synth.share_additive(rng, X), synth.share_additive(rng, Y)
    zA, zB, zC = np.zeros((4, 6), U64), np.zeros((6, 3), U64), np.zeros((4, 3), U64)
    z = oracle.beaver_matmul(xs, ys, (zA, zA), (zB, zB), (zC, zC))
    assert np.array_equal(z[0], big_matmul(X, Y))
    assert not z[1].any()


def test_beaver_matmul_each_term_matters():
    """Dropping or mis-assigning any term of Alg. 1's last two lines breaks
    reconstruction: rebuild z from the opened values term by term."""
    rng = np.random.default_rng(5)
    X, Y, xs, ys, a, b, c = deal_matmul(rng, 3, 4, 2)
    z, e, f = oracle.beaver_matmul(xs, ys, a, b, c, want_open=True)
    t = {k: big_matmul(*v) for k, v in
         dict(eb0=(e, b[0]), a0f=(a[0], f), ef=(e, f), eb1=(e, b[1]), a1f=(a[1], f)).items()}
    assert np.array_equal(z[0], c[0] + t["eb0"] + t["a0f"] + t["ef"])
    assert np.array_equal(z[1], c[1] + t["eb1"] + t["a1f"])


# ------------------------------------------------------------------ Eq. 3 (conv)
CONV_CASES = [  # B,H,W,Cin,Cout,KH,KW,pad,stride
    (1, 3, 3, 1, 1, 3, 3, 1, 1), (2, 5, 4, 3, 2, 3, 3, 1, 1), (1, 6, 6, 2, 3, 3, 3, 0, 2),
    (2, 4, 4, 5, 4, 1, 1, 0, 1), (1, 7, 5, 2, 2, 3, 3, 1, 2)]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_equals_im2col_matmul(case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(6)
    x = synth.rand_words(rng, (B, H, W, Cin)); w = synth.rand_words(rng, (KH, KW, Cin, Cout))
    direct = oracle.ring_conv2d(x, w, pad, stride)
    col = oracle.im2col(x, KH, KW, pad, stride)
    viaim = big_matmul(col, w.reshape(-1, Cout)).reshape(direct.shape)
    assert np.array_equal(direct, viaim)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_torch_float64(case):
    """Small integers keep float64 exact, so torch's conv2d is an independent
    definition of the same cross-correlation (layout NCHW / OIHW there)."""
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(7)
    xi = rng.integers(-1000, 1000, size=(B, H, W, Cin)); wi = rng.integers(-1000, 1000, size=(KH, KW, Cin, Cout))
    got = oracle.ring_conv2d(xi.astype(np.int64).view(U64), wi.astype(np.int64).view(U64), pad, stride)
    ref = torch.nn.functional.conv2d(torch.from_numpy(xi).double().permute(0, 3, 1, 2),
                                     torch.from_numpy(wi).double().permute(3, 2, 0, 1),
                                     padding=pad, stride=stride).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(oracle.to_signed(got), ref.astype(np.int64))


@pytest.mark.parametrize("case", CONV_CASES)
def test_beaver_conv_reconstructs_conv(case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(8)
    X = synth.rand_words(rng, (B, H, W, Cin)); Wt = synth.rand_words(rng, (KH, KW, Cin, Cout))
    xs, ws = synth.share_additive(rng, X), synth.share_additive(rng, Wt)

    def conv_via_bigint(A, Bf):  # independent of ring_conv2d: im2col + big ints
        col = oracle.im2col(A, KH, KW, pad, stride)
        Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, pad, stride)
        return big_matmul(col, Bf.reshape(-1, Cout)).reshape(B, Ho, Wo, Cout)

    a, b, c = synth.deal_product_triple(rng, X.shape, Wt.shape, conv_via_bigint)
    z = oracle.beaver_conv2d(xs, ws, a, b, c, pad, stride)
    assert np.array_equal(rec(z), conv_via_bigint(X, Wt))


# ------------------------------------------------- backward pass (Sec. 4.1, 4.2, 5.3)
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_gradients_match_torch_autograd(case):
    """Small integers keep float64 exact: autograd's gradients of conv2d are an
    independent definition of both transposed sums."""
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(70)
    xi = rng.integers(-300, 300, size=(B, H, W, Cin)); wi = rng.integers(-300, 300, size=(KH, KW, Cin, Cout))
    xt = torch.from_numpy(xi).double().permute(0, 3, 1, 2).requires_grad_()
    wt = torch.from_numpy(wi).double().permute(3, 2, 0, 1).requires_grad_()
    out = torch.nn.functional.conv2d(xt, wt, padding=pad, stride=stride)
    gi = rng.integers(-300, 300, size=tuple(out.permute(0, 2, 3, 1).shape))
    out.backward(torch.from_numpy(gi).double().permute(0, 3, 1, 2))
    u = lambda v: v.astype(np.int64).view(U64)
    gx = oracle.ring_conv2d_grad_x(u(gi), u(wi), xi.shape, pad, stride)
    gw = oracle.ring_conv2d_grad_w(u(xi), u(gi), KH, KW, pad, stride)
    assert np.array_equal(oracle.to_signed(gx), xt.grad.permute(0, 2, 3, 1).numpy().astype(np.int64))
    assert np.array_equal(oracle.to_signed(gw), wt.grad.permute(2, 3, 1, 0).numpy().astype(np.int64))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_gradients_are_the_adjoints_in_the_ring(case):
    """<Conv(x, w), g> = <x, grad_x(g, w)> = <w, grad_w(x, g)> holds exactly mod 2^64 for
    arbitrary 64-bit words; the forward conv is pinned above."""
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(71)
    x = synth.rand_words(rng, (B, H, W, Cin)); w = synth.rand_words(rng, (KH, KW, Cin, Cout))
    z = oracle.ring_conv2d(x, w, pad, stride)
    g = synth.rand_words(rng, z.shape)
    dot = lambda p, q: int(sum(int(a) * int(b) for a, b in zip(p.ravel(), q.ravel())) % (1 << 64))
    lhs = dot(z, g)
    assert dot(x, oracle.ring_conv2d_grad_x(g, w, x.shape, pad, stride)) == lhs
    assert dot(w, oracle.ring_conv2d_grad_w(x, g, KH, KW, pad, stride)) == lhs


def test_conv_gradients_brute_force_tiny():
    B, H, W, Cin, Cout, KH, KW, pad, stride = 1, 4, 3, 2, 2, 3, 3, 1, 1
    rng = np.random.default_rng(72)
    x = synth.rand_words(rng, (B, H, W, Cin)); w = synth.rand_words(rng, (KH, KW, Cin, Cout))
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, pad, stride)
    g = synth.rand_words(rng, (B, Ho, Wo, Cout))
    gx = np.zeros(x.shape, dtype=object); gw = np.zeros(w.shape, dtype=object)
    for b, ho, wo, kh, kw, ci, co in itertools.product(range(B), range(Ho), range(Wo), range(KH), range(KW),
                                                       range(Cin), range(Cout)):
        hi, wi = ho * stride + kh - pad, wo * stride + kw - pad
        if 0 <= hi < H and 0 <= wi < W:
            gx[b, hi, wi, ci] += int(g[b, ho, wo, co]) * int(w[kh, kw, ci, co])
            gw[kh, kw, ci, co] += int(x[b, hi, wi, ci]) * int(g[b, ho, wo, co])
    mod = np.vectorize(lambda v: v % (1 << 64), otypes=[object])
    assert np.array_equal(oracle.ring_conv2d_grad_x(g, w, x.shape, pad, stride), mod(gx).astype(U64))
    assert np.array_equal(oracle.ring_conv2d_grad_w(x, g, KH, KW, pad, stride), mod(gw).astype(U64))


@pytest.mark.parametrize("case", CONV_CASES[:3])
def test_beaver_bilinear_reconstructs_both_conv_gradients(case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(73)
    X = synth.rand_words(rng, (B, H, W, Cin)); Wt = synth.rand_words(rng, (KH, KW, Cin, Cout))
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, pad, stride)
    G = synth.rand_words(rng, (B, Ho, Wo, Cout))
    xs, ws, gs = (synth.share_additive(rng, v) for v in (X, Wt, G))
    fx = lambda g, w: oracle.ring_conv2d_grad_x(g, w, X.shape, pad, stride)
    fw = lambda x, g: oracle.ring_conv2d_grad_w(x, g, KH, KW, pad, stride)
    a, b, c = synth.deal_product_triple(rng, G.shape, Wt.shape, fx)
    assert np.array_equal(rec(oracle.beaver_bilinear(fx, gs, ws, a, b, c)), fx(G, Wt))
    a, b, c = synth.deal_product_triple(rng, X.shape, G.shape, fw)
    assert np.array_equal(rec(oracle.beaver_bilinear(fw, xs, gs, a, b, c)), fw(X, G))


def test_beaver_bilinear_with_the_matrix_product_is_alg1():
    """With product = ring_matmul the generic form must give the very shares of beaver_matmul."""
    rng = np.random.default_rng(74)
    M, K, N = 5, 7, 3
    xs = synth.share_additive(rng, synth.rand_words(rng, (M, K))); ys = synth.share_additive(rng, synth.rand_words(rng, (K, N)))
    a, b, c = synth.deal_product_triple(rng, (M, K), (K, N), oracle.ring_matmul)
    got = oracle.beaver_bilinear(oracle.ring_matmul, xs, ys, a, b, c)
    want = oracle.beaver_matmul(xs, ys, a, b, c)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])


def test_beaver_mul_elementwise():
    rng = np.random.default_rng(75)
    n = 1000
    X = synth.rand_words(rng, n); Y = synth.rand_words(rng, n)
    xs, ys = synth.share_additive(rng, X), synth.share_additive(rng, Y)
    a, b, c = synth.deal_product_triple(rng, (n,), (n,), lambda p, q: p * q)
    z = oracle.beaver_mul(xs, ys, a, b, c)
    assert np.array_equal(rec(z), X * Y)
    # the literal five terms of Alg. 1, in big integers
    e = [int(v) for v in (xs[0] - a[0]) + (xs[1] - a[1])]; f = [int(v) for v in (ys[0] - b[0]) + (ys[1] - b[1])]
    for i in range(0, n, 97):
        z0 = (int(c[0][i]) + e[i] * int(b[0][i]) + int(a[0][i]) * f[i] + e[i] * f[i]) % (1 << 64)
        z1 = (int(c[1][i]) + e[i] * int(b[1][i]) + int(a[1][i]) * f[i]) % (1 << 64)
        assert (int(z[0][i]), int(z[1][i])) == (z0, z1)


def test_relu_backward_passes_gradient_where_input_positive():
    rng = np.random.default_rng(76)
    n = 2000
    X = synth.normal_fixed(rng, (n,), 1.0); X[:3] = np.array([0, 1, -1], dtype=np.int64).view(U64)
    G = synth.normal_fixed(rng, (n,), 0.5)
    xs, gs = synth.share_additive(rng, X), synth.share_additive(rng, G)
    fwd = oracle.relu(xs, synth.deal_relu_material(rng, n))
    a, b, c = synth.deal_product_triple(rng, (n,), (n,), lambda p, q: p * q)
    gx = oracle.relu_backward(gs, fwd.s_arith, a, b, c)
    want = np.where(oracle.to_signed(X) >= 0, G, U64(0))
    assert np.array_equal(rec(gx), want)



def test_maxpool_backward_routes_gradient_to_the_window_maximum():
    """Against autograd of torch's max_pool2d on integers with a unique maximum per window."""
    rng = np.random.default_rng(77)
    B, H, W, C = 2, 6, 4, 3
    Xi = rng.permutation(B * H * W * C).reshape(B, H, W, C).astype(np.int64) - 70       # all values distinct
    Gi = rng.integers(-1000, 1000, size=(B, H // 2, W // 2, C))
    xs = synth.share_additive(rng, Xi.view(U64)); gs = synth.share_additive(rng, Gi.astype(np.int64).view(U64))
    n_out = Gi.size
    y, s1, s2 = oracle.maxpool2x2(xs, synth.deal_relu_material(rng, 2 * n_out), synth.deal_relu_material(rng, n_out),
                                  want_signs=True)
    mul = lambda p, q: p * q
    t1 = synth.deal_product_triple(rng, (2 * n_out,), (2 * n_out,), mul)
    t2 = synth.deal_product_triple(rng, (n_out,), (n_out,), mul)
    gx = oracle.maxpool2x2_backward(gs, s1, s2, t1, t2, Xi.shape)
    xt = torch.from_numpy(Xi).double().permute(0, 3, 1, 2).requires_grad_()
    torch.nn.functional.max_pool2d(xt, 2).backward(torch.from_numpy(Gi).double().permute(0, 3, 1, 2))
    assert np.array_equal(oracle.to_signed(rec(gx)), xt.grad.permute(0, 2, 3, 1).numpy().astype(np.int64))
    assert np.array_equal(oracle.to_signed(rec(y)), Xi.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4)))

# -------------------------------------------------------------------- truncation
def test_truncation_within_one_lsb_and_wrap_flag():
    rng = np.random.default_rng(9)
    vals = rng.integers(-(1 << 40), 1 << 40, size=20000).astype(np.int64)
    Z = vals.view(U64)
    z = synth.share_additive(rng, Z)
    t = oracle.truncate(z, 16)
    got = oracle.to_signed(rec(t))
    diff = got - (vals >> 16)
    assert not oracle.truncation_wraps(Z, rec(t)).any()   # |z| / 2^64 ~ 2^-24 per element
    assert set(np.unique(diff)) <= {0, 1}
    # closed form for party 0 = z0 >> 16 and party 1 = -((-z1) >> 16)
    assert np.array_equal(t[0], z[0] >> U64(16))
    assert np.array_equal(t[1], (-(((-z[1].astype(object)) % MOD) >> 16)) % MOD)
    # forced wrap: z0 = 0 and a small positive value sitting wholly in party 1
    z0 = np.zeros(4, U64); z1 = np.array([5 << 16, 1 << 20, 3, 1 << 40], dtype=U64)
    t = oracle.truncate((z0, z1), 16)
    assert oracle.truncation_wraps(z0 + z1, rec(t)).all()


def test_truncation_negative_values_floor():
    Z = np.array([-65536, -65537, -1, 65535, 65536], dtype=np.int64).view(U64)
    rng = np.random.default_rng(11)
    for _ in range(20):
        t = oracle.truncate(synth.share_additive(rng, Z), 16)
        d = oracle.to_signed(rec(t)) - np.array([-1, -2, -1, 0, 1])
        assert ((d == 0) | (d == 1)).all()


# -------------------------------------------------------------------- Beaver AND
def test_beaver_and_exhaustive_one_bit():
    """Sec. 3.2 / Alg. 4: all 2^9 one-bit assignments reconstruct X & Y."""
    for x0, x1, y0, y1, a0, a1, b0, b1, c0 in itertools.product((0, 1), repeat=9):
        c1 = ((a0 ^ a1) & (b0 ^ b1)) ^ c0
        t = oracle.beaver_and((x0, x1), (y0, y1), (a0, a1), (b0, b1), (c0, c1))
        assert (t[0] ^ t[1]) == ((x0 ^ x1) & (y0 ^ y1))


def test_beaver_and_words_bitwise():
    rng = np.random.default_rng(12)
    for _ in range(200):
        v = [int(q) for q in synth.rand_words(rng, 9)]
        c1 = ((v[4] ^ v[5]) & (v[6] ^ v[7])) ^ v[8]
        t = oracle.beaver_and(v[0:2], v[2:4], v[4:6], v[6:8], (v[8], c1))
        assert (t[0] ^ t[1]) == ((v[0] ^ v[1]) & (v[2] ^ v[3]))


# ------------------------------------------------------------- prefix adder (A2B)
def _adder_triples(rng, w):
    levels = w.bit_length() - 1
    wm = (1 << w) - 1
    a = [rng.integers(0, 1 << 64, size=2 * levels, dtype=U64) & U64(wm) for _ in range(2)]
    b = [rng.integers(0, 1 << 64, size=2 * levels, dtype=U64) & U64(wm) for _ in range(2)]
    c0 = rng.integers(0, 1 << 64, size=2 * levels, dtype=U64) & U64(wm)
    c1 = ((a[0] ^ a[1]) & (b[0] ^ b[1])) ^ c0
    return a, b, (c0, c1)


def test_adder_exhaustive_width_8():
    """Alg. 2's last step at w = 8: every (U, V) pair, random sharings/triples."""
    rng = np.random.default_rng(13)
    for U in range(256):
        a, b, c = _adder_triples(rng, 8)
        for V in range(256):
            u0 = int(rng.integers(0, 256)); v0 = int(rng.integers(0, 256))
            S = oracle.ks_add((u0, U ^ u0), (v0, V ^ v0), 8, a, b, c)
            assert (S[0] ^ S[1]) == (U + V) % 256, (U, V)


@pytest.mark.parametrize("w", [16, 32, 64])
def test_adder_random_and_carry_corners(w):
    rng = np.random.default_rng(14 + w)
    wm = (1 << w) - 1
    corners = [(wm, 1), (wm >> 1, 1), (0xAAAAAAAAAAAAAAAA & wm, 0x5555555555555555 & wm),
               (0xAAAAAAAAAAAAAAAA & wm, 0xAAAAAAAAAAAAAAAA & wm), (wm, wm), (0, 0),
               (1 << (w - 1), 1 << (w - 1)), ((1 << (w // 2)) - 1, 1)]
    rand = [(int(rng.integers(0, 1 << 64, dtype=U64)) & wm, int(rng.integers(0, 1 << 64, dtype=U64)) & wm)
            for _ in range(300)]
    for U, V in corners + rand:
        a, b, c = _adder_triples(rng, w)
        u0 = int(rng.integers(0, 1 << 64, dtype=U64)) & wm; v0 = int(rng.integers(0, 1 << 64, dtype=U64)) & wm
        S = oracle.ks_add((u0, U ^ u0), (v0, V ^ v0), w, a, b, c)
        assert (S[0] ^ S[1]) == (U + V) & wm, (hex(U), hex(V))


def _carry_outs(U, V):
    """Bit j = carry out of positions [0..j] of U + V, from plain integer addition of the low j + 1 bits."""
    g = 0
    for j in range(64):
        m = (1 << (j + 1)) - 1
        g |= (((U & m) + (V & m)) >> (j + 1)) << j
    return g


def _tree_carries_rec(rng, U, V):
    """Reconstructed carry word of the oracle's share-level prefix tree, random sharing and triples."""
    a, b, c = _adder_triples(rng, 64)
    u0, v0 = int(rng.integers(0, 1 << 64, dtype=U64)), int(rng.integers(0, 1 << 64, dtype=U64))
    G = oracle.tree_carries((u0, U ^ u0), (v0, V ^ v0), a, b, c)
    return G[0] ^ G[1]


def test_listing_tree_carries_are_the_integer_carries_exhaustive_bytes():
    """Every pair of 8-bit operands, placed at bit offsets that exercise every level of the tree
    (0: levels 0-2 only; 28 and 29: straddling the 32-bit join; 56: top byte), with the surrounding
    bits all-propagate or zero: the tree's carries are those of integer addition, position by position."""
    rng = np.random.default_rng(15)
    M64 = MOD - 1
    for off, fill in ((0, 0), (28, 0), (29, M64), (56, M64)):
        keep = M64 ^ (0xFF << off)
        for u in range(256):
            for v in range(0, 256, 1 if off == 0 else 5):
                U = ((u << off) | (fill & keep)) & M64
                V = (v << off) & M64
                assert _tree_carries_rec(rng, U, V) == _carry_outs(U, V), (off, u, v)


def test_listing_tree_carries_sixteen_bit_sweep_and_64_bit_corners():
    rng = np.random.default_rng(16)
    M64 = MOD - 1
    # a 16-bit sweep: all u in steps that hit every low pattern, v from a coprime stride, at two offsets
    for off in (0, 40):
        for u in range(0, 1 << 16, 97):
            v = (u * 40503 + 12345) & 0xFFFF
            U, V = (u << off) & M64, (v << off) & M64
            assert _tree_carries_rec(rng, U, V) == _carry_outs(U, V)
    corners = [(M64, 1), (M64 >> 1, 1), (0, 0), (M64, M64), (1 << 63, 1 << 63), (M64, 0),
               (0xAAAAAAAAAAAAAAAA, 0x5555555555555555), (0xAAAAAAAAAAAAAAAA, 0xAAAAAAAAAAAAAAAA),
               (0x5555555555555555, 0x5555555555555555), ((1 << 32) - 1, 1), ((1 << 31), (1 << 31)),
               (0x00000000FFFFFFFF, 0xFFFFFFFF00000001)] + \
              [((1 << k) - 1, 1) for k in range(1, 65)] + [(M64 ^ (1 << k), 1) for k in range(64)]
    rand = [(int(q), int(p)) for q, p in zip(synth.rand_words(rng, 500), synth.rand_words(rng, 500))]
    for U, V in corners + rand:
        U &= M64; V &= M64
        got = _tree_carries_rec(rng, U, V)
        assert got == _carry_outs(U, V), (hex(U), hex(V))
        # and hence the Kogge-Stone network's sum
        a, b, c = _adder_triples(rng, 64)
        S = oracle.ks_add((5, U ^ 5), (9, V ^ 9), 64, a, b, c)
        assert (S[0] ^ S[1]) == (U ^ V ^ ((got << 1) & M64))


def test_tree_adder_gate_wiring_bit_by_bit():
    """Which gate reads which bit and which triple bit: a prefix tree written on bit lists with index
    arithmetic only (position j of an upper half-block at level i combines with position
    (j >> i << i) - 1, the top of the lower half; all other positions enter the gate as zeros), every
    gate a one-bit Beaver AND that takes bit j of triple word 1 + 2i (carry update) / 2 + 2i (propagate
    update).  Carry shares must agree with the
    oracle's word-level tree for both parties."""
    rng = np.random.default_rng(17)

    def and1(p, q, a, b, c, t, j):
        """One-bit Beaver AND at bit j of triple t, on share pairs of bits."""
        bit = lambda w: (int(w) >> j) & 1
        o = oracle.beaver_and(p, q, (bit(a[0][t]), bit(a[1][t])), (bit(b[0][t]), bit(b[1][t])), (bit(c[0][t]), bit(c[1][t])))
        return (int(o[0]) & 1, int(o[1]) & 1)

    for _ in range(40):
        U, V = int(rng.integers(0, 1 << 64, dtype=U64)), int(rng.integers(0, 1 << 64, dtype=U64))
        u0, v0 = int(rng.integers(0, 1 << 64, dtype=U64)), int(rng.integers(0, 1 << 64, dtype=U64))
        a, b, c = _adder_triples(rng, 64)
        Us, Vs = (u0, U ^ u0), (v0, V ^ v0)
        got = oracle.tree_carries(Us, Vs, a, b, c)
        ub = [((Us[0] >> j) & 1, (Us[1] >> j) & 1) for j in range(64)]
        vb = [((Vs[0] >> j) & 1, (Vs[1] >> j) & 1) for j in range(64)]
        P = [(ub[j][0] ^ vb[j][0], ub[j][1] ^ vb[j][1]) for j in range(64)]
        G = [and1(ub[j], vb[j], a, b, c, 0, j) for j in range(64)]
        for i in range(6):
            Gn, Pn = list(G), list(P)
            for j in range(64):
                # the AND is a word operation: positions outside the upper halves enter it as shared zeros
                # (their gate output is a sharing of zero that still re-randomises the share bits)
                upper = (j >> i) & 1
                src = ((j >> i) << i) - 1
                x = P[j] if upper else (0, 0)
                t = and1(x, G[src] if upper else (0, 0), a, b, c, 1 + 2 * i, j)
                Gn[j] = (G[j][0] ^ t[0], G[j][1] ^ t[1])
                if i < 5:
                    q = and1(x, P[src] if upper else (0, 0), a, b, c, 2 + 2 * i, j)
                    Pn[j] = q if upper else (P[j][0] ^ q[0], P[j][1] ^ q[1])
            G, P = Gn, Pn
        want = tuple(sum(G[j][k] << j for j in range(64)) for k in range(2))
        assert got == want
        assert (got[0] ^ got[1]) == _carry_outs(U, V)


def test_relu_with_the_listing_tree():
    """Same reconstructed sign as with the Kogge-Stone network from different sign-bit
    shares; everything after the B2A opening depends on the opened value only, so the
    arithmetic sign shares and the outputs are the same words."""
    rng = np.random.default_rng(19)
    vals = np.concatenate([np.arange(-2048, 2049), rng.integers(-(1 << 62), 1 << 62, size=2000)]).astype(np.int64)
    X = vals.view(U64)
    xs = synth.share_additive(rng, X)
    mat = synth.deal_relu_material(rng, X.size)
    ks, tree = oracle.relu(xs, mat), oracle.relu(xs, mat, adder="tree")
    assert np.array_equal(rec(tree.y), np.maximum(vals, 0).view(U64))
    assert np.array_equal(tree.s_bit[0] ^ tree.s_bit[1], (vals < 0).astype(np.uint8))
    assert np.array_equal(rec(tree.s_arith), (vals < 0).astype(U64))
    assert np.array_equal(tree.y[0], ks.y[0]) and np.array_equal(tree.s_arith[1], ks.s_arith[1])
    assert not np.array_equal(tree.s_bit[0], ks.s_bit[0])


# --------------------------------------------------------------------------- B2A
def test_b2a_exhaustive():
    rng = np.random.default_rng(17)
    for s0, s1, rb0, rb1 in itertools.product((0, 1), repeat=4):
        for _ in range(8):
            ra0 = int(rng.integers(0, 1 << 64, dtype=U64)); ra1 = ((rb0 ^ rb1) - ra0) % MOD
            o = oracle.b2a((s0, s1), (rb0, rb1), (ra0, ra1))
            assert (o[0] + o[1]) % MOD == (s0 ^ s1)


# -------------------------------------------------------------------------- ReLU
def _relu_check(xvals, x0=None, seed=18):
    rng = np.random.default_rng(seed)
    X = np.asarray(xvals, dtype=np.int64).view(U64)
    if x0 is None:
        xs = synth.share_additive(rng, X)
    else:
        x0 = np.full(X.shape, x0, dtype=U64); xs = (x0, X - x0)
    res = oracle.relu(xs, synth.deal_relu_material(rng, X.size))
    want = np.maximum(X.view(np.int64), 0).view(U64)
    assert np.array_equal(rec(res.y), want)
    sign = (X.view(np.int64) < 0)
    assert np.array_equal((res.s_bit[0] ^ res.s_bit[1]).astype(bool), sign)
    assert np.array_equal(rec(res.s_arith), sign.astype(U64))
    return res


def test_relu_exhaustive_small_magnitude():
    _relu_check(np.arange(-4096, 4097))


@pytest.mark.parametrize("x0", [0, 1 << 63, MOD - 1, 1, (1 << 63) - 1])
def test_relu_adversarial_share_patterns(x0):
    _relu_check(np.arange(-4096, 4097), x0=x0)


def test_relu_powers_of_two_edges():
    vals = []
    for k in range(63):
        for s in (1, -1):
            for d in (-1, 0, 1):
                vals.append(s * (1 << k) + d)
    vals += [-(1 << 63), (1 << 63) - 1, 0]
    _relu_check(np.array(vals, dtype=np.int64))
    for x0 in (0, 1 << 63, MOD - 1):
        _relu_check(np.array(vals, dtype=np.int64), x0=x0)


def test_relu_trivial_a2b_masks():
    """r = 0 is a legal (if insecure) A2B sharing: (x_0, 0) and (0, x_1)."""
    rng = np.random.default_rng(19)
    X = rng.integers(-(1 << 62), 1 << 62, size=1000).astype(np.int64).view(U64)
    xs = synth.share_additive(rng, X)
    mat = synth.deal_relu_material(rng, X.size)
    mat["r"] = (np.zeros(X.size, U64), np.zeros(X.size, U64))
    assert np.array_equal(rec(oracle.relu(xs, mat).y), np.maximum(X.view(np.int64), 0).view(U64))


def test_relu_material_index_sensitivity():
    """Each of the 12 AND triples is consumed: corrupting c of any one of them
    (at a bit that can reach bit 63) changes some sign."""
    rng = np.random.default_rng(20)
    X = rng.integers(-(1 << 62), 1 << 62, size=4000).astype(np.int64).view(U64)
    xs = synth.share_additive(rng, X)
    mat = synth.deal_relu_material(rng, X.size)
    base = oracle.relu(xs, mat)
    for t in range(12):
        bad = dict(mat)
        c0 = mat["and_c"][0].copy(); c0[t] ^= U64(MOD - 1)
        bad["and_c"] = (c0, mat["and_c"][1])
        out = oracle.relu(xs, bad)
        assert not np.array_equal(out.s_bit[0] ^ out.s_bit[1], base.s_bit[0] ^ base.s_bit[1]), t


# ---------------------------------------------------------------------- max-pool
def test_maxpool_by_composition():
    rng = np.random.default_rng(21)
    B, H, W, C = 2, 6, 4, 3
    X = rng.integers(-(1 << 30), 1 << 30, size=(B, H, W, C)).astype(np.int64)
    xs = synth.share_additive(rng, X.view(U64))
    n_out = B * (H // 2) * (W // 2) * C
    out = oracle.maxpool2x2(xs, synth.deal_relu_material(rng, 2 * n_out), synth.deal_relu_material(rng, n_out))
    want = X.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4))
    assert np.array_equal(oracle.to_signed(rec(out)), want)


def test_relu_and_maxpool_commute():
    """ReLU is monotone, so ReLU(max window) = max window of ReLU: a runner may pool first and
    convert a quarter of the elements.  Both orders are exact, so the reconstructions are equal."""
    rng = np.random.default_rng(22)
    B, H, W, C = 2, 4, 6, 3
    X = rng.integers(-(1 << 30), 1 << 30, size=(B, H, W, C)).astype(np.int64)
    X[0, :2, :2, 0] = -5                     # an all-negative window: both orders give 0
    xs = synth.share_additive(rng, X.view(U64))
    n, n_out = X.size, X.size // 4
    deal = lambda k: synth.deal_relu_material(rng, k)
    relu_then_pool = oracle.maxpool2x2(oracle.relu(xs, deal(n)).y, deal(2 * n_out), deal(n_out))
    pooled = oracle.maxpool2x2(xs, deal(2 * n_out), deal(n_out))
    pool_then_relu = oracle.relu(pooled, deal(n_out)).y
    want = np.maximum(X.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4)), 0)
    assert np.array_equal(oracle.to_signed(rec(relu_then_pool)), want)
    assert np.array_equal(oracle.to_signed(rec(pool_then_relu)).reshape(want.shape), want)
    assert want[0, 0, 0, 0] == 0


# ------------------------------------------------------- fixed point vs float64
def test_tiny_layer_float64_agreement():
    """Config 0 end to end on the oracle: decoded output within 2^-12 of the
    float64 product of the decoded (quantised) inputs; ReLU exact."""
    wl = synth.config_tiny(); g = wl.layers[0]
    rng = synth.rng_for(wl.index)
    X = synth.normal_fixed(rng, (g.M, g.K), g.x_std); Wt = synth.normal_fixed(rng, (g.K, g.N), g.w_std)
    xs, ws = synth.share_additive(rng, X), synth.share_additive(rng, Wt)
    a, b, c = synth.deal_product_triple(rng, X.shape, Wt.shape, lambda A, B: A @ B)
    z = oracle.beaver_matmul(xs, ws, a, b, c)
    t = oracle.truncate(z, 16)
    assert not oracle.truncation_wraps(rec(z), rec(t)).any()
    ref = oracle.decode(X) @ oracle.decode(Wt)
    assert np.abs(oracle.decode(rec(t)) - ref).max() <= 2.0 ** -12
    res = oracle.relu(t, synth.deal_relu_material(rng, g.M * g.N))
    assert np.array_equal(oracle.to_signed(rec(res.y)), np.maximum(oracle.to_signed(rec(t)), 0))
