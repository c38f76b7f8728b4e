"""Pins for the three-party forms of the CPU oracle (Alg. 1 and Alg. 2 for N = 3;
Sec. 3.3, Sec. 5.6).  No GPU: the oracle is compared with Python big-int
arithmetic, exhaustive enumeration, closed forms and the (separately pinned)
two-party oracle on inputs where the third party holds nothing."""
import numpy as np
import pytest

import oracle
from paper_2209_13643_amd import synth

U64 = np.uint64
MOD = 1 << 64
M64 = MOD - 1


def rec3(t):
    return np.asarray(t[0], dtype=U64) + np.asarray(t[1], dtype=U64) + np.asarray(t[2], dtype=U64)


def xor3(t):
    return np.asarray(t[0]) ^ np.asarray(t[1]) ^ np.asarray(t[2])


def big_matmul(L, R):
    L = [[int(v) for v in row] for row in L]
    R = [[int(v) for v in row] for row in R]
    return np.array([[sum(L[m][k] * R[k][n] for k in range(len(R))) % MOD
                      for n in range(len(R[0]))] for m in range(len(L))], dtype=U64)


def deal_matmul3(rng, M, K, N):
    X = synth.rand_words(rng, (M, K)); Y = synth.rand_words(rng, (K, N))
    xs, ys = synth.share_additive3(rng, X), synth.share_additive3(rng, Y)
    a, b, c = synth.deal_product_triple3(rng, (M, K), (K, N), lambda A, B: A @ B)
    return X, Y, xs, ys, a, b, c


# --------------------------------------------------------------------- Alg. 1
def test_open3_is_the_sum():
    s = ([1, M64, 5], [2, 1, M64 - 4], [3, 0, 7])
    assert oracle.open3([np.array(v, dtype=U64) for v in s]).tolist() == [6, 0, 7]


@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 2), (3, 1, 4), (9, 17, 5)])
def test_beaver_matmul3_reconstructs_product(shape):
    """Sec. 3.2: the sum of the [z_i] is X*Y, for any number of parties."""
    M, K, N = shape
    rng = np.random.default_rng(31)
    X, Y, xs, ys, a, b, c = deal_matmul3(rng, M, K, N)
    z = oracle.beaver_matmul3(xs, ys, a, b, c)
    assert np.array_equal(rec3(z), big_matmul(X, Y))
    # no party's output is the product by itself
    assert not np.array_equal(z[0], big_matmul(X, Y))


def test_beaver_matmul3_is_independent_of_the_triple_and_the_sharing():
    rng = np.random.default_rng(32)
    X, Y, xs, ys, a, b, c = deal_matmul3(rng, 6, 11, 4)
    z1 = oracle.beaver_matmul3(xs, ys, a, b, c)
    xs2, ys2 = synth.share_additive3(rng, X), synth.share_additive3(rng, Y)
    a2, b2, c2 = synth.deal_product_triple3(rng, (6, 11), (11, 4), lambda A, B: A @ B)
    z2 = oracle.beaver_matmul3(xs2, ys2, a2, b2, c2)
    assert np.array_equal(rec3(z1), rec3(z2)) and not np.array_equal(z1[0], z2[0])


def test_beaver_matmul3_zero_triple_degenerates():
    """With A = B = C = 0 the opened values are X, Y themselves: party 0 ends with X*Y, the others with 0."""
    rng = np.random.default_rng(33)
    X = synth.rand_words(rng, (4, 5)); Y = synth.rand_words(rng, (5, 3))
    xs, ys = synth.share_additive3(rng, X), synth.share_additive3(rng, Y)
    zero = lambda shp: tuple(np.zeros(shp, dtype=U64) for _ in range(3))
    z = oracle.beaver_matmul3(xs, ys, zero((4, 5)), zero((5, 3)), zero((4, 3)))
    assert np.array_equal(z[0], big_matmul(X, Y)) and not z[1].any() and not z[2].any()


def test_beaver_matmul3_with_an_empty_third_party_is_the_two_party_protocol():
    """Party 2 holding zeros everywhere: parties 0 and 1 compute exactly Alg. 1 for two."""
    rng = np.random.default_rng(34)
    M, K, N = 7, 13, 5
    X = synth.rand_words(rng, (M, K)); Y = synth.rand_words(rng, (K, N))
    xs, ys = synth.share_additive(rng, X), synth.share_additive(rng, Y)
    a, b, c = synth.deal_product_triple(rng, (M, K), (K, N), lambda A, B: A @ B)
    z2 = oracle.beaver_matmul(xs, ys, a, b, c)
    pad = lambda pair, shp: (pair[0], pair[1], np.zeros(shp, dtype=U64))
    z3 = oracle.beaver_matmul3(pad(xs, (M, K)), pad(ys, (K, N)), pad(a, (M, K)), pad(b, (K, N)), pad(c, (M, N)))
    assert np.array_equal(z3[0], z2[0]) and np.array_equal(z3[1], z2[1]) and not z3[2].any()


@pytest.mark.parametrize("case", [(1, 4, 4, 2, 3, 3, 3, 1, 1), (2, 5, 6, 3, 4, 3, 3, 0, 2), (1, 3, 3, 1, 1, 1, 1, 0, 1)])
def test_beaver_conv2d3_reconstructs_the_convolution(case):
    """Eq. 3: Alg. 1 with Conv as the product; checked against the plain ring convolution of the clear values."""
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    rng = np.random.default_rng(35)
    X = synth.rand_words(rng, (B, H, W, Cin)); Wt = synth.rand_words(rng, (KH, KW, Cin, Cout))
    conv = lambda A, Bm: oracle.ring_conv2d(A, Bm, pad, stride)
    xs, ws = synth.share_additive3(rng, X), synth.share_additive3(rng, Wt)
    a, b, c = synth.deal_product_triple3(rng, X.shape, Wt.shape, conv)
    z = oracle.beaver_conv2d3(xs, ws, a, b, c, pad, stride)
    assert np.array_equal(rec3(z), conv(X, Wt))
    # third party empty: the two-party protocol
    xs2, ws2 = synth.share_additive(rng, X), synth.share_additive(rng, Wt)
    a2, b2, c2 = synth.deal_product_triple(rng, X.shape, Wt.shape, conv)
    z2 = oracle.beaver_conv2d(xs2, ws2, a2, b2, c2, pad, stride)
    pad3 = lambda pair: (pair[0], pair[1], np.zeros_like(pair[0]))
    z3 = oracle.beaver_conv2d3(pad3(xs2), pad3(ws2), pad3(a2), pad3(b2), pad3(c2), pad, stride)
    assert np.array_equal(z3[0], z2[0]) and np.array_equal(z3[1], z2[1]) and not z3[2].any()


def test_beaver_mul3_elementwise():
    rng = np.random.default_rng(36)
    n = 50
    X = synth.rand_words(rng, n); Y = synth.rand_words(rng, n)
    a, b, c = synth.deal_product_triple3(rng, n, n, lambda A, B: A * B)
    z = oracle.beaver_mul3(synth.share_additive3(rng, X), synth.share_additive3(rng, Y), a, b, c)
    want = [(int(p) * int(q)) % MOD for p, q in zip(X, Y)]
    assert [int(v) for v in rec3(z)] == want


# ----------------------------------------------------------------- truncation
def test_truncate3_is_floor_plus_the_low_carry():
    """m = z + 2^62 + r never wraps for z in [-2^62, 2^62), r < 2^63, so the result is
    floor(z / 2^bits) plus the carry of the two low parts: computed here with Python integers."""
    rng = np.random.default_rng(37)
    bits = 16
    zs = [0, 1, -1, 65535, 65536, -65536, -65537, (1 << 62) - 1, -(1 << 62), 12345678901234, -98765432109876]
    zs += [int(v) for v in rng.integers(-(1 << 61), 1 << 61, size=200)]
    zs += [int(v) for v in rng.integers(-(1 << 34), 1 << 34, size=200)]
    n = len(zs)
    rs = [0, (1 << 63) - 1, 65535, 65536] + [int(v) for v in rng.integers(0, 1 << 63, size=n - 4, dtype=U64)]
    Z = np.array([v % MOD for v in zs], dtype=U64); R = np.array(rs, dtype=U64)
    z = synth.share_additive3(rng, Z)
    r = synth.share_additive3(rng, R); rt = synth.share_additive3(rng, R >> U64(bits))
    t = oracle.truncate3(z, r, rt, bits)
    got = [int(v) for v in rec3(t).view(np.int64)]
    for zi, ri, g in zip(zs, rs, got):
        carry = (((zi + (1 << 62)) % (1 << bits)) + (ri % (1 << bits))) >> bits
        assert g == (zi >> bits) + carry, (zi, ri, g)
    # parties 1 and 2 only negate their share of r >> bits
    assert np.array_equal(t[1], (~rt[1]) + U64(1)) and np.array_equal(t[2], (~rt[2]) + U64(1))


def test_matmul3_then_truncate3_agrees_with_float64():
    rng = np.random.default_rng(38)
    M, K, N = 12, 40, 9
    xf = rng.standard_normal((M, K)); wf = rng.standard_normal((K, N)) * 0.2
    X, Wt = synth.encode_fixed(xf), synth.encode_fixed(wf)
    a, b, c = synth.deal_product_triple3(rng, (M, K), (K, N), lambda A, B: A @ B)
    z = oracle.beaver_matmul3(synth.share_additive3(rng, X), synth.share_additive3(rng, Wt), a, b, c)
    r, rt = synth.deal_trunc3_pair(rng, (M, N))
    t = oracle.truncate3(z, r, rt)
    want = oracle.decode(X) @ oracle.decode(Wt)
    assert np.abs(oracle.decode(rec3(t)) - want).max() <= 2.0 ** -12


# ----------------------------------------------------------- binary primitives
def test_beaver_and3_exhaustive_one_bit():
    """All 2^14 assignments of (x_0..2, y_0..2, a_0..2, b_0..2, c_0, c_1), 64 per word; c_2 completes c = a & b."""
    for word in range(256):
        ids = [word * 64 + k for k in range(64)]
        var = lambda j: sum(((i >> j) & 1) << k for k, i in enumerate(ids))
        X = [var(0), var(1), var(2)]; Y = [var(3), var(4), var(5)]
        a = [var(6), var(7), var(8)]; b = [var(9), var(10), var(11)]
        c01 = [var(12), var(13)]
        c = c01 + [((a[0] ^ a[1] ^ a[2]) & (b[0] ^ b[1] ^ b[2])) ^ c01[0] ^ c01[1]]
        out = oracle.beaver_and3(X, Y, a, b, c)
        assert out[0] ^ out[1] ^ out[2] == (X[0] ^ X[1] ^ X[2]) & (Y[0] ^ Y[1] ^ Y[2])


def _xor_share_int(rng, v, w):
    m = (1 << w) - 1
    s0 = int(rng.integers(0, 1 << 63)) & m; s1 = int(rng.integers(0, 1 << 63)) & m
    return [s0, s1, (v ^ s0 ^ s1) & m]


def _triples(rng, w):
    levels = w.bit_length() - 1
    cnt = 1 + 2 * levels
    wm = U64((1 << w) - 1) if w < 64 else U64(M64)
    A = synth.rand_words(rng, cnt) & wm; B = synth.rand_words(rng, cnt) & wm
    sh = lambda V: np.stack([s & wm for s in synth.share_xor3(rng, V)], axis=1)      # [cnt][3]
    return sh(A), sh(B), sh(A & B)


def test_add3_exhaustive_width_4():
    """Carry-save step + prefix network at width 4: every (u, v, w), fresh sharings and triples each time."""
    rng = np.random.default_rng(39)
    for u in range(16):
        for v in range(16):
            for w in range(16):
                ta, tb, tc = _triples(rng, 4)
                S = oracle.add3(_xor_share_int(rng, u, 4), _xor_share_int(rng, v, 4), _xor_share_int(rng, w, 4),
                                4, ta, tb, tc)
                assert S[0] ^ S[1] ^ S[2] == (u + v + w) % 16, (u, v, w)


@pytest.mark.parametrize("w", [8, 16, 32, 64])
def test_add3_random_and_carry_corners(w):
    rng = np.random.default_rng(40 + w)
    m = (1 << w) - 1
    cases = [(m, m, m), (m, 1, 0), (m, 0, 1), (m >> 1, 1, 0), (m >> 1, m >> 1, 2), (0, 0, 0), (1, 1, 1),
             (0x5555555555555555 & m, 0xAAAAAAAAAAAAAAAA & m, 1), (m, m, 1), (1 << (w - 1), 1 << (w - 1), 0)]
    cases += [tuple(int(x) & m for x in rng.integers(0, 1 << 63, size=3)) for _ in range(300)]
    if w == 64:
        cases += [tuple(int(x) for x in synth.rand_words(rng, 3)) for _ in range(300)]
    for u, v, x in cases:
        ta, tb, tc = _triples(rng, w)
        S = oracle.add3(_xor_share_int(rng, u, w), _xor_share_int(rng, v, w), _xor_share_int(rng, x, w), w, ta, tb, tc)
        assert S[0] ^ S[1] ^ S[2] == (u + v + x) & m, (u, v, x)


def test_b2a3_exhaustive():
    rng = np.random.default_rng(41)
    for bits in range(64):
        s = [(bits >> k) & 1 for k in range(3)]; rb = [(bits >> (3 + k)) & 1 for k in range(3)]
        for _ in range(4):
            ra0, ra1 = (int(v) for v in synth.rand_words(rng, 2))
            ra = [ra0, ra1, ((rb[0] ^ rb[1] ^ rb[2]) - ra0 - ra1) % MOD]
            out = oracle.b2a3(s, rb, ra)
            assert sum(out) % MOD == s[0] ^ s[1] ^ s[2]


# ----------------------------------------------------------------------- ReLU
def _relu3_check(x_signed, shares, rng):
    n = len(x_signed)
    mat = synth.deal_relu3_material(rng, n)
    res = oracle.relu3(shares, mat)
    want = np.maximum(np.array(x_signed, dtype=np.int64), 0)
    neg = (np.array(x_signed, dtype=np.int64) < 0)
    assert np.array_equal(rec3(res.y).view(np.int64), want)
    assert np.array_equal(xor3(res.s_bit), neg.astype(np.uint8))
    assert np.array_equal(rec3(res.s_arith), neg.astype(U64))
    return res


def test_relu3_exhaustive_small_magnitude_and_powers_of_two():
    rng = np.random.default_rng(42)
    xs = list(range(-4096, 4097))
    for k in range(63):
        for d in (-1, 0, 1):
            xs += [(1 << k) + d, -(1 << k) + d]
    xs += [-(1 << 63), (1 << 63) - 1]
    X = np.array([v % MOD for v in xs], dtype=U64)
    signed = X.view(np.int64).tolist()
    _relu3_check(signed, synth.share_additive3(rng, X), rng)
    # adversarial sharings: one or two shares pinned to 0, 2^63, 2^64 - 1
    for s0 in (0, 1 << 63, M64):
        for s1 in (0, 1 << 63, M64):
            a = np.full(X.shape, s0, dtype=U64); b = np.full(X.shape, s1, dtype=U64)
            _relu3_check(signed, (a, b, X - a - b), rng)
            _relu3_check(signed, (X - a - b, a, b), rng)


def test_relu3_random_words_and_material_independence():
    rng = np.random.default_rng(43)
    X = synth.rand_words(rng, 5000)
    shares = synth.share_additive3(rng, X)
    r1 = _relu3_check(X.view(np.int64).tolist(), shares, rng)
    r2 = _relu3_check(X.view(np.int64).tolist(), shares, rng)         # fresh material, same inputs
    assert not np.array_equal(r1.y[0], r2.y[0])
    # trivial A2B masks (party j keeps its word, sends zeros) are a valid special case
    mat = synth.deal_relu3_material(rng, X.size)
    mat["r0"] = tuple(np.zeros(X.size, dtype=U64) for _ in range(3)); mat["r1"] = mat["r0"]
    res = oracle.relu3(shares, mat)
    assert np.array_equal(rec3(res.y).view(np.int64), np.maximum(X.view(np.int64), 0))


def test_relu3_uses_every_triple():
    """A corrupted c word of any one of the 13 triples must change some reconstructed sign:
    the chain consumes all of them (carry patterns that exercise every level)."""
    rng = np.random.default_rng(44)
    n = 4096
    X = synth.rand_words(rng, n)
    # long carry chains: x = 2^k - 1 + (shares chosen at random) makes every level matter
    shares = synth.share_additive3(rng, X)
    mat = synth.deal_relu3_material(rng, n)
    base = xor3(oracle.relu3(shares, mat).s_bit)
    for t in range(13):
        bad = dict(mat)
        c0 = np.array(mat["and_c"][0], copy=True); c0[t] ^= U64(M64)
        bad["and_c"] = (c0, mat["and_c"][1], mat["and_c"][2])
        assert not np.array_equal(xor3(oracle.relu3(shares, bad).s_bit), base), t


def test_maxpool3_is_the_window_maximum():
    """max over 2x2 windows on reconstructed values, plain numpy as the reference; ties and negatives included."""
    rng = np.random.default_rng(45)
    B, H, W, C = 2, 6, 4, 3
    X = synth.normal_fixed(rng, (B, H, W, C), 3.0)
    X[0, 0:2, 0:2, 0] = X[0, 0, 0, 0]                      # a window of equal values
    n_out = B * (H // 2) * (W // 2) * C
    y = oracle.maxpool2x2_3(synth.share_additive3(rng, X), synth.deal_relu3_material(rng, 2 * n_out),
                            synth.deal_relu3_material(rng, n_out))
    want = X.view(np.int64).reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4))
    assert np.array_equal(rec3(y).view(np.int64), want)


# --------------------------------------------------------------- backward pass
def test_beaver_bilinear3_reconstructs_the_gradient_products():
    """Alg. 1 with the two gradient maps of a convolution in place of the product: the three
    shares reconstruct to the plain ring gradient, whatever the triple and the sharing."""
    rng = np.random.default_rng(501)
    B, H, W, Cin, Cout, KH, pad, stride = 2, 6, 5, 3, 4, 3, 1, 2
    X = synth.rand_words(rng, (B, H, W, Cin)); Wt = synth.rand_words(rng, (KH, KH, Cin, Cout))
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KH, pad, stride)
    G = synth.rand_words(rng, (B, Ho, Wo, Cout))
    gx_map = lambda g, w: oracle.ring_conv2d_grad_x(g, w, X.shape, pad, stride)
    gw_map = lambda x, g: oracle.ring_conv2d_grad_w(x, g, KH, KH, pad, stride)
    for trial in range(2):
        gs, ws, xs = (synth.share_additive3(rng, v) for v in (G, Wt, X))
        a, b, c = synth.deal_product_triple3(rng, G.shape, Wt.shape, gx_map)
        assert np.array_equal(rec3(oracle.beaver_bilinear3(gx_map, gs, ws, a, b, c)), gx_map(G, Wt))
        a, b, c = synth.deal_product_triple3(rng, X.shape, G.shape, gw_map)
        assert np.array_equal(rec3(oracle.beaver_bilinear3(gw_map, xs, gs, a, b, c)), gw_map(X, G))
    # with an empty third party it is the two-party composition word for word
    z2 = lambda n: np.zeros(n, dtype=U64)
    g2, w2 = synth.share_additive(rng, G), synth.share_additive(rng, Wt)
    a2, b2, c2 = synth.deal_product_triple(rng, G.shape, Wt.shape, gx_map)
    want = oracle.beaver_bilinear(gx_map, g2, w2, a2, b2, c2)
    pad3 = lambda pair: (pair[0], pair[1], z2(np.shape(pair[0])))
    got = oracle.beaver_bilinear3(gx_map, pad3(g2), pad3(w2), pad3(a2), pad3(b2), pad3(c2))
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]) and not got[2].any()


def test_relu_backward3_is_gradient_times_the_input_mask():
    rng = np.random.default_rng(502)
    n = 300
    X = rng.integers(-(1 << 20), 1 << 20, size=n).astype(np.int64); X[:3] = (0, -1, 1)
    G = rng.integers(-(1 << 30), 1 << 30, size=n).astype(np.int64)
    fwd = oracle.relu3(synth.share_additive3(rng, X.view(U64)), synth.deal_relu3_material(rng, n))
    t = synth.deal_product_triple3(rng, (n,), (n,), lambda p, q: p * q)
    gx = oracle.relu_backward3(synth.share_additive3(rng, G.view(U64)), fwd.s_arith, *t)
    assert np.array_equal(oracle.to_signed(rec3(gx)), np.where(X >= 0, G, 0))


def test_maxpool_backward3_routes_gradient_to_the_window_maximum():
    """Against autograd of torch's max_pool2d on integers with a unique maximum per window."""
    import torch
    rng = np.random.default_rng(503)
    B, H, W, C = 2, 4, 6, 3
    Xi = rng.permutation(B * H * W * C).reshape(B, H, W, C).astype(np.int64) - 70
    Gi = rng.integers(-1000, 1000, size=(B, H // 2, W // 2, C)).astype(np.int64)
    xs = synth.share_additive3(rng, Xi.view(U64)); gs = synth.share_additive3(rng, Gi.view(U64))
    n_out = Gi.size
    y, s1, s2 = oracle.maxpool2x2_3(xs, synth.deal_relu3_material(rng, 2 * n_out), synth.deal_relu3_material(rng, n_out),
                                    want_signs=True)
    mul = lambda p, q: p * q
    t1 = synth.deal_product_triple3(rng, (2 * n_out,), (2 * n_out,), mul)
    t2 = synth.deal_product_triple3(rng, (n_out,), (n_out,), mul)
    gx = oracle.maxpool2x2_backward3(gs, s1, s2, t1, t2, Xi.shape)
    xt = torch.from_numpy(Xi).double().permute(0, 3, 1, 2).requires_grad_()
    torch.nn.functional.max_pool2d(xt, 2).backward(torch.from_numpy(Gi).double().permute(0, 3, 1, 2))
    assert np.array_equal(oracle.to_signed(rec3(gx)), xt.grad.permute(0, 2, 3, 1).numpy().astype(np.int64))
    assert np.array_equal(oracle.to_signed(rec3(y)), Xi.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4)))
    # the sign shares reconstruct to 0 / 1
    assert set(np.unique(rec3(s1))) <= {0, 1} and set(np.unique(rec3(s2))) <= {0, 1}
