"""Seeded sweeps over ragged shapes: many small random geometries for every product the
library offers, each against the oracle bit for bit (tails in M, K, N, channels, strides,
paddings, batches; chunked and pre-opened variants picked at random)."""
import numpy as np
import pytest

import oracle
from helpers import deal_conv, deal_matmul, oracle_conv, oracle_matmul
from paper_2209_13643_amd import synth

pytestmark = pytest.mark.gpu
U64 = np.uint64


@pytest.fixture(scope="module")
def mpc():
    from paper_2209_13643_amd import mpc as m
    return m


@pytest.fixture(params=["three-streams", "single-queue"])
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
        assert np.array_equal(g, want[i]), f"{what}: party {i} differs in {(g != want[i]).sum()} of {g.size} words"


def test_random_matmul_shapes(mpc, lane):
    rng = np.random.default_rng(2024)
    for it in range(40):
        M, K, N = (int(rng.integers(1, 200)), int(rng.integers(1, 300)), int(rng.integers(1, 200)))
        batch = None if rng.integers(0, 3) else int(rng.integers(2, 5))
        print(f"random matmul {it}: {M}x{K}x{N} batch {batch}", flush=True)
        d = deal_matmul(rng, M, K, N, batch=batch)
        args = [dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c")]
        trunc = bool(rng.integers(0, 2))
        flags = mpc.MPC_TRUNCATE if trunc else 0
        kw = {}
        if rng.integers(0, 2):
            kw["f_public"] = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
            if rng.integers(0, 2):
                flags |= mpc.MPC_TWO_PHASE
        z = lane.beaver_matmul(*args, n_chunks=int(rng.integers(1, 5)), flags=flags, **kw)
        same(mpc, lane, z, oracle_matmul(d, 16 if trunc else 0), f"matmul {M}x{K}x{N}")


def test_random_conv_geometries(mpc, lane):
    rng = np.random.default_rng(2025)
    done = 0
    while done < 30:
        B, H, W = int(rng.integers(1, 4)), int(rng.integers(1, 14)), int(rng.integers(1, 14))
        Cin, Cout = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        k = int(rng.choice([1, 2, 3, 5])); pad = int(rng.integers(0, k)); stride = int(rng.integers(1, 4))
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        done += 1
        case = (B, H, W, Cin, Cout, k, k, pad, stride)
        print(f"random conv {done}: {case}", flush=True)
        d = deal_conv(rng, *case)
        x, w, a, b, c = (dev(mpc, d[q]) for q in ("x", "y", "a", "b", "c"))
        z = lane.conv2d(x, w, a, b, c, pad, stride, n_chunks=int(rng.integers(1, 4)))
        same(mpc, lane, z, oracle_conv(d), f"conv {case}")
        # prepared planes on the same layer
        f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
        right, left = lane.prepare_conv2d(a, b, f_public, pad, stride, left=bool(rng.integers(0, 2)))
        z = lane.conv2d_prepared(x, a, c, right, left, k, k, pad, stride)
        same(mpc, lane, z, oracle_conv(d), f"prepared conv {case}")


def test_random_conv_gradients(mpc, lane):
    rng = np.random.default_rng(2026)
    done = 0
    while done < 32:
        B, H, W = int(rng.integers(1, 3)), int(rng.integers(2, 12)), int(rng.integers(2, 12))
        Cin, Cout = int(rng.integers(1, 24)), int(rng.integers(1, 24))
        k = int(rng.choice([1, 2, 3, 4, 5])); pad = int(rng.integers(0, k)); stride = int(rng.integers(1, 4))
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        done += 1
        case = (B, H, W, Cin, Cout, k, k, pad, stride)
        print(f"random conv gradients {done}: {case}", flush=True)
        Ho, Wo = oracle.conv_out_hw(H, W, k, k, pad, stride)
        X = synth.rand_words(rng, (B, H, W, Cin)); Wt = synth.rand_words(rng, (k, k, Cin, Cout))
        G = synth.rand_words(rng, (B, Ho, Wo, Cout))
        xs, ws, gs = (synth.share_additive(rng, v) for v in (X, Wt, G))
        fx = lambda g, w: oracle.ring_conv2d_grad_x(g, w, X.shape, pad, stride)
        fw = lambda x, g: oracle.ring_conv2d_grad_w(x, g, k, k, pad, stride)
        a, b, c = synth.deal_product_triple(rng, G.shape, Wt.shape, fx)
        gx = lane.conv2d_grad_x(dev(mpc, gs), dev(mpc, ws), dev(mpc, a), dev(mpc, b), dev(mpc, c), pad, stride, flags=0)
        same(mpc, lane, gx, oracle.beaver_bilinear(fx, gs, ws, a, b, c), f"grad_x {case}")
        a, b, c = synth.deal_product_triple(rng, X.shape, G.shape, fw)
        gw = lane.conv2d_grad_w(dev(mpc, xs), dev(mpc, gs), dev(mpc, a), dev(mpc, b), dev(mpc, c), pad, stride, flags=0)
        same(mpc, lane, gw, oracle.beaver_bilinear(fw, xs, gs, a, b, c), f"grad_w {case}")


def test_random_relu_sizes_both_chains(mpc, lane):
    rng = np.random.default_rng(2027)
    for it in range(16):
        n = int(rng.integers(1, 3000))
        print(f"random relu {it}: n={n}", flush=True)
        xs = (synth.rand_words(rng, n), synth.rand_words(rng, n))
        mat = synth.deal_relu_material(rng, n)
        want = oracle.relu(xs, mat)
        md = mpc.material_to_device(mat)
        chunks = int(rng.integers(0, 5))
        y, sb, sa = lane.relu(dev(mpc, xs), md, n_chunks=chunks, want_sign=True)
        same(mpc, lane, y, want.y, f"relu n={n}"); same(mpc, lane, sa, want.s_arith, "sign shares")
        y, sb, sa = lane.relu(dev(mpc, xs), lane.pack_material(md), n_chunks=chunks, want_sign=True, packed=True)
        same(mpc, lane, y, want.y, f"packed relu n={n}"); same(mpc, lane, sb, want.s_bit, "packed sign bits")


# ------------------------------------------------------------------ three parties
def dev3(mpc, tri):
    return tuple(mpc.to_device(v) for v in tri)


def same3(mpc, lane, got, want, what):
    lane.sync()
    for i in range(3):
        g = mpc.to_host(got[i]).reshape(np.shape(want[i]))
        assert np.array_equal(g, want[i]), f"{what}: party {i} differs in {(g != want[i]).sum()} of {g.size} words"


def test_random_three_party_products_and_rescale(mpc, lane):
    rng = np.random.default_rng(2031)
    for it in range(16):
        if rng.integers(0, 2):
            M, K, N = (int(rng.integers(1, 160)), int(rng.integers(1, 300)), int(rng.integers(1, 160)))
            print(f"random matmul3 {it}: {M}x{K}x{N}", flush=True)
            X = synth.normal_fixed(rng, (M, K), 1.0); Y = synth.normal_fixed(rng, (K, N), 0.1)
            x, y = synth.share_additive3(rng, X), synth.share_additive3(rng, Y)
            a, b, c = synth.deal_product_triple3(rng, X.shape, Y.shape, oracle.ring_matmul)
            want = oracle.beaver_matmul3(x, y, a, b, c)
            z = lane.beaver_matmul3(dev3(mpc, x), dev3(mpc, y), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c))
        else:
            B, H, W = int(rng.integers(1, 4)), int(rng.integers(3, 12)), int(rng.integers(3, 12))
            Cin, Cout = int(rng.integers(1, 40)), int(rng.integers(1, 70))
            KH = int(rng.choice([1, 3])); pad = int(rng.integers(0, KH // 2 + 1)); stride = int(rng.integers(1, 3))
            print(f"random conv2d3 {it}: B{B} {H}x{W} {Cin}->{Cout} k{KH} pad {pad} stride {stride}", flush=True)
            conv = lambda A, Bm: oracle.ring_conv2d(A, Bm, pad, stride)
            X = synth.normal_fixed(rng, (B, H, W, Cin), 1.0); Y = synth.normal_fixed(rng, (KH, KH, Cin, Cout), 0.1)
            x, y = synth.share_additive3(rng, X), synth.share_additive3(rng, Y)
            a, b, c = synth.deal_product_triple3(rng, X.shape, Y.shape, conv)
            want = oracle.beaver_conv2d3(x, y, a, b, c, pad, stride)
            z = lane.conv2d3(dev3(mpc, x), dev3(mpc, y), dev3(mpc, a), dev3(mpc, b), dev3(mpc, c), pad, stride)
        same3(mpc, lane, z, want, "three-party product")
        r, rt = synth.deal_trunc3_pair(rng, np.shape(want[0]))
        t = lane.truncate3(z, dev3(mpc, r), dev3(mpc, rt))
        same3(mpc, lane, t, oracle.truncate3(want, r, rt), "three-party rescale")


def test_random_three_party_relu_sizes_both_chains(mpc, lane):
    rng = np.random.default_rng(2032)
    for it in range(12):
        n = int(rng.integers(1, 3000))
        print(f"random relu3 {it}: n={n}", flush=True)
        xs = tuple(synth.rand_words(rng, n) for _ in range(3))
        mat = synth.deal_relu3_material(rng, n)
        want = oracle.relu3(xs, mat)
        md = mpc.material_to_device(mat)
        y, sb, sa = lane.relu3(dev3(mpc, xs), md, want_sign=True)
        same3(mpc, lane, y, want.y, f"relu3 n={n}"); same3(mpc, lane, sa, want.s_arith, "sign shares")
        y, sb, sa = lane.relu3(dev3(mpc, xs), lane.pack_material3(md), want_sign=True, packed=True)
        same3(mpc, lane, y, want.y, f"packed relu3 n={n}"); same3(mpc, lane, sb, want.s_bit, "packed sign bits")
        same3(mpc, lane, sa, want.s_arith, "packed sign shares")
