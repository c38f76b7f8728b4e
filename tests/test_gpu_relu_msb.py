"""GPU parity of the sign-only (pruned, bit-packed) secure ReLU, mpc_relu_msb.

The pruned chain evaluates a subset of the gates of the whole-word Kogge-Stone
network with the same triple bits, so its outputs must equal the oracle's
whole-word protocol bit for bit: the oracle is fed the [12][n] material, the
library the same material after mpc_relu_pack_triples.  The packed layout
itself is checked against a numpy transcription of its definition."""
import numpy as np
import pytest

import oracle
from helpers import rec
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
        ln.set_exchange("put")          # ReLU rounds exchange by remote store instead of copy kernels
    yield ln
    ln.sync()
    ln.close()


def dev(mpc, pair):
    return (mpc.to_device(pair[0]), mpc.to_device(pair[1]))


def assert_shares_equal(got, want, what=""):
    for i in range(2):
        g = np.asarray(got[i]).reshape(np.shape(want[i]))
        if not np.array_equal(g, want[i]):
            bad = np.argwhere(g != want[i])
            raise AssertionError(f"{what}: party {i} differs at {len(bad)} of {g.size} elements, first {bad[0]}")


def level_mask(l):
    s = 2 << l
    return sum(1 << p for p in range(s - 2, 63, s))


def pack_reference(words, n):
    """[12][n] words -> packed layout, written from the layout's definition."""
    words = words.reshape(12, n)
    n64 = (n + 63) // 64 * 64
    segs = [np.concatenate([words[0], np.zeros((-n) % 4, U64)])]
    for t in range(1, 12):
        l = (t - 1) // 2; s = 2 << l
        w = np.zeros(n64, U64); w[:n] = words[t] & U64(level_mask(l))
        w = w.reshape(-1, s)
        acc = np.zeros(w.shape[0], U64)
        for k in range(s):
            acc |= w[:, k] if k == 0 else ((w[:, k] << U64(k)) | (w[:, k] >> U64(64 - k)))
        segs.append(np.concatenate([acc, np.zeros((-len(acc)) % 4, U64)]))
    return np.concatenate(segs)


def run_msb(mpc, lane, xs, mat, **kw):
    md = mpc.material_to_device(mat)
    packed = lane.pack_material(md)
    out = lane.relu(dev(mpc, xs), packed, packed=True, **kw)
    lane.sync()
    return out


@pytest.mark.parametrize("n", [1, 5, 64, 100, 1000, 4100])
def test_pack_triples_layout(mpc, lane, n):
    print(f"pack layout n={n}", flush=True)
    rng = np.random.default_rng(n)
    a = (synth.rand_words(rng, 12 * n), synth.rand_words(rng, 12 * n))
    md = {"r": dev(mpc, (a[0][:n], a[1][:n])), "and_a": dev(mpc, a), "and_b": dev(mpc, a), "and_c": dev(mpc, a)}
    got = lane.pack_material(md)["and_a"]
    for i in range(2):
        want = pack_reference(a[i], n)
        assert mpc.lib().mpc_relu_packed_words(n) == want.size
        assert np.array_equal(mpc.to_host(got[i]), want), f"party {i}"


@pytest.mark.parametrize("n", [1, 2, 3, 63, 64, 65, 255, 256, 257, 1000, 4097, 4100, 70000, 262148])
@pytest.mark.parametrize("n_chunks", [1, 3])
def test_relu_msb(mpc, lane, n, n_chunks):
    print(f"relu_msb n={n} chunks={n_chunks}", flush=True)
    rng = np.random.default_rng(1000 + n + n_chunks)
    X = rng.integers(-(1 << 40), 1 << 40, size=n).astype(np.int64).view(U64)
    X[: min(n, 9)] = np.array([0, 1, -1, 1 << 62, -(1 << 63), (1 << 63) - 1, -65536, 65536, 5],
                              dtype=np.int64).view(U64)[: min(n, 9)]
    xs = synth.share_additive(rng, X)
    mat = synth.deal_relu_material(rng, n)
    want = oracle.relu(xs, mat)
    y, sb, sa = run_msb(mpc, lane, xs, mat, n_chunks=n_chunks, want_sign=True)
    assert_shares_equal((mpc.to_host(sb[0]), mpc.to_host(sb[1])), want.s_bit, "sign bit share")
    assert_shares_equal((mpc.to_host(sa[0]), mpc.to_host(sa[1])), want.s_arith, "sign arithmetic share")
    got = (mpc.to_host(y[0]), mpc.to_host(y[1]))
    assert_shares_equal(got, want.y, "relu output")
    assert np.array_equal(rec(got).view(np.int64), np.maximum(X.view(np.int64), 0))


def test_relu_msb_uniform_words_and_carry_patterns(mpc, lane):
    """Uniform 64-bit shares, plus values whose sign hinges on one long carry
    chain (x_0 + x_1 with a run of ones meeting a single one)."""
    print("relu_msb carry patterns", flush=True)
    rng = np.random.default_rng(77)
    n = 64 * 67
    x0 = synth.rand_words(rng, n); x1 = synth.rand_words(rng, n)
    for k in range(64):                       # x0 = 2^63 - 2^k, x1 = 2^k or 2^k - 1: carry reaches bit 63 or not
        x0[2 * k] = U64((1 << 63) - (1 << k)); x1[2 * k] = U64(1 << k)
        x0[2 * k + 1] = U64((1 << 63) - (1 << k)); x1[2 * k + 1] = U64((1 << k) - 1)
    mat = synth.deal_relu_material(rng, n)
    want = oracle.relu((x0, x1), mat)
    y, sb, sa = run_msb(mpc, lane, (x0, x1), mat, want_sign=True)
    assert_shares_equal((mpc.to_host(sb[0]), mpc.to_host(sb[1])), want.s_bit, "sign bit share")
    got = (mpc.to_host(y[0]), mpc.to_host(y[1]))
    assert_shares_equal(got, want.y, "relu output")
    assert np.array_equal(rec(got).view(np.int64), np.maximum((x0 + x1).view(np.int64), 0))


@pytest.mark.parametrize("n_chunks", [0, 1, 2, 4, 8, 16])
def test_relu_msb_chunk_invariance(mpc, lane, n_chunks):
    print(f"relu_msb chunk invariance {n_chunks}", flush=True)
    rng = np.random.default_rng(321)
    n = 50000
    xs = (synth.rand_words(rng, n), synth.rand_words(rng, n))
    mat = synth.deal_relu_material(rng, n)
    y = run_msb(mpc, lane, xs, mat, n_chunks=n_chunks)
    assert_shares_equal((mpc.to_host(y[0]), mpc.to_host(y[1])), oracle.relu(xs, mat).y, "relu chunks")


def test_relu_msb_equals_whole_word_protocol(mpc, lane):
    """Same shares as mpc_relu on the same material."""
    print("relu_msb == relu", flush=True)
    rng = np.random.default_rng(5)
    n = 12345
    xs = (synth.rand_words(rng, n), synth.rand_words(rng, n))
    md = mpc.material_to_device(synth.deal_relu_material(rng, n))
    xd = dev(mpc, xs)
    a = lane.relu(xd, md); lane.sync()
    b = lane.relu(xd, lane.pack_material(md), packed=True); lane.sync()
    import torch
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


@pytest.mark.parametrize("shape", [(1, 2, 2, 1), (2, 6, 4, 3), (3, 8, 8, 16), (2, 16, 16, 64)])
def test_maxpool_msb(mpc, lane, shape):
    print(f"maxpool_msb {shape}", flush=True)
    B, H, W, C = shape
    rng = np.random.default_rng(sum(shape))
    X = rng.integers(-(1 << 30), 1 << 30, size=shape).astype(np.int64)
    xs = synth.share_additive(rng, X.view(U64))
    n_out = B * (H // 2) * (W // 2) * C
    m1, m2 = synth.deal_relu_material(rng, 2 * n_out), synth.deal_relu_material(rng, n_out)
    p1, p2 = lane.pack_material(mpc.material_to_device(m1)), lane.pack_material(mpc.material_to_device(m2))
    y = lane.maxpool2x2(dev(mpc, xs), p1, p2, packed=True)
    lane.sync()
    got = (mpc.to_host(y[0]), mpc.to_host(y[1]))
    assert_shares_equal(got, oracle.maxpool2x2(xs, m1, m2), "maxpool")
    assert np.array_equal(rec(got).view(np.int64), X.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4)))


def test_relu_msb_argument_errors(mpc, lane):
    print("relu_msb argument errors", flush=True)
    import torch
    from ctypes import byref
    n = 128
    rng = np.random.default_rng(1)
    md = lane.pack_material(mpc.material_to_device(synth.deal_relu_material(rng, n)))
    x = dev(mpc, (synth.rand_words(rng, n), synth.rand_words(rng, n)))
    y = (torch.empty_like(x[0]), torch.empty_like(x[1]))
    L = mpc.lib()
    lane.reserve(L.mpc_relu_msb_workspace_bytes(n))
    m = mpc._material(md, n, packed=True)
    assert L.mpc_relu_msb(lane._h, mpc._share(x), byref(m), mpc._share(y), 0, 1, None, None) == -1
    assert L.mpc_relu_msb(lane._h, mpc._share(x), None, mpc._share(y), n, 1, None, None) == -1
    # packed triples must be 16-byte aligned
    words = L.mpc_relu_packed_words(n)
    shifted = torch.zeros(words + 1, dtype=torch.int64, device=lane.device)[1:]
    bad = dict(md); bad["and_a"] = (shifted, md["and_a"][1])
    mb = mpc._material(bad, n, packed=True)
    assert L.mpc_relu_msb(lane._h, mpc._share(x), byref(mb), mpc._share(y), n, 1, None, None) == -1
    # a workspace that is too small is refused, not overrun
    small = mpc.Lane(0)
    small.reserve(256)
    assert L.mpc_relu_msb(small._h, mpc._share(x), byref(m), mpc._share(y), n, 1, None, None) == -2
    small.close()
    assert L.mpc_relu_msb_workspace_bytes(0) == 0 and L.mpc_relu_packed_words(0) == 0
