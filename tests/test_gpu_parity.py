"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Shares must agree bit for bit; decoded fixed-point
results must be within 2^-12 of float64 on the decoded inputs."""
import numpy as np
import pytest

import oracle
from helpers import deal_conv, deal_matmul, oracle_conv, oracle_matmul, rec
from paper_2209_13643_amd import synth

pytestmark = pytest.mark.gpu
U64 = np.uint64
TOL = 2.0 ** -12


@pytest.fixture(scope="module")
def mpc():
    from paper_2209_13643_amd import mpc as m
    return m


@pytest.fixture(params=["three-streams", "single-queue", "single-queue-put"])
def lane(mpc, request):
    """Both issue modes of a lane: party 0 / party 1 / wire on three streams
    ordered by events, or everything on one in-order queue (merged launches)."""
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
            raise AssertionError(f"{what}: party {i} differs at {len(bad)} of {g.size} elements, first {bad[0]}: "
                                 f"got {int(g[tuple(bad[0])]):#x} want {int(want[i][tuple(bad[0])]):#x}")


# ------------------------------------------------------------------- element-wise
@pytest.mark.parametrize("n", [1, 2, 255, 4097, 1 << 20])
def test_open_and_truncate(mpc, lane, n):
    print(f"open/truncate n={n}", flush=True)
    rng = np.random.default_rng(n)
    s = (synth.rand_words(rng, n), synth.rand_words(rng, n))
    out = lane.open(dev(mpc, s))
    lane.sync()
    assert np.array_equal(mpc.to_host(out), oracle.open_shares(*s))
    z = dev(mpc, s)
    lane.truncate(z, 16)
    assert_shares_equal(host(mpc, lane, z), oracle.truncate(s, 16), "truncate")


# ------------------------------------------------------------------ plain ring GEMM
RING_SHAPES = [(1, 1, 1), (5, 3, 2), (32, 32, 32), (33, 17, 65), (70, 100, 150), (300, 257, 90), (128, 2304, 64)]


@pytest.mark.parametrize("shape", RING_SHAPES)
def test_ring_matmul(mpc, lane, shape):
    M, K, N = shape
    print(f"ring_matmul {shape}", flush=True)
    rng = np.random.default_rng(M * 7 + K)
    L, R = synth.rand_words(rng, (M, K)), synth.rand_words(rng, (K, N))
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    assert np.array_equal(mpc.to_host(Z), oracle.ring_matmul(L, R))


def test_ring_matmul_extreme_digits(mpc, lane):
    """Operands whose balanced digits are all -128 / 127 / carries: the int32
    digit sums are at their largest magnitude."""
    print("ring_matmul extreme digits", flush=True)
    M, K, N = 64, 4608, 64
    pats = np.array([0x8080808080808080, 0x7F7F7F7F7F7F7F7F, 0xFFFFFFFFFFFFFFFF, 0x80, 0x8000000000000000],
                    dtype=U64)
    rng = np.random.default_rng(5)
    L = pats[rng.integers(0, 2, size=(M, K))]            # only the two extreme patterns
    R = pats[rng.integers(0, 2, size=(K, N))]
    L[::3] = pats[0]; R[:, ::2] = pats[0]                # rows/columns of all -128 digits
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    assert np.array_equal(mpc.to_host(Z), oracle.ring_matmul(L, R))


def test_ring_matmul_longest_exact_pass_worst_case(mpc):
    """The longest contraction one workgroup sums without slicing (32 736 terms), with every
    digit of many rows and columns at -128: the int32 digit sums reach 4 * 32736 * 2^14, the
    largest value the exactness bound allows.  160 output tiles keep the contraction unsplit."""
    print("ring_matmul worst-case digit sums", flush=True)
    M, K, N = 640, 32736, 2048
    lane = mpc.Lane(0); lane.use_single_queue()
    rng = np.random.default_rng(6)
    lo, hi = np.uint64(0x8080808080808080), np.uint64(0x7F7F7F7F7F7F7F7F)
    L = np.where(rng.integers(0, 2, size=(M, K)) == 1, lo, hi)
    R = np.where(rng.integers(0, 2, size=(K, N)) == 1, lo, hi)
    L[::2] = lo; R[:, ::2] = lo                          # whole rows / columns of -128 digits
    L[1] = hi; R[:, 1] = hi                              # and of +127 digits
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    assert np.array_equal(mpc.to_host(Z), oracle.ring_matmul(L, R))
    lane.close()


@pytest.mark.parametrize("shape", [(130, 70, 650), (4100, 40, 680), (200, 33, 1100)])
def test_ring_matmul_ragged_column_panels(mpc, lane, shape):
    """Outputs whose column tiles do not fill the last panel of the tile order (6 tiles of 128 columns = panels of 4 + 2;
    11 tiles of 64 columns on the 128 x 64 tile = 4 + 4 + 3; 9 tiles of 128 = 4 + 4 + 1), with ragged last tiles."""
    M, K, N = shape
    print(f"ring_matmul, ragged column panels {shape}", flush=True)
    rng = np.random.default_rng(M + 3 * K + N)
    L, R = synth.rand_words(rng, (M, K)), synth.rand_words(rng, (K, N))
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    assert np.array_equal(mpc.to_host(Z), oracle.ring_matmul(L, R))


def test_beaver_matmul_batched_ragged_column_panels(mpc, lane):
    print("beaver_matmul batched, ragged column panels", flush=True)
    d = deal_matmul(np.random.default_rng(83), 70, 40, 650, batch=3)
    z = lane.beaver_matmul(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]))
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "batched, ragged panels")


def test_ring_matmul_batched(mpc, lane):
    print("ring_matmul batched", flush=True)
    rng = np.random.default_rng(6)
    L, R = synth.rand_words(rng, (5, 40, 64)), synth.rand_words(rng, (5, 64, 48))
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    want = np.stack([oracle.ring_matmul(L[i], R[i]) for i in range(5)])
    assert np.array_equal(mpc.to_host(Z), want)


# ------------------------------------------------------------- Beaver matmul (Alg. 1)
BEAVER_SHAPES = [(1, 1, 1), (7, 5, 3), (64, 256, 128), (130, 70, 67), (257, 48, 200)]


@pytest.mark.parametrize("shape", BEAVER_SHAPES)
@pytest.mark.parametrize("trunc", [True, False])
def test_beaver_matmul(mpc, lane, shape, trunc):
    M, K, N = shape
    print(f"beaver_matmul {shape} trunc={trunc}", flush=True)
    d = deal_matmul(np.random.default_rng(M + K + N), M, K, N)
    z = lane.beaver_matmul(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]),
                           dev(mpc, d["c"]), flags=mpc.MPC_TRUNCATE if trunc else 0)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d, 16 if trunc else 0), "beaver_matmul")


def test_beaver_matmul_batched(mpc, lane):
    print("beaver_matmul batched", flush=True)
    d = deal_matmul(np.random.default_rng(77), 48, 64, 40, batch=6)
    z = lane.beaver_matmul(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]))
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "batched")


@pytest.mark.parametrize("n_chunks", [1, 2, 4, 8])
@pytest.mark.parametrize("mode", ["in-call", "pre-opened", "two-phase"])
def test_beaver_matmul_schedule_invariance(mpc, lane, n_chunks, mode):
    """Chunked openings, a pre-opened weight mask and the Alg. 3 ordering all
    give the shares of the plain Alg. 1 run (Sec. 5.10)."""
    print(f"schedule invariance chunks={n_chunks} mode={mode}", flush=True)
    d = deal_matmul(np.random.default_rng(88), 150, 96, 70)
    f_pub = None
    y = dev(mpc, d["y"])
    flags = mpc.MPC_TRUNCATE
    if mode != "in-call":
        f_pub = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
        y = None
    if mode == "two-phase":
        flags |= mpc.MPC_TWO_PHASE
    z = lane.beaver_matmul(dev(mpc, d["x"]), y, dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]),
                           f_public=f_pub, n_chunks=n_chunks, flags=flags)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "schedule")


@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 3, 2), (5, 1, 4), (1, 7, 3), (2, 3, 5)])
@pytest.mark.parametrize("n_chunks", [2, 3, 4, 8])
def test_beaver_matmul_more_chunks_than_word_pairs(mpc, lane, shape, n_chunks):
    """Fewer than two words of x per chunk: leading chunks are empty, and the weight mask
    (opened in the same call) must still be formed and exchanged."""
    M, K, N = shape
    print(f"tiny chunked matmul {shape} chunks={n_chunks}", flush=True)
    d = deal_matmul(np.random.default_rng(1000 + M * K + n_chunks), M, K, N)
    z = lane.beaver_matmul(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]),
                           dev(mpc, d["c"]), n_chunks=n_chunks, flags=mpc.MPC_TRUNCATE)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "tiny chunked")


# ---------------------------------------------------------------------- conv (Eq. 3)
CONV_CASES = [  # B,H,W,Cin,Cout,KH,KW,pad,stride
    (1, 3, 3, 1, 1, 3, 3, 1, 1), (2, 8, 8, 3, 16, 3, 3, 1, 1), (2, 9, 7, 20, 24, 3, 3, 1, 1),
    (1, 12, 12, 16, 8, 3, 3, 0, 2), (3, 10, 10, 32, 40, 1, 1, 0, 1), (2, 11, 9, 5, 7, 3, 3, 1, 2),
    (4, 16, 16, 64, 64, 3, 3, 1, 1)]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d(mpc, lane, case):
    print(f"conv2d {case}", flush=True)
    d = deal_conv(np.random.default_rng(sum(case)), *case)
    z = lane.conv2d(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]),
                    d["pad"], d["stride"])
    assert_shares_equal(host(mpc, lane, z), oracle_conv(d), "conv2d")


def test_ring_conv2d(mpc, lane):
    print("ring_conv2d", flush=True)
    rng = np.random.default_rng(9)
    x, w = synth.rand_words(rng, (2, 9, 8, 19)), synth.rand_words(rng, (3, 3, 19, 33))
    z = lane.ring_conv2d(mpc.to_device(x), mpc.to_device(w), 1, 1)
    lane.sync()
    assert np.array_equal(mpc.to_host(z), oracle.ring_conv2d(x, w, 1, 1))


# ---------------------------------------------------------------------------- ReLU
@pytest.mark.parametrize("n", [1, 2, 63, 1000, 4097, 70000])
@pytest.mark.parametrize("n_chunks", [1, 3])
def test_relu(mpc, lane, n, n_chunks):
    print(f"relu n={n} chunks={n_chunks}", flush=True)
    rng = np.random.default_rng(n + n_chunks)
    X = rng.integers(-(1 << 40), 1 << 40, size=n).astype(np.int64).view(U64)
    X[: min(n, 9)] = np.array([0, 1, -1, 1 << 62, -(1 << 63), (1 << 63) - 1, -65536, 65536, 5],
                              dtype=np.int64).view(U64)[: min(n, 9)]
    xs = synth.share_additive(rng, X)
    mat = synth.deal_relu_material(rng, n)
    want = oracle.relu(xs, mat)
    y, sb, sa = lane.relu(dev(mpc, xs), mpc.material_to_device(mat), n_chunks=n_chunks, want_sign=True)
    lane.sync()
    assert_shares_equal((mpc.to_host(sb[0]), mpc.to_host(sb[1])), want.s_bit, "sign bit share")
    assert_shares_equal((mpc.to_host(sa[0]), mpc.to_host(sa[1])), want.s_arith, "sign arithmetic share")
    got = (mpc.to_host(y[0]), mpc.to_host(y[1]))
    assert_shares_equal(got, want.y, "relu output")
    assert np.array_equal(rec(got).view(np.int64), np.maximum(X.view(np.int64), 0))


@pytest.mark.parametrize("n", [1, 2, 63, 1000, 4097, 70000])
def test_relu_with_the_listing_tree(mpc, lane, n):
    """The prefix tree of the Sec. 4.2 listing as the carry network: its sign-bit shares
    differ from the Kogge-Stone ones and must equal the oracle's tree."""
    print(f"relu tree n={n}", flush=True)
    rng = np.random.default_rng(500 + n)
    X = rng.integers(-(1 << 62), 1 << 62, size=n).astype(np.int64).view(U64)
    X[: min(n, 9)] = np.array([0, 1, -1, 1 << 62, -(1 << 63), (1 << 63) - 1, -65536, 65536, 5],
                              dtype=np.int64).view(U64)[: min(n, 9)]
    xs = synth.share_additive(rng, X)
    mat = synth.deal_relu_material(rng, n)
    want = oracle.relu(xs, mat, adder="tree")
    lane.set_adder("tree")
    y, sb, sa = lane.relu(dev(mpc, xs), mpc.material_to_device(mat), n_chunks=2, want_sign=True)
    lane.sync()
    lane.set_adder("kogge-stone")
    assert_shares_equal((mpc.to_host(sb[0]), mpc.to_host(sb[1])), want.s_bit, "sign bit share (tree)")
    assert_shares_equal((mpc.to_host(sa[0]), mpc.to_host(sa[1])), want.s_arith, "sign arithmetic share (tree)")
    assert_shares_equal((mpc.to_host(y[0]), mpc.to_host(y[1])), want.y, "relu output (tree)")
    if n >= 63:
        assert not np.array_equal(want.s_bit[0], oracle.relu(xs, mat).s_bit[0])


def test_maxpool_with_the_listing_tree(mpc, lane):
    print("maxpool tree", flush=True)
    B, H, W, C = 2, 6, 4, 3
    rng = np.random.default_rng(41)
    X = rng.integers(-(1 << 30), 1 << 30, size=(B, H, W, C)).astype(np.int64)
    xs = synth.share_additive(rng, X.view(U64))
    n_out = B * (H // 2) * (W // 2) * C
    m1, m2 = synth.deal_relu_material(rng, 2 * n_out), synth.deal_relu_material(rng, n_out)
    lane.set_adder("tree")
    y = lane.maxpool2x2(dev(mpc, xs), mpc.material_to_device(m1), mpc.material_to_device(m2))
    got = host(mpc, lane, y)
    lane.set_adder("kogge-stone")
    assert_shares_equal(got, oracle.maxpool2x2(xs, m1, m2, adder="tree"), "maxpool (tree)")
    assert np.array_equal(rec(got).view(np.int64), X.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4)))


def test_relu_exhaustive_small_magnitude(mpc, lane):
    print("relu exhaustive", flush=True)
    rng = np.random.default_rng(123)
    vals = np.arange(-4096, 4097, dtype=np.int64)
    for x0 in (None, 0, 1 << 63, (1 << 64) - 1):
        X = vals.view(U64)
        xs = synth.share_additive(rng, X) if x0 is None else (np.full(X.shape, x0, U64), X - np.full(X.shape, x0, U64))
        mat = synth.deal_relu_material(rng, X.size)
        y = lane.relu(dev(mpc, xs), mpc.material_to_device(mat))
        got = host(mpc, lane, y)
        assert_shares_equal(got, oracle.relu(xs, mat).y, "relu")
        assert np.array_equal(rec(got).view(np.int64), np.maximum(vals, 0))


@pytest.mark.parametrize("n_chunks", [1, 2, 4, 8, 16])
def test_relu_chunk_invariance(mpc, lane, n_chunks):
    print(f"relu chunk invariance {n_chunks}", flush=True)
    rng = np.random.default_rng(321)
    n = 50000
    xs = (synth.rand_words(rng, n), synth.rand_words(rng, n))
    mat = synth.deal_relu_material(rng, n)
    y = lane.relu(dev(mpc, xs), mpc.material_to_device(mat), n_chunks=n_chunks)
    assert_shares_equal(host(mpc, lane, y), oracle.relu(xs, mat).y, "relu chunks")


def test_relu_lane_chunk_size_invariance(mpc, lane):
    """The lane's automatic chunk size (what a runner shrinks when several lanes convert at once) changes no word."""
    print("relu lane chunk size", flush=True)
    rng = np.random.default_rng(322)
    n = 50000
    xs = (synth.rand_words(rng, n), synth.rand_words(rng, n))
    mat = synth.deal_relu_material(rng, n)
    want = oracle.relu(xs, mat).y
    x, m = dev(mpc, xs), mpc.material_to_device(mat)
    for elems in (4096, 1024, 0):
        lane.set_relu_chunk(elems, elems)
        assert_shares_equal(host(mpc, lane, lane.relu(x, m)), want, f"relu, {elems}-element chunks")
        packed = lane.pack_material(m)
        assert_shares_equal(host(mpc, lane, lane.relu(x, packed, packed=True)), want, f"packed relu, {elems}-element chunks")
    with pytest.raises(mpc.MpcError):
        lane.set_relu_chunk(100)


@pytest.mark.parametrize("shape", [(1, 2, 2, 1), (2, 6, 4, 3), (3, 8, 8, 16)])
def test_maxpool(mpc, lane, shape):
    print(f"maxpool {shape}", flush=True)
    B, H, W, C = shape
    rng = np.random.default_rng(sum(shape))
    X = rng.integers(-(1 << 30), 1 << 30, size=shape).astype(np.int64)
    xs = synth.share_additive(rng, X.view(U64))
    n_out = B * (H // 2) * (W // 2) * C
    m1, m2 = synth.deal_relu_material(rng, 2 * n_out), synth.deal_relu_material(rng, n_out)
    y = lane.maxpool2x2(dev(mpc, xs), mpc.material_to_device(m1), mpc.material_to_device(m2))
    got = host(mpc, lane, y)
    assert_shares_equal(got, oracle.maxpool2x2(xs, m1, m2), "maxpool")
    assert np.array_equal(rec(got).view(np.int64), X.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4)))


# ------------------------------------------------------------------ error handling
def test_argument_errors(mpc, lane):
    print("argument errors", flush=True)
    import torch
    t = torch.zeros(16, dtype=torch.int64, device="cuda:0")
    pair = (t, t)
    L = mpc.lib()
    sh = mpc._share(pair)
    null = mpc._share(None)
    h = lane._h
    lane.reserve(1 << 20)
    assert L.mpc_open(h, null, mpc._p64(t), 16) == -1
    assert L.mpc_open(h, sh, mpc._p64(t), 0) == -1
    assert L.mpc_beaver_matmul(h, sh, sh, sh, sh, sh, sh, 0, 4, 4, 1, None, 1, 0) == -1
    assert L.mpc_beaver_matmul(h, sh, sh, sh, sh, sh, sh, 4, 4, 4, 1, None, 0, 0) == -1
    assert L.mpc_beaver_matmul(h, sh, null, sh, sh, sh, sh, 4, 2, 2, 1, None, 1, 0) == -1   # no y and no f_public
    assert L.mpc_beaver_matmul(h, sh, sh, sh, sh, sh, sh, 4, 5000000, 4, 1, None, 1, 0) == -4  # K too long
    assert L.mpc_beaver_matmul(h, sh, sh, sh, sh, sh, sh, 4096, 4096, 4096, 1, None, 1, 0) == -2  # workspace
    assert L.mpc_truncate(h, sh, 16, 64) == -1
    assert L.mpc_relu(h, sh, None, sh, 16, 1, None, None) == -1
    lane.sync()


# ------------------------------------------------- small API pieces used by the runner
def test_sub_then_open_gives_weight_mask(mpc, lane):
    """mpc_sub + mpc_open = the ahead-of-time opening of W - B (Alg. 3, the early broadcast)."""
    print("sub + open", flush=True)
    rng = np.random.default_rng(55)
    W = synth.rand_words(rng, (37, 21)); B = synth.rand_words(rng, (37, 21))
    ws, bs = synth.share_additive(rng, W), synth.share_additive(rng, B)
    d = lane.sub(dev(mpc, ws), dev(mpc, bs))
    f = lane.open(d)
    lane.sync()
    assert np.array_equal(mpc.to_host(f), W - B)
    assert np.array_equal(mpc.to_host(f), oracle.open_shares(ws[0] - bs[0], ws[1] - bs[1]))


@pytest.mark.parametrize("shape", [(5, 7, 3), (64, 256, 128), (130, 70, 200)])
@pytest.mark.parametrize("left", [True, False])
def test_beaver_matmul_prepared_planes(mpc, lane, shape, left):
    """Planes of [a_i], f, b_0 + f, b_1 recoded ahead of time: the same shares as the plain call."""
    M, K, N = shape
    print(f"prepared matmul {shape} left={left}", flush=True)
    d = deal_matmul(np.random.default_rng(M * K + N), M, K, N, x_std=1.0, w_std=0.1)
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    a, b, c = dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"])
    right, lp = lane.prepare_matmul(a, b, f_public, left=left)
    for _ in range(2):                                   # the planes are reusable
        z = lane.beaver_matmul_prepared(dev(mpc, d["x"]), a, c, right, lp)
        assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "prepared matmul")


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_prepared_planes(mpc, lane, case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print(f"prepared conv {case}", flush=True)
    d = deal_conv(np.random.default_rng(sum(case) + 3), B, H, W, Cin, Cout, KH, KW, pad, stride, x_std=1.0, w_std=0.1)
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    a, b, c = dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"])
    right, lp = lane.prepare_conv2d(a, b, f_public, pad, stride)
    z = lane.conv2d_prepared(dev(mpc, d["x"]), a, c, right, lp, KH, KW, pad, stride)
    assert_shares_equal(host(mpc, lane, z), oracle_conv(d), "prepared conv")
    z = lane.conv2d_prepared(dev(mpc, d["x"]), a, c, right, None, KH, KW, pad, stride, n_chunks=3,
                             flags=mpc.MPC_TRUNCATE | mpc.MPC_TWO_PHASE)
    assert_shares_equal(host(mpc, lane, z), oracle_conv(d), "prepared conv, two-phase, chunked")


FOLDED_MATMUL = [(1, 1, 1), (5, 7, 3), (64, 256, 128), (130, 70, 200), (300, 1100, 150), (32, 512, 10), (128, 4608, 512),
                 (700, 64, 300)]


@pytest.mark.parametrize("shape", FOLDED_MATMUL)
@pytest.mark.parametrize("n_chunks", [1, 3])
def test_beaver_matmul_folded(mpc, lane, shape, n_chunks):
    """Party 0's addend folded ahead of time (c_0 - a_0 b_0): party 0 contracts one product, party 1 two,
    and every output word is Alg. 1's.  Shapes cover one-tile outputs whose contraction is sliced (the two
    parties then get different slice counts), many tiles, ragged edges, and a rescale-free call."""
    M, K, N = shape
    print(f"folded matmul {shape} chunks={n_chunks}", flush=True)
    d = deal_matmul(np.random.default_rng(M * K + N + 9), M, K, N)
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    a, b, c = dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"])
    right, lp = lane.prepare_matmul(a, b, f_public)
    c0f = lane.fold_matmul(a, b, c)
    lane.sync()
    assert np.array_equal(mpc.to_host(c0f), d["c"][0] - oracle.ring_matmul(d["a"][0], d["b"][0]))
    for trunc in (True, False):
        z = lane.beaver_matmul_prepared(dev(mpc, d["x"]), a, (c0f, c[1]), right, lp, n_chunks=n_chunks,
                                        flags=(mpc.MPC_TRUNCATE if trunc else 0) | mpc.MPC_FOLDED)
        assert_shares_equal(host(mpc, lane, z), oracle_matmul(d, 16 if trunc else 0), "folded matmul")


def test_beaver_matmul_folded_batched(mpc, lane):
    print("folded matmul batched", flush=True)
    d = deal_matmul(np.random.default_rng(78), 48, 64, 40, batch=6)
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    a, b, c = dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"])
    right, lp = lane.prepare_matmul(a, b, f_public)
    c0f = lane.fold_matmul(a, b, c)
    z = lane.beaver_matmul_prepared(dev(mpc, d["x"]), a, (c0f, c[1]), right, lp, flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "folded batched")


@pytest.mark.parametrize("shape", [(1, 1, 1), (5, 7, 3), (64, 256, 128), (130, 70, 200), (300, 1100, 150), (700, 64, 300)])
def test_beaver_matmul_folded_two_shared_operands(mpc, lane, shape):
    """The folded call on a product of two shared operands (f opens in the call, only a_1's and b_1's planes and
    the folded addend come from the offline phase): every output word is Alg. 1's."""
    M, K, N = shape
    print(f"folded matmul, y shared {shape}", flush=True)
    d = deal_matmul(np.random.default_rng(M * K + N + 21), M, K, N)
    x, y, a, b, c = (dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c"))
    right, lp = lane.prepare_matmul(a, b, None)
    c0f = lane.fold_matmul(a, b, c)
    for trunc in (True, False):
        z = lane.beaver_matmul_folded(x, y, a, b, (c0f, c[1]), right, lp, flags=mpc.MPC_TRUNCATE if trunc else 0)
        assert_shares_equal(host(mpc, lane, z), oracle_matmul(d, 16 if trunc else 0), "folded matmul, y shared")
    # chunked masking gives the same words
    z = lane.beaver_matmul_folded(x, y, a, b, (c0f, c[1]), right, lp, n_chunks=3)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "folded matmul, y shared, chunked")
    lib = mpc.lib()
    none = mpc._share(None)
    z2 = (z[0].clone(), z[1].clone())
    args = (lane._h, mpc._share(x), none, mpc._share(a), mpc._share(b), mpc._share((c0f, c[1])), mpc._share(z2),
            right.data_ptr(), lp.data_ptr(), M, K, N, 1, 1, 0)
    assert lib.mpc_beaver_matmul_folded(*args) == -1          # MPC_EINVAL: y missing
    args = args[:7] + (None,) + args[8:]
    assert lib.mpc_beaver_matmul_folded(*args) == -1          # MPC_EINVAL: no prepared planes
    lane.sync()


def test_beaver_matmul_folded_attention_heads(mpc, lane):
    """Per-head Q * K^T (right operand stored [N][K]) and A * V as batched folded calls."""
    print("folded attention products", flush=True)
    rng = np.random.default_rng(91)
    heads, S, dh = 6, 80, 64
    # Q * K^T: K is stored [S][dh] = [N][K]
    d = deal_matmul(rng, S, dh, S, batch=heads)
    tr = lambda pair: (np.ascontiguousarray(pair[0].transpose(0, 2, 1)), np.ascontiguousarray(pair[1].transpose(0, 2, 1)))
    x, a, c = dev(mpc, d["x"]), dev(mpc, d["a"]), dev(mpc, d["c"])
    yT, bT = dev(mpc, tr(d["y"])), dev(mpc, tr(d["b"]))
    right, lp = lane.prepare_matmul(a, bT, None, flags=mpc.MPC_TRANS_Y)
    c0f = lane.fold_matmul(a, bT, c, flags=mpc.MPC_TRANS_Y)
    z = lane.beaver_matmul_folded(x, yT, a, bT, (c0f, c[1]), right, lp, flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_Y)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "folded Q K^T")
    # A * V
    d = deal_matmul(rng, S, S, dh, batch=heads)
    x, y, a, b, c = (dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c"))
    right, lp = lane.prepare_matmul(a, b, None)
    c0f = lane.fold_matmul(a, b, c)
    z = lane.beaver_matmul_folded(x, y, a, b, (c0f, c[1]), right, lp)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "folded A V")


@pytest.mark.parametrize("case", CONV_CASES + [(2, 4, 4, 512, 96, 3, 3, 1, 1), (3, 16, 16, 3, 64, 3, 3, 1, 1)])
def test_conv2d_folded(mpc, lane, case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print(f"folded conv {case}", flush=True)
    d = deal_conv(np.random.default_rng(sum(case) + 4), B, H, W, Cin, Cout, KH, KW, pad, stride)
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    a, b, c = dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"])
    right, lp = lane.prepare_conv2d(a, b, f_public, pad, stride)
    c0f = lane.fold_conv2d(a, b, c, pad, stride)
    for _ in range(2):
        z = lane.conv2d_prepared(dev(mpc, d["x"]), a, (c0f, c[1]), right, lp, KH, KW, pad, stride,
                                 flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
        assert_shares_equal(host(mpc, lane, z), oracle_conv(d), "folded conv")
    # what the folded call cannot be combined with is refused before anything is enqueued
    with pytest.raises(mpc.MpcError):
        lane.conv2d_prepared(dev(mpc, d["x"]), a, (c0f, c[1]), right, None, KH, KW, pad, stride,
                             flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
    with pytest.raises(mpc.MpcError):
        lane.conv2d_prepared(dev(mpc, d["x"]), a, (c0f, c[1]), right, lp, KH, KW, pad, stride,
                             flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED | mpc.MPC_TWO_PHASE)


@pytest.fixture()
def small_tile_everywhere(mpc):
    """Every unsliced GEMM launch on 64 x 64 workgroup tiles of half-width waves, whatever its size."""
    mpc.set_gemm_small_tile(1 << 20, 1)
    yield
    mpc.set_gemm_small_tile()


@pytest.mark.parametrize("shape", RING_SHAPES + [(640, 96, 700)])
def test_ring_matmul_on_small_tiles(mpc, lane, small_tile_everywhere, shape):
    M, K, N = shape
    print(f"ring_matmul, small tiles {shape}", flush=True)
    rng = np.random.default_rng(M * 11 + K)
    L, R = synth.rand_words(rng, (M, K)), synth.rand_words(rng, (K, N))
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    assert np.array_equal(mpc.to_host(Z), oracle.ring_matmul(L, R))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_plain_and_folded_on_small_tiles(mpc, lane, small_tile_everywhere, case):
    B, H, W, Cin, Cout, KH, KW, pad, stride = case
    print(f"conv, small tiles {case}", flush=True)
    d = deal_conv(np.random.default_rng(sum(case) + 5), B, H, W, Cin, Cout, KH, KW, pad, stride)
    x, y, a, b, c = (dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c"))
    z = lane.conv2d(x, y, a, b, c, pad, stride)
    assert_shares_equal(host(mpc, lane, z), oracle_conv(d), "conv on small tiles")
    f_public = mpc.to_device((d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1]))
    right, lp = lane.prepare_conv2d(a, b, f_public, pad, stride)
    c0f = lane.fold_conv2d(a, b, c, pad, stride)
    z = lane.conv2d_prepared(x, a, (c0f, c[1]), right, lp, KH, KW, pad, stride, flags=mpc.MPC_TRUNCATE | mpc.MPC_FOLDED)
    assert_shares_equal(host(mpc, lane, z), oracle_conv(d), "folded conv on small tiles")


def test_beaver_matmul_batched_and_extreme_digits_on_small_tiles(mpc, lane, small_tile_everywhere):
    print("batched matmul and extreme digits, small tiles", flush=True)
    d = deal_matmul(np.random.default_rng(79), 48, 64, 40, batch=6)
    z = lane.beaver_matmul(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]))
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "batched on small tiles")
    M, K, N = 200, 4608, 200                 # 200 tiles: enough workgroups that the contraction stays unsliced
    pats = np.array([0x8080808080808080, 0x7F7F7F7F7F7F7F7F], dtype=U64)
    rng = np.random.default_rng(8)
    L = pats[rng.integers(0, 2, size=(M, K))]; R = pats[rng.integers(0, 2, size=(K, N))]
    L[::3] = pats[0]; R[:, ::2] = pats[0]
    Z = lane.ring_matmul(mpc.to_device(L), mpc.to_device(R))
    lane.sync()
    assert np.array_equal(mpc.to_host(Z), oracle.ring_matmul(L, R))


def test_graph_capture_replays(mpc):
    """A secure layer (Beaver matmul + ReLU) recorded once and replayed on fresh inputs in the same
    buffers, with eager work and synchronisation between the replays: every replay equals the oracle."""
    import torch
    print("graph capture", flush=True)
    lane = mpc.Lane(0); lane.use_single_queue()
    M, K, N = 64, 256, 128
    rng = np.random.default_rng(77)
    deals = [deal_matmul(rng, M, K, N, x_std=1.0, w_std=1.0 / 16) for _ in range(3)]
    mat = synth.deal_relu_material(rng, M * N)
    md = mpc.material_to_device(mat)
    d0 = deals[0]
    buf = {k: dev(mpc, d0[k]) for k in ("x", "y", "a", "b", "c")}
    z = (torch.empty_like(buf["c"][0]), torch.empty_like(buf["c"][1]))
    y = (torch.empty_like(z[0]), torch.empty_like(z[1]))

    def layer():
        lane.beaver_matmul(buf["x"], buf["y"], buf["a"], buf["b"], buf["c"], out=z)
        lane.relu(z, md, out=y)
    layer(); lane.sync()                                  # eager warm-up: attributes set, workspace sized
    with lane.capture() as cap:
        layer()
    graph = cap.graph
    assert mpc.lib().mpc_ctx_capture_end(lane._h, None) == -1            # no capture open any more
    for d in deals:
        for k in buf:
            for i in range(2):
                buf[k][i].copy_(mpc.to_device(d[k][i]))
        torch.cuda.synchronize()
        graph.launch(lane)
        lane.sync()
        want = oracle.relu(oracle_matmul(d), mat).y
        assert_shares_equal((mpc.to_host(y[0]), mpc.to_host(y[1])), want, "graph replay")
        # eager work between replays, on the same lane and workspace
        other = lane.relu(dev(mpc, d["c"]), md)
        lane.sync()
        assert_shares_equal((mpc.to_host(other[0]), mpc.to_host(other[1])), oracle.relu(d["c"], mat).y, "eager between replays")
    three = mpc.Lane(0)
    assert mpc.lib().mpc_ctx_capture_begin(three._h) == -1               # three streams: not capturable
    three.close()
    graph.close(); lane.close()


def test_add_is_the_local_sum(mpc, lane):
    print("add", flush=True)
    rng = np.random.default_rng(68)
    n = 4099
    X, Y = synth.rand_words(rng, n), synth.rand_words(rng, n)
    xs, ys = synth.share_additive(rng, X), synth.share_additive(rng, Y)
    got = host(mpc, lane, lane.add(dev(mpc, xs), dev(mpc, ys)))
    assert_shares_equal(got, (xs[0] + ys[0], xs[1] + ys[1]), "add")
    assert np.array_equal(rec(got), X + Y)


def test_profiling_regions(mpc, lane):
    print("profiling regions", flush=True)
    d = deal_matmul(np.random.default_rng(66), 96, 64, 80)
    args = [dev(mpc, d[k]) for k in ("x", "y", "a", "b", "c")]
    lane.beaver_matmul(*args)                        # not recorded
    lane.set_profiling(True); lane.profile_reset()
    for _ in range(3):
        z = lane.beaver_matmul(*args)
    n = 96 * 80
    y = lane.relu(z, mpc.material_to_device(synth.deal_relu_material(np.random.default_rng(67), n)))
    lane.set_profiling(False)
    lane.beaver_matmul(*args)                        # not recorded either
    gemm_ms, gemm_n = lane.profile(mpc.PROF_GEMM_KERNEL)
    lin_ms, lin_n = lane.profile(mpc.PROF_LINEAR)
    relu_ms, relu_n = lane.profile(mpc.PROF_RELU)
    assert (gemm_n, lin_n, relu_n) == (3, 3, 1)
    assert 0 < gemm_ms <= lin_ms and relu_ms > 0
    samples = lane.profile_samples(mpc.PROF_LINEAR)
    assert len(samples) == 3 and all(t > 0 for t in samples) and abs(sum(samples) - lin_ms) < 1e-6
    lane.profile_reset()
    assert lane.profile_samples(mpc.PROF_LINEAR) == []
    assert lane.profile(mpc.PROF_LINEAR) == (0.0, 0)
    assert_shares_equal(host(mpc, lane, z), oracle_matmul(d), "result unaffected by profiling")


def test_mfma_rate_measurement_aid(mpc):
    """The roofline's measurement aid runs, ends, and reports a plausible rate: some POP/s, never above what the
    matrix cores can issue (which operand pattern is faster in so short a run depends on the clock's ramp)."""
    print("mfma rate", flush=True)
    lane = mpc.Lane(0, single_queue=True)
    zero = lane.mfma_rate(False, iters=500, launches=4)
    rand = lane.mfma_rate(True, iters=500, launches=4)
    assert 0.5e15 < rand < 6e15 and 0.5e15 < zero < 6e15, (zero, rand)
    with pytest.raises(mpc.MpcError):
        lane.mfma_rate(True, iters=0)
    lane.close()
