"""Parity at the full sizes of the five workloads, in the launch configuration
the benchmark times (single-queue lane, automatic ReLU chunking).

Linear layers: inputs and triples are dealt on the host (triple products by the
oracle) and every output share is compared bit for bit.  Secure ReLU at the
large sizes: material is drawn on the device by the seeded dealer (a
random-number source, not the code under test), downloaded slab by slab, and
the oracle recomputes every element: all output words (y, sign bits, sign
shares) of both parties are compared; the whole output is also checked through
the property rec(y) == max(rec(x), 0)."""
import numpy as np
import pytest
import torch

import oracle
from helpers import deal_conv, deal_matmul, oracle_conv, oracle_matmul, rec
from paper_2209_13643_amd import synth

pytestmark = pytest.mark.gpu
U64 = np.uint64
TOL = 2.0 ** -12


@pytest.fixture(scope="module")
def mods():
    from paper_2209_13643_amd import dealer, mpc, pipeline
    return mpc, dealer, pipeline


@pytest.fixture()
def lane(mods):
    ln = mods[0].Lane(0)
    ln.use_single_queue()
    yield ln
    ln.sync()
    ln.close()


def dev(mpc, pair):
    return (mpc.to_device(pair[0]), mpc.to_device(pair[1]))


def assert_equal_shares(mpc, got, want, what):
    for i in range(2):
        g = mpc.to_host(got[i]).reshape(want[i].shape)
        assert np.array_equal(g, want[i]), f"{what}: party {i}: {(g != want[i]).sum()} of {g.size} words differ"


def relu_sampled_check(mpc, dealer, lane, z, seed, slab=4 << 20):
    """Full-size secure ReLU on device shares z: every output word of both parties against the oracle
    (elements are independent, so the oracle runs slab by slab on the downloaded material), plus the
    reconstruction property on the device."""
    n = z[0].numel()
    g = dealer.gen(seed, lane.device)
    mat = dealer.relu_material(g, n, lane.device)
    y, sb, sa = lane.relu(z, mat, want_sign=True)
    lane.sync()
    rz = (z[0] + z[1]).view(-1); ry = (y[0] + y[1]).view(-1)
    assert torch.equal(ry, torch.clamp(rz, min=0)), "rec(y) != max(rec(x), 0)"
    assert torch.equal((sb[0] ^ sb[1]).view(-1).bool(), rz < 0)
    assert torch.equal((sa[0] + sa[1]).view(-1), (rz < 0).to(torch.int64))
    for lo in range(0, n, slab):
        hi = min(n, lo + slab)
        take = lambda t: mpc.to_host(t.view(-1)[lo:hi])
        take12 = lambda t: mpc.to_host(t.view(12, n)[:, lo:hi].contiguous())
        sub = {k: (take(mat[k][0]), take(mat[k][1])) for k in ("r", "rb", "ra", "ma", "mb", "mc")}
        for k in ("and_a", "and_b", "and_c"):
            sub[k] = (take12(mat[k][0]), take12(mat[k][1]))
        want = oracle.relu((take(z[0]), take(z[1])), sub)
        for i in range(2):
            assert np.array_equal(take(y[i]), want.y[i]), f"relu y, party {i}, elements {lo}..{hi}"
            assert np.array_equal(take(sb[i]), want.s_bit[i]), f"relu sign bits, party {i}, elements {lo}..{hi}"
            assert np.array_equal(take(sa[i]), want.s_arith[i]), f"relu sign shares, party {i}, elements {lo}..{hi}"
        del sub, want
    # the sign-only packed chain on the same material, packed on the device: every word of
    # every output equals the whole-word protocol's, which was just checked
    packed = lane.pack_material(mat)
    for k in ("and_a", "and_b", "and_c"):
        del mat[k]
    y2, sb2, sa2 = lane.relu(z, packed, want_sign=True, packed=True)
    lane.sync()
    for i in range(2):
        assert torch.equal(y2[i], y[i]) and torch.equal(sb2[i], sb[i]) and torch.equal(sa2[i], sa[i]), \
            f"mpc_relu_msb differs from mpc_relu, party {i}"
    return y


def float_check(d, z_rec_u64, conv):
    """Decoded output within 2^-12 of float64 on the decoded inputs (sampled rows)."""
    got = oracle.decode(z_rec_u64)
    if conv:
        x = torch.from_numpy(oracle.decode(d["X"])).permute(0, 3, 1, 2)[:2]
        w = torch.from_numpy(oracle.decode(d["Y"])).permute(3, 2, 0, 1)
        ref = torch.nn.functional.conv2d(x, w, padding=d["pad"], stride=d["stride"]).permute(0, 2, 3, 1).numpy()
        got = got[:2]
    else:
        ref = oracle.decode(d["X"])[..., :64, :] @ oracle.decode(d["Y"])
        got = got[..., :64, :]
    assert np.abs(got - ref).max() <= TOL


def test_config1_vgg_block_full(mods, lane):
    mpc, dealer, _ = mods
    L = synth.config_vgg_block().layers[0]
    print("config 1 full: conv 64x16x16x128 -> 128 + relu", flush=True)
    rng = synth.rng_for(1)
    d = deal_conv(rng, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, x_std=L.x_std, w_std=L.w_std)
    z = lane.conv2d(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]), L.pad, L.stride)
    lane.sync()
    want = oracle_conv(d)
    assert_equal_shares(mpc, z, want, "conv")
    assert not oracle.truncation_wraps(rec(oracle_conv(d, 0)), rec(want)).any()
    float_check(d, rec(want), conv=True)
    # the ReLU of this config fits on the host: full bit-exact comparison
    mat = synth.deal_relu_material(rng, L.B * L.Ho * L.Wo * L.Cout)
    md = mpc.material_to_device(mat)
    y = lane.relu(z, md)
    lane.sync()
    want_y = oracle.relu(want, mat).y
    assert_equal_shares(mpc, y, want_y, "relu")
    y2 = lane.relu(z, lane.pack_material(md), packed=True)
    lane.sync()
    assert_equal_shares(mpc, y2, want_y, "relu, sign-only packed chain")


def test_config2_resnet_bottleneck_full(mods, lane):
    mpc, dealer, _ = mods
    rng = synth.rng_for(2)
    for li, L in enumerate(synth.config_resnet_bottleneck().layers):
        print(f"config 2 full: {L.name} {L.gemm_mkn}", flush=True)
        d = deal_conv(rng, L.B, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride, x_std=L.x_std, w_std=L.w_std)
        z = lane.conv2d(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]), L.pad, L.stride)
        lane.sync()
        want = oracle_conv(d)
        assert_equal_shares(mpc, z, want, L.name)
        float_check(d, rec(want), conv=True)
        relu_sampled_check(mpc, dealer, lane, z, seed=200 + li)
        del d, z, want
        torch.cuda.empty_cache()


def test_config3_transformer_full(mods, lane):
    mpc, dealer, _ = mods
    rng = synth.rng_for(3)
    for li, L in enumerate(synth.config_transformer().layers):
        print(f"config 3 full: {L.name} {L.M}x{L.K}x{L.N} batch {L.batch}", flush=True)
        d = deal_matmul(rng, L.M, L.K, L.N, batch=L.batch if L.batch > 1 else None, x_std=L.x_std, w_std=L.w_std)
        z = lane.beaver_matmul(dev(mpc, d["x"]), dev(mpc, d["y"]), dev(mpc, d["a"]), dev(mpc, d["b"]), dev(mpc, d["c"]))
        lane.sync()
        want = oracle_matmul(d)
        assert_equal_shares(mpc, z, want, L.name)
        float_check(d, rec(want), conv=False)
        if L.relu:
            relu_sampled_check(mpc, dealer, lane, z, seed=300 + li)
        del d, z, want
        torch.cuda.empty_cache()


def test_config1_backward_full(mods, lane):
    """Both gradient products of the configs[1] convolution at full size, opened masks of the
    forward pass reused, and the ReLU backward on its 2 097 152 outputs: every share bit for bit."""
    mpc, dealer, _ = mods
    L = synth.config_vgg_block().layers[0]
    print("config 1 backward, full size", flush=True)
    rng = synth.rng_for(1, 5)
    X = synth.normal_fixed(rng, (L.B, L.H, L.W, L.Cin), L.x_std); Wt = synth.normal_fixed(rng, (L.KH, L.KW, L.Cin, L.Cout), L.w_std)
    G = synth.normal_fixed(rng, (L.B, L.Ho, L.Wo, L.Cout), 0.5)
    xs, ws, gs = (synth.share_additive(rng, v) for v in (X, Wt, G))
    fx = lambda g, w: oracle.ring_conv2d_grad_x(g, w, X.shape, L.pad, L.stride)
    fw = lambda x, g: oracle.ring_conv2d_grad_w(x, g, L.KH, L.KW, L.pad, L.stride)
    a, b, c = synth.deal_product_triple(rng, G.shape, Wt.shape, fx)
    want = oracle.truncate(oracle.beaver_bilinear(fx, gs, ws, a, b, c), 16)
    f_public = mpc.to_device((ws[0] - b[0]) + (ws[1] - b[1]))
    gx = lane.conv2d_grad_x(dev(mpc, gs), None, dev(mpc, a), dev(mpc, b), dev(mpc, c), L.pad, L.stride, f_public=f_public)
    lane.sync()
    assert_equal_shares(mpc, gx, want, "grad_x")
    a, b, c = synth.deal_product_triple(rng, X.shape, G.shape, fw)
    want = oracle.truncate(oracle.beaver_bilinear(fw, xs, gs, a, b, c), 16)
    e_public = mpc.to_device((xs[0] - a[0]) + (xs[1] - a[1]))
    gw = lane.conv2d_grad_w(None, dev(mpc, gs), dev(mpc, a), dev(mpc, b), dev(mpc, c), L.pad, L.stride, e_public=e_public)
    lane.sync()
    assert_equal_shares(mpc, gw, want, "grad_w")
    ref = torch.nn.functional.conv2d(torch.from_numpy(oracle.decode(X)).permute(3, 0, 1, 2),
                                     torch.from_numpy(oracle.decode(G)).permute(3, 0, 1, 2), padding=L.pad).permute(2, 3, 0, 1).numpy()
    assert np.abs(oracle.decode(rec(want)) - ref).max() <= 2.0 ** -12 * 4   # 16384-term sums of truncated products
    # ReLU backward
    n = G.size
    s = (rng.integers(0, 2, size=n) == 1)
    sa = synth.share_additive(rng, s.astype(U64))
    t = synth.deal_product_triple(rng, (n,), (n,), lambda p, q: p * q)
    gflat = (gs[0].reshape(-1), gs[1].reshape(-1))
    got = lane.relu_backward(dev(mpc, gflat), dev(mpc, sa), *[dev(mpc, q) for q in t])
    lane.sync()
    assert_equal_shares(mpc, got, oracle.relu_backward(gflat, sa, *t), "relu backward")


def test_config3_dense_backward_full(mods, lane):
    """x^T g and g w^T of the BERT-base output projection (4096 x 768 x 768) at full size."""
    mpc, dealer, _ = mods
    L = [l for l in synth.config_transformer().layers if l.name == "out"][0]
    print("config 3 dense backward, full size", flush=True)
    rng = synth.rng_for(3, 5)
    X = synth.normal_fixed(rng, (L.M, L.K), 1.0); Wt = synth.normal_fixed(rng, (L.K, L.N), L.w_std)
    G = synth.normal_fixed(rng, (L.M, L.N), 0.5)
    xs, ws, gs = (synth.share_additive(rng, v) for v in (X, Wt, G))
    tp = lambda pair: tuple(np.ascontiguousarray(p.T) for p in pair)
    a, b, c = synth.deal_product_triple(rng, (L.K, L.M), (L.M, L.N), oracle.ring_matmul)
    want = oracle.truncate(oracle.beaver_matmul(tp(xs), gs, a, b, c), 16)
    gw = lane.beaver_matmul(dev(mpc, xs), dev(mpc, gs), dev(mpc, tp(a)), dev(mpc, b), dev(mpc, c),
                            flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_X)
    lane.sync()
    assert_equal_shares(mpc, gw, want, "grad_w")
    a, bt, c = synth.deal_product_triple(rng, (L.M, L.N), (L.N, L.K), oracle.ring_matmul)
    want = oracle.truncate(oracle.beaver_matmul(gs, tp(ws), a, bt, c), 16)
    gx = lane.beaver_matmul(dev(mpc, gs), dev(mpc, ws), dev(mpc, a), dev(mpc, tp(bt)), dev(mpc, c),
                            flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_Y)
    lane.sync()
    assert_equal_shares(mpc, gx, want, "grad_x")


@pytest.mark.parametrize("packed_relu", [False, True], ids=["whole-word-relu", "sign-only-packed-relu"])
def test_config4_vgg16_pipeline_full(mods, packed_relu):
    """Batch 128 = 4 micro-batches of 32 through the whole VGG16-CIFAR network:
    the inter-batch pipeline (one lane per micro-batch) gives exactly the shares
    of the serial run, and every layer's reconstructed output equals the plain
    fixed-point layer on its reconstructed input (conv within +-1 ulp of the
    truncation, ReLU and max-pool exact)."""
    mpc, dealer, pipeline = mods
    wl = synth.config_vgg16_pipeline(32)
    layers = wl.layers
    n_mb = 4
    print("config 4 full: VGG16-CIFAR, 4 x 32 images", flush=True)
    lanes = [mpc.Lane(0) for _ in range(n_mb)]
    for ln in lanes:
        ln.use_single_queue()
    g = dealer.gen(synth.BASE_SEED + wl.index, lanes[0].device)
    weights = pipeline.deal_weights(g, layers, lanes[0].device)
    states, xs = [], []
    for m in range(n_mb):
        states.append(pipeline.deal_microbatch(lanes[m], g, layers, weights, packed_relu=packed_relu))
        xs.append(dealer.share(g, dealer.normal_fixed(g, (32, 32, 32, 3), 1.0, lanes[0].device)))
    torch.cuda.synchronize()
    keep_a, keep_b = [], []
    serial = [pipeline.forward(lanes[0], layers, states[m], xs[m], keep_a) for m in range(n_mb)]
    lanes[0].sync()
    piped = pipeline.forward_pipelined(lanes, layers, states, xs, keep_b)
    for ln in lanes:
        ln.sync()
    for m in range(n_mb):
        for i in range(2):
            assert torch.equal(serial[m][i], piped[m][i]), f"micro-batch {m}, party {i}: pipelined != serial"
    # layer-by-layer properties on micro-batch 0 (keep_a holds its intermediates first)
    x = xs[0]
    it = iter(keep_a)
    for L, st, (W, _) in zip(layers, states[0], weights):
        z = next(it)
        rx = (x[0] + x[1]); rz = (z[0] + z[1])
        if isinstance(L, synth.Conv):
            xin = rx.view(L.B, L.H, L.W, L.Cin).double().permute(0, 3, 1, 2)
            ref = torch.nn.functional.conv2d(xin.cpu(), W.double().permute(3, 2, 0, 1).cpu(), padding=L.pad).permute(0, 2, 3, 1)
        else:
            ref = rx.view(L.M, L.K).double().cpu() @ W.double().cpu()
        exact = torch.floor(ref / 65536.0)           # products are exact in float64 at these magnitudes
        diff = rz.view(ref.shape).cpu().double() - exact
        assert diff.min() >= 0 and diff.max() <= 1, f"{L.name}: truncated product off by {diff.min()}..{diff.max()}"
        x = z
        if st.relu is not None:
            y = next(it)
            assert torch.equal(y[0] + y[1], torch.clamp(rz, min=0)), f"{L.name}: relu"
            x = y
        if st.pool1 is not None:
            p = next(it)
            ry = (x[0] + x[1]).view(L.B, L.Ho // 2, 2, L.Wo // 2, 2, L.Cout)
            assert torch.equal((p[0] + p[1]), ry.amax(dim=(2, 4))), f"{L.name}: max-pool"
            x = p
    for ln in lanes:
        ln.close()


def test_config4_four_lanes_device_dealt_every_micro_batch_against_oracle(mods):
    """The benchmark's step as it is launched (batch 128 = 4 micro-batches of 32 on four lanes, folded prepared
    calls, remote-store exchange, outputs allocated ahead of the pass) on material dealt on the device: every
    micro-batch's shares, triples and ReLU / pool material are downloaded, the oracle runs the whole network on
    them, and every layer's output shares of all four micro-batches are compared word for word.  The device
    dealer forms C = A * B with the library's own ring product: for the first and the last convolution and the
    last dense layer the oracle recomputes C from the downloaded A and B."""
    from helpers import oracle_forward
    mpc, dealer, pipeline = mods
    wl = synth.config_vgg16_pipeline(32)
    layers = wl.layers
    n_mb = 4
    print("config 4, four lanes, device-dealt: dealing", flush=True)
    lanes = [mpc.Lane(0) for _ in range(n_mb)]
    for ln in lanes:
        ln.use_single_queue(); ln.set_exchange("put")
    g = dealer.gen(synth.BASE_SEED + wl.index + 500, lanes[0].device)
    weights = pipeline.deal_weights(g, layers, lanes[0].device)
    states, xs, outs = [], [], []
    for m in range(n_mb):
        st = pipeline.deal_microbatch(lanes[m], g, layers, weights)
        xs.append(dealer.share(g, dealer.normal_fixed(g, (32, 32, 32, 3), 1.0, lanes[0].device)))
        torch.cuda.synchronize()
        pipeline.prepare_layers(lanes[m], layers, st, fold=True)
        states.append(st); outs.append(pipeline.alloc_outputs(lanes[m], layers, st))
    for _ in range(2):                        # the second pass overwrites the first one's outputs in place
        pipeline.forward_pipelined(lanes, layers, states, xs, [], outs_per_mb=outs)
    for ln in lanes:
        ln.sync()
    h = lambda t: mpc.to_host(t)
    pair = lambda p: (h(p[0]), h(p[1]))

    def host_material(mat):
        if mat is None:
            return None
        n = mat["r"][0].numel()
        out = {k: pair(mat[k]) for k in ("r", "rb", "ra", "ma", "mb", "mc")}
        for k in ("and_a", "and_b", "and_c"):
            out[k] = tuple(h(mat[k][i].view(12, n)) for i in range(2))
        return out

    last_conv = max(i for i, L in enumerate(layers) if isinstance(L, synth.Conv))
    for m in range(n_mb):
        print(f"micro-batch {m}: download, oracle forward, compare", flush=True)
        host = []
        for li, (L, st) in enumerate(zip(layers, states[m])):
            host.append(dict(w=pair(st.w), a=pair(st.a), b=pair(st.b), c=pair(st.c), relu=host_material(st.relu),
                             pool1=host_material(st.pool1), pool2=host_material(st.pool2), pool_first=False))
            if li in (0, last_conv, len(layers) - 1):
                A, Bm = host[-1]["a"][0] + host[-1]["a"][1], host[-1]["b"][0] + host[-1]["b"][1]
                C = oracle.ring_conv2d(A, Bm, L.pad, L.stride) if isinstance(L, synth.Conv) else oracle.ring_matmul(A, Bm)
                assert np.array_equal(host[-1]["c"][0] + host[-1]["c"][1], C), f"micro-batch {m}, {L.name}: dealt C != A * B"
        want = oracle_forward(layers, host, pair(xs[m]))
        for li, (L, o) in enumerate(zip(layers, outs[m])):
            got = o["p"] if "p" in o else o["y"] if "y" in o else o["z"]
            assert_equal_shares(mpc, got, want[li], f"micro-batch {m}, layer {li} ({L.name})")
        del host, want
    for ln in lanes:
        ln.close()


def test_config4_one_micro_batch_every_share_against_oracle(mods, lane):
    """One micro-batch of config 4 at its full size (32 images) with inputs, triples and material
    dealt on the host: every layer's output shares, both parties, against the oracle word for word;
    the sign-only packed chain on the same material gives the same words."""
    from helpers import deal_network_host, oracle_forward
    mpc, dealer, pipeline = mods
    wl = synth.config_vgg16_pipeline(32)
    layers = wl.layers
    rng = synth.rng_for(wl.index, 21)
    print("config 4, 32 images: dealing on the host", flush=True)
    host, _ = deal_network_host(rng, layers)
    xs = synth.share_additive(rng, synth.normal_fixed(rng, (32, 32, 32, 3), 1.0))
    print("oracle forward", flush=True)
    want = oracle_forward(layers, host, xs)
    for packed in (False, True):
        print(f"device forward, packed={packed}", flush=True)
        x = dev(mpc, xs)
        keep = []
        for li, (L, st) in enumerate(zip(layers, host)):
            def mat(m):
                if m is None:
                    return None
                md = mpc.material_to_device(m)
                return lane.pack_material(md) if packed else md
            state = pipeline.LayerState(w=dev(mpc, st["w"]), a=dev(mpc, st["a"]), b=dev(mpc, st["b"]), c=dev(mpc, st["c"]),
                                        relu=mat(st["relu"]), pool1=mat(st["pool1"]), pool2=mat(st["pool2"]), packed=packed)
            x = pipeline.run_layer(lane, L, state, x, keep)
            lane.sync()
            assert_equal_shares(mpc, x, want[li], f"layer {li} ({L.name}), packed={packed}")
            keep.clear(); del state
            torch.cuda.empty_cache()


def test_config1_with_three_parties(mods, lane):
    """configs[1] at full size with three simulated parties: the convolution's three output shares
    against the oracle word for word (inputs and triple dealt on the host), then the masked rescale
    and the secure ReLU on device-dealt material: the oracle recomputes every element, plus the
    reconstruction properties."""
    mpc, dealer, _ = mods
    wl = synth.config_vgg_block(); L = wl.layers[0]
    rng = synth.rng_for(wl.index, 33)
    conv = lambda A, Bm: oracle.ring_conv2d(A, Bm, L.pad, L.stride)
    X = synth.normal_fixed(rng, (L.B, L.H, L.W, L.Cin), L.x_std)
    Wt = synth.normal_fixed(rng, (L.KH, L.KW, L.Cin, L.Cout), L.w_std)
    x, w = synth.share_additive3(rng, X), synth.share_additive3(rng, Wt)
    a, b, c = synth.deal_product_triple3(rng, X.shape, Wt.shape, conv)
    want = oracle.beaver_conv2d3(x, w, a, b, c, L.pad, L.stride)
    d3 = lambda tri: tuple(mpc.to_device(v) for v in tri)
    z = lane.conv2d3(d3(x), d3(w), d3(a), d3(b), d3(c), L.pad, L.stride)
    lane.sync()
    for i in range(3):
        assert np.array_equal(mpc.to_host(z[i]), want[i]), f"conv2d3 party {i}"
    # rescale
    n = z[0].numel()
    r, rt = synth.deal_trunc3_pair(rng, want[0].shape)
    want_t = oracle.truncate3(want, r, rt)
    t = lane.truncate3(z, d3(r), d3(rt)); lane.sync()
    for i in range(3):
        assert np.array_equal(mpc.to_host(t[i]), want_t[i]), f"truncate3 party {i}"
    ref = torch.nn.functional.conv2d(torch.from_numpy(oracle.decode(X)).permute(0, 3, 1, 2),
                                     torch.from_numpy(oracle.decode(Wt)).permute(3, 2, 0, 1), padding=L.pad, stride=L.stride)
    got = oracle.decode(want_t[0] + want_t[1] + want_t[2])
    assert np.abs(got - ref.permute(0, 2, 3, 1).numpy()).max() <= TOL
    # secure ReLU, material drawn on the device
    g = dealer.gen(4242, lane.device)
    mat = dealer.relu3_material(g, n, lane.device)
    y, sb, sa = lane.relu3(t, mat, want_sign=True); lane.sync()
    rz = (t[0] + t[1] + t[2]).view(-1); ry = (y[0] + y[1] + y[2]).view(-1)
    assert torch.equal(ry, torch.clamp(rz, min=0)), "rec(y) != max(rec(x), 0)"
    assert torch.equal((sb[0] ^ sb[1] ^ sb[2]).view(-1).bool(), rz < 0)
    assert torch.equal((sa[0] + sa[1] + sa[2]).view(-1), (rz < 0).to(torch.int64))
    # every element: the whole material is downloaded and the oracle recomputes the call
    take = lambda q: mpc.to_host(q.view(-1))
    take13 = lambda q: mpc.to_host(q.view(13, n))
    sub = {k: tuple(take(q) for q in mat[k]) for k in ("r0", "r1", "rb", "ra", "ma", "mb", "mc")}
    for k in ("and_a", "and_b", "and_c"):
        sub[k] = tuple(take13(q) for q in mat[k])
    res = oracle.relu3(tuple(take(q) for q in t), sub)
    for i in range(3):
        assert np.array_equal(take(y[i]), res.y[i].reshape(-1)), f"relu3, party {i}"
        assert np.array_equal(take(sa[i]), res.s_arith[i].reshape(-1)), f"relu3 sign shares, party {i}"
        assert np.array_equal(take(sb[i]), res.s_bit[i].reshape(-1)), f"relu3 sign bits, party {i}"
    # the sign-only chain on the same material, packed on the device: the same words everywhere
    # (whole-word run), and the oracle recomputation again
    yp, sbp, sap = lane.relu3(t, lane.pack_material3(mat), want_sign=True, packed=True); lane.sync()
    for i in range(3):
        assert torch.equal(yp[i], y[i]) and torch.equal(sbp[i], sb[i]) and torch.equal(sap[i], sa[i]), f"relu3 packed, party {i}"
        assert np.array_equal(take(yp[i]), res.y[i].reshape(-1)), f"relu3 packed, party {i}"
