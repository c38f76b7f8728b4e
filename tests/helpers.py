"""Shared dealing helpers for the parity tests: all inputs come from the seeded
generators, all triple products and expected values from the CPU oracle."""
import numpy as np

import oracle
from paper_2209_13643_amd import synth

U64 = np.uint64


def rec(pair):
    return np.asarray(pair[0], dtype=U64) + np.asarray(pair[1], dtype=U64)


def batched(fn):
    """Lift a 2-D product to a leading batch dimension."""
    def f(A, B):
        if A.ndim == 2:
            return fn(A, B)
        return np.stack([fn(A[i], B[i]) for i in range(A.shape[0])])
    return f


def deal_matmul(rng, M, K, N, batch=None, x_std=None, w_std=None):
    xs_shape = (M, K) if batch is None else (batch, M, K)
    ws_shape = (K, N) if batch is None else (batch, K, N)
    X = synth.rand_words(rng, xs_shape) if x_std is None else synth.normal_fixed(rng, xs_shape, x_std)
    Y = synth.rand_words(rng, ws_shape) if w_std is None else synth.normal_fixed(rng, ws_shape, w_std)
    xs, ys = synth.share_additive(rng, X), synth.share_additive(rng, Y)
    a, b, c = synth.deal_product_triple(rng, xs_shape, ws_shape, batched(oracle.ring_matmul))
    return dict(X=X, Y=Y, x=xs, y=ys, a=a, b=b, c=c)


def oracle_matmul(d, truncate_bits=16):
    """Oracle output shares for a dealt (possibly batched) Beaver matmul."""
    if d["X"].ndim == 2:
        z = oracle.beaver_matmul(d["x"], d["y"], d["a"], d["b"], d["c"])
    else:
        zs = [oracle.beaver_matmul(*[(d[k][0][i], d[k][1][i]) for k in ("x", "y", "a", "b", "c")])
              for i in range(d["X"].shape[0])]
        z = (np.stack([q[0] for q in zs]), np.stack([q[1] for q in zs]))
    return oracle.truncate(z, truncate_bits) if truncate_bits else z


def deal_conv(rng, B, H, W, Cin, Cout, KH, KW, pad, stride, x_std=None, w_std=None):
    X = synth.rand_words(rng, (B, H, W, Cin)) if x_std is None else synth.normal_fixed(rng, (B, H, W, Cin), x_std)
    Wt = synth.rand_words(rng, (KH, KW, Cin, Cout)) if w_std is None else \
        synth.normal_fixed(rng, (KH, KW, Cin, Cout), w_std)
    xs, ws = synth.share_additive(rng, X), synth.share_additive(rng, Wt)
    a, b, c = synth.deal_product_triple(rng, X.shape, Wt.shape,
                                        lambda A, Bf: oracle.ring_conv2d(A, Bf, pad, stride))
    return dict(X=X, Y=Wt, x=xs, y=ws, a=a, b=b, c=c, pad=pad, stride=stride)


def oracle_conv(d, truncate_bits=16):
    z = oracle.beaver_conv2d(d["x"], d["y"], d["a"], d["b"], d["c"], d["pad"], d["stride"])
    return oracle.truncate(z, truncate_bits) if truncate_bits else z


# ----------------------------------------------------------- whole networks (host)
def deal_network_host(rng, layers, weights=None, pool_first=False):
    """Per-layer shares / triples / material as numpy arrays for one micro-batch.
    `weights`: list of (W, (w0, w1)) to reuse across micro-batches, or None to draw them.
    `pool_first`: layers with ReLU and max-pool get their ReLU material at the pooled size."""
    states, wout = [], []
    for li, L in enumerate(layers):
        conv = isinstance(L, synth.Conv)
        wshape = (L.KH, L.KW, L.Cin, L.Cout) if conv else (L.K, L.N)
        if weights is None:
            W = synth.normal_fixed(rng, wshape, L.w_std); wsh = synth.share_additive(rng, W)
        else:
            W, wsh = weights[li]
        wout.append((W, wsh))
        if conv:
            prod = lambda A, Bf, L=L: oracle.ring_conv2d(A, Bf, L.pad, L.stride)
            a, b, c = synth.deal_product_triple(rng, (L.B, L.H, L.W, L.Cin), wshape, prod)
            n_out = L.B * L.Ho * L.Wo * L.Cout
        else:
            a, b, c = synth.deal_product_triple(rng, (L.M, L.K), wshape, oracle.ring_matmul)
            n_out = L.M * L.N
        st = dict(W=W, w=wsh, a=a, b=b, c=c, relu=None, pool1=None, pool2=None)
        st["pool_first"] = bool(pool_first and conv and L.pool and L.relu)
        if L.relu:
            st["relu"] = synth.deal_relu_material(rng, n_out // 4 if st["pool_first"] else n_out)
        if conv and L.pool:
            n_pool = L.B * (L.Ho // 2) * (L.Wo // 2) * L.Cout
            st["pool1"] = synth.deal_relu_material(rng, 2 * n_pool)
            st["pool2"] = synth.deal_relu_material(rng, n_pool)
        states.append(st)
    return states, wout


def oracle_forward(layers, states, x):
    """Oracle run of the whole network; returns the list of every layer's output shares."""
    outs = []
    for L, st in zip(layers, states):
        if isinstance(L, synth.Conv):
            xs = (x[0].reshape(L.B, L.H, L.W, L.Cin), x[1].reshape(L.B, L.H, L.W, L.Cin))
            z = oracle.truncate(oracle.beaver_conv2d(xs, st["w"], st["a"], st["b"], st["c"], L.pad, L.stride), 16)
        else:
            xs = (x[0].reshape(L.M, L.K), x[1].reshape(L.M, L.K))
            z = oracle.truncate(oracle.beaver_matmul(xs, st["w"], st["a"], st["b"], st["c"]), 16)
        if st.get("pool_first"):
            z = oracle.maxpool2x2(z, st["pool1"], st["pool2"])
            z = oracle.relu((z[0].reshape(-1), z[1].reshape(-1)), st["relu"]).y
            z = (z[0].reshape(L.B, L.Ho // 2, L.Wo // 2, L.Cout), z[1].reshape(L.B, L.Ho // 2, L.Wo // 2, L.Cout))
        else:
            if st["relu"] is not None:
                z = oracle.relu(z, st["relu"]).y
            if st["pool1"] is not None:
                z = oracle.maxpool2x2(z, st["pool1"], st["pool2"])
        outs.append(z)
        x = z
    return outs


# ------------------------------------------------ whole networks, three parties
def deal_network_host3(rng, layers, weights=None, pool_first=False):
    """deal_network_host for three parties: every share a triple, plus the rescale pair of every layer."""
    states, wout = [], []
    for li, L in enumerate(layers):
        conv = isinstance(L, synth.Conv)
        wshape = (L.KH, L.KW, L.Cin, L.Cout) if conv else (L.K, L.N)
        if weights is None:
            W = synth.normal_fixed(rng, wshape, L.w_std); wsh = synth.share_additive3(rng, W)
        else:
            W, wsh = weights[li]
        wout.append((W, wsh))
        if conv:
            prod = lambda A, Bf, L=L: oracle.ring_conv2d(A, Bf, L.pad, L.stride)
            a, b, c = synth.deal_product_triple3(rng, (L.B, L.H, L.W, L.Cin), wshape, prod)
            n_out = L.B * L.Ho * L.Wo * L.Cout
        else:
            a, b, c = synth.deal_product_triple3(rng, (L.M, L.K), wshape, oracle.ring_matmul)
            n_out = L.M * L.N
        r, rt = synth.deal_trunc3_pair(rng, c[0].shape)
        st = dict(W=W, w=wsh, a=a, b=b, c=c, r=r, rt=rt, relu=None, pool1=None, pool2=None)
        st["pool_first"] = bool(pool_first and conv and L.pool and L.relu)
        if L.relu:
            st["relu"] = synth.deal_relu3_material(rng, n_out // 4 if st["pool_first"] else n_out)
        if conv and L.pool:
            n_pool = L.B * (L.Ho // 2) * (L.Wo // 2) * L.Cout
            st["pool1"] = synth.deal_relu3_material(rng, 2 * n_pool)
            st["pool2"] = synth.deal_relu3_material(rng, n_pool)
        states.append(st)
    return states, wout


def oracle_forward3(layers, states, x):
    outs = []
    for L, st in zip(layers, states):
        if isinstance(L, synth.Conv):
            xs = tuple(v.reshape(L.B, L.H, L.W, L.Cin) for v in x)
            z = oracle.beaver_conv2d3(xs, st["w"], st["a"], st["b"], st["c"], L.pad, L.stride)
        else:
            xs = tuple(v.reshape(L.M, L.K) for v in x)
            z = oracle.beaver_matmul3(xs, st["w"], st["a"], st["b"], st["c"])
        z = oracle.truncate3(z, st["r"], st["rt"], 16)
        if st.get("pool_first"):
            z = oracle.maxpool2x2_3(z, st["pool1"], st["pool2"])
            z = oracle.relu3(z, st["relu"]).y
        else:
            if st["relu"] is not None:
                z = oracle.relu3(z, st["relu"]).y
            if st["pool1"] is not None:
                z = oracle.maxpool2x2_3(z, st["pool1"], st["pool2"])
        outs.append(z)
        x = z
    return outs


# ------------------------------------------------------- whole networks: training
def deal_backward_host(rng, layers, states):
    """Gradient triples per layer: forward masks of weights / activations reused."""
    mul = lambda p, q: p * q
    out = []
    for li, (L, st) in enumerate(zip(layers, states)):
        conv = isinstance(L, synth.Conv)
        A = rec(st["a"]); Bm = rec(st["b"])
        gshape = (L.B, L.Ho, L.Wo, L.Cout) if conv else (L.M, L.N)
        n_out = int(np.prod(gshape))
        Ag = synth.rand_words(rng, gshape); Bg = synth.rand_words(rng, gshape)
        if conv:
            Cw = oracle.ring_conv2d_grad_w(A, Bg, L.KH, L.KW, L.pad, L.stride)
            Cx = oracle.ring_conv2d_grad_x(Ag, Bm, A.shape, L.pad, L.stride) if li > 0 else None
        else:
            Cw = oracle.ring_matmul(np.ascontiguousarray(A.T), Bg)
            Cx = oracle.ring_matmul(Ag, np.ascontiguousarray(Bm.T)) if li > 0 else None
        bs = dict(gw=dict(a=st["a"], b=synth.share_additive(rng, Bg), c=synth.share_additive(rng, Cw)),
                  gx=None if Cx is None else dict(a=synth.share_additive(rng, Ag), b=st["b"], c=synth.share_additive(rng, Cx)),
                  relu_t=None, pool_t1=None, pool_t2=None)
        if st["relu"] is not None:
            bs["relu_t"] = synth.deal_product_triple(rng, (n_out,), (n_out,), mul)
        if st["pool1"] is not None:
            n_pool = n_out // 4
            bs["pool_t1"] = synth.deal_product_triple(rng, (2 * n_pool,), (2 * n_pool,), mul)
            bs["pool_t2"] = synth.deal_product_triple(rng, (n_pool,), (n_pool,), mul)
        out.append(bs)
    return out


def oracle_train_step(layers, states, bstates, x, gout):
    """Oracle forward (keeping inputs and sign shares) and backward; returns the final
    forward output and the per-layer weight-gradient shares."""
    tape = []
    for L, st in zip(layers, states):
        t = dict(x=x)
        if isinstance(L, synth.Conv):
            xs = (x[0].reshape(L.B, L.H, L.W, L.Cin), x[1].reshape(L.B, L.H, L.W, L.Cin))
            z = oracle.truncate(oracle.beaver_conv2d(xs, st["w"], st["a"], st["b"], st["c"], L.pad, L.stride), 16)
        else:
            xs = (x[0].reshape(L.M, L.K), x[1].reshape(L.M, L.K))
            z = oracle.truncate(oracle.beaver_matmul(xs, st["w"], st["a"], st["b"], st["c"]), 16)
        if st["relu"] is not None:
            r = oracle.relu(z, st["relu"]); z = r.y; t["relu_sign"] = r.s_arith
        if st["pool1"] is not None:
            t["pool_in_shape"] = z[0].shape
            z, s1, s2 = oracle.maxpool2x2(z, st["pool1"], st["pool2"], want_signs=True); t["pool_signs"] = (s1, s2)
        tape.append(t); x = z
    out = x
    g = gout
    grads = [None] * len(layers)
    tp = lambda pair: tuple(np.ascontiguousarray(p.T) for p in pair)
    for li in range(len(layers) - 1, -1, -1):
        L, st, bs, t = layers[li], states[li], bstates[li], tape[li]
        if st["pool1"] is not None:
            g = oracle.maxpool2x2_backward(g, t["pool_signs"][0], t["pool_signs"][1], bs["pool_t1"], bs["pool_t2"], t["pool_in_shape"])
        if st["relu"] is not None:
            g = oracle.relu_backward((g[0].reshape(-1), g[1].reshape(-1)), t["relu_sign"], *bs["relu_t"])
        xin = t["x"]
        if isinstance(L, synth.Conv):
            gs = (g[0].reshape(L.B, L.Ho, L.Wo, L.Cout), g[1].reshape(L.B, L.Ho, L.Wo, L.Cout))
            xs = (xin[0].reshape(L.B, L.H, L.W, L.Cin), xin[1].reshape(L.B, L.H, L.W, L.Cin))
            fw = lambda p, q, L=L: oracle.ring_conv2d_grad_w(p, q, L.KH, L.KW, L.pad, L.stride)
            gw = oracle.truncate(oracle.beaver_bilinear(fw, xs, gs, bs["gw"]["a"], bs["gw"]["b"], bs["gw"]["c"]), 16)
            gx = None
            if bs["gx"] is not None:
                fx = lambda p, q, L=L: oracle.ring_conv2d_grad_x(p, q, (L.B, L.H, L.W, L.Cin), L.pad, L.stride)
                gx = oracle.truncate(oracle.beaver_bilinear(fx, gs, st["w"], bs["gx"]["a"], bs["gx"]["b"], bs["gx"]["c"]), 16)
        else:
            gs = (g[0].reshape(L.M, L.N), g[1].reshape(L.M, L.N))
            xs = (xin[0].reshape(L.M, L.K), xin[1].reshape(L.M, L.K))
            gw = oracle.truncate(oracle.beaver_matmul(tp(xs), gs, tp(bs["gw"]["a"]), bs["gw"]["b"], bs["gw"]["c"]), 16)
            gx = None
            if bs["gx"] is not None:
                gx = oracle.truncate(oracle.beaver_matmul(gs, tp(st["w"]), bs["gx"]["a"], tp(bs["gx"]["b"]), bs["gx"]["c"]), 16)
        grads[li] = gw
        g = gx
    return out, grads


def deal_backward_host3(rng, layers, states):
    """deal_backward_host for three parties; every gradient product also gets a rescale pair."""
    mul = lambda p, q: p * q
    rec3 = lambda t: np.asarray(t[0], U64) + np.asarray(t[1], U64) + np.asarray(t[2], U64)
    out = []
    for li, (L, st) in enumerate(zip(layers, states)):
        conv = isinstance(L, synth.Conv)
        A = rec3(st["a"]); Bm = rec3(st["b"])
        gshape = (L.B, L.Ho, L.Wo, L.Cout) if conv else (L.M, L.N)
        n_out = int(np.prod(gshape))
        Ag = synth.rand_words(rng, gshape); Bg = synth.rand_words(rng, gshape)
        if conv:
            Cw = oracle.ring_conv2d_grad_w(A, Bg, L.KH, L.KW, L.pad, L.stride)
            Cx = oracle.ring_conv2d_grad_x(Ag, Bm, A.shape, L.pad, L.stride) if li > 0 else None
        else:
            Cw = oracle.ring_matmul(np.ascontiguousarray(A.T), Bg)
            Cx = oracle.ring_matmul(Ag, np.ascontiguousarray(Bm.T)) if li > 0 else None
        rw, rtw = synth.deal_trunc3_pair(rng, Cw.shape)
        bs = dict(gw=dict(a=st["a"], b=synth.share_additive3(rng, Bg), c=synth.share_additive3(rng, Cw), r=rw, rt=rtw),
                  gx=None, relu_t=None, pool_t1=None, pool_t2=None)
        if Cx is not None:
            rx, rtx = synth.deal_trunc3_pair(rng, Cx.shape)
            bs["gx"] = dict(a=synth.share_additive3(rng, Ag), b=st["b"], c=synth.share_additive3(rng, Cx), r=rx, rt=rtx)
        if st["relu"] is not None:
            bs["relu_t"] = synth.deal_product_triple3(rng, (n_out,), (n_out,), mul)
        if st["pool1"] is not None:
            n_pool = n_out // 4
            bs["pool_t1"] = synth.deal_product_triple3(rng, (2 * n_pool,), (2 * n_pool,), mul)
            bs["pool_t2"] = synth.deal_product_triple3(rng, (n_pool,), (n_pool,), mul)
        out.append(bs)
    return out


def oracle_train_step3(layers, states, bstates, x, gout):
    """oracle_train_step for three parties: forward with the tape, backward with a masked
    rescale after every gradient product."""
    tape = []
    for L, st in zip(layers, states):
        t = dict(x=x)
        if isinstance(L, synth.Conv):
            xs = tuple(v.reshape(L.B, L.H, L.W, L.Cin) for v in x)
            z = oracle.beaver_conv2d3(xs, st["w"], st["a"], st["b"], st["c"], L.pad, L.stride)
        else:
            xs = tuple(v.reshape(L.M, L.K) for v in x)
            z = oracle.beaver_matmul3(xs, st["w"], st["a"], st["b"], st["c"])
        z = oracle.truncate3(z, st["r"], st["rt"], 16)
        if st["relu"] is not None:
            r = oracle.relu3(z, st["relu"]); z = r.y; t["relu_sign"] = r.s_arith
        if st["pool1"] is not None:
            t["pool_in_shape"] = z[0].shape
            z, s1, s2 = oracle.maxpool2x2_3(z, st["pool1"], st["pool2"], want_signs=True); t["pool_signs"] = (s1, s2)
        tape.append(t); x = z
    out = x
    g = gout
    grads = [None] * len(layers)
    for li in range(len(layers) - 1, -1, -1):
        L, st, bs, t = layers[li], states[li], bstates[li], tape[li]
        if st["pool1"] is not None:
            g = oracle.maxpool2x2_backward3(g, t["pool_signs"][0], t["pool_signs"][1], bs["pool_t1"], bs["pool_t2"], t["pool_in_shape"])
        if st["relu"] is not None:
            g = oracle.relu_backward3(tuple(v.reshape(-1) for v in g), t["relu_sign"], *bs["relu_t"])
        xin = t["x"]
        if isinstance(L, synth.Conv):
            gs = tuple(v.reshape(L.B, L.Ho, L.Wo, L.Cout) for v in g)
            xs = tuple(v.reshape(L.B, L.H, L.W, L.Cin) for v in xin)
            fw = lambda p, q, L=L: oracle.ring_conv2d_grad_w(p, q, L.KH, L.KW, L.pad, L.stride)
            fx = lambda p, q, L=L: oracle.ring_conv2d_grad_x(p, q, (L.B, L.H, L.W, L.Cin), L.pad, L.stride)
        else:
            gs = tuple(v.reshape(L.M, L.N) for v in g)
            xs = tuple(v.reshape(L.M, L.K) for v in xin)
            fw = lambda p, q: oracle.ring_matmul(np.ascontiguousarray(p.T), q)
            fx = lambda p, q: oracle.ring_matmul(p, np.ascontiguousarray(q.T))
        gw = oracle.truncate3(oracle.beaver_bilinear3(fw, xs, gs, bs["gw"]["a"], bs["gw"]["b"], bs["gw"]["c"]),
                              bs["gw"]["r"], bs["gw"]["rt"], 16)
        gx = None
        if bs["gx"] is not None:
            gx = oracle.truncate3(oracle.beaver_bilinear3(fx, gs, st["w"], bs["gx"]["a"], bs["gx"]["b"], bs["gx"]["c"]),
                                  bs["gx"]["r"], bs["gx"]["rt"], 16)
        grads[li] = gw
        g = gx
    return out, grads
