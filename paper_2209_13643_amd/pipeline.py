"""Multi-layer secure forward pass and the inter-batch pipeline (Sec. 4.3).

A network is a list of `synth.Conv` / `synth.Gemm` layer descriptions.  Each
micro-batch runs on its own lane (one library context = one in-order queue with
its own workspace); layers are issued layer-major over the micro-batches, so
the MFMA-bound Beaver GEMM of one micro-batch executes while the HBM-bound
secure ReLU of another is streaming - the paper's two-thread linear /
non-linear overlap, realised with HIP queues instead of host threads.

Only call sequencing lives here: every protocol step is a library call.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

from . import dealer, mpc, synth


@dataclass
class LayerState:
    """Device-resident shares and offline material of one layer for one micro-batch."""
    w: tuple                      # weight shares (shared by all micro-batches)
    a: tuple
    b: tuple
    c: tuple
    f_public: torch.Tensor | None = None     # W - B opened ahead of time (Alg. 3)
    relu: dict | None = None
    pool1: dict | None = None
    pool2: dict | None = None
    packed: bool = False          # ReLU / pool material in the packed layout of mpc_relu_msb
    right: torch.Tensor | None = None   # prepared digit planes of f, b_0 + f, b_1 (prepare_layers)
    left: torch.Tensor | None = None    # prepared digit planes of a_0, a_1
    pool_first: bool = False      # pooled layer evaluated as ReLU(maxpool(z)): the ReLU material covers the pooled size
    c_fold: tuple | None = None   # (c_0 - a_0 b_0, c_1): addends of the folded prepared call (prepare_layers(fold=True))


def with_batch(layers, batch: int):
    """Copy of the layer list with the conv batch / FC row count set to `batch`."""
    out = []
    for L in layers:
        if isinstance(L, synth.Conv):
            out.append(synth.Conv(L.name, batch, L.H, L.W, L.Cin, L.Cout, L.KH, L.KW, L.pad, L.stride,
                                  L.x_std, L.w_std, L.relu, L.pool))
        else:
            out.append(synth.Gemm(L.name, batch, L.K, L.N, L.x_std, L.w_std, L.batch, L.relu))
    return out


def deal_weights(g, layers, device):
    """Additive shares of every layer's fixed-point weights."""
    ws = []
    for L in layers:
        shape = (L.KH, L.KW, L.Cin, L.Cout) if isinstance(L, synth.Conv) else (L.K, L.N)
        W = dealer.normal_fixed(g, shape, L.w_std, device)
        ws.append((W, dealer.share(g, W)))
    return ws


def deal_microbatch(lane: mpc.Lane, g, layers, weights, packed_relu: bool = False, pool_first: bool = False) -> list:
    """Triples and ReLU / pool material for one micro-batch (offline phase stand-in).
    packed_relu: material for the sign-only carry chain (mpc_relu_msb / mpc_maxpool2x2_msb).
    pool_first: layers with ReLU and max-pool are evaluated as ReLU(maxpool(z)) - the same function, since
    max and ReLU commute, on a quarter of the ReLU elements; their ReLU material is dealt for the pooled size."""
    dev = lane.device
    states = []
    for L, (W, wsh) in zip(layers, weights):
        if isinstance(L, synth.Conv):
            A = dealer.rand_words(g, (L.B, L.H, L.W, L.Cin), dev); Bm = dealer.rand_words(g, W.shape, dev)
            lane.wait_torch()            # A, Bm were written on torch's stream
            C = lane.ring_conv2d(A, Bm, L.pad, L.stride)
            n_out = L.B * L.Ho * L.Wo * L.Cout
        else:
            A = dealer.rand_words(g, (L.M, L.K), dev); Bm = dealer.rand_words(g, W.shape, dev)
            lane.wait_torch()
            C = lane.ring_matmul(A, Bm)
            n_out = L.M * L.N
        lane.sync()
        st = LayerState(w=wsh, a=dealer.share(g, A), b=dealer.share(g, Bm), c=dealer.share(g, C), packed=packed_relu)
        pooled = isinstance(L, synth.Conv) and L.pool
        st.pool_first = pool_first and pooled and L.relu
        if L.relu:
            n_relu = L.B * (L.Ho // 2) * (L.Wo // 2) * L.Cout if st.pool_first else n_out
            st.relu = dealer.relu_material(g, n_relu, dev, packed=packed_relu)
        if pooled:
            n_pool = L.B * (L.Ho // 2) * (L.Wo // 2) * L.Cout
            st.pool1 = dealer.relu_material(g, 2 * n_pool, dev, packed=packed_relu)
            st.pool2 = dealer.relu_material(g, n_pool, dev, packed=packed_relu)
        states.append(st)
    torch.cuda.synchronize(dev)
    return states


def preopen_weights(lane: mpc.Lane, states):
    """Alg. 3's early broadcast of the weight masks, ahead of the forward pass: open W - B of every layer."""
    for st in states:
        d = lane.sub(st.w, st.b)
        st.f_public = lane.open(d)
    lane.sync()


def prepare_layers(lane: mpc.Lane, layers, states, fold: bool = False):
    """Recode the input-independent operands of every layer once (the triples' [a_i] and, from the
    opened weight mask, f, b_0 + f, b_1) and keep their digit planes resident: run_layer then only
    masks, exchanges and recodes the activation.  Opens the weight masks first if that was not done.
    fold: also form party 0's folded addend c_0 - a_0 b_0, so that the online call contracts three
    ring products instead of four (MPC_FOLDED)."""
    if any(st.f_public is None for st in states):
        preopen_weights(lane, states)
    for L, st in zip(layers, states):
        if isinstance(L, synth.Conv):
            st.right, st.left = lane.prepare_conv2d(st.a, st.b, st.f_public, L.pad, L.stride)
            if fold:
                st.c_fold = (lane.fold_conv2d(st.a, st.b, st.c, L.pad, L.stride), st.c[1])
        else:
            st.right, st.left = lane.prepare_matmul(st.a, st.b, st.f_public)
            if fold:
                st.c_fold = (lane.fold_matmul(st.a, st.b, st.c), st.c[1])
    lane.sync()


def alloc_outputs(lane: mpc.Lane, layers, states):
    """Output tensors of every call of one forward pass on `lane`, allocated once: a pass that is given
    them (run_layer's `out`) allocates nothing, so a serving loop can reuse them step after step (a lane
    executes its calls in order: step k+1 overwrites a tensor only after step k's readers have run)."""
    dev = lane.device
    pair = lambda shape: tuple(torch.empty(shape, dtype=torch.int64, device=dev) for _ in range(2))
    bufs = []
    for L, st in zip(layers, states):
        if isinstance(L, synth.Conv):
            full, pooled = (L.B, L.Ho, L.Wo, L.Cout), (L.B, L.Ho // 2, L.Wo // 2, L.Cout)
        else:
            full, pooled = (L.M, L.N), None
        b = dict(z=pair(full))
        if st.pool1 is not None:
            b["p"] = pair(pooled)
        if st.relu is not None:
            b["y"] = pair(pooled if st.pool_first else full)
        bufs.append(b)
    return bufs


def run_layer(lane: mpc.Lane, L, st: LayerState, x, keep: list, n_chunks=1, relu_chunks=0, flags=mpc.MPC_TRUNCATE,
              out: dict | None = None):
    """One secure layer on one lane: linear (+ ReLU) (+ 2x2 max-pool).  Returns output shares.
    Every tensor the layer produces is appended to `keep`: the calls only enqueue work and torch's
    allocator knows nothing about the lane's queue, so nothing may be freed (and handed out again)
    before the caller has synchronised the lane.  With `out` (one entry of alloc_outputs) the calls
    write into those tensors instead and nothing is allocated."""
    o = out or {}
    y_arg = None if st.f_public is not None else st.w
    if isinstance(L, synth.Conv):
        xs = (x[0].view(L.B, L.H, L.W, L.Cin), x[1].view(L.B, L.H, L.W, L.Cin))
        if st.right is not None and st.c_fold is not None:
            z = lane.conv2d_prepared(xs, st.a, st.c_fold, st.right, st.left, L.KH, L.KW, L.pad, L.stride,
                                     n_chunks=n_chunks, flags=flags | mpc.MPC_FOLDED, out=o.get("z"))
        elif st.right is not None:
            z = lane.conv2d_prepared(xs, st.a, st.c, st.right, st.left, L.KH, L.KW, L.pad, L.stride,
                                     n_chunks=n_chunks, flags=flags, out=o.get("z"))
        else:
            z = lane.conv2d(xs, y_arg, st.a, st.b, st.c, L.pad, L.stride, f_public=st.f_public,
                            n_chunks=n_chunks, flags=flags, out=o.get("z"))
    else:
        xs = (x[0].view(L.M, L.K), x[1].view(L.M, L.K))
        if st.right is not None and st.c_fold is not None:
            z = lane.beaver_matmul_prepared(xs, st.a, st.c_fold, st.right, st.left, n_chunks=n_chunks,
                                            flags=flags | mpc.MPC_FOLDED, out=o.get("z"))
        elif st.right is not None:
            z = lane.beaver_matmul_prepared(xs, st.a, st.c, st.right, st.left, n_chunks=n_chunks, flags=flags, out=o.get("z"))
        else:
            z = lane.beaver_matmul(xs, y_arg, st.a, st.b, st.c, f_public=st.f_public, n_chunks=n_chunks, flags=flags,
                                   out=o.get("z"))
    outs = [z]
    if st.pool_first:
        z = lane.maxpool2x2(z, st.pool1, st.pool2, n_chunks=relu_chunks, packed=st.packed, out=o.get("p")); outs.append(z)
        z = lane.relu(z, st.relu, n_chunks=relu_chunks, packed=st.packed, out=o.get("y")); outs.append(z)
        if out is None:
            keep.extend(outs)
        return z
    if st.relu is not None:
        z = lane.relu(z, st.relu, n_chunks=relu_chunks, packed=st.packed, out=o.get("y")); outs.append(z)
    if st.pool1 is not None:
        z = lane.maxpool2x2(z, st.pool1, st.pool2, n_chunks=relu_chunks, packed=st.packed, out=o.get("p")); outs.append(z)
    if out is None:
        keep.extend(outs)
    return z


def forward(lane: mpc.Lane, layers, states, x, keep: list, outs=None, **kw):
    """All layers on one lane.  Every intermediate tensor is appended to `keep`:
    the calls only enqueue work, and torch's allocator knows nothing about the
    lane's queue, so nothing may be freed (and handed out again) until the
    caller has synchronised the lane.  `outs` (alloc_outputs): preallocated tensors instead."""
    for li, (L, st) in enumerate(zip(layers, states)):
        x = run_layer(lane, L, st, x, keep, out=outs[li] if outs is not None else None, **kw)
    return x


def forward_interlinear(lane: mpc.Lane, wlane: mpc.Lane, layers, states, x, keep: list, **kw):
    """Inter-linear pipeline across layers (Alg. 3, Sec. 4.1): the weight mask W - B of layer l+1 is
    opened on a second lane while layer l computes; the compute lane waits (on the device) for that
    opening only when it reaches layer l+1.  Same shares as forward()."""
    def open_mask(st):
        d = wlane.sub(st.w, st.b)
        st.f_public = wlane.open(d)
        keep.extend([d, st.f_public])
    open_mask(states[0])
    for li, (L, st) in enumerate(zip(layers, states)):
        lane.wait_for(wlane)                       # this layer's mask has arrived
        if li + 1 < len(layers):
            open_mask(states[li + 1])              # next layer's mask travels while this layer computes
        x = run_layer(lane, L, st, x, keep, **kw)
    return x


class ChunkedLinear:
    """One secure linear layer with real overlap inside the layer (Alg. 3, Sec. 4.1): the input's rows (images of a
    convolution, rows of a dense layer) are cut into chunks, and chunk k runs as a folded prepared call on
    lanes[k % len(lanes)].  A Beaver product is separable over the rows of its left operand, so every chunk is a
    complete call on its slices of x, a and c (the right-operand planes are shared), and the output words are those
    of the one-call layer; while one lane's call is in its MFMA-bound GEMM, the other lane's call masks, exchanges
    and recodes its chunk, which is HBM-bound.  Slices along the leading dimension are contiguous: nothing is copied.

    Offline (constructor): the right-operand planes once, and per chunk the planes of its a_1 rows; the folded addend
    c_0 - a_0 b_0 is formed for the whole layer and sliced."""

    def __init__(self, lanes, L, st: LayerState, n_chunks: int = 2):
        self.lanes, self.L, self.conv = list(lanes), L, isinstance(L, synth.Conv)
        rows = st.a[0].shape[0]
        if not self.conv and st.a[0].dim() != 2:
            raise ValueError("batched products are already many independent calls: run them on lanes as they are")
        if n_chunks < 1 or n_chunks > rows:
            raise ValueError("between one chunk and one chunk per row")
        l0 = self.lanes[0]
        if self.conv:
            self.right, _ = l0.prepare_conv2d(st.a, st.b, st.f_public, L.pad, L.stride, left=False)
            c0f = l0.fold_conv2d(st.a, st.b, st.c, L.pad, L.stride)
        else:
            self.right, _ = l0.prepare_matmul(st.a, st.b, st.f_public, left=False)
            c0f = l0.fold_matmul(st.a, st.b, st.c)
        self.c = (c0f, st.c[1])
        self.bounds = [rows * k // n_chunks for k in range(n_chunks + 1)]
        self.a, self.left = [], []
        for k in range(n_chunks):
            sl = slice(self.bounds[k], self.bounds[k + 1])
            a = (st.a[0][sl], st.a[1][sl])
            ln = self.lanes[k % len(self.lanes)]
            if self.conv:
                _, lp = ln.prepare_conv2d(a, st.b, None, L.pad, L.stride, right=False)
            else:
                _, lp = ln.prepare_matmul(a, st.b, None, right=False)
            self.a.append(a); self.left.append(lp)
        for ln in self.lanes:
            ln.sync()

    def __call__(self, x, out, after: mpc.Lane | None = None, flags=mpc.MPC_TRUNCATE):
        """Issue all chunks; `out` = (z_0, z_1) of the whole layer's shape.  `after`: the lane that produced x (every
        chunk lane waits for it on the device).  Call join() on the lane that consumes `out`."""
        L = self.L
        for ln in self.lanes if after is not None else ():
            if ln is not after:
                ln.wait_for(after)
        for k, (a, lp) in enumerate(zip(self.a, self.left)):
            sl = slice(self.bounds[k], self.bounds[k + 1])
            ln = self.lanes[k % len(self.lanes)]
            xs, cs, zs = (x[0][sl], x[1][sl]), (self.c[0][sl], self.c[1][sl]), (out[0][sl], out[1][sl])
            if self.conv:
                ln.conv2d_prepared(xs, a, cs, self.right, lp, L.KH, L.KW, L.pad, L.stride, flags=flags | mpc.MPC_FOLDED, out=zs)
            else:
                ln.beaver_matmul_prepared(xs, a, cs, self.right, lp, flags=flags | mpc.MPC_FOLDED, out=zs)
        return out

    def join(self, consumer: mpc.Lane):
        """The consumer's next call waits (on the device) for every chunk lane."""
        for ln in self.lanes:
            if ln is not consumer:
                consumer.wait_for(ln)


RELU_CHUNK_ELEMS = 1 << 20      # the library's default chunk of the whole-word conversions (one lane at a time)


def share_cache(lanes, on: bool = True):
    """Lanes that convert at the same time share the last-level cache: give each the default conversion chunk divided
    by their number (so that a chunk's exchanged words and carried state still fit their share), or restore the
    default.  Chunking never changes a result."""
    n = len(lanes)
    for ln in lanes:
        ln.set_relu_chunk(max(1 << 16, RELU_CHUNK_ELEMS // n) if on and n > 1 else 0)


def forward_pipelined(lanes, layers, states_per_mb, xs, keep: list, outs_per_mb=None, **kw):
    """Inter-batch pipeline: micro-batch m on lanes[m]; layer-major issue order."""
    cur = list(xs)
    share_cache(lanes)
    try:
        for li, L in enumerate(layers):
            for m, lane in enumerate(lanes):
                cur[m] = run_layer(lane, L, states_per_mb[m][li], cur[m], keep,
                                   out=outs_per_mb[m][li] if outs_per_mb is not None else None, **kw)
    finally:
        share_cache(lanes, False)           # chunk sizes are read when a call is issued: the lanes are back to the default
    return cur


# ------------------------------------------------------------------ three parties
@dataclass
class LayerState3:
    """One layer's shares and offline material for one micro-batch, three parties (triples of tensors)."""
    w: tuple
    a: tuple
    b: tuple
    c: tuple
    r: tuple                      # rescale pair: shares of r and of r >> 16
    rt: tuple
    f_public: torch.Tensor | None = None
    relu: dict | None = None
    pool1: dict | None = None
    pool2: dict | None = None
    packed: bool = False          # ReLU / pool material in the packed layout: sign-only chain (mpc_relu3_msb)
    pool_first: bool = False      # pooled layer evaluated as ReLU(maxpool(z)): the ReLU material covers the pooled size
    right: torch.Tensor | None = None   # prepared digit planes of f, b_0 + f, b_1, b_2 (prepare_layers3)
    left: torch.Tensor | None = None    # prepared digit planes of a_0, a_1, a_2


def deal_weights3(g, layers, device):
    ws = []
    for L in layers:
        shape = (L.KH, L.KW, L.Cin, L.Cout) if isinstance(L, synth.Conv) else (L.K, L.N)
        W = dealer.normal_fixed(g, shape, L.w_std, device)
        ws.append((W, dealer.share3(g, W)))
    return ws


def deal_microbatch3(lane: mpc.Lane, g, layers, weights, packed_relu: bool = False, pool_first: bool = False) -> list:
    """Triples, rescale pairs and ReLU / pool material of one micro-batch for three parties.
    packed_relu: material for the sign-only carry chain (mpc_relu3_msb / mpc_maxpool3_msb).
    pool_first: as in deal_microbatch (pooled layers run as ReLU(maxpool(z)))."""
    dev = lane.device
    states = []
    for L, (W, wsh) in zip(layers, weights):
        if isinstance(L, synth.Conv):
            A = dealer.rand_words(g, (L.B, L.H, L.W, L.Cin), dev); Bm = dealer.rand_words(g, W.shape, dev)
            lane.wait_torch()
            C = lane.ring_conv2d(A, Bm, L.pad, L.stride)
            n_out = L.B * L.Ho * L.Wo * L.Cout
        else:
            A = dealer.rand_words(g, (L.M, L.K), dev); Bm = dealer.rand_words(g, W.shape, dev)
            lane.wait_torch()
            C = lane.ring_matmul(A, Bm)
            n_out = L.M * L.N
        lane.sync()
        r = dealer.rand_words(g, C.shape, dev) & ((1 << 63) - 1)
        st = LayerState3(w=wsh, a=dealer.share3(g, A), b=dealer.share3(g, Bm), c=dealer.share3(g, C),
                         r=dealer.share3(g, r), rt=dealer.share3(g, r >> dealer.FRAC_BITS), packed=packed_relu)
        st.pool_first = pool_first and isinstance(L, synth.Conv) and L.pool and L.relu
        if L.relu:
            st.relu = dealer.relu3_material(g, n_out // 4 if st.pool_first else n_out, dev, packed=packed_relu)
        if isinstance(L, synth.Conv) and L.pool:
            n_pool = L.B * (L.Ho // 2) * (L.Wo // 2) * L.Cout
            st.pool1 = dealer.relu3_material(g, 2 * n_pool, dev, packed=packed_relu)
            st.pool2 = dealer.relu3_material(g, n_pool, dev, packed=packed_relu)
        states.append(st)
    torch.cuda.synchronize(dev)
    return states


def preopen_weights3(lane: mpc.Lane, states):
    """Alg. 3's early broadcast of the weight masks with three parties."""
    for st in states:
        st.f_public = lane.open3(lane.sub3(st.w, st.b))
    lane.sync()


def prepare_layers3(lane: mpc.Lane, layers, states):
    """prepare_layers for three parties: the planes of every layer's input-independent operands, recoded once."""
    if any(st.f_public is None for st in states):
        preopen_weights3(lane, states)
    for L, st in zip(layers, states):
        if isinstance(L, synth.Conv):
            st.right, st.left = lane.prepare_conv2d3(st.a, st.b, st.f_public, L.pad, L.stride)
        else:
            st.right, st.left = lane.prepare_matmul3(st.a, st.b, st.f_public)
    lane.sync()


def run_layer3(lane: mpc.Lane, L, st: LayerState3, x, keep: list):
    """One secure layer with three parties: linear, masked rescale (+ ReLU) (+ 2x2 max-pool)."""
    y_arg = None if st.f_public is not None else st.w
    if isinstance(L, synth.Conv):
        xs = tuple(v.view(L.B, L.H, L.W, L.Cin) for v in x)
        if st.right is not None:
            z = lane.conv2d3_prepared(xs, st.a, st.c, st.right, st.left, L.KH, L.KW, L.pad, L.stride)
        else:
            z = lane.conv2d3(xs, y_arg, st.a, st.b, st.c, L.pad, L.stride, f_public=st.f_public)
    else:
        xs = tuple(v.view(L.M, L.K) for v in x)
        if st.right is not None:
            z = lane.beaver_matmul3_prepared(xs, st.a, st.c, st.right, st.left)
        else:
            z = lane.beaver_matmul3(xs, y_arg, st.a, st.b, st.c, f_public=st.f_public)
    lane.truncate3(z, st.r, st.rt)
    outs = [z]
    if st.pool_first:
        z = lane.maxpool3(z, st.pool1, st.pool2, packed=st.packed); outs.append(z)
        z = lane.relu3(z, st.relu, packed=st.packed); outs.append(z)
        keep.extend(outs)
        return z
    if st.relu is not None:
        z = lane.relu3(z, st.relu, packed=st.packed); outs.append(z)
    if st.pool1 is not None:
        z = lane.maxpool3(z, st.pool1, st.pool2, packed=st.packed); outs.append(z)
    keep.extend(outs)
    return z


def forward3(lane: mpc.Lane, layers, states, x, keep: list):
    for L, st in zip(layers, states):
        x = run_layer3(lane, L, st, x, keep)
    return x


def forward_pipelined3(lanes, layers, states_per_mb, xs, keep: list):
    """Inter-batch pipeline with three parties: micro-batch m on lanes[m], layer-major issue order."""
    cur = list(xs)
    share_cache(lanes)
    try:
        for li, L in enumerate(layers):
            for m, lane in enumerate(lanes):
                cur[m] = run_layer3(lane, L, states_per_mb[m][li], cur[m], keep)
    finally:
        share_cache(lanes, False)
    return cur


# ------------------------------------------------------------------ training step
@dataclass
class BackwardState3:
    """Gradient triples and rescale pairs of one layer for one micro-batch, three parties."""
    gx: dict | None               # input gradient: a (mask of g), b (= forward weight mask), c, r, rt
    gw: dict                      # weight gradient: a (= forward activation mask), b (mask of g), c, r, rt
    relu_t: tuple | None = None
    pool_t1: tuple | None = None
    pool_t2: tuple | None = None


def deal_backward3(lane: mpc.Lane, g, layers, states) -> list:
    """deal_backward for three parties: the forward masks are reused, every gradient product
    gets a rescale pair of its own."""
    dev = lane.device
    out = []
    for li, (L, st) in enumerate(zip(layers, states)):
        A = st.a[0] + st.a[1] + st.a[2]; Bm = st.b[0] + st.b[1] + st.b[2]
        conv = isinstance(L, synth.Conv)
        gshape = (L.B, L.Ho, L.Wo, L.Cout) if conv else (L.M, L.N)
        n_out = A.new_empty(gshape).numel()
        Ag = dealer.rand_words(g, gshape, dev); Bg = dealer.rand_words(g, gshape, dev)
        lane.wait_torch()
        if conv:
            Cw = lane.ring_conv2d_grad_w(A, Bg, L.KH, L.KW, L.pad, L.stride)
            Cx = lane.ring_conv2d_grad_x(Ag, Bm, A.shape, L.pad, L.stride) if li > 0 else None
        else:
            AT = A.transpose(0, 1).contiguous(); BT = Bm.transpose(0, 1).contiguous()
            lane.wait_torch()
            Cw = lane.ring_matmul(AT, Bg)
            Cx = lane.ring_matmul(Ag, BT) if li > 0 else None
        lane.sync()
        rw, rtw = dealer.trunc3_pair(g, Cw.shape, dev)
        gx = None
        if Cx is not None:
            rx, rtx = dealer.trunc3_pair(g, Cx.shape, dev)
            gx = dict(a=dealer.share3(g, Ag), b=st.b, c=dealer.share3(g, Cx), r=rx, rt=rtx)
        bs = BackwardState3(gx=gx, gw=dict(a=st.a, b=dealer.share3(g, Bg), c=dealer.share3(g, Cw), r=rw, rt=rtw))
        if st.relu is not None:
            bs.relu_t = dealer.mul_triple3(g, n_out, dev)
        if st.pool1 is not None:
            n_pool = n_out // 4
            bs.pool_t1 = dealer.mul_triple3(g, 2 * n_pool, dev); bs.pool_t2 = dealer.mul_triple3(g, n_pool, dev)
        out.append(bs)
    torch.cuda.synchronize(dev)
    return out


def forward_train3(lane: mpc.Lane, layers, states, x, keep: list):
    """forward3 that keeps every layer's input shares and the sign shares of its conversions (the tape)."""
    tape = []
    for L, st in zip(layers, states):
        rec = dict(x=x)
        y_arg = None if st.f_public is not None else st.w
        if isinstance(L, synth.Conv):
            xs = tuple(v.view(L.B, L.H, L.W, L.Cin) for v in x)
            z = lane.conv2d3(xs, y_arg, st.a, st.b, st.c, L.pad, L.stride, f_public=st.f_public)
        else:
            xs = tuple(v.view(L.M, L.K) for v in x)
            z = lane.beaver_matmul3(xs, y_arg, st.a, st.b, st.c, f_public=st.f_public)
        lane.truncate3(z, st.r, st.rt)
        keep.append(z)
        if st.relu is not None:
            z, sb, sa = lane.relu3(z, st.relu, want_sign=True, packed=st.packed)
            rec["relu_sign"] = sa; keep.extend([z, sb, sa])
        if st.pool1 is not None:
            rec["pool_in_shape"] = tuple(z[0].shape)
            z, s1, s2 = lane.maxpool3(z, st.pool1, st.pool2, packed=st.packed, want_signs=True)
            rec["pool_signs"] = (s1, s2); keep.extend([z, s1, s2])
        tape.append(rec)
        x = z
    return x, tape


def backward3(lane: mpc.Lane, layers, states, bstates, tape, gout, keep: list):
    """backward for three parties: max-pool backward, ReLU backward, then the two gradient
    products of the layer, each followed by its masked rescale.  Returns the weight-gradient shares."""
    g = gout
    grads = [None] * len(layers)
    for li in range(len(layers) - 1, -1, -1):
        L, st, bs, rec = layers[li], states[li], bstates[li], tape[li]
        if st.pool1 is not None:
            B, H, W, C = rec["pool_in_shape"]
            gp = tuple(v.view(B, H // 2, W // 2, C) for v in g)
            g = lane.maxpool3_backward(gp, rec["pool_signs"][0], rec["pool_signs"][1], bs.pool_t1, bs.pool_t2, (B, H, W, C))
            keep.append(g)
        if st.relu is not None:
            g = lane.relu3_backward(tuple(v.reshape(-1) for v in g), rec["relu_sign"], *bs.relu_t)
            keep.append(g)
        x = rec["x"]
        w_arg = None if st.f_public is not None else st.w
        gx = None
        if isinstance(L, synth.Conv):
            gs = tuple(v.view(L.B, L.Ho, L.Wo, L.Cout) for v in g)
            xs = tuple(v.view(L.B, L.H, L.W, L.Cin) for v in x)
            gw = lane.conv2d3_grad_w(xs, gs, bs.gw["a"], bs.gw["b"], bs.gw["c"], L.pad, L.stride)
            if bs.gx is not None:
                gx = lane.conv2d3_grad_x(gs, w_arg, bs.gx["a"], bs.gx["b"], bs.gx["c"], L.pad, L.stride, f_public=st.f_public)
        else:
            gs = tuple(v.view(L.M, L.N) for v in g)
            xs = tuple(v.view(L.M, L.K) for v in x)
            gw = lane.beaver_matmul3(xs, gs, bs.gw["a"], bs.gw["b"], bs.gw["c"], flags=mpc.MPC_TRANS_X)
            if bs.gx is not None:
                gx = lane.beaver_matmul3(gs, w_arg, bs.gx["a"], bs.gx["b"], bs.gx["c"], f_public=st.f_public, flags=mpc.MPC_TRANS_Y)
        lane.truncate3(gw, bs.gw["r"], bs.gw["rt"])
        if gx is not None:
            lane.truncate3(gx, bs.gx["r"], bs.gx["rt"])
        grads[li] = gw
        keep.extend([gw, gx])
        g = gx
    return grads


def sgd_step3(lane: mpc.Lane, states, grads, lr_pairs, lr_shift: int):
    """w <- w - 2^-lr_shift * grad_w with three parties: one more masked rescale of the gradient
    (in place; lr_pairs[l] = the offline pair (r, r >> lr_shift) of layer l) and a local
    subtraction.  Weight masks opened ahead of time are opened again."""
    for st, gw, (r, rt) in zip(states, grads, lr_pairs):
        lane.truncate3(gw, r, rt, bits=lr_shift)
        lane.sub3(st.w, tuple(v.view(st.w[0].shape) for v in gw), out=st.w)
        if st.f_public is not None:
            st.f_public = lane.open3(lane.sub3(st.w, st.b))


@dataclass
class BackwardState:
    """Gradient triples of one layer for one micro-batch (offline material)."""
    gx: dict | None               # input gradient: a (mask of g), b (= forward weight mask), c
    gw: dict                      # weight gradient: a (= forward activation mask), b (mask of g), c
    relu_t: tuple | None = None   # element-wise triple of the ReLU backward
    pool_t1: tuple | None = None  # element-wise triples of the max-pool backward (2 n_out / n_out words)
    pool_t2: tuple | None = None


def deal_backward(lane: mpc.Lane, g, layers, states) -> list:
    """Gradient triples for every layer; the forward masks of weights and activations are
    reused, so the values opened in the forward pass serve again (Sec. 4.1, backward pass)."""
    dev = lane.device
    out = []
    for li, (L, st) in enumerate(zip(layers, states)):
        A = st.a[0] + st.a[1]; Bm = st.b[0] + st.b[1]
        conv = isinstance(L, synth.Conv)
        gshape = (L.B, L.Ho, L.Wo, L.Cout) if conv else (L.M, L.N)
        n_out = A.new_empty(gshape).numel()
        Ag = dealer.rand_words(g, gshape, dev); Bg = dealer.rand_words(g, gshape, dev)
        lane.wait_torch()
        if conv:
            Cw = lane.ring_conv2d_grad_w(A, Bg, L.KH, L.KW, L.pad, L.stride)
            Cx = lane.ring_conv2d_grad_x(Ag, Bm, A.shape, L.pad, L.stride) if li > 0 else None
        else:
            AT = A.transpose(0, 1).contiguous(); BT = Bm.transpose(0, 1).contiguous()
            lane.wait_torch()
            Cw = lane.ring_matmul(AT, Bg)
            Cx = lane.ring_matmul(Ag, BT) if li > 0 else None
        lane.sync()
        bs = BackwardState(gx=None if Cx is None else dict(a=dealer.share(g, Ag), b=st.b, c=dealer.share(g, Cx)),
                           gw=dict(a=st.a, b=dealer.share(g, Bg), c=dealer.share(g, Cw)))
        if st.relu is not None:
            bs.relu_t = dealer.mul_triple(g, n_out, dev)
        if st.pool1 is not None:
            n_pool = n_out // 4
            bs.pool_t1 = dealer.mul_triple(g, 2 * n_pool, dev); bs.pool_t2 = dealer.mul_triple(g, n_pool, dev)
        out.append(bs)
    torch.cuda.synchronize(dev)
    return out


def forward_train(lane: mpc.Lane, layers, states, x, keep: list, **kw):
    """Forward pass that keeps what the backward pass reuses: every layer's input
    shares and the sign shares of its ReLU / max-pool conversions (the tape)."""
    tape = []
    for L, st in zip(layers, states):
        rec = dict(x=x)
        y_arg = None if st.f_public is not None else st.w
        if isinstance(L, synth.Conv):
            xs = (x[0].view(L.B, L.H, L.W, L.Cin), x[1].view(L.B, L.H, L.W, L.Cin))
            z = lane.conv2d(xs, y_arg, st.a, st.b, st.c, L.pad, L.stride, f_public=st.f_public)
        else:
            xs = (x[0].view(L.M, L.K), x[1].view(L.M, L.K))
            z = lane.beaver_matmul(xs, y_arg, st.a, st.b, st.c, f_public=st.f_public)
        keep.append(z)
        if st.relu is not None:
            z, sb, sa = lane.relu(z, st.relu, want_sign=True, packed=st.packed, **kw)
            rec["relu_sign"] = sa; keep.extend([z, sb, sa])
        if st.pool1 is not None:
            rec["pool_in_shape"] = tuple(z[0].shape)
            z, s1, s2 = lane.maxpool2x2(z, st.pool1, st.pool2, packed=st.packed, want_signs=True)
            rec["pool_signs"] = (s1, s2); keep.extend([z, s1, s2])
        tape.append(rec)
        x = z
    return x, tape


def backward(lane: mpc.Lane, layers, states, bstates, tape, gout, keep: list):
    """Backward pass: per layer (last to first) max-pool backward, ReLU backward, then the
    weight gradient x^T g / Conv-gradient and the input gradient (Sec. 5.3).  Returns the
    list of weight-gradient shares, first layer first."""
    g = gout
    grads = [None] * len(layers)
    for li in range(len(layers) - 1, -1, -1):
        L, st, bs, rec = layers[li], states[li], bstates[li], tape[li]
        conv = isinstance(L, synth.Conv)
        if st.pool1 is not None:
            B, H, W, C = rec["pool_in_shape"]
            gp = (g[0].view(B, H // 2, W // 2, C), g[1].view(B, H // 2, W // 2, C))
            g = lane.maxpool2x2_backward(gp, rec["pool_signs"][0], rec["pool_signs"][1], bs.pool_t1, bs.pool_t2, (B, H, W, C))
            keep.append(g)
        if st.relu is not None:
            gf = (g[0].reshape(-1), g[1].reshape(-1))
            g = lane.relu_backward(gf, rec["relu_sign"], *bs.relu_t)
            keep.append(g)
        x = rec["x"]
        if conv:
            gs = (g[0].view(L.B, L.Ho, L.Wo, L.Cout), g[1].view(L.B, L.Ho, L.Wo, L.Cout))
            xs = (x[0].view(L.B, L.H, L.W, L.Cin), x[1].view(L.B, L.H, L.W, L.Cin))
            gw = lane.conv2d_grad_w(xs, gs, bs.gw["a"], bs.gw["b"], bs.gw["c"], L.pad, L.stride)
            gx = None
            if bs.gx is not None:
                gx = lane.conv2d_grad_x(gs, None if st.f_public is not None else st.w, bs.gx["a"], bs.gx["b"], bs.gx["c"],
                                        L.pad, L.stride, f_public=st.f_public)
        else:
            gs = (g[0].view(L.M, L.N), g[1].view(L.M, L.N))
            xs = (x[0].view(L.M, L.K), x[1].view(L.M, L.K))
            gw = lane.beaver_matmul(xs, gs, bs.gw["a"], bs.gw["b"], bs.gw["c"], flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_X)
            gx = None
            if bs.gx is not None:
                gx = lane.beaver_matmul(gs, None if st.f_public is not None else st.w, bs.gx["a"], bs.gx["b"], bs.gx["c"],
                                        f_public=st.f_public, flags=mpc.MPC_TRUNCATE | mpc.MPC_TRANS_Y)
        grads[li] = gw
        keep.extend([gw, gx])
        g = gx
    return grads


def sgd_step(lane: mpc.Lane, states, grads, lr_shift: int):
    """w <- w - 2^-lr_shift * grad_w on shares: a local truncation of the gradient (in
    place) and a local subtraction.  Weight masks opened ahead of time are opened again."""
    for st, gw in zip(states, grads):
        lane.truncate(gw, lr_shift)
        lane.sub(st.w, (gw[0].view(st.w[0].shape), gw[1].view(st.w[1].shape)), out=st.w)
        if st.f_public is not None:
            st.f_public = lane.open(lane.sub(st.w, st.b))
