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


def deal_microbatch(lane: mpc.Lane, g, layers, weights, packed_relu: bool = False) -> list:
    """Triples and ReLU / pool material for one micro-batch (offline phase stand-in).
    packed_relu: material for the sign-only carry chain (mpc_relu_msb / mpc_maxpool2x2_msb)."""
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
        if L.relu:
            st.relu = dealer.relu_material(g, n_out, dev, packed=packed_relu)
        if isinstance(L, synth.Conv) and L.pool:
            n_pool = L.B * (L.Ho // 2) * (L.Wo // 2) * L.Cout
            st.pool1 = dealer.relu_material(g, 2 * n_pool, dev, packed=packed_relu)
            st.pool2 = dealer.relu_material(g, n_pool, dev, packed=packed_relu)
        states.append(st)
    torch.cuda.synchronize(dev)
    return states


def preopen_weights(lane: mpc.Lane, states):
    """Alg. 3, lines 2-5, ahead of the forward pass: open W - B of every layer."""
    for st in states:
        d = lane.sub(st.w, st.b)
        st.f_public = lane.open(d)
    lane.sync()


def run_layer(lane: mpc.Lane, L, st: LayerState, x, n_chunks=1, relu_chunks=0, flags=mpc.MPC_TRUNCATE):
    """One secure layer on one lane: linear (+ ReLU) (+ 2x2 max-pool).  Returns output shares."""
    y_arg = None if st.f_public is not None else st.w
    if isinstance(L, synth.Conv):
        xs = (x[0].view(L.B, L.H, L.W, L.Cin), x[1].view(L.B, L.H, L.W, L.Cin))
        z = lane.conv2d(xs, y_arg, st.a, st.b, st.c, L.pad, L.stride, f_public=st.f_public,
                        n_chunks=n_chunks, flags=flags)
    else:
        xs = (x[0].view(L.M, L.K), x[1].view(L.M, L.K))
        z = lane.beaver_matmul(xs, y_arg, st.a, st.b, st.c, f_public=st.f_public, n_chunks=n_chunks, flags=flags)
    outs = [z]
    if st.relu is not None:
        z = lane.relu(z, st.relu, n_chunks=relu_chunks, packed=st.packed); outs.append(z)
    if st.pool1 is not None:
        z = lane.maxpool2x2(z, st.pool1, st.pool2, n_chunks=relu_chunks, packed=st.packed); outs.append(z)
    run_layer.last_intermediates = outs      # kept alive by the caller through `keep`
    return z


def forward(lane: mpc.Lane, layers, states, x, keep: list, **kw):
    """All layers on one lane.  Every intermediate tensor is appended to `keep`:
    the calls only enqueue work, and torch's allocator knows nothing about the
    lane's queue, so nothing may be freed (and handed out again) until the
    caller has synchronised the lane."""
    for L, st in zip(layers, states):
        x = run_layer(lane, L, st, x, **kw)
        keep.extend(run_layer.last_intermediates)
    return x


def forward_pipelined(lanes, layers, states_per_mb, xs, keep: list, **kw):
    """Inter-batch pipeline: micro-batch m on lanes[m]; layer-major issue order."""
    cur = list(xs)
    for li, L in enumerate(layers):
        for m, lane in enumerate(lanes):
            cur[m] = run_layer(lane, L, states_per_mb[m][li], cur[m], **kw)
            keep.extend(run_layer.last_intermediates)
    return cur
