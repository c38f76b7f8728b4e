"""Device-side synthetic dealer: the stand-in for the offline phase.

Produces, directly in HBM, the inputs of the online phase for a workload:
additive shares of fixed-point tensors, Beaver triples (C = A*B through the
library's own plain ring product, `mpc_ring_matmul` / `mpc_ring_conv2d`), and
secure-ReLU material.  Everything here runs before the timed region; the paper
excludes the offline phase from its measurements as well (Sec. 5.2, Sec. 5.9).
torch is used as a random-number source and for the element-wise relations the
material has to satisfy; none of this is on the online path.
"""
from __future__ import annotations

import math

import torch

from . import mpc

FRAC_BITS = 16


def gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def rand_words(g, shape, device):
    """Uniform 64-bit words (as int64 bit patterns)."""
    hi = torch.randint(-(1 << 31), 1 << 31, shape, generator=g, device=device, dtype=torch.int64)
    lo = torch.randint(0, 1 << 32, shape, generator=g, device=device, dtype=torch.int64)
    return (hi << 32) | lo


def normal_fixed(g, shape, std, device):
    v = torch.randn(shape, generator=g, device=device, dtype=torch.float64) * std
    return torch.round(v * float(1 << FRAC_BITS)).to(torch.int64)


def share(g, value):
    """Additive shares.  Like everything in this module the result is produced by
    torch on torch's current stream: synchronise (or Lane.wait_torch()) before a
    lane reads it."""
    s0 = rand_words(g, value.shape, value.device)
    return s0, value - s0


def share_xor(g, value):
    s0 = rand_words(g, value.shape, value.device)
    return s0, value ^ s0


def conv_layer(lane: "mpc.Lane", g, B, H, W, Cin, Cout, KH, KW, pad, stride, x_std, w_std):
    dev = lane.device
    X = normal_fixed(g, (B, H, W, Cin), x_std, dev)
    Wt = normal_fixed(g, (KH, KW, Cin, Cout), w_std, dev)
    A = rand_words(g, X.shape, dev); Bm = rand_words(g, Wt.shape, dev)
    lane.wait_torch()                # A, Bm were written on torch's stream
    C = lane.ring_conv2d(A, Bm, pad, stride)
    lane.sync()
    d = dict(X=X, W=Wt, x=share(g, X), w=share(g, Wt), a=share(g, A), b=share(g, Bm), c=share(g, C))
    d["f_public"] = Wt - Bm          # epsilon = W - B, opened ahead of time (Alg. 3)
    torch.cuda.synchronize(dev)
    return d


def matmul_layer(lane: "mpc.Lane", g, M, K, N, x_std, w_std, batch=None):
    dev = lane.device
    xs = (M, K) if batch is None else (batch, M, K)
    ws = (K, N) if batch is None else (batch, K, N)
    X = normal_fixed(g, xs, x_std, dev); Wt = normal_fixed(g, ws, w_std, dev)
    A = rand_words(g, xs, dev); Bm = rand_words(g, ws, dev)
    lane.wait_torch()
    C = lane.ring_matmul(A, Bm)
    lane.sync()
    d = dict(X=X, W=Wt, x=share(g, X), w=share(g, Wt), a=share(g, A), b=share(g, Bm), c=share(g, C))
    d["f_public"] = Wt - Bm
    torch.cuda.synchronize(dev)
    return d


def conv_backward(lane: "mpc.Lane", g, fwd: dict, pad: int, stride: int, g_std: float = 0.5) -> dict:
    """Output-gradient shares and the two gradient triples of a conv layer dealt by
    conv_layer: the input-gradient triple reuses the forward weight mask (so the
    opened W - B serves again), the filter-gradient triple the forward activation mask."""
    dev = lane.device
    A = fwd["a"][0] + fwd["a"][1]; Bm = fwd["b"][0] + fwd["b"][1]
    KH, KW = Bm.shape[0], Bm.shape[1]
    G = normal_fixed(g, fwd["c"][0].shape, g_std, dev)
    Ag = rand_words(g, G.shape, dev); Bg = rand_words(g, G.shape, dev)
    lane.wait_torch()
    d = dict(G=G, g=share(g, G))
    if KH == KW:
        Cx = lane.ring_conv2d_grad_x(Ag, Bm, A.shape, pad, stride); lane.sync()
        d["gx"] = dict(a=share(g, Ag), b=fwd["b"], c=share(g, Cx), f_public=fwd["f_public"])
    Cw = lane.ring_conv2d_grad_w(A, Bg, KH, KW, pad, stride); lane.sync()
    d["gw"] = dict(a=fwd["a"], b=share(g, Bg), c=share(g, Cw), e_public=fwd["X"] - A)
    torch.cuda.synchronize(dev)
    return d


def matmul_backward(lane: "mpc.Lane", g, fwd: dict, g_std: float = 0.5) -> dict:
    """The same for a dense layer dealt by matmul_layer (2-D or batched):
    grad_x = g w^T (triple A_g, B^T -> C), grad_w = x^T g (triple A^T, B_g -> C)."""
    dev = lane.device
    A = fwd["a"][0] + fwd["a"][1]; Bm = fwd["b"][0] + fwd["b"][1]
    G = normal_fixed(g, fwd["c"][0].shape, g_std, dev)
    Ag = rand_words(g, G.shape, dev); Bg = rand_words(g, G.shape, dev)
    BmT = Bm.transpose(-1, -2).contiguous(); AT = A.transpose(-1, -2).contiguous()
    lane.wait_torch()
    Cx = lane.ring_matmul(Ag, BmT); lane.sync()
    Cw = lane.ring_matmul(AT, Bg); lane.sync()
    d = dict(G=G, g=share(g, G),
             gx=dict(a=share(g, Ag), b=fwd["b"], c=share(g, Cx), f_public=fwd["f_public"]),
             gw=dict(a=fwd["a"], b=share(g, Bg), c=share(g, Cw)))
    torch.cuda.synchronize(dev)
    return d


def mul_triple(g, n: int, device):
    """Element-wise multiplication triple on n words."""
    a = rand_words(g, (n,), device); b = rand_words(g, (n,), device)
    t = (share(g, a), share(g, b), share(g, a * b))
    torch.cuda.synchronize(device)
    return t


def relu_material(g, n: int, device, packed: bool = False) -> dict:
    """Secure-ReLU material for n elements.  packed=True draws the AND triples
    directly in the packed layout of mpc_relu_msb (uniform words satisfy the
    bit-wise triple relation in any layout)."""
    m = {}
    m["r"] = (rand_words(g, (n,), device), rand_words(g, (n,), device))
    tshape = (mpc.lib().mpc_relu_packed_words(n),) if packed else (mpc.N_AND_TRIPLES, n)
    a = (rand_words(g, tshape, device), rand_words(g, tshape, device))
    b = (rand_words(g, tshape, device), rand_words(g, tshape, device))
    m["and_a"], m["and_b"] = a, b
    m["and_c"] = share_xor(g, (a[0] ^ a[1]) & (b[0] ^ b[1]))
    rb = tuple(torch.randint(0, 2, (n,), generator=g, device=device, dtype=torch.uint8) for _ in range(2))
    m["rb"] = rb
    m["ra"] = share(g, (rb[0] ^ rb[1]).to(torch.int64))
    ma = (rand_words(g, (n,), device), rand_words(g, (n,), device))
    mb = (rand_words(g, (n,), device), rand_words(g, (n,), device))
    m["ma"], m["mb"] = ma, mb
    m["mc"] = share(g, (ma[0] + ma[1]) * (mb[0] + mb[1]))
    torch.cuda.synchronize(device)      # torch filled these on its own stream; the lanes use theirs
    return m


# ---------------------------------------------------------------- three parties
def share3(g, value):
    s0 = rand_words(g, value.shape, value.device); s1 = rand_words(g, value.shape, value.device)
    return s0, s1, value - s0 - s1


def share_xor3(g, value):
    s0 = rand_words(g, value.shape, value.device); s1 = rand_words(g, value.shape, value.device)
    return s0, s1, value ^ s0 ^ s1


def conv_layer3(lane: "mpc.Lane", g, B, H, W, Cin, Cout, KH, KW, pad, stride, x_std, w_std):
    """A convolution layer's inputs, triple and rescale pair for three parties."""
    dev = lane.device
    X = normal_fixed(g, (B, H, W, Cin), x_std, dev)
    Wt = normal_fixed(g, (KH, KW, Cin, Cout), w_std, dev)
    A = rand_words(g, X.shape, dev); Bm = rand_words(g, Wt.shape, dev)
    lane.wait_torch()
    C = lane.ring_conv2d(A, Bm, pad, stride)
    lane.sync()
    d = dict(X=X, W=Wt, x=share3(g, X), w=share3(g, Wt), a=share3(g, A), b=share3(g, Bm), c=share3(g, C))
    r = rand_words(g, C.shape, dev) & ((1 << 63) - 1)          # uniform in [0, 2^63)
    d["r"], d["rt"] = share3(g, r), share3(g, r >> FRAC_BITS)
    torch.cuda.synchronize(dev)
    return d


def relu3_material(g, n: int, device, packed: bool = False) -> dict:
    """Three-party secure-ReLU material for n elements (13 AND triples, two A2B masks per party).
    packed=True draws the AND triples directly in the packed layout of mpc_relu3_msb (uniform
    words satisfy the bit-wise triple relation in any layout)."""
    w = lambda shape: rand_words(g, shape, device)
    m = {"r0": tuple(w((n,)) for _ in range(3)), "r1": tuple(w((n,)) for _ in range(3))}
    tshape = (mpc.lib().mpc_relu3_packed_words(n),) if packed else (mpc.N_AND_TRIPLES3, n)
    A, Bm = w(tshape), w(tshape)
    m["and_a"], m["and_b"], m["and_c"] = share_xor3(g, A), share_xor3(g, Bm), share_xor3(g, A & Bm)
    bits = [torch.randint(0, 2, (n,), generator=g, device=device, dtype=torch.uint8) for _ in range(3)]
    m["rb"] = tuple(bits)
    m["ra"] = share3(g, (bits[0] ^ bits[1] ^ bits[2]).to(torch.int64))
    MA, MB = w((n,)), w((n,))
    m["ma"], m["mb"], m["mc"] = share3(g, MA), share3(g, MB), share3(g, MA * MB)
    torch.cuda.synchronize(device)
    return m


def mul_triple3(g, n: int, device):
    """Element-wise multiplication triple on n words, three parties."""
    a = rand_words(g, (n,), device); b = rand_words(g, (n,), device)
    t = (share3(g, a), share3(g, b), share3(g, a * b))
    torch.cuda.synchronize(device)
    return t


def trunc3_pair(g, shape, device, bits: int = FRAC_BITS):
    """Offline pair of the three-party rescale: shares of r in [0, 2^63) and of r >> bits."""
    r = rand_words(g, shape, device) & ((1 << 63) - 1)
    return share3(g, r), share3(g, r >> bits)


def he_std(fan_in: int) -> float:
    return math.sqrt(2.0 / fan_in)
