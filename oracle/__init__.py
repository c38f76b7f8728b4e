"""CPU oracle for the secure-layer hot path (two parties, ring Z_2^64; the
three-party forms of Alg. 1 / Alg. 2 at the end).

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``; never by the GPU library or its
Python binding.  The arithmetic lives in ``mpc_oracle.c`` (plain C, uint64
wrap-around, straight loops); this module is a ctypes shim plus a handful of
plain-definition checkers on reconstructed values and a second, independent
adder form (the divide-and-conquer prefix tree of the paper's Sec. 4.2 listing)
used only to cross-check the Kogge-Stone form.

Parity status: values of individual shares are not fixed by the paper (it prints
no worked example), so share bit patterns are "parity unpinned" by the paper
itself; every function here is pinned by identities, closed forms, exhaustive
enumeration and library special cases in ``tests/test_oracle_*.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mpc_oracle.c")
_LIB = os.path.join(_HERE, "libmpc_oracle.so")

U64 = np.uint64
_P64 = ctypes.POINTER(ctypes.c_uint64)
_P8 = ctypes.POINTER(ctypes.c_uint8)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (portable x86-64-v3 code, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(
            ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC",
             "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    """The compiled oracle.  MPC_ORACLE_LIB names another build of mpc_oracle.c to load instead: the
    mutation test points it at copies with a planted mistake, to show that the pins notice."""
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(os.environ.get("MPC_ORACLE_LIB") or build())
    return _lib


def _w(a):
    a = np.ascontiguousarray(a, dtype=U64)
    return a, a.ctypes.data_as(_P64)


def _b(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(_P8)


def n_threads() -> int:
    """Threads the OpenMP loops will use (OMP_NUM_THREADS or all cores)."""
    v = os.environ.get("OMP_NUM_THREADS")
    return int(v) if v else (os.cpu_count() or 1)


# --------------------------------------------------------------------- ring ops
def ring_matmul(L, R):
    """Z = L @ R mod 2^64 (plain definition)."""
    L, pl = _w(L); R, pr = _w(R)
    M, K = L.shape; K2, N = R.shape
    assert K == K2
    Z = np.empty((M, N), dtype=U64)
    lib().orc_ring_matmul(pl, pr, Z.ctypes.data_as(_P64), M, K, N)
    return Z


def conv_out_hw(H, W, KH, KW, pad, stride):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def ring_conv2d(x, w, pad, stride):
    """Direct NHWC x [KH,KW,Cin,Cout] cross-correlation mod 2^64, zero padding."""
    x, px = _w(x); w, pw = _w(w)
    B, H, W, Cin = x.shape; KH, KW, Cin2, Cout = w.shape
    assert Cin == Cin2
    Ho, Wo = conv_out_hw(H, W, KH, KW, pad, stride)
    z = np.empty((B, Ho, Wo, Cout), dtype=U64)
    lib().orc_ring_conv2d(px, pw, z.ctypes.data_as(_P64), B, H, W, Cin, Cout, KH, KW, pad, stride)
    return z


def im2col(x, KH, KW, pad, stride):
    x, px = _w(x)
    B, H, W, Cin = x.shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, pad, stride)
    col = np.empty((B * Ho * Wo, KH * KW * Cin), dtype=U64)
    lib().orc_im2col(px, col.ctypes.data_as(_P64), B, H, W, Cin, KH, KW, pad, stride)
    return col


# --------------------------------------------------------------- Alg. 1 / Eq. 3
def open_shares(s0, s1):
    """Reconstruct a two-party additive sharing (Sec. 3.1)."""
    s0, p0 = _w(s0); s1, p1 = _w(s1)
    out = np.empty_like(s0)
    lib().orc_open(p0, p1, out.ctypes.data_as(_P64), s0.size)
    return out


def beaver_matmul(x, y, a, b, c, want_open=False):
    """Alg. 1 on matrices.  x, y, a, b, c are pairs (party 0, party 1)."""
    (x0, px0), (x1, px1) = _w(x[0]), _w(x[1])
    (y0, py0), (y1, py1) = _w(y[0]), _w(y[1])
    (a0, pa0), (a1, pa1) = _w(a[0]), _w(a[1])
    (b0, pb0), (b1, pb1) = _w(b[0]), _w(b[1])
    (c0, pc0), (c1, pc1) = _w(c[0]), _w(c[1])
    M, K = x0.shape; _, N = y0.shape
    z0 = np.empty((M, N), dtype=U64); z1 = np.empty((M, N), dtype=U64)
    e = np.empty((M, K), dtype=U64) if want_open else None
    f = np.empty((K, N), dtype=U64) if want_open else None
    lib().orc_beaver_matmul(px0, px1, py0, py1, pa0, pa1, pb0, pb1, pc0, pc1,
                            z0.ctypes.data_as(_P64), z1.ctypes.data_as(_P64), M, K, N,
                            e.ctypes.data_as(_P64) if want_open else None,
                            f.ctypes.data_as(_P64) if want_open else None)
    return ((z0, z1), e, f) if want_open else (z0, z1)


def beaver_conv2d(x, w, a, b, c, pad, stride):
    """Eq. 3: Alg. 1 with Conv as the product.  NHWC / [KH,KW,Cin,Cout]."""
    (x0, px0), (x1, px1) = _w(x[0]), _w(x[1])
    (w0, pw0), (w1, pw1) = _w(w[0]), _w(w[1])
    (a0, pa0), (a1, pa1) = _w(a[0]), _w(a[1])
    (b0, pb0), (b1, pb1) = _w(b[0]), _w(b[1])
    (c0, pc0), (c1, pc1) = _w(c[0]), _w(c[1])
    B, H, W, Cin = x0.shape; KH, KW, _, Cout = w0.shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, pad, stride)
    z0 = np.empty((B, Ho, Wo, Cout), dtype=U64); z1 = np.empty_like(z0)
    lib().orc_beaver_conv2d(px0, px1, pw0, pw1, pa0, pa1, pb0, pb1, pc0, pc1,
                            z0.ctypes.data_as(_P64), z1.ctypes.data_as(_P64),
                            B, H, W, Cin, Cout, KH, KW, pad, stride)
    return z0, z1


def truncate(z, bits=16):
    """Local two-party truncation; returns new arrays."""
    z0 = np.array(z[0], dtype=U64, copy=True); z1 = np.array(z[1], dtype=U64, copy=True)
    lib().orc_truncate(z0.ctypes.data_as(_P64), z1.ctypes.data_as(_P64), z0.size, bits)
    return z0, z1


# ---------------------------------------------------------------- backward pass
def ring_conv2d_grad_x(g, w, x_shape, pad, stride):
    """Gradient of ring_conv2d w.r.t. its input: the transpose of the forward sum."""
    g, pg = _w(g); w, pw = _w(w)
    B, H, W, Cin = x_shape; KH, KW, Cin2, Cout = w.shape
    assert Cin == Cin2 and g.shape == (B,) + conv_out_hw(H, W, KH, KW, pad, stride) + (Cout,)
    gx = np.empty((B, H, W, Cin), dtype=U64)
    lib().orc_ring_conv2d_grad_x(pg, pw, gx.ctypes.data_as(_P64), B, H, W, Cin, Cout, KH, KW, pad, stride)
    return gx


def ring_conv2d_grad_w(x, g, KH, KW, pad, stride):
    """Gradient of ring_conv2d w.r.t. its filter."""
    x, px = _w(x); g, pg = _w(g)
    B, H, W, Cin = x.shape; Cout = g.shape[-1]
    assert g.shape == (B,) + conv_out_hw(H, W, KH, KW, pad, stride) + (Cout,)
    gw = np.empty((KH, KW, Cin, Cout), dtype=U64)
    lib().orc_ring_conv2d_grad_w(px, pg, gw.ctypes.data_as(_P64), B, H, W, Cin, Cout, KH, KW, pad, stride)
    return gw


def beaver_bilinear(product, p, q, a, b, c):
    """Alg. 1 / Eq. 3 with any bilinear `product(left, right)` in place of Conv:
    open e = p - a and f = q - b, then [z_0] = [c_0] + product(e, [b_0]) + product([a_0], f)
    + product(e, f) and [z_1] = [c_1] + product(e, [b_1]) + product([a_1], f).
    Used for the two gradient products of a layer (Sec. 4.1, backward pass)."""
    e = open_shares(np.asarray(p[0], U64) - np.asarray(a[0], U64), np.asarray(p[1], U64) - np.asarray(a[1], U64))
    f = open_shares(np.asarray(q[0], U64) - np.asarray(b[0], U64), np.asarray(q[1], U64) - np.asarray(b[1], U64))
    z0 = np.asarray(c[0], U64) + product(e, b[0]) + product(a[0], f) + product(e, f)
    z1 = np.asarray(c[1], U64) + product(e, b[1]) + product(a[1], f)
    return z0, z1


def beaver_mul(x, y, a, b, c):
    """Alg. 1 element by element (no rescale)."""
    arrs = [_w(v[i]) for v in (x, y, a, b, c) for i in range(2)]
    z0 = np.empty_like(arrs[0][0]); z1 = np.empty_like(z0)
    lib().orc_beaver_mul(*[p for _, p in arrs], z0.ctypes.data_as(_P64), z1.ctypes.data_as(_P64), ctypes.c_size_t(z0.size))
    return z0, z1


def relu_backward(g, s_arith, a, b, c):
    """Backward of ReLU (Sec. 4.2 / 5.3): output gradient times the input mask
    1 - s, the mask shares being [1 - s]_0 = 1 - [s]_0, [1 - s]_1 = -[s]_1 kept
    from the forward conversion.  One element-wise Alg. 1, no rescale (the mask
    is an integer)."""
    m = (U64(1) - np.asarray(s_arith[0], U64), U64(0) - np.asarray(s_arith[1], U64))
    return beaver_mul(g, m, a, b, c)


# ------------------------------------------------------------------ binary side
def beaver_and(X, Y, a, b, c):
    """Beaver AND on one word pair: all arguments are 2-sequences of ints."""
    arrs = [np.array(v, dtype=U64) for v in (X, Y, a, b, c)]
    out = np.zeros(2, dtype=U64)
    lib().orc_beaver_and(*[v.ctypes.data_as(_P64) for v in arrs], out.ctypes.data_as(_P64))
    return int(out[0]), int(out[1])


def ks_add(U, V, w, ta, tb, tc):
    """XOR shares of (U+V) mod 2^w via the Kogge-Stone network.
    U, V: 2-sequences; ta/tb/tc: pairs of arrays with 2*log2(w) words each."""
    Ua = np.array(U, dtype=U64); Va = np.array(V, dtype=U64)
    t = [np.ascontiguousarray(v, dtype=U64) for v in (ta[0], ta[1], tb[0], tb[1], tc[0], tc[1])]
    S = np.zeros(2, dtype=U64)
    lib().orc_ks_add(Ua.ctypes.data_as(_P64), Va.ctypes.data_as(_P64), w,
                     *[v.ctypes.data_as(_P64) for v in t], S.ctypes.data_as(_P64))
    return int(S[0]), int(S[1])


def b2a(s, rb, ra):
    sa = np.array(s, dtype=np.uint8); rba = np.array(rb, dtype=np.uint8)
    raa = np.array(ra, dtype=U64); out = np.zeros(2, dtype=U64)
    lib().orc_b2a(sa.ctypes.data_as(_P8), rba.ctypes.data_as(_P8),
                  raa.ctypes.data_as(_P64), out.ctypes.data_as(_P64))
    return int(out[0]), int(out[1])


class _ReluMaterialC(ctypes.Structure):
    _fields_ = [("r", _P64 * 2), ("ta", _P64 * 2), ("tb", _P64 * 2), ("tc", _P64 * 2),
                ("rb", _P8 * 2), ("ra", _P64 * 2),
                ("ma", _P64 * 2), ("mb", _P64 * 2), ("mc", _P64 * 2)]


@dataclass
class ReluResult:
    y: tuple          # output shares (y_0, y_1)
    s_bit: tuple      # XOR shares of the sign bit, uint8
    s_arith: tuple    # additive shares of the sign bit


ADDERS = {"kogge-stone": 0, "tree": 1}


def relu(x, mat, adder="kogge-stone") -> ReluResult:
    """Secure ReLU on additive shares x = (x_0, x_1).

    ``mat`` is a mapping with keys r, and_a, and_b, and_c ([12, n] each),
    rb (uint8), ra, ma, mb, mc; every value a pair (party 0, party 1).
    ``adder``: "kogge-stone", or "tree" for the prefix tree of the listing in Sec. 4.2."""
    x0, px0 = _w(np.ravel(x[0])); x1, px1 = _w(np.ravel(x[1]))
    n = x0.size
    keep = []
    m = _ReluMaterialC()

    def put(field, key, conv, size):
        for p in range(2):
            arr, ptr = conv(np.ravel(mat[key][p]))
            assert arr.size == size, (key, arr.size, size)
            keep.append(arr)
            getattr(m, field)[p] = ptr

    put("r", "r", _w, n)
    put("ta", "and_a", _w, 12 * n); put("tb", "and_b", _w, 12 * n); put("tc", "and_c", _w, 12 * n)
    put("rb", "rb", _b, n); put("ra", "ra", _w, n)
    put("ma", "ma", _w, n); put("mb", "mb", _w, n); put("mc", "mc", _w, n)
    y0 = np.empty(n, dtype=U64); y1 = np.empty(n, dtype=U64)
    sb0 = np.empty(n, dtype=np.uint8); sb1 = np.empty(n, dtype=np.uint8)
    sa0 = np.empty(n, dtype=U64); sa1 = np.empty(n, dtype=U64)
    lib().orc_relu_adder(px0, px1, ctypes.byref(m), y0.ctypes.data_as(_P64), y1.ctypes.data_as(_P64),
                         ctypes.c_size_t(n), sb0.ctypes.data_as(_P8), sb1.ctypes.data_as(_P8),
                         sa0.ctypes.data_as(_P64), sa1.ctypes.data_as(_P64), ctypes.c_int(ADDERS[adder]))
    shp = np.shape(x[0])
    return ReluResult((y0.reshape(shp), y1.reshape(shp)), (sb0.reshape(shp), sb1.reshape(shp)),
                      (sa0.reshape(shp), sa1.reshape(shp)))


def tree_carries(U, V, ta, tb, tc):
    """Carry shares of the listing's prefix tree for one XOR-shared word pair;
    ta, tb, tc: (12 words of party 0, 12 words of party 1)."""
    arr = lambda v: np.array(v, dtype=U64)
    Ua, Va = arr(U), arr(V)
    t = [arr(q[p]) for q in (ta, tb, tc) for p in range(2)]
    G = np.zeros(2, dtype=U64)
    lib().orc_tree_carries(Ua.ctypes.data_as(_P64), Va.ctypes.data_as(_P64), *[q.ctypes.data_as(_P64) for q in t],
                           G.ctypes.data_as(_P64))
    return int(G[0]), int(G[1])


# ------------------------------------------------------------------ max-pooling
def pool_level1(x):
    """One party's local gather for the first tournament level (NHWC, 2x2/2)."""
    x, px = _w(x); B, H, W, C = x.shape
    d = np.empty(2 * B * (H // 2) * (W // 2) * C, dtype=U64)
    lib().orc_pool_level1(px, d.ctypes.data_as(_P64), B, H, W, C)
    return d


def pool_level2(x, r1):
    x, px = _w(x); r1, pr = _w(r1); B, H, W, C = x.shape
    n = B * (H // 2) * (W // 2) * C
    v = np.empty(n, dtype=U64); d2 = np.empty(n, dtype=U64)
    lib().orc_pool_level2(px, pr, v.ctypes.data_as(_P64), d2.ctypes.data_as(_P64), B, H, W, C)
    return v, d2


def maxpool2x2(x, mat1, mat2, want_signs=False, adder="kogge-stone"):
    """max over 2x2 windows by max(p,q) = q + ReLU(p-q), two tournament levels.
    mat1 covers 2*n_out elements, mat2 n_out elements.  Returns output shares;
    with want_signs also the additive sign shares of the two conversions (what the
    backward pass keeps)."""
    B, H, W, C = np.shape(x[0])
    d1 = (pool_level1(x[0]), pool_level1(x[1]))
    c1 = relu(d1, mat1, adder); r1 = c1.y
    v0, d20 = pool_level2(x[0], r1[0]); v1, d21 = pool_level2(x[1], r1[1])
    c2 = relu((d20, d21), mat2, adder); r2 = c2.y
    shp = (B, H // 2, W // 2, C)
    y = ((v0 + r2[0]).reshape(shp), (v1 + r2[1]).reshape(shp))
    return (y, c1.s_arith, c2.s_arith) if want_signs else y


def maxpool2x2_backward(g, s1, s2, t1, t2, x_shape):
    """Backward of maxpool2x2 (Sec. 5.3: element-wise products with the masks kept
    from the forward conversions).  With m = 1 - s the mask of a conversion,
    out = v + ReLU(u - v) gives grad_u = g*m2, grad_v = g - grad_u; one level down
    u = p01 + ReLU(p00 - p01) gives grad_p00 = grad_u*m1, grad_p01 = grad_u - grad_p00,
    and likewise v with (p10, p11).  t2 / t1: element-wise triples on n_out / 2*n_out
    words (pairs interleaved as in pool_level1).  Returns shares shaped like the input."""
    B, H, W, C = x_shape
    g0, g1 = (np.asarray(v, U64).reshape(-1) for v in g)
    gu = relu_backward((g0, g1), s2, *t2)
    gv = (g0 - gu[0], g1 - gu[1])
    G1 = tuple(np.stack([gu[i], gv[i]], axis=1).reshape(-1) for i in range(2))
    P = relu_backward(G1, s1, *t1)
    out = []
    for i in range(2):
        Pi = P[i].reshape(B, H // 2, W // 2, C, 2)
        gui = gu[i].reshape(B, H // 2, W // 2, C); gvi = gv[i].reshape(B, H // 2, W // 2, C)
        gx = np.empty((B, H // 2, 2, W // 2, 2, C), dtype=U64)
        gx[:, :, 0, :, 0, :] = Pi[..., 0];       gx[:, :, 0, :, 1, :] = gui - Pi[..., 0]
        gx[:, :, 1, :, 0, :] = Pi[..., 1];       gx[:, :, 1, :, 1, :] = gvi - Pi[..., 1]
        out.append(gx.reshape(B, H, W, C))
    return tuple(out)


# ---------------------------------------------------------------- three parties
_PP64 = ctypes.c_void_p * 3


def _w3(arrs):
    """Three contiguous uint64 arrays and the array of their pointers."""
    keep = [np.ascontiguousarray(a, dtype=U64) for a in arrs]
    assert len(keep) == 3
    return keep, _PP64(*[a.ctypes.data for a in keep])


def _out3(shape, dtype=U64):
    keep = [np.empty(shape, dtype=dtype) for _ in range(3)]
    return keep, _PP64(*[a.ctypes.data for a in keep])


def open3(s):
    """Reconstruct a three-party additive sharing (Sec. 3.1)."""
    k, ps = _w3(s)
    out = np.empty_like(k[0])
    lib().orc3_open(ps, out.ctypes.data_as(_P64), ctypes.c_size_t(out.size))
    return out


def beaver_mul3(x, y, a, b, c):
    """Alg. 1 element by element; every argument a triple (party 0, 1, 2)."""
    kx, px = _w3(x); ky, py = _w3(y); ka, pa = _w3(a); kb, pb = _w3(b); kc, pc = _w3(c)
    z, pz = _out3(kx[0].shape)
    lib().orc3_beaver_mul(px, py, pa, pb, pc, pz, ctypes.c_size_t(kx[0].size))
    return tuple(z)


def beaver_matmul3(x, y, a, b, c):
    """Alg. 1 on matrices with three parties."""
    kx, px = _w3(x); ky, py = _w3(y); ka, pa = _w3(a); kb, pb = _w3(b); kc, pc = _w3(c)
    M, K = kx[0].shape; _, N = ky[0].shape
    z, pz = _out3((M, N))
    lib().orc3_beaver_matmul(px, py, pa, pb, pc, pz, M, K, N)
    return tuple(z)


def beaver_conv2d3(x, w, a, b, c, pad, stride):
    """Eq. 3 with three parties.  NHWC / [KH,KW,Cin,Cout]."""
    kx, px = _w3(x); kw, pw = _w3(w); ka, pa = _w3(a); kb, pb = _w3(b); kc, pc = _w3(c)
    B, H, W, Cin = kx[0].shape; KH, KW, _, Cout = kw[0].shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, pad, stride)
    z, pz = _out3((B, Ho, Wo, Cout))
    lib().orc3_beaver_conv2d(px, pw, pa, pb, pc, pz, B, H, W, Cin, Cout, KH, KW, pad, stride)
    return tuple(z)


def truncate3(z, r, rt, bits=16):
    """Masked three-party truncation with the offline pair ([r], [r >> bits]); returns new arrays."""
    kz = [np.array(v, dtype=U64, copy=True) for v in z]
    pz = _PP64(*[a.ctypes.data for a in kz])
    kr, pr = _w3(r); kt, pt = _w3(rt)
    lib().orc3_truncate(pz, pr, pt, ctypes.c_size_t(kz[0].size), bits)
    return tuple(kz)


def beaver_and3(X, Y, a, b, c):
    """One Beaver AND on XOR-shared words; every argument three python ints."""
    arrs = [np.array(v, dtype=U64) for v in (X, Y, a, b, c)]
    out = np.zeros(3, dtype=U64)
    lib().orc3_beaver_and(*[q.ctypes.data_as(_P64) for q in arrs], out.ctypes.data_as(_P64))
    return tuple(int(v) for v in out)


def add3(U, V, W, w, ta, tb, tc):
    """XOR shares of (U + V + W) mod 2^w from XOR shares (three ints each) of the
    addends; ta, tb, tc: [1 + 2*log2(w)][3] triple words."""
    arrs = [np.array(v, dtype=U64) for v in (U, V, W)]
    t = [np.ascontiguousarray(v, dtype=U64) for v in (ta, tb, tc)]
    S = np.zeros(3, dtype=U64)
    lib().orc3_add3(arrs[0].ctypes.data_as(_P64), arrs[1].ctypes.data_as(_P64), arrs[2].ctypes.data_as(_P64),
                    ctypes.c_int(w), *[q.ctypes.data_as(_P64) for q in t], S.ctypes.data_as(_P64))
    return tuple(int(v) for v in S)


def b2a3(s, rb, ra):
    sa = np.array(s, dtype=np.uint8); rba = np.array(rb, dtype=np.uint8)
    raa = np.array(ra, dtype=U64); out = np.zeros(3, dtype=U64)
    lib().orc3_b2a(sa.ctypes.data_as(_P8), rba.ctypes.data_as(_P8),
                   raa.ctypes.data_as(_P64), out.ctypes.data_as(_P64))
    return tuple(int(v) for v in out)


class _Relu3MaterialC(ctypes.Structure):
    _fields_ = [(k, _PP64) for k in ("r0", "r1", "ta", "tb", "tc", "rb", "ra", "ma", "mb", "mc")]


def relu3(x, mat) -> ReluResult:
    """Secure ReLU with three parties.  ``mat``: keys r0, r1, and_a, and_b, and_c
    ([13, n] each), rb (uint8), ra, ma, mb, mc; every value a triple of arrays."""
    kx, px = _w3([np.ravel(v) for v in x])
    n = kx[0].size
    keep = []
    m = _Relu3MaterialC()
    for field, key, dt, size in (("r0", "r0", U64, n), ("r1", "r1", U64, n), ("ta", "and_a", U64, 13 * n),
                                 ("tb", "and_b", U64, 13 * n), ("tc", "and_c", U64, 13 * n),
                                 ("rb", "rb", np.uint8, n), ("ra", "ra", U64, n),
                                 ("ma", "ma", U64, n), ("mb", "mb", U64, n), ("mc", "mc", U64, n)):
        arrs = [np.ascontiguousarray(np.ravel(v), dtype=dt) for v in mat[key]]
        assert len(arrs) == 3 and all(a.size == size for a in arrs), key
        keep.append(arrs)
        setattr(m, field, _PP64(*[a.ctypes.data for a in arrs]))
    y, py = _out3(n); sb, psb = _out3(n, np.uint8); sa, psa = _out3(n)
    lib().orc3_relu(px, ctypes.byref(m), py, ctypes.c_size_t(n), psb, psa)
    shp = np.shape(x[0])
    return ReluResult(tuple(v.reshape(shp) for v in y), tuple(v.reshape(shp) for v in sb),
                      tuple(v.reshape(shp) for v in sa))


def maxpool2x2_3(x, mat1, mat2, want_signs=False):
    """Three-party 2x2 max-pool by max(p,q) = q + ReLU(p-q): the local gathers of
    maxpool2x2 on every party's share, the two conversions by relu3.  With
    want_signs also the additive sign shares of the two conversions."""
    B, H, W, C = np.shape(x[0])
    c1 = relu3(tuple(pool_level1(x[p]) for p in range(3)), mat1); r1 = c1.y
    lv2 = [pool_level2(x[p], r1[p]) for p in range(3)]
    c2 = relu3(tuple(q[1] for q in lv2), mat2); r2 = c2.y
    shp = (B, H // 2, W // 2, C)
    y = tuple((lv2[p][0] + r2[p]).reshape(shp) for p in range(3))
    return (y, c1.s_arith, c2.s_arith) if want_signs else y


def beaver_bilinear3(product, p, q, a, b, c):
    """beaver_bilinear with three parties (Alg. 1 for N = 3): e = p - a and f = q - b
    opened from three shares; party 0 adds product(e, f)."""
    u = lambda v: np.asarray(v, U64)
    e = open3(tuple(u(p[i]) - u(a[i]) for i in range(3)))
    f = open3(tuple(u(q[i]) - u(b[i]) for i in range(3)))
    z = [u(c[i]) + product(e, b[i]) + product(a[i], f) for i in range(3)]
    z[0] = z[0] + product(e, f)
    return tuple(z)


def relu_backward3(g, s_arith, a, b, c):
    """relu_backward with three parties: mask shares [1 - s]_0 = 1 - [s]_0, [1 - s]_i = -[s]_i."""
    m = tuple(U64(1 if i == 0 else 0) - np.asarray(s_arith[i], U64) for i in range(3))
    return beaver_mul3(g, m, a, b, c)


def maxpool2x2_backward3(g, s1, s2, t1, t2, x_shape):
    """maxpool2x2_backward with three parties: the same two element-wise products
    (Sec. 5.3) and local sums, on triples of shares."""
    B, H, W, C = x_shape
    gs = tuple(np.asarray(v, U64).reshape(-1) for v in g)
    gu = relu_backward3(gs, s2, *t2)
    gv = tuple(gs[i] - gu[i] for i in range(3))
    G1 = tuple(np.stack([gu[i], gv[i]], axis=1).reshape(-1) for i in range(3))
    P = relu_backward3(G1, s1, *t1)
    out = []
    for i in range(3):
        Pi = P[i].reshape(B, H // 2, W // 2, C, 2)
        gui = gu[i].reshape(B, H // 2, W // 2, C); gvi = gv[i].reshape(B, H // 2, W // 2, C)
        gx = np.empty((B, H // 2, 2, W // 2, 2, C), dtype=U64)
        gx[:, :, 0, :, 0, :] = Pi[..., 0];       gx[:, :, 0, :, 1, :] = gui - Pi[..., 0]
        gx[:, :, 1, :, 0, :] = Pi[..., 1];       gx[:, :, 1, :, 1, :] = gvi - Pi[..., 1]
        out.append(gx.reshape(B, H, W, C))
    return tuple(out)


# --------------------------------------------- checkers on reconstructed values
def to_signed(u):
    return np.asarray(u, dtype=U64).view(np.int64)


def decode(u, frac_bits=16):
    """Fixed-point decode of reconstructed ring values to float64."""
    return to_signed(u).astype(np.float64) / float(1 << frac_bits)


def truncation_wraps(z_rec, t_rec, bits=16):
    """Boolean mask of elements where local truncation left the +-1 band
    around floor(z / 2^bits) (the share-wrap event)."""
    want = to_signed(z_rec) >> bits
    got = to_signed(t_rec)
    return np.abs(got - want) > 1
