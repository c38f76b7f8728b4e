"""The ring identities the folded calls rest on, checked on the CPU against the oracle's literal Alg. 1 / Eq. 3:
party 0's output share c_0 + e*b_0 + a_0*f + e*f equals (c_0 - a_0*b_0) + (x_0 + e_1)*(b_0 + f), and when the right
operand is a share too, b_0 + f = y_0 + f_1.  Party 1's share is the oracle's own formula.  (The HIP path's parity
tests compare its folded calls with the same oracle outputs word for word; this file pins the algebra by itself.)"""
import numpy as np
import pytest

import oracle
from helpers import deal_conv, deal_matmul


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 2), (17, 33, 9)])
def test_folded_party0_share_matmul(shape):
    M, K, N = shape
    d = deal_matmul(np.random.default_rng(M * 100 + K * 10 + N), M, K, N)
    z = oracle.beaver_matmul(d["x"], d["y"], d["a"], d["b"], d["c"])
    e = [d["x"][i] - d["a"][i] for i in range(2)]
    f = [d["y"][i] - d["b"][i] for i in range(2)]
    c0_folded = d["c"][0] - oracle.ring_matmul(d["a"][0], d["b"][0])
    # weight form: f is public ahead of time, party 0 holds the planes of b_0 + f
    z0 = c0_folded + oracle.ring_matmul(d["x"][0] + e[1], d["b"][0] + (f[0] + f[1]))
    assert np.array_equal(z0, z[0])
    # two shared operands: b_0 + f is party 0's own share plus the word it receives
    assert np.array_equal(d["b"][0] + (f[0] + f[1]), d["y"][0] + f[1])
    z0 = c0_folded + oracle.ring_matmul(d["x"][0] + e[1], d["y"][0] + f[1])
    assert np.array_equal(z0, z[0])
    # party 1 keeps Alg. 1's form: c_1 + e*b_1 + a_1*f
    E, F = e[0] + e[1], f[0] + f[1]
    assert np.array_equal(d["c"][1] + oracle.ring_matmul(E, d["b"][1]) + oracle.ring_matmul(d["a"][1], F), z[1])


def test_folded_party0_share_conv():
    d = deal_conv(np.random.default_rng(77), 2, 6, 5, 3, 4, 3, 3, 1, 2)
    z = oracle.beaver_conv2d(d["x"], d["y"], d["a"], d["b"], d["c"], d["pad"], d["stride"])
    conv = lambda A, B: oracle.ring_conv2d(A, B, d["pad"], d["stride"])
    e1 = d["x"][1] - d["a"][1]
    F = (d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1])
    z0 = (d["c"][0] - conv(d["a"][0], d["b"][0])) + conv(d["x"][0] + e1, d["b"][0] + F)
    assert np.array_equal(z0, z[0])


def test_fold_is_not_symmetric_for_free():
    """Folding party 1 the same way would need the extra product e*f: (a_1 + e)(b_1 + f) over-counts it."""
    d = deal_matmul(np.random.default_rng(5), 4, 6, 3)
    z = oracle.beaver_matmul(d["x"], d["y"], d["a"], d["b"], d["c"])
    E = (d["x"][0] - d["a"][0]) + (d["x"][1] - d["a"][1])
    F = (d["y"][0] - d["b"][0]) + (d["y"][1] - d["b"][1])
    folded1 = (d["c"][1] - oracle.ring_matmul(d["a"][1], d["b"][1])) + oracle.ring_matmul(d["a"][1] + E, d["b"][1] + F)
    assert np.array_equal(folded1 - oracle.ring_matmul(E, F), z[1])
    assert not np.array_equal(folded1, z[1])


def test_beaver_product_is_separable_over_rows():
    """What the row-chunked layer rests on: Alg. 1 / Eq. 3 on a slice of the left operand's rows (images), with the
    same slices of a and c and the whole right operand, gives the same slice of every output share."""
    d = deal_matmul(np.random.default_rng(41), 11, 7, 5)
    z = oracle.beaver_matmul(d["x"], d["y"], d["a"], d["b"], d["c"])
    for lo, hi in ((0, 4), (4, 11), (10, 11)):
        cut = lambda k: (d[k][0][lo:hi], d[k][1][lo:hi])
        zs = oracle.beaver_matmul(cut("x"), d["y"], cut("a"), d["b"], cut("c"))
        assert np.array_equal(zs[0], z[0][lo:hi]) and np.array_equal(zs[1], z[1][lo:hi])
    d = deal_conv(np.random.default_rng(42), 3, 5, 6, 2, 3, 3, 3, 1, 1)
    z = oracle.beaver_conv2d(d["x"], d["y"], d["a"], d["b"], d["c"], d["pad"], d["stride"])
    cut = lambda k: (d[k][0][1:3], d[k][1][1:3])
    zs = oracle.beaver_conv2d(cut("x"), d["y"], cut("a"), d["b"], cut("c"), d["pad"], d["stride"])
    assert np.array_equal(zs[0], z[0][1:3]) and np.array_equal(zs[1], z[1][1:3])
