"""The oracle against small examples worked by hand from the algorithms' statements
(tests/golden/worked_examples.json: every entry cites the passage it instantiates)."""
import json
import os

import numpy as np

import oracle

U64 = np.uint64
MOD = 1 << 64
G = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "worked_examples.json")))


def w(v):
    """ring elements: a negative entry n stands for 2^64 + n"""
    return np.array([int(q) % MOD for q in np.ravel(v)], dtype=U64).reshape(np.shape(v))


def parties(entry, key):
    return tuple(w([v]) for v in entry[key])


def ints(arrs):
    return [int(a.ravel()[0]) for a in arrs]


def want(entry, key):
    return [int(v) % MOD for v in entry[key]]


def test_alg1_two_parties():
    for name in ("alg1_two_parties", "alg1_wraps_mod_2_64"):
        e = G[name]
        z = oracle.beaver_mul(*[parties(e, k) for k in "xyabc"])
        assert ints(z) == want(e, "z"), name
        # the same numbers as 1x1 matrices
        m = lambda k: tuple(a.reshape(1, 1) for a in parties(e, k))
        assert ints(oracle.beaver_matmul(*[m(k) for k in "xyabc"])) == want(e, "z"), name


def test_alg1_three_parties():
    e = G["alg1_three_parties"]
    assert ints(oracle.beaver_mul3(*[parties(e, k) for k in "xyabc"])) == want(e, "z")
    m = lambda k: tuple(a.reshape(1, 1) for a in parties(e, k))
    assert ints(oracle.beaver_matmul3(*[m(k) for k in "xyabc"])) == want(e, "z")


def test_beaver_and():
    e = G["beaver_and_4_bit"]
    assert list(oracle.beaver_and(e["X"], e["Y"], e["a"], e["b"], e["c"])) == e["T"]


def test_adders():
    for name in ("adder_8_bit_full_ripple", "adder_8_bit_carry_chain"):
        e = G[name]
        levels = e["width"].bit_length() - 1
        zero = ([0] * (2 * levels), [0] * (2 * levels))
        assert list(oracle.ks_add(e["U"], e["V"], e["width"], zero, zero, zero)) == e["S"], name
    e = G["carry_save_three_addends_4_bit"]
    levels = e["width"].bit_length() - 1
    zero = np.zeros((1 + 2 * levels, 3), dtype=U64)
    assert list(oracle.add3(e["U"], e["V"], e["W"], e["width"], zero, zero, zero)) == e["S"]


def test_truncations():
    e = G["truncate_two_parties_plus_one"]
    t = oracle.truncate(parties(e, "z"), e["bits"])
    assert ints(t) == want(e, "t")
    e = G["truncate_three_parties_low_carry"]
    t = oracle.truncate3(parties(e, "z"), parties(e, "r"), parties(e, "rt"), e["bits"])
    assert ints(t) == want(e, "t")


def test_b2a():
    e = G["b2a_shared_random_bit"]
    assert list(oracle.b2a(e["s"], e["rb"], want(e, "ra"))) == want(e, "out")


def test_relu_with_zero_material():
    n = 1
    z64 = lambda k=n: (np.zeros(k, dtype=U64), np.zeros(k, dtype=U64))
    mat = {"r": z64(), "and_a": z64(12 * n), "and_b": z64(12 * n), "and_c": z64(12 * n),
           "rb": (np.zeros(n, dtype=np.uint8), np.zeros(n, dtype=np.uint8)), "ra": z64(), "ma": z64(), "mb": z64(), "mc": z64()}
    for case in G["relu_zero_material"]["cases"]:
        x = tuple(w([v]) for v in case["x"])
        assert ints(oracle.relu(x, mat).y) == [int(v) % MOD for v in case["y"]], case
