"""Do the oracle's pins notice a mistake?  Each case plants one plausible error in a copy of
oracle/mpc_oracle.c (a dropped term, a wrong sign, index, shift or operand), builds it, and runs the
pin suites (tests/test_oracle_pins.py, test_oracle_three_party.py, test_oracle_golden.py) against that
build in a child process: the suites must fail.  Everything here happens on the CPU."""
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mpc_oracle.c")
SUITES = ["tests/test_oracle_golden.py", "tests/test_oracle_pins.py", "tests/test_oracle_three_party.py"]

# (name, text in the source - must occur exactly once -, replacement)
MUTANTS = [
    ("mask adds instead of subtracting", "e[i] = x[i] - a[i];", "e[i] = x[i] + a[i];"),
    ("element-wise product without the e*f term", "z0[i] = c0[i] + e * b0[i] + a0[i] * f + e * f;", "z0[i] = c0[i] + e * b0[i] + a0[i] * f;"),
    ("matrix product reads the left operand transposed", "const u64 l = L[(size_t)m * K + k];", "const u64 l = L[(size_t)k * M + m];"),
    ("party 1 of the matrix product uses party 0's b", "orc_ring_matmul(e, b1, t, M, K, N);", "orc_ring_matmul(e, b0, t, M, K, N);"),
    ("convolution protocol without Conv(e, f)", "CONV(e, f);   for (size_t i = 0; i < nz; ++i) z0[i] += t[i];", ""),
    ("convolution pads on the wrong side", "const int hi = ho * stride + kh - pad;\n                    if (hi < 0 || hi >= H) continue;\n                    for (int kw = 0; kw < KW; ++kw) {\n                        const int wi = wo * stride + kw - pad;\n                        if (wi < 0 || wi >= W) continue;\n                        const u64* xi",
     "const int hi = ho * stride + kh + pad;\n                    if (hi < 0 || hi >= H) continue;\n                    for (int kw = 0; kw < KW; ++kw) {\n                        const int wi = wo * stride + kw - pad;\n                        if (wi < 0 || wi >= W) continue;\n                        const u64* xi"),
    ("filter gradient accumulates x*x", "for (int co = 0; co < Cout; ++co) wr[co] += xv * go[co];", "for (int co = 0; co < Cout; ++co) wr[co] += xv * xv;"),
    ("input gradient ignores the stride", "const int hi = ho * stride + kh - pad;\n                    if (hi < 0 || hi >= H) continue;\n                    for (int kw = 0; kw < KW; ++kw) {\n                        const int wi = wo * stride + kw - pad;\n                        if (wi < 0 || wi >= W) continue;\n                        u64* xo",
     "const int hi = ho + kh - pad;\n                    if (hi < 0 || hi >= H) continue;\n                    for (int kw = 0; kw < KW; ++kw) {\n                        const int wi = wo * stride + kw - pad;\n                        if (wi < 0 || wi >= W) continue;\n                        u64* xo"),
    ("party 1 truncates like party 0", "z1[i] = (u64)0 - (((u64)0 - z1[i]) >> bits);", "z1[i] = z1[i] >> bits;"),
    ("Beaver AND without d & g", "out[0] = c[0] ^ (d & b[0]) ^ (g & a[0]) ^ (d & g);", "out[0] = c[0] ^ (d & b[0]) ^ (g & a[0]);"),
    ("A2B: party 1 forgets its mask", "V[0] = r[1];         V[1] = x[1] ^ r[1];", "V[0] = r[1];         V[1] = x[1];"),
    ("prefix level shifts by l + 1 instead of 2^l", "    for (int l = 0; l < levels; ++l) {\n        const int d = 1 << l;\n        const u64 Gs[2]", "    for (int l = 0; l < levels; ++l) {\n        const int d = l + 1;\n        const u64 Gs[2]"),
    ("generate update uses the shifted propagate", "beaver_and(P, Gs, ta[1 + 2 * l], tb[1 + 2 * l], tc[1 + 2 * l], T);", "beaver_and(P, Ps, ta[1 + 2 * l], tb[1 + 2 * l], tc[1 + 2 * l], T);"),
    ("tree adder spreads one position too low", "for (int k = 1; k <= half; ++k) mu |= (u64)1 << k;", "for (int k = 0; k < half; ++k) mu |= (u64)1 << k;"),
    ("sign takes the carry out of bit 63", "const u64 s[2] = { (P0[0] >> 63) ^ ((G[0] >> 62) & 1),\n                           (P0[1] >> 63) ^ ((G[1] >> 62) & 1) };",
     "const u64 s[2] = { (P0[0] >> 63) ^ ((G[0] >> 63) & 1),\n                           (P0[1] >> 63) ^ ((G[1] >> 63) & 1) };"),
    ("B2A without the factor two", "const u64 sa[2] = { ra[0] + v - 2 * v * ra[0], ra[1] - 2 * v * ra[1] };", "const u64 sa[2] = { ra[0] + v - v * ra[0], ra[1] - v * ra[1] };"),
    ("select: both parties hold the public one", "const u64 m[2] = { (u64)1 - sa[0], (u64)0 - sa[1] };", "const u64 m[2] = { (u64)1 - sa[0], (u64)1 - sa[1] };"),
    ("max-pool second level compares the wrong way", "d2[o] = u - v;", "d2[o] = v - u;"),
    ("three parties: matrix product without e*f", "if (p == 0) { orc_ring_matmul(e, f, t, M, K, N); for (size_t i = 0; i < mn; ++i) z[p][i] += t[i]; }", ""),
    ("three parties: rescale keeps the offset", "z[0][i] = (m >> bits) - ((u64)1 << (62 - bits)) - rt[0][i];", "z[0][i] = (m >> bits) - rt[0][i];"),
    ("three parties: AND opened from two parties only", "for (int p = 0; p < NP; ++p) { d ^= X[p] ^ a[p]; g ^= Y[p] ^ b[p]; }", "for (int p = 0; p < 2; ++p) { d ^= X[p] ^ a[p]; g ^= Y[p] ^ b[p]; }"),
    ("three parties: carry word is not the majority", "K[p] = ((T[p] ^ W[p]) << 1) & wm;", "K[p] = (T[p] << 1) & wm;"),
    ("three parties: both ANDs of a level share a triple", "beaver_and3(P, Ps, ta[3 + 2 * l], tb[3 + 2 * l], tc[3 + 2 * l], Pn);", "beaver_and3(P, Ps, ta[2 + 2 * l], tb[2 + 2 * l], tc[2 + 2 * l], Pn);"),
    ("three parties: A2B sends both masks to the same peer", "Wd[j][(j + 2) % NP] = r1[j];", "Wd[j][(j + 1) % NP] = r1[j];"),
]


def run_mutant(case, tmp):
    idx, (name, old, new) = case
    text = open(SRC).read()
    if text.count(old) != 1:
        return name, "the source no longer contains this text exactly once"
    src = os.path.join(tmp, f"mutant{idx}.c"); lib = os.path.join(tmp, f"mutant{idx}.so")
    open(src, "w").write(text.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC", "-w", "-o", lib, src])
    env = dict(os.environ, MPC_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    try:
        rc = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *SUITES], cwd=ROOT, env=env,
                            stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=300).returncode
    except subprocess.TimeoutExpired:
        rc = -1
    return name, None if rc != 0 else "the pin suites still pass"


def test_every_planted_mistake_is_noticed():
    with tempfile.TemporaryDirectory() as tmp:
        with ThreadPoolExecutor(max_workers=4) as pool:
            results = list(pool.map(lambda c: run_mutant(c, tmp), enumerate(MUTANTS)))
    missed = [f"{name}: {why}" for name, why in results if why]
    assert not missed, "undetected: " + "; ".join(missed)


def test_the_unmodified_source_passes_under_the_same_harness():
    """The harness itself: an unmutated copy, built and run the same way, passes (so a failure above is the mutation's)."""
    with tempfile.TemporaryDirectory() as tmp:
        lib = os.path.join(tmp, "plain.so")
        subprocess.check_call(["gcc", "-O1", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC", "-w", "-o", lib, SRC])
        env = dict(os.environ, MPC_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
        rc = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_golden.py"],
                            cwd=ROOT, env=env, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=300).returncode
        assert rc == 0
