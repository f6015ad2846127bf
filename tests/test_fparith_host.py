"""The exact fp64 modular arithmetic of the GPU path (csrc/fparith.hpp), compiled for the host and checked against
Python integers at the edges of the ranges its comments claim: operands of +-(p-1), lazy values of several p, primes
just below 2^50 and a small one, ties of the centred reduction, and the eight-term accumulation of a base conversion.
No GPU: the header is plain C++ (its fused multiply-adds are spelled out, and contraction is off as in the GPU build)."""
import ctypes
import os
import random
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = r"""
#include "fparith.hpp"
extern "C" {
double t_mulmod(double a, double b, double p, double pinv) { return fp_mulmod(a, b, p, pinv); }
double t_norm(double v, double p, double pinv) { return fp_norm(v, p, pinv); }
uint64_t t_canonical(double v, double p, double pinv) { return fp_canonical(v, p, pinv); }
double t_from_u64(uint64_t x) { return fp_from_u64(x); }
uint64_t t_to_u64(double v) { return fp_to_u64(v); }
double t_centred(uint64_t x, double p, double half) { return fp_centred_from_u64(x, p, half); }
}
"""


@pytest.fixture(scope="module")
def fp(tmp_path_factory):
    d = tmp_path_factory.mktemp("fparith")
    src, lib = d / "w.cpp", d / "libw.so"
    src.write_text(SRC)
    inc = os.path.join(ROOT, "paper_1810_00845_amd", "csrc")
    base = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-shared", "-fPIC", "-I", inc, str(src), "-o", str(lib)]
    if subprocess.run(base[:4] + ["-mfma"] + base[4:], capture_output=True).returncode != 0:   # fma in hardware if there
        subprocess.run(base, check=True)
    l = ctypes.CDLL(str(lib))
    D, U = ctypes.c_double, ctypes.c_uint64
    l.t_mulmod.restype = D; l.t_mulmod.argtypes = [D] * 4
    l.t_norm.restype = D; l.t_norm.argtypes = [D] * 3
    l.t_canonical.restype = U; l.t_canonical.argtypes = [D] * 3
    l.t_from_u64.restype = D; l.t_from_u64.argtypes = [U]
    l.t_to_u64.restype = U; l.t_to_u64.argtypes = [D]
    l.t_centred.restype = D; l.t_centred.argtypes = [U, D, D]
    return l


def primes():
    from oracle import Oracle
    big = Oracle(15, [50, 50, 50], 3, 50, seed=1).primes[:2]        # the largest primes = 1 mod 2^16 below 2^50
    small = Oracle(12, [36, 40], 2, 45, seed=1).primes              # 36-, 40- and 45-bit primes
    return [int(p) for p in list(big) + list(small)]


def is_int(x):
    return x == int(x)


def test_mulmod_is_exact_and_in_range_at_the_extremes(fp):
    rnd = random.Random(5)
    for p in primes():
        pf, pinv = float(p), 1.0 / float(p)
        edge = [p - 1, -(p - 1), (p - 1) // 2, -((p - 1) // 2), (p + 1) // 2, 1, -1, 0, int(0.55 * p), -int(0.55 * p)]
        lazy = [int(6.2 * p), -int(6.2 * p), int(5.1 * p), 2 ** 53 - 1, -(2 ** 53 - 1)]
        cases = [(a, b) for a in edge + lazy for b in edge] + \
                [(rnd.randrange(-int(6.2 * p), int(6.2 * p)), rnd.randrange(-p // 2, p // 2)) for _ in range(3000)]
        for a, b in cases:
            r = fp.t_mulmod(float(a), float(b), pf, pinv)
            assert is_int(r) and (int(r) - a * b) % p == 0, (p, a, b, r)
            assert abs(r) <= p / 2 + 3 * 2.0 ** -53 * abs(a * b) + 1, (p, a, b, r)


def test_norm_and_canonical_at_ties_and_lazy_values(fp):
    rnd = random.Random(6)
    for p in primes():
        pf, pinv, half = float(p), 1.0 / float(p), (p - 1) // 2
        vals = [0, 1, -1, half, -half, half + 1, -(half + 1), p - 1, p, p + 1, -p]
        for k in range(-8, 9):                       # lazy values around every multiple of p the transforms can reach
            for d in (-half - 1, -half, -1, 0, 1, half, half + 1):
                v = k * p + d
                if abs(v) < 2 ** 53:
                    vals.append(v)
        vals += [rnd.randrange(-(2 ** 53) + 1, 2 ** 53) for _ in range(3000)]
        for v in vals:
            r = fp.t_norm(float(v), pf, pinv)
            assert is_int(r) and (int(r) - v) % p == 0 and abs(r) <= p / 2 * (1 + 2.0 ** -48) + abs(v) * 2.0 ** -52, (p, v, r)
            c = fp.t_canonical(float(v), pf, pinv)
            assert 0 <= c < p and (c - v) % p == 0, (p, v, c)
        # what the base conversion relies on: a value of at most 0.6 p in magnitude (a modular product's output) is
        # reduced to THE centred representative, ties included
        for v in [half, half + 1, -half, -half - 1, int(0.6 * p), -int(0.6 * p)] + [rnd.randrange(-int(0.6 * p), int(0.6 * p)) for _ in range(2000)]:
            r = int(fp.t_norm(float(v), pf, pinv))
            want = v % p
            want = want - p if want > half else want
            assert r == want, (p, v, r, want)


def test_integer_conversions(fp):
    for x in (0, 1, 2 ** 32 - 1, 2 ** 32, 2 ** 50 - 27, 2 ** 52 - 1):
        assert fp.t_from_u64(x) == float(x) and fp.t_to_u64(float(x)) == x
    for p in primes():
        half = (p - 1) // 2
        for x in (0, 1, half, half + 1, p - 1):
            want = x - p if x > half else x
            assert fp.t_centred(x, float(p), float(half)) == float(want)


def test_eight_term_sums_stay_exact(fp):
    """A base conversion adds eight modular products before it normalises, the inner product up to eight digits: the
    sum of eight lazy products of centred operands is an exact integer below 2^53, congruent to the true sum."""
    rnd = random.Random(7)
    for p in primes():
        pf, pinv = float(p), 1.0 / float(p)
        for trial in range(300):
            worst = trial < 8
            ys = [(p - 1) // 2 * (1 if (trial >> i) & 1 else -1) if worst else rnd.randrange(-p // 2, p // 2) for i in range(8)]
            hs = [int(0.55 * p) if worst else rnd.randrange(-int(0.55 * p), int(0.55 * p)) for _ in range(8)]
            s, true = 0.0, 0
            for y, h in zip(ys, hs):
                s += fp.t_mulmod(float(y), float(h), pf, pinv)
                true += y * h
                assert abs(s) < 2 ** 53 and is_int(s)
            assert (int(s) - true) % p == 0
            assert (fp.t_canonical(s, pf, pinv) - true) % p == 0
