"""Pins of the CPU oracle against things other than itself.

Every check here compares the oracle with brute force in Python integers, a
closed form, an invariant of the mathematics, or a stored vector -- chosen so
that a dropped term, a wrong sign or index, or a transposed operand anywhere
in the oracle fails at least one of them.  No GPU.
"""
import cmath
import math
import os

import numpy as np
import pytest

from oracle import Ct, Oracle, OracleError, Pt, lib, round_half_away

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brv(x, bits):
    return int(format(x, "0%db" % bits)[::-1], 2) if bits else 0


def crt_lift(residues, primes):
    """Non-negative CRT lift with Python integers."""
    Q = math.prod(primes)
    x = 0
    for r, q in zip(residues, primes):
        hat = Q // q
        x += int(r) * pow(hat, -1, q) * hat
    return x % Q


def centred(x, Q):
    return x - Q if x > Q // 2 else x


def negacyclic_mul(a, b, q):
    n = len(a)
    c = [0] * n
    for i in range(n):
        for j in range(n):
            k = i + j
            if k < n:
                c[k] = (c[k] + a[i] * b[j]) % q
            else:
                c[k - n] = (c[k - n] - a[i] * b[j]) % q
    return c


# ---------------------------------------------------------------- primes ----
def test_primes_trial_division_and_order():
    L = lib()
    for log_n, bits in [(5, 20), (10, 30), (12, 32)]:
        two_n = 2 << log_n
        used = []
        for _ in range(4):
            arr = (np.array(used, dtype=np.uint64) if used else np.zeros(1, dtype=np.uint64))
            p = int(L.orc_next_prime(bits, log_n, arr.ctypes.data_as(
                __import__("ctypes").POINTER(__import__("ctypes").c_uint64)), len(used)))
            assert p < (1 << bits) and p % two_n == 1
            assert all(p % d for d in range(2, int(math.isqrt(p)) + 1))
            # nothing between the previous pick (or 2^bits) and p was skipped wrongly
            hi = used[-1] if used else (1 << bits) + 1
            c = hi - two_n
            while c > p:
                assert any(c % d == 0 for d in range(2, int(math.isqrt(c)) + 1))
                c -= two_n
            used.append(p)
        assert len(set(used)) == 4


def test_is_prime_known_values():
    L = lib()
    for p in [2, 3, 37, 41, 1073692673, (1 << 61) - 1, 18446744073709551557]:
        assert L.orc_is_prime(p) == 1
    # 0, 1, a Carmichael number, strong pseudoprimes to the bases {2,3,5,7} and to the
    # first nine primes, a square of a prime, a product of two 32-bit primes
    for c in [0, 1, 561, 3215031751, 3825123056546413051, 4294967291 ** 2, 4294967291 * 4294967279]:
        assert L.orc_is_prime(c) == 0


def test_context_primes_and_psi():
    o = Oracle(8, [30, 30, 40], 3, 50, seed=1)
    assert o.K == 1 and o.alpha == 1
    assert len(set(o.primes)) == 4
    psi = np.zeros(4, dtype=np.uint64)
    import ctypes
    lib().orc_get_psi(o._h, psi.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))
    for q, w in zip(o.primes, psi):
        assert q % (2 * o.N) == 1
        assert pow(int(w), o.N, q) == q - 1
        assert pow(int(w), 2 * o.N, q) == 1
    o2 = Oracle(8, [30] * 5, 2, 30, seed=1)  # alpha = 3 special primes, all distinct from the q_i
    assert o2.K == 3 and len(set(o2.primes)) == 8
    assert o2.primes == sorted(o2.primes, reverse=True)  # same size: strictly descending picks


# ------------------------------------------------------------------ prng ----
def test_prng_stored_vectors():
    for line in open(os.path.join(GOLDEN, "prng_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        seed, kind, ctr, idx, val = line.split()
        assert lib().orc_rnd(int(seed), int(kind), int(ctr), int(idx)) == int(val, 16)


def test_prng_streams_differ_and_look_uniform():
    L = lib()
    a = np.array([L.orc_rnd(5, 2, 0, i) for i in range(4096)], dtype=np.uint64)
    b = np.array([L.orc_rnd(5, 2, 1, i) for i in range(4096)], dtype=np.uint64)
    c = np.array([L.orc_rnd(5, 3, 0, i) for i in range(4096)], dtype=np.uint64)
    assert len(set(a.tolist()) | set(b.tolist()) | set(c.tolist())) == 3 * 4096
    for v in (a, b, c):
        bits = np.unpackbits(v.view(np.uint8))
        assert abs(bits.mean() - 0.5) < 0.01
        counts = np.bincount((v % np.uint64(16)).astype(np.int64), minlength=16)
        chi2 = ((counts - 256.0) ** 2 / 256.0).sum()
        assert chi2 < 50.0  # 15 dof, p ~ 1e-5


def test_gauss_table_matches_pmf_definition():
    import mpmath as mp
    mp.mp.dps = 80
    sigma = mp.mpf("3.2")
    w = [mp.e ** (-(mp.mpf(x) ** 2) / (2 * sigma ** 2)) for x in range(0, 20)]
    total = w[0] + 2 * sum(w[1:])
    tab = np.zeros(19, dtype=np.uint64)
    import ctypes
    lib().orc_gauss_table(tab.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))
    cum = mp.mpf(0)
    for k in range(19):
        cum += w[0] if k == 0 else 2 * w[k]
        assert int(tab[k]) == int(mp.floor(mp.mpf(2) ** 63 * cum / total))
    # exact moments of the tabulated distribution
    probs = np.diff(np.concatenate([[0.0], tab.astype(np.float64), [2.0 ** 63]])) / 2.0 ** 63
    var = sum(p * k * k for k, p in enumerate(probs))
    assert abs(math.sqrt(var) - 3.2) < 1e-6


def test_gauss_and_ternary_samplers():
    L = lib()
    xs = np.array([L.orc_gauss_from_word(L.orc_rnd(3, 3, 0, i)) for i in range(40000)])
    assert np.abs(xs).max() <= 19
    assert abs(xs.mean()) < 0.06 and abs(xs.std() - 3.2) < 0.05
    # magnitude = number of table entries <= v, sign = low bit
    assert L.orc_gauss_from_word(0) == 0 and L.orc_gauss_from_word(1) == 0
    assert L.orc_gauss_from_word((1149872836518706973 << 1) | 1) == -1
    assert L.orc_gauss_from_word((1149872836518706972 << 1)) == 0
    assert L.orc_gauss_from_word((1 << 64) - 1) == -19 and L.orc_gauss_from_word((1 << 64) - 2) == 19
    ts = np.array([L.orc_ternary_from_word(L.orc_rnd(3, 1, 0, i)) for i in range(30000)])
    for v in (-1, 0, 1):
        assert abs((ts == v).mean() - 1 / 3) < 0.01
    assert [L.orc_ternary_from_word(w) for w in (0, 1, 2, 3, 4, 5)] == [0, 1, -1, 0, 1, -1]


@pytest.mark.parametrize("sigma", [0.8, 1.5, 3.19, 6.0, 10.0])
def test_gauss_table_for_other_sigmas(sigma):
    """The computed tables against the pmf's definition at 80 digits: entries within 8 units of 2^-63 (the long double
    computation carries 64 bits), strictly increasing, tail cut at floor(6 sigma), variance of the tabulated
    distribution = sigma^2 up to the cut."""
    import ctypes
    import mpmath as mp
    mp.mp.dps = 80
    K = int(math.floor(6 * sigma))
    tab = np.zeros(60, dtype=np.uint64)
    assert lib().orc_gauss_table_for(ctypes.c_double(sigma), tab.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))) == K
    s = mp.mpf(sigma)                      # the double's exact value, as the C code sees it
    w = [mp.e ** (-(mp.mpf(x) ** 2) / (2 * s ** 2)) for x in range(K + 1)]
    total = w[0] + 2 * sum(w[1:])
    cum = mp.mpf(0)
    for k in range(K):
        cum += w[0] if k == 0 else 2 * w[k]
        assert abs(int(tab[k]) - int(mp.floor(mp.mpf(2) ** 63 * cum / total))) <= 8
        assert k == 0 or tab[k] > tab[k - 1]
    probs = np.diff(np.concatenate([[0.0], tab[:K].astype(np.float64), [2.0 ** 63]])) / 2.0 ** 63
    var = sum(p * k * k for k, p in enumerate(probs))
    assert abs(math.sqrt(var) - sigma) < 2e-3 * sigma


def test_gauss_table_rejects_bad_sigmas_and_keeps_the_literal_one():
    import ctypes
    tab, lit = np.zeros(60, dtype=np.uint64), np.zeros(19, dtype=np.uint64)
    p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))
    for bad in (0.0, -1.0, 0.2, 10.5, float("nan")):
        assert lib().orc_gauss_table_for(ctypes.c_double(bad), p(tab)) == 0
    assert lib().orc_gauss_table_for(ctypes.c_double(3.2), p(tab)) == 19
    lib().orc_gauss_table(p(lit))
    assert np.array_equal(tab[:19], lit)


def test_error_polynomials_follow_the_context_sigma():
    """Encryption noise of a context made with sigma = 1.5: decrypting a fresh encryption of zero gives
    e0 + e1 s + ... whose spread follows sigma; compared with the default context on the same seed."""
    spread = {}
    for sigma in (1.5, 3.2, 6.0):
        o = Oracle(10, [40], 1, 45, seed=5, sigma=sigma)
        ct = o.encrypt(o.pt_from_coeffs(np.zeros(o.N, dtype=np.int64), 1.0, 1))
        spread[sigma] = np.std(np.array(o.pt_coeffs(o.decrypt(ct)), dtype=np.float64))
    # noise of a fresh ciphertext = e0 + e1 s + v e_pk-like terms, each proportional to sigma
    assert 0.4 < spread[1.5] / spread[3.2] < 0.55 and 1.7 < spread[6.0] / spread[3.2] < 2.05


@pytest.mark.parametrize("log_n,h", [(4, 1), (4, 16), (10, 64), (12, 192)])
def test_fixed_hamming_weight_secret(log_n, h):
    o = Oracle(log_n, [40], 1, 45, seed=9, secret_kind=1, hamming_weight=h)
    s = o.secret_coeffs()
    assert np.count_nonzero(s) == h and set(np.unique(s)) <= {-1, 0, 1}
    if h >= 64:      # signs and positions both look uniform
        assert 0.3 < (s == 1).sum() / h < 0.7
        pos = np.nonzero(s)[0]
        assert abs(pos.mean() / o.N - 0.5) < 0.12 and (pos < o.N // 2).sum() > h // 4
    # another seed moves the support; the uniform ternary secret of the same seed is a different one
    assert not np.array_equal(s, Oracle(log_n, [40], 1, 45, seed=10, secret_kind=1, hamming_weight=h).secret_coeffs()) or h == 1 << log_n
    assert np.count_nonzero(Oracle(log_n, [40], 1, 45, seed=9).secret_coeffs()) != h or log_n == 4
    # the scheme works with it: encrypt / decrypt round trip
    m = np.arange(o.N, dtype=np.int64) - o.N // 2
    ct = o.encrypt(o.pt_from_coeffs(m << 20, 1.0, 1))
    got = np.array(o.pt_coeffs(o.decrypt(ct)), dtype=np.int64)
    assert np.abs(got - (m << 20)).max() < 1 << 12


def test_fixed_hamming_weight_positions_are_uniform_over_seeds():
    """Brute force on a tiny ring: over many seeds every position is hit equally often (N = 16, h = 4: 1/4 each)."""
    hits = np.zeros(16)
    for seed in range(600):
        hits += Oracle(4, [30], 1, 40, seed=seed, secret_kind=1, hamming_weight=4).secret_coeffs() != 0
    assert np.abs(hits / 600 - 0.25).max() < 0.07


def test_bad_secret_parameters_are_rejected():
    for kw in (dict(secret_kind=2), dict(secret_kind=1, hamming_weight=0), dict(secret_kind=1, hamming_weight=17), dict(sigma=0.0)):
        with pytest.raises(Exception):
            Oracle(4, [30], 1, 40, seed=1, **kw)


# ------------------------------------------------------------------- ntt ----
@pytest.mark.parametrize("log_n", [2, 5, 8])
def test_ntt_is_the_defining_sum(log_n):
    o = Oracle(log_n, [30, 45], 1, 50, seed=2)
    import ctypes
    psis = np.zeros(o.L + o.K, dtype=np.uint64)
    lib().orc_get_psi(o._h, psis.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))
    rng = np.random.default_rng(log_n)
    for prime in range(o.L + o.K):
        q, psi = o.primes[prime], int(psis[prime])
        a = [int(x) for x in rng.integers(0, q, o.N)]
        got = o.ntt(np.array(a, dtype=np.uint64), prime)
        for i in range(o.N):
            e = 2 * brv(i, log_n) + 1
            want = sum(a[j] * pow(psi, e * j, q) for j in range(o.N)) % q
            assert int(got[i]) == want
        back = o.ntt(got, prime, inverse=True)
        assert back.tolist() == a
        # NTT(X) lists the evaluation points themselves
        x = np.zeros(o.N, dtype=np.uint64)
        x[1] = 1
        pts = o.ntt(x, prime)
        assert [int(v) for v in pts] == [pow(psi, 2 * brv(i, log_n) + 1, q) for i in range(o.N)]


@pytest.mark.parametrize("log_n", [1, 4, 6])
def test_ntt_product_is_schoolbook_negacyclic_convolution(log_n):
    o = Oracle(log_n, [40], 1, 59, seed=3)
    rng = np.random.default_rng(10 + log_n)
    for prime in range(2):
        q = o.primes[prime]
        a = [int(x) for x in rng.integers(0, q, o.N)]
        b = [int(x) for x in rng.integers(0, q, o.N)]
        fa = o.ntt(np.array(a, dtype=np.uint64), prime)
        fb = o.ntt(np.array(b, dtype=np.uint64), prime)
        prod = np.array([(int(x) * int(y)) % q for x, y in zip(fa, fb)], dtype=np.uint64)
        got = o.ntt(prod, prime, inverse=True)
        assert got.tolist() == negacyclic_mul(a, b, q)


# ---------------------------------------------------------------- encode ----
def test_encode_constant_and_unit_vectors():
    o = Oracle(5, [40, 40], 1, 50, seed=4)
    scale = 2.0 ** 30
    coef = o.encode_coeffs(np.ones(o.slots), scale)
    assert coef[0] == 2 ** 30 and not coef[1:].any()
    # a single slot set: evaluate the rounded polynomial at every root by brute force
    for j in (0, 3, o.slots - 1):
        z = np.zeros(o.slots)
        z[j] = 1.0
        coef = o.encode_coeffs(z, scale)
        for jj in range(o.slots):
            zeta = cmath.exp(1j * math.pi * pow(5, jj, 2 * o.N) / o.N)
            val = sum(int(coef[k]) * zeta ** k for k in range(o.N)) / scale
            assert abs(val - (1.0 if jj == j else 0.0)) < o.N / scale
    # imaginary parts travel too
    z = np.zeros(o.slots, dtype=complex)
    z[2] = 1j
    coef = o.encode_coeffs(z, scale)
    zeta = cmath.exp(1j * math.pi * pow(5, 2, 2 * o.N) / o.N)
    val = sum(int(coef[k]) * zeta ** k for k in range(o.N)) / scale
    assert abs(val - 1j) < o.N / scale


def test_encode_decode_roundtrip_and_rounding_error():
    o = Oracle(8, [50, 50, 50], 3, 55, seed=5)
    rng = np.random.default_rng(0)
    z = rng.uniform(-1, 1, o.slots) + 1j * rng.uniform(-1, 1, o.slots)
    for scale in (2.0 ** 20, 2.0 ** 45):
        pt = o.encode(z, scale, 3)
        got = o.decode(pt)
        # rounding moves each coefficient by at most 1/2 -> each slot by at most N/(2*scale);
        # typical is sqrt(N/12)/scale (the O(sqrt N) encoding error of Sec. "HEAAN")
        assert np.abs(got - z).max() <= o.N / (2 * scale)
        if scale < 2.0 ** 40:  # above that the decode's own float rounding shows
            assert np.abs(got - z).std() < 3 * math.sqrt(o.N / 12) / scale
    # fewer values than slots: the rest are zero
    pt = o.encode(z[:10], 2.0 ** 30, 2)
    got = o.decode(pt)
    assert np.abs(got[:10] - z[:10]).max() < 1e-6 and np.abs(got[10:]).max() < 1e-6


def test_encode_product_is_slotwise_product():
    o = Oracle(6, [50, 50], 1, 55, seed=6)
    rng = np.random.default_rng(1)
    z1 = rng.uniform(-1, 1, o.slots)
    z2 = rng.uniform(-1, 1, o.slots) + 1j * rng.uniform(-1, 1, o.slots)
    s = 2.0 ** 30
    a, b = o.encode_coeffs(z1, s), o.encode_coeffs(z2, s)
    Q = o.primes[0] * o.primes[1]
    c = [centred(x, Q) for x in negacyclic_mul([int(x) for x in a], [int(x) for x in b], Q)]
    got = o.decode(o.pt_from_coeffs(c, s * s, 2))
    assert np.abs(got - z1 * z2).max() < 1e-6


def test_pt_coeffs_is_centred_crt():
    o = Oracle(4, [30, 31, 32], 1, 40, seed=8)
    vals = [0, 1, -1, 2 ** 45, -(2 ** 45), 12345678901234567, -98765432109876543, 7, -7, 2 ** 80, -(2 ** 80),
            3, 4, 5, 6, -6]
    pt = o.pt_from_coeffs(vals, 1.0, 3)
    assert o.pt_coeffs(pt) == vals
    co = o.pt_export(pt)
    for i in range(3):
        assert co[i].tolist() == [v % o.primes[i] for v in vals]


# ------------------------------------------------------- automorphism -------
def test_order_of_five_and_galois_elt():
    for log_n in (3, 6, 12):
        two_n = 2 << log_n
        assert pow(5, 1 << (log_n - 1), two_n) == 1
        assert pow(5, 1 << (log_n - 2), two_n) != 1
        assert lib().orc_galois_elt(log_n, 7) == pow(5, 7, two_n)


def test_automorphism_is_evaluation_at_power(small_oracle):
    o = small_oracle
    import ctypes
    u64p = ctypes.POINTER(ctypes.c_uint64)
    psis = np.zeros(o.L + o.K, dtype=np.uint64)
    lib().orc_get_psi(o._h, psis.ctypes.data_as(u64p))
    rng = np.random.default_rng(2)
    for prime, g in [(0, 5), (1, 25), (3, pow(5, 11, 2 * o.N)), (2, 2 * o.N - 1)]:
        q, psi = o.primes[prime], int(psis[prime])
        a = np.array(rng.integers(0, q, o.N), dtype=np.uint64)
        out = np.zeros_like(a)
        lib().orc_automorph_coeff(o._h, a.ctypes.data_as(u64p), g, prime, out.ctypes.data_as(u64p))
        for e in range(1, 2 * o.N, 2):  # every primitive 2N-th root psi^e
            x = pow(psi, e, q)
            lhs = sum(int(out[k]) * pow(x, k, q) for k in range(o.N)) % q
            rhs = sum(int(a[k]) * pow(x, g * k, q) for k in range(o.N)) % q
            assert lhs == rhs
    # composition
    a = np.array(rng.integers(0, o.primes[0], o.N), dtype=np.uint64)
    t1, t2, t3 = (np.zeros_like(a) for _ in range(3))
    lib().orc_automorph_coeff(o._h, a.ctypes.data_as(u64p), 5, 0, t1.ctypes.data_as(u64p))
    lib().orc_automorph_coeff(o._h, t1.ctypes.data_as(u64p), 125, 0, t2.ctypes.data_as(u64p))
    lib().orc_automorph_coeff(o._h, a.ctypes.data_as(u64p), 625, 0, t3.ctypes.data_as(u64p))
    assert t2.tolist() == t3.tolist()


def test_automorphism_rotates_slots_left():
    o = Oracle(6, [50, 50], 1, 55, seed=9)
    import ctypes
    u64p = ctypes.POINTER(ctypes.c_uint64)
    rng = np.random.default_rng(3)
    z = rng.uniform(-1, 1, o.slots) + 1j * rng.uniform(-1, 1, o.slots)
    pt = o.encode(z, 2.0 ** 40, 2)
    for r in (1, 5, o.slots - 1):
        out = np.zeros_like(pt.data)
        lib().orc_automorph_ntt(o._h, pt.data.ctypes.data_as(u64p), o.galois_elt(r), 0, 2, out.ctypes.data_as(u64p))
        got = o.decode(Pt(out, pt.scale))
        assert np.abs(got - np.roll(z, -r)).max() < 1e-8


# ------------------------------------------------------ base conversion -----
def _base_conv(o, rows, src, dst):
    import ctypes
    u64p = ctypes.POINTER(ctypes.c_uint64)
    ptrs = (u64p * len(src))(*[r.ctypes.data_as(u64p) for r in rows])
    srcs = (ctypes.c_int * len(src))(*src)
    out = np.zeros(o.N, dtype=np.uint64)
    lib().orc_base_conv(o._h, ptrs, srcs, len(src), dst, out.ctypes.data_as(u64p))
    return out


def test_base_conversion_bigint_identity():
    o = Oracle(4, [35, 36, 37, 38, 39, 40], 2, 41, seed=10)  # alpha = K = 3
    rng = np.random.default_rng(4)
    for src in ([0, 1, 2], [3, 4, 5], [6, 7, 8], [4], [0, 5]):
        cs = [o.primes[i] for i in src]
        D = math.prod(cs)
        xs = [int(rng.integers(0, 2 ** 62)) * int(rng.integers(0, 2 ** 62)) % D for _ in range(o.N)]
        xs[0], xs[1], xs[2] = 0, D - 1, D // 2
        rows = [np.array([x % c for x in xs], dtype=np.uint64) for c in cs]
        for dst in range(o.L + o.K):
            if dst in src:
                continue
            got = _base_conv(o, rows, src, dst)
            t = o.primes[dst]
            for k, x in enumerate(xs):
                big = 0
                for c in cs:
                    hat = D // c
                    y = (x % c) * pow(hat, -1, c) % c
                    if y > c // 2:
                        y -= c
                    big += y * hat
                assert big % D == x % D                      # it is x plus a multiple of D ...
                assert abs(big) <= len(cs) * D // 2          # ... a small one, centred
                assert int(got[k]) == big % t
        if len(src) == 1:  # one source prime: exactly the centred representative
            got = _base_conv(o, rows, src, (src[0] + 1) % 9)
            t = o.primes[(src[0] + 1) % 9]
            assert got.tolist() == [centred(x, D) % t for x in xs]


# ----------------------------------------------------------------- keys -----
def _poly_mul_ntt(o, a, b, prime):
    q = o.primes[prime]
    return np.array([(int(x) * int(y)) % q for x, y in zip(a, b)], dtype=np.uint64)


def test_switch_key_relation_without_noise():
    o = Oracle(5, [30, 31, 32, 33, 34], 2, 40, seed=11, noise=False)  # alpha 3: digits {0,1,2},{3,4}
    o.keygen()
    o.gen_rot_keys([3])
    g = o.galois_elt(3)
    s = o.secret_coeffs()
    P = math.prod(o.primes[o.L:])
    total = o.L + o.K
    # independent targets in coefficient form, Python integers
    s2 = negacyclic_mul([int(x) for x in s], [int(x) for x in s], 1 << 200)
    s2 = [centred(x, 1 << 200) for x in s2]
    sg = [0] * o.N
    for i in range(o.N):
        t = (i * g) % (2 * o.N)
        if t < o.N:
            sg[t] = int(s[i])
        else:
            sg[t - o.N] = -int(s[i])
    for key_id, target in ((0, s2), (g, sg)):
        key = o.keys[key_id]
        for j in range(o.dnum):
            for i in range(total):
                q = o.primes[i]
                s_ntt = o.ntt(np.array([int(x) % q for x in s], dtype=np.uint64), i)
                lhs = (key[j, 0, i].astype(object) + _poly_mul_ntt(o, key[j, 1, i], s_ntt, i).astype(object)) % q
                lhs = o.ntt(np.array(lhs.tolist(), dtype=np.uint64), i, inverse=True)
                in_digit = i < o.L and i // o.alpha == j
                want = [((P % q) * t) % q if in_digit else 0 for t in target]
                assert lhs.tolist() == want


def test_switch_key_noise_is_small_and_shared_across_primes():
    o = Oracle(5, [30, 31, 32], 3, 40, seed=12)
    o.keygen()
    s = o.secret_coeffs()
    key = o.keys[0]
    errs = []
    for i in range(o.L + o.K):
        q = o.primes[i]
        s_ntt = o.ntt(np.array([int(x) % q for x in s], dtype=np.uint64), i)
        lhs = (key[1, 0, i].astype(object) + _poly_mul_ntt(o, key[1, 1, i], s_ntt, i).astype(object)) % q
        co = o.ntt(np.array(lhs.tolist(), dtype=np.uint64), i, inverse=True)
        if i == 1:  # remove P*s^2 on the digit's own prime
            s2 = negacyclic_mul([int(x) % q for x in s], [int(x) % q for x in s], q)
            P = o.primes[3] % q
            co = np.array([(int(c) - P * t) % q for c, t in zip(co, s2)], dtype=np.uint64)
        errs.append([centred(int(c), q) for c in co])
    assert all(e == errs[0] for e in errs)
    assert max(abs(x) for x in errs[0]) <= 19 and any(errs[0])


# ------------------------------------------------- encrypt / decrypt --------
def test_encrypt_decrypt_identity_without_noise():
    o = Oracle(6, [40, 41, 42], 1, 50, seed=13, noise=False)
    rng = np.random.default_rng(5)
    m = [int(x) for x in rng.integers(-2 ** 50, 2 ** 50, o.N)]
    pt = o.pt_from_coeffs(m, 1.0, 3)
    ct = o.encrypt(pt)
    assert o.pt_coeffs(o.decrypt(ct)) == m
    ct2 = o.encrypt(pt)
    assert not np.array_equal(ct.data, ct2.data)  # fresh randomness per encryption
    # c1 is the uniform polynomial of the stream (coefficient form), c0 = m - a*s
    c1 = o.export(ct)[1]
    for i in range(3):
        q = o.primes[i]
        want = [lib().orc_rnd(13, 2, 0, i * o.N + k) % q for k in range(o.N)]
        assert c1[i].tolist() == want
    s = [int(x) for x in o.secret_coeffs()]
    q = o.primes[0]
    a_s = negacyclic_mul([int(x) for x in c1[0]], [x % q for x in s], q)
    assert o.export(ct)[0][0].tolist() == [(mm - t) % q for mm, t in zip(m, a_s)]


def test_encrypt_noise_is_bounded_gaussian():
    o = Oracle(8, [40, 41], 1, 50, seed=14)
    m = [0] * o.N
    ct = o.encrypt(o.pt_from_coeffs(m, 1.0, 2))
    e = o.pt_coeffs(o.decrypt(ct))
    assert max(abs(x) for x in e) <= 19
    assert 2.0 < np.std(e) < 4.5
    want = [lib().orc_gauss_from_word(lib().orc_rnd(14, 3, 0, k)) for k in range(o.N)]
    assert e == want


# ----------------------------------------------------- key switching --------
def test_mod_down_bigint_identity():
    o = Oracle(4, [35, 36, 37, 38], 2, 39, seed=15)  # K = 2
    import ctypes
    u64p = ctypes.POINTER(ctypes.c_uint64)
    rng = np.random.default_rng(6)
    for l in (4, 3, 1):
        qs, ps = o.primes[:l], o.primes[o.L:]
        Q, P = math.prod(qs), math.prod(ps)
        xs = [int(rng.integers(0, 2 ** 62)) ** 3 % (Q * P) for _ in range(o.N)]
        acc = np.zeros((l + o.K, o.N), dtype=np.uint64)
        for i, q in enumerate(qs + ps):
            acc[i] = np.array([x % q for x in xs], dtype=np.uint64)
        # the oracle works in NTT form
        for i in range(l):
            acc[i] = o.ntt(acc[i], i)
        for m in range(o.K):
            acc[l + m] = o.ntt(acc[l + m], o.L + m)
        out = np.zeros((l, o.N), dtype=np.uint64)
        lib().orc_mod_down(o._h, acc.ctypes.data_as(u64p), l, out.ctypes.data_as(u64p))
        for i in range(l):
            out[i] = o.ntt(out[i], i, inverse=True)
        for k, x in enumerate(xs):
            big = 0
            for p in ps:
                hat = P // p
                y = (x % p) * pow(hat, -1, p) % p
                if y > p // 2:
                    y -= p
                big += y * hat
            assert (x - big) % P == 0
            want = (x - big) // P
            assert abs(want - x / P) <= o.K / 2 + 0.5 + 1e-9
            assert [int(out[i][k]) for i in range(l)] == [want % q for q in qs]


@pytest.mark.parametrize("q_bits,dnum,levels", [([30, 31, 32], 3, (3, 2, 1)), ([30, 31, 32, 33, 34], 2, (5, 4, 3, 2)),
                                                ([30, 31, 32, 33], 1, (4, 2))])
def test_key_switch_exact_relation_without_noise(q_bits, dnum, levels):
    o = Oracle(5, q_bits, dnum, 36, seed=16, noise=False)
    o.keygen()
    s = [int(x) for x in o.secret_coeffs()]
    h = sum(abs(x) for x in s)
    rng = np.random.default_rng(7)
    for l in levels:
        qs = o.primes[:l]
        Q = math.prod(qs)
        d_int = [int(rng.integers(0, 2 ** 62)) ** 4 % Q for _ in range(o.N)]
        d = np.stack([o.ntt(np.array([x % q for x in d_int], dtype=np.uint64), i) for i, q in enumerate(qs)])
        ks0, ks1 = o.key_switch(d, 0)
        got = o.pt_coeffs(o.decrypt(Ct(np.stack([ks0, ks1]), 1.0)))
        s2 = negacyclic_mul(s, s, Q)
        want = negacyclic_mul(d_int, s2, Q)
        rho = [centred((g - w) % Q, Q) for g, w in zip(got, want)]
        assert max(abs(x) for x in rho) <= (o.K / 2 + 0.5) * (1 + h)


def test_relinearize_and_rotate_against_plain_slots():
    o = Oracle(8, [50, 50, 50, 50], 2, 55, seed=17)
    o.keygen()
    o.gen_rot_keys([1, 3, o.slots - 4, 4])
    rng = np.random.default_rng(8)
    z1 = rng.uniform(-1, 1, o.slots)
    z2 = rng.uniform(-1, 1, o.slots)
    s = 2.0 ** 40
    c1, c2 = o.encrypt(o.encode(z1, s, 4)), o.encrypt(o.encode(z2, s, 4))
    dec = lambda c: o.decode(o.decrypt(c)).real
    tol = 1e-7
    assert np.abs(dec(c1) - z1).max() < tol
    assert np.abs(dec(o.add(c1, c2)) - (z1 + z2)).max() < tol
    assert np.abs(dec(o.sub(c1, c2)) - (z1 - z2)).max() < tol
    m3 = o.mul_no_relin(c1, c2)
    assert m3.polys == 3 and np.abs(dec(m3) - z1 * z2).max() < tol
    m2 = o.relinearize(m3)
    assert m2.polys == 2 and np.abs(dec(m2) - z1 * z2).max() < tol
    assert np.array_equal(o.mul(c1, c2).data, m2.data)
    r = o.rescale(m2)
    assert r.limbs == 3 and abs(r.scale - s * s / o.primes[3]) < 1e-3 * r.scale
    assert np.abs(dec(r) - z1 * z2).max() < 1e-6
    for k in (1, 3):
        assert np.abs(dec(o.rot_left(c1, k)) - np.roll(z1, -k)).max() < tol
    assert np.abs(dec(o.rot_right(c1, 4)) - np.roll(z1, 4)).max() < tol
    assert np.abs(dec(o.rot_left(o.rot_left(c1, 1), 3)) - np.roll(z1, -4)).max() < tol
    assert np.abs(dec(o.rot_right(o.rot_left(c1, 4), 4)) - z1).max() < tol
    assert np.array_equal(o.rot_left(c1, 0).data, c1.data)
    assert np.array_equal(o.rot_left(c1, o.slots).data, c1.data)
    # rotation at a lower level uses the same key restricted to the limbs present
    low = o.rescale(o.mul_scalar(c1, 1.0, o.primes[3]))
    assert low.limbs == 3 and np.abs(dec(o.rot_left(low, 3)) - np.roll(z1, -3)).max() < tol
    low2 = o.rescale(o.mul_scalar(low, 1.0, o.primes[2]))
    assert low2.limbs == 2 and np.abs(dec(o.rot_left(low2, 1)) - np.roll(z1, -1)).max() < tol


def test_plain_and_scalar_ops_against_plain_slots():
    o = Oracle(7, [50, 50, 50], 3, 55, seed=18)
    rng = np.random.default_rng(9)
    z = rng.uniform(-1, 1, o.slots)
    w = rng.uniform(-1, 1, o.slots)
    s = 2.0 ** 40
    c = o.encrypt(o.encode(z, s, 3))
    dec = lambda x: o.decode(o.decrypt(x)).real
    pw = o.encode(w, s, 3)
    assert np.abs(dec(o.add_plain(c, pw)) - (z + w)).max() < 1e-7
    assert np.abs(dec(o.sub_plain(c, pw)) - (z - w)).max() < 1e-7
    assert np.abs(dec(o.mul_plain(c, pw)) - z * w).max() < 1e-7
    assert np.abs(dec(o.add_scalar(c, 0.625)) - (z + 0.625)).max() < 1e-7
    assert np.abs(dec(o.sub_scalar(c, -1.5)) - (z + 1.5)).max() < 1e-7
    m = o.mul_scalar(c, -0.3, 2.0 ** 30)
    assert abs(m.scale - s * 2.0 ** 30) == 0 and np.abs(dec(m) + 0.3 * z).max() < 1e-7
    assert np.array_equal(o.mul_scalar(c, 1.0, 1.0).data, c.data)
    # scalar add on a scale beyond 2^63
    big = o.mul_plain(c, pw)
    assert np.abs(dec(o.add_scalar(big, 0.25)) - (z * w + 0.25)).max() < 1e-7


def test_rescale_bigint_identity():
    o = Oracle(5, [33, 34, 35, 36], 1, 40, seed=19)
    rng = np.random.default_rng(10)
    for l in (4, 3, 2):
        qs = o.primes[:l]
        Q, ql = math.prod(qs), qs[-1]
        h = ql // 2
        xs = [[int(rng.integers(0, 2 ** 62)) ** 3 % Q for _ in range(o.N)] for _ in range(2)]
        xs[0][0], xs[0][1], xs[0][2] = 0, ql - h - 1, ql - h  # around the rounding boundary
        coeff = np.zeros((2, l, o.N), dtype=np.uint64)
        for p in range(2):
            for i, q in enumerate(qs):
                coeff[p, i] = np.array([x % q for x in xs[p]], dtype=np.uint64)
        ct = o.import_ct(coeff, float(ql) * 4.0)
        out = o.rescale(ct)
        assert out.limbs == l - 1 and out.scale == 4.0
        got = o.export(out)
        for p in range(2):
            for k, x in enumerate(xs[p]):
                want = (x + h) // ql
                assert [int(got[p, i, k]) for i in range(l - 1)] == [want % q for q in qs[:-1]]


def test_division_profile_and_error_paths():
    o = Oracle(5, [30, 31, 32], 3, 40, seed=20)
    o.keygen()
    c = o.encrypt(o.encode([0.5], 2.0 ** 20, 3))
    assert o.max_scalar_div(c, float("inf")) == o.primes[2]
    assert o.max_scalar_div(c, o.primes[2]) == 1      # strictly below the bound
    assert o.max_scalar_div(c, o.primes[2] + 1) == o.primes[2]
    assert np.array_equal(o.div_scalar(c, 1).data, c.data)
    with pytest.raises(OracleError):
        o.div_scalar(c, o.primes[1])
    low = o.rescale(o.rescale(c))
    assert low.limbs == 1 and o.max_scalar_div(low, float("inf")) == 1
    with pytest.raises(OracleError):
        o.rescale(low)
    with pytest.raises(OracleError):
        o.add(c, low)
    with pytest.raises(OracleError):
        o.add(c, o.mul_scalar(c, 1.0, 2.0))
    with pytest.raises(OracleError):
        o.rot_left(c, 1)  # no key generated for this amount


def test_round_half_away():
    assert [round_half_away(v) for v in (0.5, -0.5, 1.5, 2.5, -2.5, 0.49999999999999994, 1e300 % 7.0)] == \
        [1, -1, 2, 3, -3, 0, round_half_away(1e300 % 7.0)]
    assert round_half_away(2.0 ** 80) == 2 ** 80 and round_half_away(-(2.0 ** 53 + 2)) == -(2 ** 53 + 2)


def test_add_of_two_and_three_polynomial_ciphertexts_is_exact_on_the_plaintext():
    """add / sub of operands with different polynomial counts (a two-polynomial ciphertext is a three-polynomial one
    with c2 = 0): decryption is linear, so the decrypted coefficients of the sum are exactly the sums of the decrypted
    coefficients modulo every prime -- an identity that does not go through the addition's own code.  A planted
    mistake (c2 dropped) breaks it."""
    o = Oracle(8, [40, 36, 30], 3, 50, seed=41)
    o.keygen()
    rng = np.random.default_rng(4)
    za, zb, zc = (rng.uniform(-1, 1, o.slots) for _ in range(3))
    a = o.encrypt(o.encode(za, 2.0 ** 20, 3))
    b = o.encrypt(o.encode(zb, 2.0 ** 20, 3))
    c = o.encrypt(o.encode(zc, 2.0 ** 40, 3))
    three = o.mul_no_relin(a, b)                                  # scale 2^40, three polynomials
    assert three.polys == 3 and c.polys == 2
    q = np.asarray(o.primes[:3], dtype=object)[:, None]
    dec = lambda ct: o.pt_export(o.decrypt(ct)).astype(object)
    for first, second, sign in ((three, c, 1), (c, three, 1), (three, c, -1)):
        out = o.add(first, second) if sign == 1 else o.sub(first, second)
        assert out.polys == 3 and out.scale == three.scale
        assert np.array_equal(dec(out), (dec(first) + sign * dec(second)) % q)
    with pytest.raises(Exception):
        o.sub(c, three)                                           # a two-polynomial minuend has no c2 to subtract from
    # the value: slot-wise za zb + zc
    got = o.decode(o.decrypt(o.add(three, c))).real
    assert np.abs(got - (za * zb + zc)).max() <= 1e-3
    # planted mistake: the sum with c2 left out decrypts to something else
    from oracle.ckks import Ct
    out = o.add(three, c)
    wrong = Ct(out.data[:2].copy(), out.scale)
    assert not np.array_equal(dec(wrong), (dec(three) + dec(c)) % q)
