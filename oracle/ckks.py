"""Python face of the CPU oracle (TEST INFRASTRUCTURE, not product code).

Thin ctypes layer over ``ckks_oracle.c`` plus the few steps that are easier to
read with Python integers: the centred CRT lift used by decode, and the exact
rounding of real scalars to integers.  Only ``tests/``, the smoke check and the
``cpu_baseline`` leg of the benchmark may import this package; it shares no
code with the GPU library.

Names follow the HISA table of the CHET paper (Fig. "Instructions of the
HISA"); everything below that table is the plain definition of RNS-CKKS with
hybrid key switching, see the header of ``ckks_oracle.c``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ckks_oracle.c")
_LIB = os.path.join(_HERE, "libckks_oracle.so")

u64p = C.POINTER(C.c_uint64)
i64p = C.POINTER(C.c_int64)
f64p = C.POINTER(C.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no vector intrinsics)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_int), C.c_int, C.c_int, C.c_uint64, C.c_int]
        L.orc_create_ex.restype = C.c_void_p
        L.orc_create_ex.argtypes = L.orc_create.argtypes + [C.c_double, C.c_int, C.c_int]
        L.orc_gauss_table_for.restype = C.c_int
        L.orc_gauss_table_for.argtypes = [C.c_double, u64p]
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_rnd.restype = C.c_uint64
        L.orc_rnd.argtypes = [C.c_uint64] * 4
        L.orc_gauss_from_word.restype = C.c_int64
        L.orc_gauss_from_word.argtypes = [C.c_uint64]
        L.orc_ternary_from_word.restype = C.c_int64
        L.orc_ternary_from_word.argtypes = [C.c_uint64]
        L.orc_is_prime.argtypes = [C.c_uint64]
        L.orc_next_prime.restype = C.c_uint64
        L.orc_next_prime.argtypes = [C.c_int, C.c_int, u64p, C.c_int]
        L.orc_find_psi.restype = C.c_uint64
        L.orc_find_psi.argtypes = [C.c_uint64, C.c_int]
        L.orc_galois_elt.restype = C.c_uint64
        L.orc_galois_elt.argtypes = [C.c_int, C.c_uint64]
        L.orc_mulmod.restype = C.c_uint64
        L.orc_mulmod.argtypes = [C.c_uint64] * 3
        L.orc_powmod.restype = C.c_uint64
        L.orc_powmod.argtypes = [C.c_uint64] * 3
        for name in ("orc_num_primes", "orc_num_special", "orc_alpha"):
            getattr(L, name).argtypes = [C.c_void_p]
        vp = C.c_void_p
        L.orc_get_primes.argtypes = [vp, u64p]
        L.orc_get_psi.argtypes = [vp, u64p]
        L.orc_get_secret_coef.argtypes = [vp, i64p]
        L.orc_gauss_table.argtypes = [u64p]
        L.orc_ntt.argtypes = [vp, C.c_int, u64p]
        L.orc_intt.argtypes = [vp, C.c_int, u64p]
        L.orc_sample_uniform.argtypes = [vp, C.c_uint64, C.c_uint64, C.c_int, u64p]
        L.orc_sample_error.argtypes = [vp, C.c_uint64, C.c_uint64, i64p]
        L.orc_signed_to_ntt.argtypes = [vp, i64p, C.c_int, u64p]
        L.orc_encode.argtypes = [C.c_int, f64p, f64p, C.c_uint64, C.c_double, i64p]
        L.orc_decode.argtypes = [C.c_int, f64p, f64p, C.c_uint64, C.c_double, f64p, f64p]
        L.orc_encrypt.argtypes = [vp, u64p, C.c_int, C.c_uint64, u64p]
        L.orc_decrypt.argtypes = [vp, u64p, C.c_int, C.c_int, u64p]
        L.orc_to_coeff.argtypes = [vp, u64p, C.c_int, C.c_int]
        L.orc_to_ntt.argtypes = [vp, u64p, C.c_int, C.c_int]
        L.orc_add.argtypes = [vp, u64p, u64p, C.c_int, C.c_int, C.c_int, u64p]
        L.orc_add_plain.argtypes = [vp, u64p, u64p, C.c_int, C.c_int, C.c_int, u64p]
        L.orc_add_const.argtypes = [vp, u64p, u64p, C.c_int, C.c_int, C.c_int, u64p]
        L.orc_mul_plain.argtypes = [vp, u64p, u64p, C.c_int, C.c_int, u64p]
        L.orc_mul_const.argtypes = [vp, u64p, u64p, C.c_int, C.c_int, u64p]
        L.orc_mul_no_relin.argtypes = [vp, u64p, u64p, C.c_int, u64p]
        L.orc_automorph_coeff.argtypes = [vp, u64p, C.c_uint64, C.c_int, u64p]
        L.orc_automorph_ntt.argtypes = [vp, u64p, C.c_uint64, C.c_int, C.c_int, u64p]
        L.orc_base_conv.argtypes = [vp, C.POINTER(u64p), C.POINTER(C.c_int), C.c_int, C.c_int, u64p]
        L.orc_gen_switch_key.argtypes = [vp, C.c_uint64, u64p, u64p]
        L.orc_secret_squared.argtypes = [vp, u64p]
        L.orc_secret_automorph.argtypes = [vp, C.c_uint64, u64p]
        L.orc_mod_down.argtypes = [vp, u64p, C.c_int, u64p]
        L.orc_mod_down_rescale.argtypes = [vp, u64p, C.c_int, u64p]
        L.orc_key_switch.argtypes = [vp, u64p, C.c_int, u64p, u64p, u64p]
        L.orc_key_switch_acc.argtypes = [vp, u64p, C.c_int, u64p, u64p, u64p]
        L.orc_fma_const.argtypes = [vp, u64p, u64p, u64p, C.POINTER(C.c_int), C.c_int]
        L.orc_fma_plain.argtypes = [vp, u64p, u64p, u64p, C.POINTER(C.c_int), C.c_int]
        L.orc_rotate.argtypes = [vp, u64p, C.c_int, C.c_uint64, u64p, u64p]
        L.orc_relinearize.argtypes = [vp, u64p, C.c_int, u64p, u64p]
        L.orc_rescale.argtypes = [vp, u64p, C.c_int, C.c_int, u64p]
    return _lib


def _p(a: np.ndarray):
    assert a.dtype == np.uint64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(u64p)


def round_half_away(v: float) -> int:
    """Nearest integer to the exact value of the double v, ties away from zero."""
    f = Fraction(v)
    m = (abs(f) + Fraction(1, 2)).__floor__()
    return -m if f < 0 else m


class OracleError(Exception):
    """Raised where the GPU library returns an error code (same conditions)."""


@dataclass
class Pt:
    data: np.ndarray  # [l][N] uint64, NTT form
    scale: float

    @property
    def limbs(self) -> int:
        return self.data.shape[0]


@dataclass
class Ct:
    data: np.ndarray  # [polys][l][N] uint64, NTT form
    scale: float

    @property
    def polys(self) -> int:
        return self.data.shape[0]

    @property
    def limbs(self) -> int:
        return self.data.shape[1]


class Oracle:
    """One parameter set + secret key + evaluation keys."""

    def __init__(self, log_n, q_bits, dnum, special_bits, seed, noise=True, sigma=3.2, secret_kind=0, hamming_weight=0):
        """sigma: parameter of the error distribution; secret_kind 0: uniform ternary secret, 1: exactly
        hamming_weight non-zero coefficients (see orc_create_ex)."""
        self.log_n, self.N, self.slots = log_n, 1 << log_n, 1 << (log_n - 1)
        self.L, self.dnum = len(q_bits), dnum
        qb = (C.c_int * len(q_bits))(*q_bits)
        self._h = lib().orc_create_ex(log_n, len(q_bits), qb, dnum, special_bits, seed, 1 if noise else 0,
                                      float(sigma), int(secret_kind), int(hamming_weight))
        if not self._h:
            raise OracleError("bad parameters")
        self.K = lib().orc_num_special(self._h)
        self.alpha = lib().orc_alpha(self._h)
        buf = np.zeros(self.L + self.K, dtype=np.uint64)
        lib().orc_get_primes(self._h, _p(buf))
        self.primes = [int(x) for x in buf]  # q_0..q_{L-1}, p_0..p_{K-1}
        self.seed = seed
        self.enc_counter = 0
        self.keys = {}  # key_id (0 = relin, else galois element) -> [dnum][2][L+K][N]

    def __del__(self):
        try:
            lib().orc_destroy(self._h)
        except Exception:
            pass

    # ---- raw transforms -------------------------------------------------
    def ntt(self, a: np.ndarray, prime: int, inverse=False) -> np.ndarray:
        out = np.ascontiguousarray(a, dtype=np.uint64).copy()
        (lib().orc_intt if inverse else lib().orc_ntt)(self._h, prime, _p(out))
        return out

    def secret_coeffs(self) -> np.ndarray:
        s = np.zeros(self.N, dtype=np.int64)
        lib().orc_get_secret_coef(self._h, s.ctypes.data_as(i64p))
        return s

    # ---- keys -----------------------------------------------------------
    def keygen(self):
        """Relinearisation key (key id 0): switches from s^2 to s."""
        tgt = np.zeros((self.L + self.K, self.N), dtype=np.uint64)
        lib().orc_secret_squared(self._h, _p(tgt))
        key = np.zeros((self.dnum, 2, self.L + self.K, self.N), dtype=np.uint64)
        lib().orc_gen_switch_key(self._h, 0, _p(tgt), _p(key))
        self.keys[0] = key

    def galois_elt(self, steps: int) -> int:
        return int(lib().orc_galois_elt(self.log_n, steps % self.slots))

    def gen_rot_keys(self, left_steps):
        """Rotation-key selection (Sec. "Rotation Keys Selection"): one key per distinct amount."""
        for r in left_steps:
            r %= self.slots
            if r == 0:
                continue
            g = self.galois_elt(r)
            if g in self.keys:
                continue
            tgt = np.zeros((self.L + self.K, self.N), dtype=np.uint64)
            lib().orc_secret_automorph(self._h, g, _p(tgt))
            key = np.zeros((self.dnum, 2, self.L + self.K, self.N), dtype=np.uint64)
            lib().orc_gen_switch_key(self._h, g, _p(tgt), _p(key))
            self.keys[g] = key

    # ---- encode / decode --------------------------------------------------
    def encode_coeffs(self, values, scale: float) -> np.ndarray:
        """Complex (or real) slot vector -> signed integer coefficients [N]."""
        v = np.asarray(values)
        re = np.ascontiguousarray(v.real, dtype=np.float64)
        im = np.ascontiguousarray(v.imag, dtype=np.float64) if np.iscomplexobj(v) else None
        coef = np.zeros(self.N, dtype=np.int64)
        lib().orc_encode(self.log_n, re.ctypes.data_as(f64p),
                         im.ctypes.data_as(f64p) if im is not None else None,
                         len(re), float(scale), coef.ctypes.data_as(i64p))
        return coef

    def pt_from_coeffs(self, coeffs, scale: float, limbs: int) -> Pt:
        """Signed integer coefficients (any size) -> plaintext in NTT form."""
        data = np.zeros((limbs, self.N), dtype=np.uint64)
        ints = [int(x) for x in coeffs]
        assert len(ints) == self.N
        for i in range(limbs):
            q = self.primes[i]
            data[i] = np.array([x % q for x in ints], dtype=np.uint64)
        lib().orc_to_ntt(self._h, _p(data), 1, limbs)
        return Pt(data, float(scale))

    def encode(self, values, scale: float, limbs: int) -> Pt:
        return self.pt_from_coeffs(self.encode_coeffs(values, scale), scale, limbs)

    def pt_coeffs(self, pt: Pt):
        """Centred CRT lift of the plaintext's coefficients: list of Python ints."""
        l = pt.limbs
        co = pt.data.copy()
        lib().orc_to_coeff(self._h, _p(co), 1, l)
        qs = self.primes[:l]
        Q = 1
        for q in qs:
            Q *= q
        # x = sum_i [x_i * (Q/q_i)^-1]_{q_i} * (Q/q_i)  mod Q, then centre
        terms = []
        for q in qs:
            hat = Q // q
            terms.append((hat, pow(hat % q, -1, q), q))
        out = []
        rows = [co[i].tolist() for i in range(l)]
        for k in range(self.N):
            x = 0
            for i, (hat, inv, q) in enumerate(terms):
                x += ((rows[i][k] * inv) % q) * hat
            x %= Q
            if x > Q // 2:
                x -= Q
            out.append(x)
        return out

    def decode(self, pt: Pt, count=None) -> np.ndarray:
        count = self.slots if count is None else count
        m = self.pt_coeffs(pt)
        hi = np.array([float(x) for x in m], dtype=np.float64)
        lo = np.array([float(x - int(h)) for x, h in zip(m, hi)], dtype=np.float64)
        re = np.zeros(count, dtype=np.float64)
        im = np.zeros(count, dtype=np.float64)
        lib().orc_decode(self.log_n, hi.ctypes.data_as(f64p), lo.ctypes.data_as(f64p), count,
                         float(pt.scale), re.ctypes.data_as(f64p), im.ctypes.data_as(f64p))
        return re + 1j * im

    # ---- encryption profile ----------------------------------------------
    def encrypt(self, pt: Pt) -> Ct:
        l = pt.limbs
        ct = np.zeros((2, l, self.N), dtype=np.uint64)
        lib().orc_encrypt(self._h, _p(pt.data), l, self.enc_counter, _p(ct))
        self.enc_counter += 1
        return Ct(ct, pt.scale)

    def decrypt(self, ct: Ct) -> Pt:
        pt = np.zeros((ct.limbs, self.N), dtype=np.uint64)
        lib().orc_decrypt(self._h, _p(ct.data), ct.polys, ct.limbs, _p(pt))
        return Pt(pt, ct.scale)

    def copy(self, ct: Ct) -> Ct:
        return Ct(ct.data.copy(), ct.scale)

    def export(self, ct: Ct) -> np.ndarray:
        """Coefficient form, canonical residues, [polys][l][N]."""
        co = ct.data.copy()
        lib().orc_to_coeff(self._h, _p(co), ct.polys, ct.limbs)
        return co

    def import_ct(self, coeff: np.ndarray, scale: float) -> Ct:
        d = np.ascontiguousarray(coeff, dtype=np.uint64).copy()
        lib().orc_to_ntt(self._h, _p(d), d.shape[0], d.shape[1])
        return Ct(d, float(scale))

    def pt_export(self, pt: Pt) -> np.ndarray:
        co = pt.data.copy()
        lib().orc_to_coeff(self._h, _p(co), 1, pt.limbs)
        return co

    # ---- add / sub --------------------------------------------------------
    @staticmethod
    def _same_scale(a: float, b: float) -> bool:
        return abs(a - b) <= 2.0 ** -30 * max(abs(a), abs(b))

    def _check_pair(self, a, b, need_scale=True):
        if a.limbs != b.limbs:
            raise OracleError("level mismatch")
        if need_scale and not self._same_scale(a.scale, b.scale):
            raise OracleError("scale mismatch")

    def add(self, a: Ct, b: Ct, subtract=False) -> Ct:
        self._check_pair(a, b)
        if a.polys != b.polys:
            # a two-polynomial ciphertext is a three-polynomial one with c2 = 0
            if a.polys < b.polys and subtract:
                raise OracleError("size mismatch")
            polys = max(a.polys, b.polys)
            pad = lambda c: Ct(np.concatenate([c.data, np.zeros((polys - c.polys,) + c.data.shape[1:], np.uint64)]), c.scale)
            a, b = pad(a), pad(b)
        out = np.zeros_like(a.data)
        lib().orc_add(self._h, _p(a.data), _p(b.data), a.polys, a.limbs, int(subtract), _p(out))
        return Ct(out, a.scale)

    def sub(self, a: Ct, b: Ct) -> Ct:
        return self.add(a, b, subtract=True)

    def add_plain(self, a: Ct, p: Pt, subtract=False) -> Ct:
        self._check_pair(a, p)
        out = np.zeros_like(a.data)
        lib().orc_add_plain(self._h, _p(a.data), _p(p.data), a.polys, a.limbs, int(subtract), _p(out))
        return Ct(out, a.scale)

    def sub_plain(self, a: Ct, p: Pt) -> Ct:
        return self.add_plain(a, p, subtract=True)

    def _int_mod_primes(self, v: int, l: int) -> np.ndarray:
        return np.array([v % self.primes[i] for i in range(l)], dtype=np.uint64)

    def add_scalar(self, a: Ct, x: float, subtract=False) -> Ct:
        """Adds round(x * scale) to the constant coefficient of c0."""
        v = self._int_mod_primes(round_half_away(float(x) * a.scale), a.limbs)
        out = np.zeros_like(a.data)
        lib().orc_add_const(self._h, _p(a.data), _p(v), a.polys, a.limbs, int(subtract), _p(out))
        return Ct(out, a.scale)

    def sub_scalar(self, a: Ct, x: float) -> Ct:
        return self.add_scalar(a, x, subtract=True)

    # ---- multiply ---------------------------------------------------------
    def mul_plain(self, a: Ct, p: Pt) -> Ct:
        self._check_pair(a, p, need_scale=False)
        out = np.zeros_like(a.data)
        lib().orc_mul_plain(self._h, _p(a.data), _p(p.data), a.polys, a.limbs, _p(out))
        return Ct(out, a.scale * p.scale)

    def mul_scalar(self, a: Ct, x: float, x_scale: float) -> Ct:
        """Every residue times round(x * x_scale); the scale grows by x_scale."""
        v = self._int_mod_primes(round_half_away(float(x) * float(x_scale)), a.limbs)
        out = np.zeros_like(a.data)
        lib().orc_mul_const(self._h, _p(a.data), _p(v), a.polys, a.limbs, _p(out))
        return Ct(out, a.scale * float(x_scale))

    def mul_int(self, a: Ct, v: int, x_scale: float) -> Ct:
        """Every residue times the integer v (fixed-point weight already rounded)."""
        vm = self._int_mod_primes(int(v), a.limbs)
        out = np.zeros_like(a.data)
        lib().orc_mul_const(self._h, _p(a.data), _p(vm), a.polys, a.limbs, _p(out))
        return Ct(out, a.scale * float(x_scale))

    def mul_no_relin(self, a: Ct, b: Ct) -> Ct:
        self._check_pair(a, b, need_scale=False)
        if a.polys != 2 or b.polys != 2:
            raise OracleError("size mismatch")
        out = np.zeros((3, a.limbs, self.N), dtype=np.uint64)
        lib().orc_mul_no_relin(self._h, _p(a.data), _p(b.data), a.limbs, _p(out))
        return Ct(out, a.scale * b.scale)

    def relinearize(self, a: Ct) -> Ct:
        if a.polys == 2:
            return self.copy(a)
        if 0 not in self.keys:
            raise OracleError("no key")
        out = np.zeros((2, a.limbs, self.N), dtype=np.uint64)
        lib().orc_relinearize(self._h, _p(a.data), a.limbs, _p(self.keys[0]), _p(out))
        return Ct(out, a.scale)

    def mul(self, a: Ct, b: Ct) -> Ct:
        return self.relinearize(self.mul_no_relin(a, b))

    # ---- rotations --------------------------------------------------------
    def rot_left(self, a: Ct, steps: int) -> Ct:
        r = steps % self.slots
        if r == 0:
            return self.copy(a)
        if a.polys != 2:
            raise OracleError("size mismatch")
        g = self.galois_elt(r)
        if g not in self.keys:
            raise OracleError("no key")
        out = np.zeros_like(a.data)
        lib().orc_rotate(self._h, _p(a.data), a.limbs, g, _p(self.keys[g]), _p(out))
        return Ct(out, a.scale)

    def rot_right(self, a: Ct, steps: int) -> Ct:
        return self.rot_left(a, self.slots - (steps % self.slots))

    def key_switch(self, d: np.ndarray, key_id: int):
        """Raw key switch of one NTT-form polynomial [l][N] -> (ks0, ks1)."""
        l = d.shape[0]
        ks0 = np.zeros((l, self.N), dtype=np.uint64)
        ks1 = np.zeros((l, self.N), dtype=np.uint64)
        lib().orc_key_switch(self._h, _p(np.ascontiguousarray(d)), l, _p(self.keys[key_id]), _p(ks0), _p(ks1))
        return ks0, ks1

    # ---- the key switch in two halves, for sums formed before the division by P ----
    def ext_primes(self, l: int):
        """Indices (into self.primes) of the l + K limbs a key-switch accumulator lives on."""
        return list(range(l)) + [self.L + m for m in range(self.K)]

    def key_switch_acc(self, d: np.ndarray, key_id: int):
        """Decompose, ModUp and inner product with the key: the accumulators (acc_b, acc_a), each [l + K][N], whose
        mod_down gives the key switch of d."""
        l = d.shape[0]
        acc_b = np.zeros((l + self.K, self.N), dtype=np.uint64)
        acc_a = np.zeros((l + self.K, self.N), dtype=np.uint64)
        lib().orc_key_switch_acc(self._h, _p(np.ascontiguousarray(d)), l, _p(self.keys[key_id]), _p(acc_b), _p(acc_a))
        return acc_b, acc_a

    def mod_down(self, acc: np.ndarray, l: int) -> np.ndarray:
        out = np.zeros((l, self.N), dtype=np.uint64)
        lib().orc_mod_down(self._h, _p(np.ascontiguousarray(acc)), l, _p(out))
        return out

    def mod_down_rescale(self, acc: np.ndarray, l: int) -> np.ndarray:
        """acc [l + K][N] (NTT form) divided by q_{l-1} P in one base conversion: [l - 1][N]."""
        out = np.zeros((l - 1, self.N), dtype=np.uint64)
        lib().orc_mod_down_rescale(self._h, _p(np.ascontiguousarray(acc)), l, _p(out))
        return out

    def automorph_ntt(self, x: np.ndarray, g: int) -> np.ndarray:
        """sigma_g of an NTT-form polynomial [l][N] on the primes q_0..q_{l-1}."""
        out = np.zeros_like(x)
        lib().orc_automorph_ntt(self._h, _p(np.ascontiguousarray(x)), g, 0, x.shape[0], _p(out))
        return out

    def fma_const(self, acc: np.ndarray, x: np.ndarray, v: int, primes):
        """acc += x * v limb-wise on the listed primes (in place)."""
        idx = (C.c_int * len(primes))(*primes)
        w = np.array([int(v) % self.primes[i] for i in primes], dtype=np.uint64)
        lib().orc_fma_const(self._h, _p(acc), _p(np.ascontiguousarray(x)), _p(w), idx, len(primes))

    def fma_plain(self, acc: np.ndarray, x: np.ndarray, pt: np.ndarray, primes):
        """acc += x (.) pt slot-wise on the listed primes (in place)."""
        idx = (C.c_int * len(primes))(*primes)
        lib().orc_fma_plain(self._h, _p(acc), _p(np.ascontiguousarray(x)), _p(np.ascontiguousarray(pt)), idx, len(primes))

    def residues_ntt(self, coeffs, primes) -> np.ndarray:
        """Signed integer coefficients -> NTT-form residues on the listed primes, [len(primes)][N]."""
        co = np.ascontiguousarray(coeffs, dtype=np.int64)
        out = np.zeros((len(primes), self.N), dtype=np.uint64)
        for k, i in enumerate(primes):
            lib().orc_signed_to_ntt(self._h, co.ctypes.data_as(i64p), i, _p(out[k]))
        return out

    # ---- division profile -------------------------------------------------
    def max_scalar_div(self, a: Ct, ub: float) -> int:
        """The last coprime modulus of a if it is below ub, else 1 (RNS reading of maxScalarDiv)."""
        if a.limbs > 1 and self.primes[a.limbs - 1] < ub:
            return self.primes[a.limbs - 1]
        return 1

    def div_scalar(self, a: Ct, d: int) -> Ct:
        if d == 1:
            return self.copy(a)
        if a.limbs < 2:
            raise OracleError("depth exhausted")
        if d != self.primes[a.limbs - 1]:
            raise OracleError("bad divisor")
        out = np.zeros((a.polys, a.limbs - 1, self.N), dtype=np.uint64)
        lib().orc_rescale(self._h, _p(a.data), a.polys, a.limbs, _p(out))
        return Ct(out, a.scale / float(d))

    def rescale(self, a: Ct) -> Ct:
        if a.limbs < 2:
            raise OracleError("depth exhausted")
        return self.div_scalar(a, self.primes[a.limbs - 1])
