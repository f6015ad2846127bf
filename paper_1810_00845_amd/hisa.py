"""Thin Python binding of libhisa (argument marshalling only).

Every method forwards to the C-ABI entry point of the same name in
``include/hisa.h``; all arithmetic runs in the HIP kernels of the library.
PyTorch is used for what it is good at here: the HIP stream the work is
enqueued on and raw device buffers for ``ntt_raw``.  There is no CPU fallback:
loading fails loudly when the library has not been built, and creating a
context fails when there is no GPU.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhisa.so")

MAX_Q = 48
CONV_SCALAR, CONV_MASKED, CONV_PLAIN = 0, 1, 2
CHW_ROTATE_INPUTS, CHW_ROTATE_SUMS, CHW_ROTATE_SUMS_TAPS = 0, 1, 2
PAD_SAME, PAD_SAME_MASKED = 1, 2

ERRORS = {0: "OK", -1: "ARG", -2: "LEVEL_MISMATCH", -3: "SCALE_MISMATCH", -4: "NO_KEY", -5: "BAD_DIVISOR",
          -6: "DEPTH_EXHAUSTED", -7: "OOM", -8: "HIP", -9: "SIZE"}


class HisaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("HISA_ERR_%s (%d): %s" % (ERRORS.get(code, "?"), code, msg))
        self.code = code


class Params(C.Structure):
    _fields_ = [("log_n", C.c_uint32), ("num_q", C.c_uint32), ("q_bits", C.c_uint32 * MAX_Q), ("dnum", C.c_uint32),
                ("special_bits", C.c_uint32), ("noise", C.c_uint32), ("seed", C.c_uint64), ("sigma", C.c_double),
                ("secret_kind", C.c_uint32), ("hamming_weight", C.c_uint32)]


class TensorStruct(C.Structure):
    _fields_ = [("batch", C.c_uint32), ("channels", C.c_uint32), ("height", C.c_uint32), ("width", C.c_uint32),
                ("h_stride", C.c_uint32), ("w_stride", C.c_uint32), ("offset", C.c_uint32), ("clean", C.c_uint32),
                ("c_inner", C.c_uint32), ("c_stride", C.c_uint32), ("cts", C.POINTER(C.c_void_p))]


class OpCounts(C.Structure):
    _fields_ = [(name, C.c_uint64) for name in ("rot_left", "rot_shared", "rot_summed", "relinearize", "mul", "mul_plain", "mul_scalar",
                                                "add", "rescale", "mac_plain", "mac_scalar", "key_switch_calls")] + \
               [("min_limbs", C.c_uint32), ("reserved", C.c_uint32), ("limb_sum", C.c_uint64 * 12), ("limb_sq_sum", C.c_uint64 * 12)]


class Calibration(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("fma_f64", "mul_f64", "add_f64", "rndne_add_f64", "mul_lo_u64", "mul_hi_u64", "copy_GBs")] + \
               [("copy_bytes", C.c_uint64), ("clock_mhz", C.c_double), ("compute_units", C.c_uint32), ("reserved", C.c_uint32)]


class MacExtents(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_taps", "ic", "oc", "batch", "log_n", "limbs", "polys", "lq", "gap")] + \
               [("ct_words", C.c_uint64), ("tap_words", C.POINTER(C.c_uint64))] + \
               [(n, C.c_uint64) for n in ("tap0_words", "out_words", "x2_tap_words", "x2_words", "x2_extent", "out2_extent",
                                          "w_words", "w_stride_t", "w_stride_oc", "w_extent")]


def check_mac_extents(tap_words, **fields):
    """hisa_check_mac_extents: the library's error code (0 = every access inside its allocation) for one
    multiply-accumulate launch described by its shape fields and the words behind each pointer; host only."""
    taps = (C.c_uint64 * len(tap_words))(*[int(t) for t in tap_words])
    a = MacExtents(n_taps=len(tap_words), tap_words=C.cast(taps, C.POINTER(C.c_uint64)), **{k: int(v) for k, v in fields.items()})
    fn = load().hisa_check_mac_extents
    fn.argtypes = [C.POINTER(MacExtents)]
    fn.restype = C.c_int
    return fn(C.byref(a))


class ConvGeom(C.Structure):
    _fields_ = [("fh", C.c_uint32), ("fw", C.c_uint32), ("stride", C.c_uint32), ("pad_same", C.c_uint32),
                ("mode", C.c_uint32), ("shared_moddown", C.c_uint32), ("chw_schedule", C.c_uint32)]


_lib = None


def load():
    """dlopen libhisa.so; raises if it was not built (python -m paper_1810_00845_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libhisa.so is missing: build it with `python -m paper_1810_00845_amd.build`; "
                              "there is no CPU fallback")
        # PyTorch ships its own HIP runtime; import it first so that libhisa binds to that same
        # runtime (streams and device pointers are only valid within one runtime instance).
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        _lib.hisa_last_error.restype = C.c_char_p
        _lib.hisa_last_error.argtypes = [C.c_void_p]
    return _lib


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double)) if a is not None else None


class _Handle:
    __slots__ = ("ctx", "h")

    def __init__(self, ctx, h):
        self.ctx, self.h = ctx, h

    def free(self):
        if self.h and self.ctx._h:
            load().hisa_free(C.c_void_p(self.ctx._h), C.c_void_p(self.h))
        self.h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Plaintext(_Handle):
    @property
    def limbs(self):
        l = C.c_uint32()
        self.ctx._ck(load().hisa_pt_info(C.c_void_p(self.h), C.byref(l), None))
        return l.value

    @property
    def scale(self):
        s = C.c_double()
        self.ctx._ck(load().hisa_pt_info(C.c_void_p(self.h), None, C.byref(s)))
        return s.value


class Ciphertext(_Handle):
    def info(self):
        l, p, s = C.c_uint32(), C.c_uint32(), C.c_double()
        self.ctx._ck(load().hisa_ct_info(C.c_void_p(self.h), C.byref(l), C.byref(p), C.byref(s)))
        return l.value, p.value, s.value

    @property
    def limbs(self):
        return self.info()[0]

    @property
    def polys(self):
        return self.info()[1]

    @property
    def scale(self):
        return self.info()[2]


class Context:
    """One parameter set on one GPU (see hisa_create)."""

    def __init__(self, log_n, q_bits, dnum, special_bits, seed, noise=True, stream=None, sigma=0.0, secret_kind=0,
                 hamming_weight=0):
        """sigma: parameter of the error distribution (0: 3.2); secret_kind 1: a secret with exactly hamming_weight
        non-zero coefficients instead of the uniform ternary one."""
        lib = load()
        prm = Params()
        prm.log_n, prm.num_q, prm.dnum = log_n, len(q_bits), dnum
        for i, b in enumerate(q_bits):
            prm.q_bits[i] = b
        prm.special_bits, prm.noise, prm.seed = special_bits, 1 if noise else 0, seed
        prm.sigma, prm.secret_kind, prm.hamming_weight = float(sigma), int(secret_kind), int(hamming_weight)
        if stream is None:
            import torch
            if not torch.cuda.is_available():
                raise HisaError(-8, "no GPU visible to PyTorch; libhisa has no CPU fallback")
            stream = torch.cuda.current_stream().cuda_stream
        self._h = None
        h = C.c_void_p()
        rc = lib.hisa_create(C.byref(prm), C.c_void_p(stream), C.byref(h))
        if rc != 0:
            msg = lib.hisa_last_error(h).decode() if h.value else "hisa_create failed"
            if h.value:
                lib.hisa_destroy(h)
            raise HisaError(rc, msg)
        self._h = h.value
        self.log_n, self.N, self.slots = log_n, 1 << log_n, 1 << (log_n - 1)
        self.L, self.dnum = len(q_bits), dnum
        a = C.c_uint32()
        self._ck(lib.hisa_get_alpha(self._vp, C.byref(a)))
        self.alpha = self.K = a.value
        q = (C.c_uint64 * self.L)()
        p = (C.c_uint64 * self.K)()
        self._ck(lib.hisa_get_primes(self._vp, q, p))
        self.primes = [int(x) for x in q] + [int(x) for x in p]

    @property
    def _vp(self):
        return C.c_void_p(self._h)

    def _ck(self, rc):
        if rc != 0:
            raise HisaError(rc, load().hisa_last_error(self._vp).decode())

    def close(self):
        if self._h:
            load().hisa_destroy(self._vp)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def sync(self):
        self._ck(load().hisa_sync(self._vp))

    # ---- keys ----
    def keygen(self):
        self._ck(load().hisa_keygen(self._vp))

    def gen_rot_keys(self, left_steps):
        arr = (C.c_int32 * len(left_steps))(*[int(s) for s in left_steps])
        self._ck(load().hisa_gen_rot_keys(self._vp, arr, C.c_size_t(len(left_steps))))

    def galois_elt(self, steps):
        g = C.c_uint64()
        self._ck(load().hisa_galois_elt(self._vp, C.c_int32(steps), C.byref(g)))
        return g.value

    # ---- plaintexts ----
    def _new_pt(self, h):
        return Plaintext(self, h.value)

    def _new_ct(self, h):
        return Ciphertext(self, h if isinstance(h, int) else h.value)

    def encode(self, values, scale, limbs):
        v = np.asarray(values)
        re = np.ascontiguousarray(v.real, dtype=np.float64)
        im = np.ascontiguousarray(v.imag, dtype=np.float64) if np.iscomplexobj(v) else None
        h = C.c_void_p()
        self._ck(load().hisa_encode(self._vp, _dp(re), _dp(im), C.c_size_t(len(re)), C.c_double(scale),
                                    C.c_uint32(limbs), C.byref(h)))
        return self._new_pt(h)

    def decode(self, pt, count=None):
        count = self.slots if count is None else count
        re, im = np.zeros(count), np.zeros(count)
        self._ck(load().hisa_decode(self._vp, C.c_void_p(pt.h), _dp(re), _dp(im), C.c_size_t(count)))
        return re + 1j * im

    def pt_from_coeffs(self, coeffs, scale, limbs):
        a = np.ascontiguousarray(coeffs, dtype=np.int64)
        assert a.shape == (self.N,)
        h = C.c_void_p()
        self._ck(load().hisa_pt_from_coeffs(self._vp, a.ctypes.data_as(C.POINTER(C.c_int64)), C.c_double(scale),
                                            C.c_uint32(limbs), C.byref(h)))
        return self._new_pt(h)

    def pt_export(self, pt):
        out = np.zeros((pt.limbs, self.N), dtype=np.uint64)
        self._ck(load().hisa_pt_export(self._vp, C.c_void_p(pt.h), out.ctypes.data_as(C.POINTER(C.c_uint64))))
        return out

    # ---- encryption profile ----
    def encrypt(self, pt):
        h = C.c_void_p()
        self._ck(load().hisa_encrypt(self._vp, C.c_void_p(pt.h), C.byref(h)))
        return self._new_ct(h)

    def encrypt_batch(self, pts):
        n = len(pts)
        arr = (C.c_void_p * n)(*[p.h for p in pts])
        out = (C.c_void_p * n)()
        self._ck(load().hisa_encrypt_batch(self._vp, arr, C.c_size_t(n), out))
        return [self._new_ct(int(out[i])) for i in range(n)]

    def set_enc_counter(self, c):
        self._ck(load().hisa_set_enc_counter(self._vp, C.c_uint64(c)))

    def decrypt(self, ct):
        h = C.c_void_p()
        self._ck(load().hisa_decrypt(self._vp, C.c_void_p(ct.h), C.byref(h)))
        return self._new_pt(h)

    def copy(self, ct):
        h = C.c_void_p()
        self._ck(load().hisa_copy(self._vp, C.c_void_p(ct.h), C.byref(h)))
        return self._new_ct(h)

    # ---- generic call helpers ----
    def _out(self, fn, *args):
        h = C.c_void_p()
        self._ck(getattr(load(), fn)(self._vp, *args, C.byref(h)))
        return self._new_ct(h)

    def _inplace(self, fn, *args):
        self._ck(getattr(load(), fn)(self._vp, *args))

    def add(self, a, b): return self._out("hisa_add", C.c_void_p(a.h), C.c_void_p(b.h))
    def sub(self, a, b): return self._out("hisa_sub", C.c_void_p(a.h), C.c_void_p(b.h))
    def add_assign(self, a, b): self._inplace("hisa_add_assign", C.c_void_p(a.h), C.c_void_p(b.h))
    def sub_assign(self, a, b): self._inplace("hisa_sub_assign", C.c_void_p(a.h), C.c_void_p(b.h))
    def add_plain(self, a, p): return self._out("hisa_add_plain", C.c_void_p(a.h), C.c_void_p(p.h))
    def sub_plain(self, a, p): return self._out("hisa_sub_plain", C.c_void_p(a.h), C.c_void_p(p.h))
    def add_plain_assign(self, a, p): self._inplace("hisa_add_plain_assign", C.c_void_p(a.h), C.c_void_p(p.h))
    def sub_plain_assign(self, a, p): self._inplace("hisa_sub_plain_assign", C.c_void_p(a.h), C.c_void_p(p.h))
    def add_scalar(self, a, x): return self._out("hisa_add_scalar", C.c_void_p(a.h), C.c_double(x))
    def sub_scalar(self, a, x): return self._out("hisa_sub_scalar", C.c_void_p(a.h), C.c_double(x))
    def add_scalar_assign(self, a, x): self._inplace("hisa_add_scalar_assign", C.c_void_p(a.h), C.c_double(x))
    def sub_scalar_assign(self, a, x): self._inplace("hisa_sub_scalar_assign", C.c_void_p(a.h), C.c_double(x))
    def mul(self, a, b): return self._out("hisa_mul", C.c_void_p(a.h), C.c_void_p(b.h))
    def mul_assign(self, a, b): self._inplace("hisa_mul_assign", C.c_void_p(a.h), C.c_void_p(b.h))
    def mul_no_relin(self, a, b): return self._out("hisa_mul_no_relin", C.c_void_p(a.h), C.c_void_p(b.h))
    def relinearize(self, a): self._inplace("hisa_relinearize", C.c_void_p(a.h))
    def mul_plain(self, a, p): return self._out("hisa_mul_plain", C.c_void_p(a.h), C.c_void_p(p.h))
    def mul_plain_assign(self, a, p): self._inplace("hisa_mul_plain_assign", C.c_void_p(a.h), C.c_void_p(p.h))

    def mul_scalar(self, a, x, x_scale):
        return self._out("hisa_mul_scalar", C.c_void_p(a.h), C.c_double(x), C.c_double(x_scale))

    def mul_scalar_assign(self, a, x, x_scale):
        self._inplace("hisa_mul_scalar_assign", C.c_void_p(a.h), C.c_double(x), C.c_double(x_scale))

    def rot_left(self, a, steps): return self._out("hisa_rot_left", C.c_void_p(a.h), C.c_int32(steps))
    def rot_right(self, a, steps): return self._out("hisa_rot_right", C.c_void_p(a.h), C.c_int32(steps))
    def rot_left_assign(self, a, steps): self._inplace("hisa_rot_left_assign", C.c_void_p(a.h), C.c_int32(steps))
    def rot_right_assign(self, a, steps): self._inplace("hisa_rot_right_assign", C.c_void_p(a.h), C.c_int32(steps))

    def rot_left_noalloc(self, a, steps, out):
        """rotLeft into the existing ciphertext `out`; the library allocates nothing on the device."""
        self._inplace("hisa_rot_left_noalloc", C.c_void_p(a.h), C.c_int32(steps), C.c_void_p(out.h))

    def max_scalar_div(self, a, ub):
        d = C.c_uint64()
        self._ck(load().hisa_max_scalar_div(self._vp, C.c_void_p(a.h), C.c_double(ub), C.byref(d)))
        return d.value

    def div_scalar(self, a, d): self._inplace("hisa_div_scalar", C.c_void_p(a.h), C.c_uint64(d))
    def rescale(self, a): self._inplace("hisa_rescale", C.c_void_p(a.h))

    # ---- batched forms ----
    @staticmethod
    def _harr(cts):
        return (C.c_void_p * len(cts))(*[c.h for c in cts])

    def _batch_out(self, fn, n, *args):
        out = (C.c_void_p * n)()
        self._ck(getattr(load(), fn)(self._vp, *args, out))
        return [self._new_ct(int(out[i])) for i in range(n)]

    def rot_left_batch(self, cts, steps):
        return self._batch_out("hisa_rot_left_batch", len(cts), self._harr(cts), C.c_size_t(len(cts)), C.c_int32(steps))

    def rot_left_hoisted_batch(self, cts, steps):
        """[len(steps)][len(cts)] rotated ciphertexts; the decomposition of c1 is shared by all steps."""
        n, ns = len(cts), len(steps)
        arr = (C.c_void_p * (n * ns))()
        st = (C.c_int32 * ns)(*[int(x) for x in steps])
        self._ck(load().hisa_rot_left_hoisted_batch(self._vp, self._harr(cts), C.c_size_t(n), st, C.c_size_t(ns), arr))
        return [[self._new_ct(int(arr[s * n + i])) for i in range(n)] for s in range(ns)]

    def rot_left_sum_batch(self, terms, steps):
        """terms[s][b]: out[b] = sum over s of rotLeft(terms[s][b], steps[s]), one division by P per output."""
        ns, n = len(steps), len(terms[0])
        assert len(terms) == ns and all(len(t) == n for t in terms)
        flat = [c for t in terms for c in t]
        arr = (C.c_void_p * n)()
        st = (C.c_int32 * ns)(*[int(x) for x in steps])
        self._ck(load().hisa_rot_left_sum_batch(self._vp, self._harr(flat), C.c_size_t(n), st, C.c_size_t(ns), arr))
        return [self._new_ct(int(arr[i])) for i in range(n)]

    def set_merge_doublings(self, max_doublings):
        """FC / matmul rotate-and-add chains as sums of rotations: 0 (off) or 2..4 consecutive doublings per sum."""
        self._ck(load().hisa_set_merge_doublings(self._vp, C.c_uint32(max_doublings)))

    def set_fused_rescale(self, on):
        """Layers divide by q_{l-1} P in one base conversion where their divScalar directly follows the division by P."""
        self._ck(load().hisa_set_fused_rescale(self._vp, C.c_uint32(1 if on else 0)))

    def add_batch(self, a, b):
        return self._batch_out("hisa_add_batch", len(a), self._harr(a), self._harr(b), C.c_size_t(len(a)))

    def mul_plain_batch(self, a, p):
        return self._batch_out("hisa_mul_plain_batch", len(a), self._harr(a), C.c_void_p(p.h), C.c_size_t(len(a)))

    def mul_no_relin_batch(self, a, b):
        return self._batch_out("hisa_mul_no_relin_batch", len(a), self._harr(a), self._harr(b), C.c_size_t(len(a)))

    def relinearize_batch(self, cts):
        self._ck(load().hisa_relinearize_batch(self._vp, self._harr(cts), C.c_size_t(len(cts))))

    def rescale_batch(self, cts):
        self._ck(load().hisa_rescale_batch(self._vp, self._harr(cts), C.c_size_t(len(cts))))

    def ct_random_batch(self, n, limbs, scale, counter):
        return self._batch_out("hisa_ct_random_batch", n, C.c_size_t(n), C.c_uint32(limbs), C.c_double(scale),
                               C.c_uint64(counter))

    # ---- parity / debug surface ----
    def ct_export(self, ct):
        l, p, _ = ct.info()
        out = np.zeros((p, l, self.N), dtype=np.uint64)
        self._ck(load().hisa_ct_export(self._vp, C.c_void_p(ct.h), out.ctypes.data_as(C.POINTER(C.c_uint64))))
        return out

    def ct_import(self, coeff, scale):
        a = np.ascontiguousarray(coeff, dtype=np.uint64)
        h = C.c_void_p()
        self._ck(load().hisa_ct_import(self._vp, a.ctypes.data_as(C.POINTER(C.c_uint64)), C.c_uint32(a.shape[0]),
                                       C.c_uint32(a.shape[1]), C.c_double(scale), C.byref(h)))
        return self._new_ct(h)

    def ct_import_batch(self, coeff, scale):
        a = np.ascontiguousarray(coeff, dtype=np.uint64)
        n = a.shape[0]
        out = (C.c_void_p * n)()
        self._ck(load().hisa_ct_import_batch(self._vp, a.ctypes.data_as(C.POINTER(C.c_uint64)), C.c_size_t(n),
                                             C.c_uint32(a.shape[1]), C.c_uint32(a.shape[2]), C.c_double(scale), out))
        return [self._new_ct(int(out[i])) for i in range(n)]

    def ntt_raw(self, dev_tensor, prime_index, inverse=False):
        """In-place transform of a contiguous int64 CUDA tensor [n_polys, N] (bit pattern = uint64)."""
        assert dev_tensor.is_cuda and dev_tensor.is_contiguous() and dev_tensor.element_size() == 8
        assert dev_tensor.shape[-1] == self.N
        n_polys = dev_tensor.numel() // self.N
        self._ck(load().hisa_ntt_raw(self._vp, C.c_void_p(dev_tensor.data_ptr()), C.c_uint32(prime_index),
                                     C.c_size_t(n_polys), C.c_int(1 if inverse else 0)))

    # ---- tensor layer ----
    def tensor_encrypt(self, x, scale, limbs, h_stride=None, w_stride=1, offset=0, c_inner=1, c_stride=0):
        """x[batch][channels][height][width] -> clean CipherTensor, HW-tiled or (c_inner > 1) CHW-tiled."""
        x = np.ascontiguousarray(x, dtype=np.float64)
        b, c, h, w = x.shape
        t = CipherTensor(self, [None] * (b * -(-c // c_inner)), b, c, h, w, h_stride if h_stride else w * w_stride, w_stride,
                         offset, 1, c_inner, c_stride)
        st, arr = t._struct()
        self._ck(load().hisa_tensor_encrypt(self._vp, _dp(x), C.c_double(scale), C.c_uint32(limbs), C.byref(st)))
        t._adopt(st, arr)
        return t

    def tensor_decrypt(self, t):
        out = np.zeros((t.batch, t.channels, t.height, t.width))
        st, _arr = t._struct()
        self._ck(load().hisa_tensor_decrypt(self._vp, C.byref(st), _dp(out)))
        return out

    def _layer(self, fn, t, n_out_cts, *args):
        st, _arr = t._struct()
        out = CipherTensor(self, [None] * n_out_cts, 0, 0, 0, 0, 0, 0, 0, 0, 1, 0)
        ost, oarr = out._struct()
        self._ck(getattr(load(), fn)(self._vp, C.byref(st), *args, C.byref(ost)))
        out._adopt(ost, oarr)
        return out

    def conv2d(self, t, w, fh, fw, stride=1, pad_same=False, mode=CONV_SCALAR, shared_moddown=False, chw_schedule=0):
        w = np.ascontiguousarray(w, dtype=np.float64)
        assert w.shape[:3] == (fh, fw, t.channels)
        oc = w.shape[3]
        g = ConvGeom(fh, fw, stride, int(pad_same), mode, 1 if shared_moddown else 0, chw_schedule)
        return self._layer("hisa_conv2d", t, t.batch * -(-oc // t.c_inner), _dp(w), C.c_uint32(oc), C.byref(g))

    def conv2d_prepare(self, like, w, fh, fw, stride=1, pad_same=False, mode=CONV_SCALAR, shared_moddown=False, chw_schedule=0):
        """Converts conv weights once for tensors laid out like `like`; returns a plan for conv2d_apply (free with
        conv_plan_free)."""
        w = np.ascontiguousarray(w, dtype=np.float64)
        assert w.shape[:3] == (fh, fw, like.channels)
        oc = w.shape[3]
        g = ConvGeom(fh, fw, stride, int(pad_same), mode, 1 if shared_moddown else 0, chw_schedule)
        st, _arr = like._struct()
        plan = C.c_void_p()
        self._ck(load().hisa_conv2d_prepare(self._vp, C.byref(st), _dp(w), C.c_uint32(oc), C.byref(g), C.byref(plan)))
        return (plan, -(-oc // like.c_inner))

    def conv2d_apply(self, t, plan):
        return self._layer("hisa_conv2d_apply", t, t.batch * plan[1], plan[0])

    def conv2d_apply_multi(self, t, plans):
        """conv2d_apply of every plan on the same tensor, the rotations of the inputs shared between the plans."""
        st, _arr = t._struct()
        outs = [CipherTensor(self, [None] * (t.batch * p[1]), 0, 0, 0, 0, 0, 0, 0, 0, 1, 0) for p in plans]
        structs = [o._struct() for o in outs]
        plan_arr = (C.c_void_p * len(plans))(*[p[0] for p in plans])
        out_arr = (C.c_void_p * len(plans))(*[C.addressof(ost) for ost, _ in structs])
        self._ck(load().hisa_conv2d_apply_multi(self._vp, C.byref(st), plan_arr, C.c_size_t(len(plans)), out_arr))
        for o, (ost, oarr) in zip(outs, structs):
            o._adopt(ost, oarr)
        return outs

    def conv_plan_free(self, plan):
        self._ck(load().hisa_conv_plan_free(self._vp, plan[0]))

    def conv2d_fixed(self, t, w_int, w_scale, pt_coeffs, pt_scale, oc, fh, fw, stride=1, pad_same=False, mode=CONV_SCALAR, shared_moddown=False,
                     chw_schedule=0):
        i64p = C.POINTER(C.c_int64)
        wi = np.ascontiguousarray(w_int, dtype=np.int64) if w_int is not None else None
        pc = np.ascontiguousarray(pt_coeffs, dtype=np.int64) if pt_coeffs is not None else None
        g = ConvGeom(fh, fw, stride, int(pad_same), mode, 1 if shared_moddown else 0, chw_schedule)
        return self._layer("hisa_conv2d_fixed", t, t.batch * -(-oc // t.c_inner), wi.ctypes.data_as(i64p) if wi is not None else None,
                           C.c_double(w_scale), pc.ctypes.data_as(i64p) if pc is not None else None, C.c_double(pt_scale),
                           C.c_uint32(oc), C.byref(g))

    def fc(self, t, w):
        w = np.ascontiguousarray(w, dtype=np.float64)
        out_features = w.shape[0]
        assert w.size == out_features * t.channels * t.height * t.width
        return self._layer("hisa_fc", t, t.batch * out_features, _dp(w), C.c_uint32(out_features))

    def fc_prepare(self, like, w):
        """Encodes fc weights once for tensors laid out like `like`; returns a plan for fc_apply (free with
        fc_plan_free)."""
        w = np.ascontiguousarray(w, dtype=np.float64)
        out_features = w.shape[0]
        assert w.size == out_features * like.channels * like.height * like.width
        st, _arr = like._struct()
        plan = C.c_void_p()
        self._ck(load().hisa_fc_prepare(self._vp, C.byref(st), _dp(w), C.c_uint32(out_features), C.byref(plan)))
        return (plan, out_features)

    def fc_apply(self, t, plan):
        return self._layer("hisa_fc_apply", t, t.batch * plan[1], plan[0])

    def fc_plan_free(self, plan):
        self._ck(load().hisa_fc_plan_free(self._vp, plan[0]))

    def fc_fixed(self, t, pt_coeffs, pt_scale):
        pc = np.ascontiguousarray(pt_coeffs, dtype=np.int64)
        out_features = pc.shape[0]
        assert pc.shape == (out_features, t.channels, self.N)
        return self._layer("hisa_fc_fixed", t, t.batch * out_features, pc.ctypes.data_as(C.POINTER(C.c_int64)),
                           C.c_double(pt_scale), C.c_uint32(out_features))

    def tensor_mask(self, t):
        """The masking multiply: same tensor, one level lower, zeros outside the elements."""
        return self._layer("hisa_tensor_mask", t, len(t.cts))

    def tensor_mask_fixed(self, t, mask_coeffs, mask_scale):
        mc = np.ascontiguousarray(mask_coeffs, dtype=np.int64)
        assert mc.shape == (-(-t.channels // t.c_inner), self.N)
        return self._layer("hisa_tensor_mask_fixed", t, len(t.cts), mc.ctypes.data_as(C.POINTER(C.c_int64)), C.c_double(mask_scale))

    def tensor_add_bias(self, t, bias):
        """bias[c] onto the elements of channel c, in place (one addPlain per ciphertext)."""
        b = np.ascontiguousarray(bias, dtype=np.float64)
        assert b.shape == (t.channels,)
        st, _arr = t._struct()
        self._ck(load().hisa_tensor_add_bias(self._vp, C.byref(st), _dp(b)))
        return t

    def tensor_add_bias_fixed(self, t, bias_coeffs):
        bc = np.ascontiguousarray(bias_coeffs, dtype=np.int64)
        assert bc.shape == (-(-t.channels // t.c_inner), self.N)
        st, _arr = t._struct()
        self._ck(load().hisa_tensor_add_bias_fixed(self._vp, C.byref(st), bc.ctypes.data_as(C.POINTER(C.c_int64))))
        return t

    def tensor_to_chw(self, t, c_inner, c_stride):
        """Clean HW-tiled tensor -> CHW-tiled (c_inner channels per ciphertext, c_stride slots apart)."""
        return self._layer("hisa_tensor_to_chw", t, t.batch * -(-t.channels // c_inner), C.c_uint32(c_inner), C.c_uint32(c_stride))

    def tensor_to_hw(self, t):
        """CHW-tiled tensor -> clean HW-tiled tensor, one level lower."""
        return self._layer("hisa_tensor_to_hw", t, t.batch * t.channels)

    def tensor_to_hw_fixed(self, t, mask_coeffs, mask_scale):
        mc = np.ascontiguousarray(mask_coeffs, dtype=np.int64)
        assert mc.shape == (self.N,)
        return self._layer("hisa_tensor_to_hw_fixed", t, t.batch * t.channels, mc.ctypes.data_as(C.POINTER(C.c_int64)),
                           C.c_double(mask_scale))

    def tensor_layout_rot_steps(self, t, c_inner=1, c_stride=0):
        return self._steps("hisa_tensor_layout_rot_steps", t, C.c_uint32(c_inner), C.c_uint32(c_stride))

    def matmul_geometry(self, t, out_features, replicas):
        """(block length P, replicas used R, number of output ciphertexts) of matmul on tensors laid out like t."""
        st, _arr = t._struct()
        block, used, n_out = C.c_uint32(), C.c_uint32(), C.c_uint32()
        self._ck(load().hisa_matmul_geometry(self._vp, C.byref(st), C.c_uint32(out_features), C.c_uint32(replicas),
                                             C.byref(block), C.byref(used), C.byref(n_out)))
        return block.value, used.value, n_out.value

    def matmul(self, t, w, replicas):
        """Homomorphic matmul with replicas: w[OUT][C][H][W] -> CHW-tiled tensor of OUT 1x1 channels."""
        w = np.ascontiguousarray(w, dtype=np.float64)
        out_features = w.shape[0]
        assert w.size == out_features * t.channels * t.height * t.width
        n_out = self.matmul_geometry(t, out_features, replicas)[2]
        return self._layer("hisa_matmul", t, n_out, _dp(w), C.c_uint32(out_features), C.c_uint32(replicas))

    def matmul_fixed(self, t, pt_coeffs, pt_scale, mask_coeffs, mask_scale, out_features, replicas):
        i64p = C.POINTER(C.c_int64)
        pc = np.ascontiguousarray(pt_coeffs, dtype=np.int64)
        mc = np.ascontiguousarray(mask_coeffs, dtype=np.int64) if mask_coeffs is not None else None
        _block, used, n_out = self.matmul_geometry(t, out_features, replicas)
        per = -(-t.channels // t.c_inner)
        assert pc.shape == (-(-out_features // used), per, self.N) and (mc is None or mc.shape == (per, self.N))
        return self._layer("hisa_matmul_fixed", t, n_out, pc.ctypes.data_as(i64p), C.c_double(pt_scale),
                           mc.ctypes.data_as(i64p) if mc is not None else None, C.c_double(mask_scale),
                           C.c_uint32(out_features), C.c_uint32(replicas))

    def matmul_prepare(self, like, w, replicas):
        """Encodes matmul weights once for tensors laid out like `like`; returns a plan for matmul_apply (free with
        matmul_plan_free)."""
        w = np.ascontiguousarray(w, dtype=np.float64)
        out_features = w.shape[0]
        assert w.size == out_features * like.channels * like.height * like.width
        st, _arr = like._struct()
        plan = C.c_void_p()
        self._ck(load().hisa_matmul_prepare(self._vp, C.byref(st), _dp(w), C.c_uint32(out_features), C.c_uint32(replicas),
                                            C.byref(plan)))
        return (plan, self.matmul_geometry(like, out_features, replicas)[2] // like.batch)

    def matmul_apply(self, t, plan):
        return self._layer("hisa_matmul_apply", t, t.batch * plan[1], plan[0])

    def matmul_plan_free(self, plan):
        self._ck(load().hisa_matmul_plan_free(self._vp, plan[0]))

    def matmul_rot_steps(self, t, replicas):
        return self._steps("hisa_matmul_rot_steps", t, C.c_uint32(replicas))

    def sum_pool2x2(self, t):
        return self._layer("hisa_sum_pool2x2", t, len(t.cts))

    def avg_pool2x2(self, t):
        """The 2x2 mean: the sum pool at four times the scale (no ciphertext operation for the 1/4)."""
        return self._layer("hisa_avg_pool2x2", t, len(t.cts))

    def poly2_act(self, t, a, b):
        return self._layer("hisa_poly2_act", t, len(t.cts), C.c_double(a), C.c_double(b))

    def _steps(self, fn, t, *args):
        st, _arr = t._struct()
        buf = (C.c_int32 * 1024)()      # a CHW-tiled convolution alone can ask for 257 amounts
        n = C.c_size_t()
        self._ck(getattr(load(), fn)(self._vp, C.byref(st), *args, buf, C.c_size_t(1024), C.byref(n)))
        return [int(buf[i]) for i in range(n.value)]

    def conv2d_rot_steps(self, t, fh, fw, stride=1, pad_same=False, chw_schedule=0):
        g = ConvGeom(fh, fw, stride, int(pad_same), 0, 0, chw_schedule)
        return self._steps("hisa_conv2d_rot_steps", t, C.byref(g))

    def fc_rot_steps(self, t):
        return self._steps("hisa_fc_rot_steps", t)

    def pool_rot_steps(self, t):
        return self._steps("hisa_pool_rot_steps", t)

    # ---- analysis backend ----
    def analysis_begin(self):
        """From here to analysis_end the calls on this context are dry runs that only record."""
        self._ck(load().hisa_analysis_begin(self._vp))

    check_mac_extents = staticmethod(check_mac_extents)   # needs no context: a pure host check

    def analysis_end(self):
        """(operation counts as a dict incl. 'min_limbs', 'limb_sum' = {operation: limbs summed over its occurrences} and
        'limb_sq_sum' (their squares), sorted left-rotation amounts that needed a key)."""
        counts, n = OpCounts(), C.c_size_t()
        buf = (C.c_int32 * 4096)()
        self._ck(load().hisa_analysis_end(self._vp, C.byref(counts), buf, C.c_size_t(4096), C.byref(n)))
        d = {name: int(getattr(counts, name)) for name, _ in OpCounts._fields_ if name not in ("reserved", "limb_sum", "limb_sq_sum")}
        d["limb_sum"] = {name: int(counts.limb_sum[i]) for i, (name, _) in enumerate(OpCounts._fields_[:12])}
        d["limb_sq_sum"] = {name: int(counts.limb_sq_sum[i]) for i, (name, _) in enumerate(OpCounts._fields_[:12])}
        return d, [int(buf[i]) for i in range(n.value)]

    def profile_enable(self, on=True):
        self._ck(load().hisa_profile_enable(self._vp, C.c_int(1 if on else 0)))

    def calibrate(self):
        """Measured issue rates (T lane-ops/s) and copy bandwidth (GB/s) of this GPU, as a dict."""
        c = Calibration()
        self._ck(load().hisa_calibrate(self._vp, C.byref(c)))
        return {n: getattr(c, n) for n, _ in Calibration._fields_ if n != "reserved"}

    def profile_read(self):
        """{kernel name: (launches, total ms)} since the last read."""
        buf = C.create_string_buffer(1 << 16)
        self._ck(load().hisa_profile_read(self._vp, buf, C.c_size_t(len(buf))))
        out = {}
        for line in buf.value.decode().splitlines():
            name, cnt, ms = line.split("\t")
            out[name] = (int(cnt), float(ms))
        return out

    def key_export(self, key_id):
        out = np.zeros((self.dnum, 2, self.L + self.K, self.N), dtype=np.uint64)
        self._ck(load().hisa_key_export(self._vp, C.c_uint64(key_id), out.ctypes.data_as(C.POINTER(C.c_uint64))))
        return out

    def secret_export(self):
        out = np.zeros(self.N, dtype=np.int64)
        self._ck(load().hisa_secret_export(self._vp, out.ctypes.data_as(C.POINTER(C.c_int64))))
        return out


class CipherTensor:
    """Vector of ciphertexts + layout metadata (the paper's CipherTensor; HW-tiled when c_inner == 1, CHW-tiled with
    c_inner channels per ciphertext, c_stride slots apart, otherwise)."""

    def __init__(self, ctx, cts, batch, channels, height, width, h_stride, w_stride, offset, clean, c_inner=1, c_stride=0):
        self.ctx, self.cts = ctx, cts
        self.batch, self.channels, self.height, self.width = batch, channels, height, width
        self.h_stride, self.w_stride, self.offset, self.clean = h_stride, w_stride, offset, clean
        self.c_inner, self.c_stride = max(1, c_inner), c_stride

    def meta(self):
        return (self.batch, self.channels, self.height, self.width, self.h_stride, self.w_stride, self.offset, self.clean,
                self.c_inner, self.c_stride)

    def shaped_like(self, cts=None, **kw):
        t = CipherTensor(self.ctx, self.cts if cts is None else cts, *self.meta())
        for k, v in kw.items():
            setattr(t, k, v)
        return t

    def _struct(self):
        n = len(self.cts)
        arr = (C.c_void_p * n)(*[(c.h if c is not None else None) for c in self.cts])
        st = TensorStruct(self.batch, self.channels, self.height, self.width, self.h_stride, self.w_stride, self.offset,
                          self.clean, self.c_inner, self.c_stride, C.cast(arr, C.POINTER(C.c_void_p)))
        return st, arr

    def _adopt(self, st, arr):
        self.batch, self.channels, self.height, self.width = st.batch, st.channels, st.height, st.width
        self.h_stride, self.w_stride, self.offset, self.clean = st.h_stride, st.w_stride, st.offset, st.clean
        self.c_inner, self.c_stride = max(1, st.c_inner), st.c_stride
        self.cts = [Ciphertext(self.ctx, int(arr[i])) for i in range(len(arr))]

    def free(self):
        for c in self.cts:
            if c is not None:
                c.free()
        self.cts = []
