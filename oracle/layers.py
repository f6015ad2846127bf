"""Oracle side of the HW-tiled tensor kernels (TEST INFRASTRUCTURE, not product code).

The schedules of the paper's runtime (Sec. "Runtime"; Algorithm 1 for conv2d
with VALID padding, its SAME-padding variant with a mask, homomorphic matmul
without replicas, pooling, degree-2 activation) written as plain loops over the
oracle's HISA instructions, one instruction per statement, in the paper's
order.  Each layer also returns the fixed-point integers it used, so that a
test can hand the very same integers to another implementation.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

from .ckks import Oracle, round_half_away

CONV_SCALAR, CONV_MASKED, CONV_PLAIN = 0, 1, 2
MASK_SCALE = 2.0 ** 25


@dataclass
class OTensor:
    cts: list            # batch*channels ciphertexts, index b*channels + c
    batch: int
    channels: int
    height: int
    width: int
    h_stride: int
    w_stride: int
    offset: int
    clean: int


def plane_slots(h, w, hs, ws, off):
    return [off + y * hs + x * ws for y in range(h) for x in range(w)]


def tensor_encrypt(o: Oracle, x, scale, limbs, h_stride=None, w_stride=1, offset=0) -> OTensor:
    b, c, h, w = x.shape
    hs = h_stride if h_stride else w * w_stride
    cts = []
    for bi in range(b):
        for ci in range(c):
            z = np.zeros(o.slots)
            z[plane_slots(h, w, hs, w_stride, offset)] = x[bi, ci].reshape(-1)
            cts.append(o.encrypt(o.encode(z, scale, limbs)))
    return OTensor(cts, b, c, h, w, hs, w_stride, offset, 1)


def tensor_decrypt(o: Oracle, t: OTensor):
    out = np.zeros((t.batch, t.channels, t.height, t.width))
    sl = plane_slots(t.height, t.width, t.h_stride, t.w_stride, t.offset)
    for i, ct in enumerate(t.cts):
        z = o.decode(o.decrypt(ct)).real
        out[i // t.channels, i % t.channels] = z[sl].reshape(t.height, t.width)
    return out


def conv2d(o: Oracle, t: OTensor, w, stride=1, pad_same=False, mode=CONV_SCALAR):
    """Algorithm 1.  w[FH][FW][IC][OC].  Returns (output tensor, dict of the integers used)."""
    fh, fw, ic_n, oc_n = w.shape
    assert ic_n == t.channels
    l = t.cts[0].limbs
    q_last = float(o.primes[l - 1])
    if pad_same:
        assert t.clean, "SAME padding needs zeros around the plane"
        oh, ow = -(-t.height // stride), -(-t.width // stride)
        ph, pw = fh // 2, fw // 2
    else:
        oh, ow = (t.height - fh) // stride + 1, (t.width - fw) // stride + 1
        ph = pw = 0
    valid = np.zeros(o.slots)
    valid[plane_slots(oh, ow, t.h_stride * stride, t.w_stride * stride, t.offset)] = 1.0
    ints = {"w_int": None, "w_scale": 1.0, "pt_coeffs": None, "pt_scale": 1.0}
    if mode == CONV_PLAIN:
        pt_scale = q_last
        coeffs = np.zeros((fh, fw, ic_n, oc_n, o.N), dtype=np.int64)
        for idx in np.ndindex(fh, fw, ic_n, oc_n):
            coeffs[idx] = o.encode_coeffs(float(w[idx]) * valid, pt_scale)
        ints.update(pt_coeffs=coeffs, pt_scale=pt_scale)
    else:
        w_scale = q_last / MASK_SCALE if mode == CONV_MASKED else q_last
        w_int = np.zeros(w.shape, dtype=np.int64)
        for idx in np.ndindex(*w.shape):
            w_int[idx] = round_half_away(float(w[idx]) * w_scale)   # FixedPrecision(weight, plainLogP)
        ints.update(w_int=w_int, w_scale=w_scale)
        if mode == CONV_MASKED:
            ints.update(pt_coeffs=o.encode_coeffs(valid, MASK_SCALE), pt_scale=MASK_SCALE)
    out = conv2d_fixed(o, t, ints, oc_n, fh, fw, stride, pad_same, mode)
    return out, ints


def conv2d_fixed(o: Oracle, t: OTensor, ints, oc_n, fh, fw, stride, pad_same, mode):
    l = t.cts[0].limbs
    ph, pw = (fh // 2, fw // 2) if pad_same else (0, 0)
    if pad_same:
        oh, ow = -(-t.height // stride), -(-t.width // stride)
    else:
        oh, ow = (t.height - fh) // stride + 1, (t.width - fw) // stride + 1
    rotated = {}  # the rotations do not depend on (b, oc): computed once ("code motion" of Sec. "Runtime")

    def rot(b, ic, fy, fx):
        key = (b, ic, fy, fx)
        if key not in rotated:
            r = (fy - ph) * t.h_stride + (fx - pw) * t.w_stride
            rotated[key] = o.rot_left(t.cts[b * t.channels + ic], r % o.slots)
        return rotated[key]

    mask_pt = None
    if mode == CONV_MASKED:
        mask_pt = o.pt_from_coeffs(ints["pt_coeffs"], ints["pt_scale"], l)
    outs = []
    for b in range(t.batch):
        for oc in range(oc_n):
            acc = None
            for ic in range(t.channels):
                for fy in range(fh):
                    for fx in range(fw):
                        temp = rot(b, ic, fy, fx)
                        if mode == CONV_PLAIN:
                            pt = o.pt_from_coeffs(ints["pt_coeffs"][fy, fx, ic, oc], ints["pt_scale"], l)
                            temp = o.mul_plain(temp, pt)
                        else:
                            temp = o.mul_int(temp, int(ints["w_int"][fy, fx, ic, oc]), ints["w_scale"])
                        acc = temp if acc is None else o.add(acc, temp)
            if mode == CONV_MASKED:
                acc = o.mul_plain(acc, mask_pt)
            outs.append(o.div_scalar(acc, o.max_scalar_div(acc, float("inf"))))
    # Without the masking multiply the slots outside the valid outputs hold sums over neighbouring slots; only a
    # 1x1 filter at stride 1 reads no neighbour, so there a clean input stays clean.
    pointwise = fh == 1 and fw == 1 and stride == 1
    clean = 1 if mode != CONV_SCALAR or (pointwise and t.clean) else 0
    return OTensor(outs, t.batch, oc_n, oh, ow, t.h_stride * stride, t.w_stride * stride, t.offset, clean)


def fc(o: Oracle, t: OTensor, w):
    """w[OUT][C][H][W].  Returns (output tensor, plaintext coefficients [OUT][C][N], their scale)."""
    out_n = w.shape[0]
    l = t.cts[0].limbs
    if t.height == 1 and t.width == 1:
        wt = np.ascontiguousarray(w.reshape(out_n, t.channels).T).reshape(1, 1, t.channels, out_n)
        out, ints = conv2d(o, t, wt, mode=CONV_SCALAR)
        return out, ints
    pt_scale = float(o.primes[l - 1])
    sl = plane_slots(t.height, t.width, t.h_stride, t.w_stride, t.offset)
    coeffs = np.zeros((out_n, t.channels, o.N), dtype=np.int64)
    for k in range(out_n):
        for c in range(t.channels):
            z = np.zeros(o.slots)
            z[sl] = np.asarray(w[k, c], dtype=np.float64).reshape(-1)
            coeffs[k, c] = o.encode_coeffs(z, pt_scale)
    return fc_fixed(o, t, coeffs, pt_scale), {"pt_coeffs": coeffs, "pt_scale": pt_scale}


def fc_reduce_steps(o: Oracle, t: OTensor):
    """Rotation amounts of the log-step sum over a plane (Sec. "Homomorphic Tensor Operations": reductions over
    equally strided elements take log-many rotations with additions in between).  Along the width the amounts are
    w_stride * 2^k, along the height h_stride * 2^k, each up to the next power of two of the dimension; the padding
    positions this reads are zero after the masked multiply.  That needs the padded rows not to overlap and the padded
    plane not to wrap around the slot vector; otherwise (or if it is not shorter) the sum runs over the contiguous
    power-of-two window 1, 2, 4, ... that covers the plane."""
    span = (t.height - 1) * t.h_stride + (t.width - 1) * t.w_stride
    window = []
    while (1 << len(window)) < span + 1:
        window.append(1 << len(window))
    wl = max(t.width - 1, 0).bit_length()
    hl = max(t.height - 1, 0).bit_length()
    fits = (t.w_stride << wl) <= t.h_stride and \
        t.offset + ((1 << hl) - 1) * t.h_stride + ((1 << wl) - 1) * t.w_stride < o.slots
    strided = [t.w_stride << k for k in range(wl)] + [t.h_stride << k for k in range(hl)]
    return strided if fits and len(strided) < len(window) else window


def fc_fixed(o: Oracle, t: OTensor, coeffs, pt_scale):
    out_n = coeffs.shape[0]
    l = t.cts[0].limbs
    steps = fc_reduce_steps(o, t)
    outs = []
    for b in range(t.batch):
        for k in range(out_n):
            acc = None
            for c in range(t.channels):
                temp = o.mul_plain(t.cts[b * t.channels + c], o.pt_from_coeffs(coeffs[k, c], pt_scale, l))
                acc = temp if acc is None else o.add(acc, temp)
            acc = o.rescale(acc)
            for r in steps:               # rotate-and-add: slot `offset` collects every element of the plane
                acc = o.add(acc, o.rot_left(acc, r))
            outs.append(acc)
    return OTensor(outs, t.batch, out_n, 1, 1, 1, 1, t.offset, 0)


def sum_pool2x2(o: Oracle, t: OTensor):
    outs = []
    for ct in t.cts:
        acc = ct
        for r in (t.w_stride, t.h_stride, t.h_stride + t.w_stride):
            acc = o.add(acc, o.rot_left(ct, r))
        outs.append(acc)
    return replace(t, cts=outs, height=t.height // 2, width=t.width // 2, h_stride=2 * t.h_stride,
                   w_stride=2 * t.w_stride, clean=0)


def poly2_act(o: Oracle, t: OTensor, a, b):
    """x^2 + (b/a) x, the factor a being left to the next layer."""
    outs = []
    for ct in t.cts:
        acc = o.mul(ct, ct)
        if b != 0.0:
            acc = o.add(acc, o.mul_scalar(ct, b / a, ct.scale))
        outs.append(o.rescale(acc))
    return replace(t, cts=outs)


def rot_steps_conv(o: Oracle, t: OTensor, fh, fw, pad_same=False):
    ph, pw = (fh // 2, fw // 2) if pad_same else (0, 0)
    return sorted({((fy - ph) * t.h_stride + (fx - pw) * t.w_stride) % o.slots for fy in range(fh) for fx in range(fw)} - {0})
