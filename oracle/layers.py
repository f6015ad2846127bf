"""Oracle side of the HW-tiled tensor kernels (TEST INFRASTRUCTURE, not product code).

The schedules of the paper's runtime (Sec. "Runtime"; Algorithm 1 for conv2d
with VALID padding, its SAME-padding variant with a mask, homomorphic matmul
without and with replicas (the latter with a CHW-tiled output), CHW-tiled
conv2d, the masking multiply, the conversions between the two tilings,
pooling, degree-2 activation) written as plain loops over the
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
    c_inner: int = 1     # channels per ciphertext: 1 = HW-tiling, more = CHW-tiling (cts index b*ceil(C/c_inner) + c//c_inner)
    c_stride: int = 0    # slots between two channels of one ciphertext


def cts_per_image(t: OTensor):
    return -(-t.channels // t.c_inner)


def tensor_slots(t: OTensor):
    """Slots of the elements of one ciphertext, channel-major: element (c mod c_inner, y, x) sits in slot
    offset + (c mod c_inner)*c_stride + y*h_stride + x*w_stride (Sec. "Runtime": physical strides per inner dimension)."""
    return [t.offset + cl * t.c_stride + y * t.h_stride + x * t.w_stride
            for cl in range(t.c_inner) for y in range(t.height) for x in range(t.width)]


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


def tensor_encrypt_chw(o: Oracle, x, scale, limbs, c_inner, c_stride, h_stride=None, w_stride=1, offset=0) -> OTensor:
    """CHW-tiling: c_inner channels per ciphertext, c_stride slots apart."""
    b, c, h, w = x.shape
    hs = h_stride if h_stride else w * w_stride
    t = OTensor([], b, c, h, w, hs, w_stride, offset, 1, c_inner, c_stride)
    sl = np.asarray(tensor_slots(t)).reshape(c_inner, h * w)
    assert len(set(sl.reshape(-1).tolist())) == sl.size and sl.max() < o.slots
    for bi in range(b):
        for j in range(cts_per_image(t)):
            z = np.zeros(o.slots)
            for cl in range(min(c_inner, c - j * c_inner)):
                z[sl[cl]] = x[bi, j * c_inner + cl].reshape(-1)
            t.cts.append(o.encrypt(o.encode(z, scale, limbs)))
    return t


def tensor_decrypt(o: Oracle, t: OTensor):
    if t.c_inner > 1:
        out = np.zeros((t.batch, t.channels, t.height, t.width))
        sl = np.asarray(tensor_slots(t)).reshape(t.c_inner, t.height, t.width)
        per = cts_per_image(t)
        for i, ct in enumerate(t.cts):
            z = o.decode(o.decrypt(ct)).real
            for cl in range(min(t.c_inner, t.channels - (i % per) * t.c_inner)):
                out[i // per, (i % per) * t.c_inner + cl] = z[sl[cl]]
        return out
    out = np.zeros((t.batch, t.channels, t.height, t.width))
    sl = plane_slots(t.height, t.width, t.h_stride, t.w_stride, t.offset)
    for i, ct in enumerate(t.cts):
        z = o.decode(o.decrypt(ct)).real
        out[i // t.channels, i % t.channels] = z[sl].reshape(t.height, t.width)
    return out


class SharedModDown:
    """sum_k weight_k * rotLeft(x_k, amount_k) with the division by P taken once for the whole sum instead of once per
    rotation (the rotations of a convolution are only ever used inside such sums): every rotated term contributes its
    key-switch accumulators -- on the l + K limbs, before the division -- times the weight taken on those same limbs,
    and sigma(c0) times the weight on the l limbs; an unrotated term contributes weight * (c0, c1); at the end
    (ModDown(E_b) + Z_0, ModDown(E_a) + Z_1).  Up to the rounding of the division this is the sum of the rotated
    ciphertexts; ciphertext bits differ from the term-by-term schedule.  The accumulators of an (input, amount) pair
    are computed once and shared by all the sums over the same inputs."""

    def __init__(self, o: Oracle, inputs):
        self.o, self.inputs = o, inputs
        self.acc = {}      # (input index, amount) -> (acc_b, acc_a, sigma(c0))
        self.res = {}      # (weight key, basis) -> residues of a plaintext weight

    def rotated(self, i, amount):
        if (i, amount) not in self.acc:
            ct, g = self.inputs[i], self.o.galois_elt(amount)
            if g not in self.o.keys:
                raise KeyError("no key for rotation by %d" % amount)
            acc_b, acc_a = self.o.key_switch_acc(self.o.automorph_ntt(ct.data[1], g), g)
            self.acc[(i, amount)] = (acc_b, acc_a, self.o.automorph_ntt(ct.data[0], g))
        return self.acc[(i, amount)]

    def total(self, terms, scale, rescale=False):
        """terms: (input index, rotLeft amount, weight, weight key); weight is an integer (key None) or an array of N
        signed plaintext coefficients (key: anything hashable that names it).  Returns the sum as a ciphertext.
        rescale: the sum's divScalar by the last modulus is taken together with the division by P -- the terms without
        a rotation enter the accumulators times P, and the whole is divided by q_{l-1} P in one base conversion
        (mod_down_rescale): one limb fewer, scale / q_{l-1}."""
        from .ckks import Ct
        o = self.o
        l = self.inputs[0].limbs
        ext, qs = o.ext_primes(l), list(range(l))
        e_b = np.zeros((l + o.K, o.N), dtype=np.uint64)
        e_a = np.zeros((l + o.K, o.N), dtype=np.uint64)
        z = np.zeros((2, l, o.N), dtype=np.uint64)

        def fma(acc, x, w, wkey, primes, basis):
            if wkey is None:
                o.fma_const(acc, x, int(w), primes)
            else:
                if (wkey, basis) not in self.res:
                    self.res[(wkey, basis)] = o.residues_ntt(w, primes)
                o.fma_plain(acc, x, self.res[(wkey, basis)], primes)

        any_rotated = False
        for i, amount, w, wkey in terms:
            if amount % o.slots == 0:
                fma(z[0], self.inputs[i].data[0], w, wkey, qs, "q")
                fma(z[1], self.inputs[i].data[1], w, wkey, qs, "q")
            else:
                acc_b, acc_a, r0 = self.rotated(i, amount % o.slots)
                fma(e_b, acc_b, w, wkey, ext, "ext")
                fma(e_a, acc_a, w, wkey, ext, "ext")
                fma(z[0], r0, w, wkey, qs, "q")
                any_rotated = True
        if rescale:
            assert l >= 2
            return divide_by_p_and_last(o, e_b, e_a, z, l, scale)
        out = Ct(z, scale)
        if any_rotated:
            out = o.add(Ct(np.stack([o.mod_down(e_b, l), o.mod_down(e_a, l)]), scale), out)
        return out


def conv2d(o: Oracle, t: OTensor, w, stride=1, pad_same=False, mode=CONV_SCALAR, shared_moddown=False, fused_rescale=False):
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
    out = conv2d_fixed(o, t, ints, oc_n, fh, fw, stride, pad_same, mode, shared_moddown, fused_rescale)
    return out, ints


def conv2d_fixed(o: Oracle, t: OTensor, ints, oc_n, fh, fw, stride, pad_same, mode, shared_moddown=False, fused_rescale=False):
    """shared_moddown: the sum over (input channel, tap) goes through SharedModDown.  fused_rescale (with
    shared_moddown, scalar weights without the masking multiply): that sum's division by P and the divScalar are one
    division."""
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
        shared = SharedModDown(o, t.cts[b * t.channels:(b + 1) * t.channels]) if shared_moddown else None
        for oc in range(oc_n):
            if shared is not None:
                amount = lambda fy, fx: ((fy - ph) * t.h_stride + (fx - pw) * t.w_stride) % o.slots
                if mode == CONV_PLAIN:
                    terms = [(ic, amount(fy, fx), ints["pt_coeffs"][fy, fx, ic, oc], (fy, fx, ic, oc))
                             for ic in range(t.channels) for fy in range(fh) for fx in range(fw)]
                    acc = shared.total(terms, t.cts[0].scale * ints["pt_scale"])
                else:
                    terms = [(ic, amount(fy, fx), int(ints["w_int"][fy, fx, ic, oc]), None)
                             for ic in range(t.channels) for fy in range(fh) for fx in range(fw)]
                    one = fused_rescale and mode == CONV_SCALAR
                    acc = shared.total(terms, t.cts[0].scale * ints["w_scale"], rescale=one)
                    if one:
                        outs.append(acc)
                        continue
                if mode == CONV_MASKED:
                    acc = o.mul_plain(acc, mask_pt)
                outs.append(o.div_scalar(acc, o.max_scalar_div(acc, float("inf"))))
                continue
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


def fc(o: Oracle, t: OTensor, w, merge=0):
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
    return fc_fixed(o, t, coeffs, pt_scale, merge), {"pt_coeffs": coeffs, "pt_scale": pt_scale}


def fc_reduce_steps(o: Oracle, t: OTensor):
    """Rotation amounts of the log-step sum over a plane (Sec. "Homomorphic Tensor Operations": reductions over
    equally strided elements take log-many rotations with additions in between).  Along the width the amounts are
    w_stride * 2^k, along the height h_stride * 2^k, each up to the next power of two of the dimension; the padding
    positions this reads are zero after the masked multiply.  That needs the padded rows not to overlap and the padded
    plane not to wrap around the slot vector; otherwise (or if it is not shorter) the sum runs over the contiguous
    power-of-two window 1, 2, 4, ... that covers the plane."""
    return reduce_steps(t, o.slots)


def reduce_steps(t: OTensor, limit):
    """The same rule for the elements of one ciphertext of a tensor with c_inner channels (a third strided
    dimension, c_stride * 2^k, whose padded planes must not overlap either); the padded elements have to stay
    below slot `limit`."""
    span = (t.c_inner - 1) * t.c_stride + (t.height - 1) * t.h_stride + (t.width - 1) * t.w_stride
    window = []
    while (1 << len(window)) < span + 1:
        window.append(1 << len(window))
    wl = max(t.width - 1, 0).bit_length()
    hl = max(t.height - 1, 0).bit_length()
    cl = max(t.c_inner - 1, 0).bit_length()
    fits = (t.w_stride << wl) <= t.h_stride and (t.c_inner == 1 or (t.h_stride << hl) <= t.c_stride) and \
        t.offset + ((1 << cl) - 1) * t.c_stride + ((1 << hl) - 1) * t.h_stride + ((1 << wl) - 1) * t.w_stride < limit
    strided = [t.w_stride << k for k in range(wl)] + [t.h_stride << k for k in range(hl)] + \
        [t.c_stride << k for k in range(cl)]
    return strided if fits and len(strided) < len(window) else window


def merge_doublings(steps, merge):
    """Rotate-and-add steps s, 2s, 4s, .. add up all multiples of s below 2^k s: up to `merge` consecutive doublings
    are taken as ONE sum of the 2^c - 1 rotations by s, 2s, 3s, .. of the same ciphertext (one decomposition, one
    division by P: SharedModDown) instead of c rotations one after the other.  Returns the groups of amounts;
    merge < 2 leaves every step a group of its own."""
    groups = []
    i = 0
    while i < len(steps):
        c = 1
        while merge >= 2 and c < merge and i + c < len(steps) and steps[i + c] == 2 * steps[i + c - 1]:
            c += 1
        groups.append([steps[i]] if c == 1 else [m * steps[i] for m in range(1, 1 << c)])
        i += c
    return groups


def rotate_and_add(o: Oracle, x, groups, right=False):
    """x += rot(x, a) for the single amounts, x = sum over {0} + group of rot(x, a) with one division by P for the
    others (rotLeft amounts; right: rotRight amounts)."""
    for grp in groups:
        amounts = [(o.slots - a) % o.slots for a in grp] if right else [a % o.slots for a in grp]
        if len(amounts) == 1:
            x = o.add(x, o.rot_right(x, grp[0]) if right else o.rot_left(x, amounts[0]))
        else:
            x = SharedModDown(o, [x]).total([(0, 0, 1, None)] + [(0, a, 1, None) for a in amounts], x.scale)
    return x


def matmul_geometry(o: Oracle, t: OTensor, replicas):
    """Block length P (the power of two that covers every element slot of a ciphertext), the number of replicas R
    actually used (a power of two, at most `replicas` and at most slots / P), the rotRight amounts that build the
    replicas (log-many, adding in between) and the rotLeft amounts of the reduction inside a block
    (Sec. "Homomorphic Tensor Operations", matmul and CHW paragraphs)."""
    top = t.offset + (t.c_inner - 1) * t.c_stride + (t.height - 1) * t.h_stride + (t.width - 1) * t.w_stride + 1
    block = 1 << (top - 1).bit_length()
    assert block <= o.slots
    r = 1
    while 2 * r <= min(replicas, o.slots // block):
        r *= 2
    replicate = [block << k for k in range(r.bit_length() - 1)]
    return block, r, replicate, reduce_steps(t, block if r > 1 else o.slots)


def matmul(o: Oracle, t: OTensor, w, replicas, merge=0):
    """Homomorphic matmul with replicas.  w[OUT][C][H][W].  Returns (CHW-tiled output tensor with R 1x1 channels per
    ciphertext, dict of the fixed-point integers used)."""
    out_n = w.shape[0]
    w = np.asarray(w, dtype=np.float64).reshape(out_n, t.channels, t.height * t.width)
    block, r, _, _ = matmul_geometry(o, t, replicas)
    l = t.cts[0].limbs
    per = cts_per_image(t)
    sl = np.asarray(tensor_slots(t)).reshape(t.c_inner, t.height * t.width)
    needs_mask = r > 1 and not t.clean
    ints = {"mask_coeffs": None, "mask_scale": 1.0}
    if needs_mask:   # 0/1 on the element slots, encoded at the scale of the modulus the divScalar removes
        mask_scale = float(o.primes[l - 1])
        masks = np.zeros((per, o.N), dtype=np.int64)
        for j in range(per):
            z = np.zeros(o.slots)
            z[sl[:min(t.c_inner, t.channels - j * t.c_inner)].reshape(-1)] = 1.0
            masks[j] = o.encode_coeffs(z, mask_scale)
        ints.update(mask_coeffs=masks, mask_scale=mask_scale)
        l -= 1
    pt_scale = float(o.primes[l - 1])
    groups = -(-out_n // r)
    coeffs = np.zeros((groups, per, o.N), dtype=np.int64)
    for g in range(groups):
        for j in range(per):
            z = np.zeros(o.slots)
            for rep in range(min(r, out_n - g * r)):
                for cl in range(min(t.c_inner, t.channels - j * t.c_inner)):
                    z[rep * block + sl[cl]] = w[g * r + rep, j * t.c_inner + cl]
            coeffs[g, j] = o.encode_coeffs(z, pt_scale)
    ints.update(pt_coeffs=coeffs, pt_scale=pt_scale)
    return matmul_fixed(o, t, ints, out_n, replicas, merge), ints


def matmul_fixed(o: Oracle, t: OTensor, ints, out_n, replicas, merge=0):
    """1. (input not clean, R > 1) mulPlain by the 0/1 mask + divScalar, so that step 2 copies zeros and not leftovers;
    2. log2 R times x += rotRight(x, P 2^k): R copies of the elements, P slots apart;  3. per group g of R outputs:
    sum over the input ciphertexts of mulPlain(x_j, weights of outputs gR..gR+R-1, output gR+r on the r-th copy),
    divScalar;  4. rotate-and-add inside the blocks: output gR+r ends in slot r P + offset.  merge: steps 2 and 4 take
    up to that many consecutive doublings as one sum of rotations (merge_doublings)."""
    block, r, replicate, reduce = matmul_geometry(o, t, replicas)
    per = cts_per_image(t)
    groups = -(-out_n // r)
    outs = []
    for b in range(t.batch):
        xs = t.cts[b * per:(b + 1) * per]
        if r > 1:
            if not t.clean:
                masked = []
                for j, x in enumerate(xs):
                    pt = o.pt_from_coeffs(ints["mask_coeffs"][j], ints["mask_scale"], x.limbs)
                    temp = o.mul_plain(x, pt)
                    masked.append(o.div_scalar(temp, o.max_scalar_div(temp, float("inf"))))
                xs = masked
            xs = [rotate_and_add(o, x, merge_doublings(replicate, merge), right=True) for x in xs]
        for g in range(groups):
            acc = None
            for j, x in enumerate(xs):
                temp = o.mul_plain(x, o.pt_from_coeffs(ints["pt_coeffs"][g, j], ints["pt_scale"], x.limbs))
                acc = temp if acc is None else o.add(acc, temp)
            acc = o.rescale(acc)
            outs.append(rotate_and_add(o, acc, merge_doublings(reduce, merge)))
    return OTensor(outs, t.batch, out_n, 1, 1, 1, 1, t.offset, 0, r, block)


def fc_fixed(o: Oracle, t: OTensor, coeffs, pt_scale, merge=0):
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
            # rotate-and-add: slot `offset` collects every element of the plane
            outs.append(rotate_and_add(o, acc, merge_doublings(steps, merge)))
    return OTensor(outs, t.batch, out_n, 1, 1, 1, 1, t.offset, 0)


def sum_pool2x2(o: Oracle, t: OTensor, merge=0):
    """x + rot(x, w_stride) + rot(x, h_stride) + rot(x, h_stride + w_stride); merge >= 2: as one sum with a single
    division by P (the chain x += rot(x, w_stride); x += rot(x, h_stride) merged, as in merge_doublings)."""
    outs = []
    for ct in t.cts:
        amounts = (t.w_stride, t.h_stride, t.h_stride + t.w_stride)
        if merge >= 2:
            outs.append(SharedModDown(o, [ct]).total([(0, 0, 1, None)] + [(0, r, 1, None) for r in amounts], ct.scale))
            continue
        acc = ct
        for r in amounts:
            acc = o.add(acc, o.rot_left(ct, r))
        outs.append(acc)
    return replace(t, cts=outs, height=t.height // 2, width=t.width // 2, h_stride=2 * t.h_stride,
                   w_stride=2 * t.w_stride, clean=0)


def avg_pool2x2(o: Oracle, t: OTensor, merge=0):
    """The 2x2 average: the sum pool with the scale of every output ciphertext taken four times as large -- a
    ciphertext stands for (integer polynomial) / scale, so this is the division by 4, exact and free of any
    ciphertext operation (no level, no noise)."""
    from .ckks import Ct
    s = sum_pool2x2(o, t, merge)
    return replace(s, cts=[Ct(ct.data, 4.0 * ct.scale) for ct in s.cts])


def divide_by_p_and_last(o: Oracle, e_b, e_a, z, l, scale):
    """(ModDown(e_b) + z_0, ModDown(e_a) + z_1) followed by the divScalar by q_{l-1}, as ONE division by q_{l-1} P: z enters
    the accumulators times P first."""
    from .ckks import Ct
    p_all = 1
    for m in range(o.K):
        p_all *= int(o.primes[o.L + m])
    qs = list(range(l))
    o.fma_const(e_b[:l], z[0], p_all, qs)
    o.fma_const(e_a[:l], z[1], p_all, qs)
    return Ct(np.stack([o.mod_down_rescale(e_b, l), o.mod_down_rescale(e_a, l)]), scale / float(o.primes[l - 1]))


def poly2_act(o: Oracle, t: OTensor, a, b, fused_rescale=False):
    """x^2 + (b/a) x, the factor a being left to the next layer.  fused_rescale: the linear term joins (d0, d1) of the
    unrelinearised square, and the relinearisation's division by P is taken together with the divScalar."""
    outs = []
    for ct in t.cts:
        if fused_rescale:
            sq = o.mul_no_relin(ct, ct)
            z = sq.data[:2].copy()
            if b != 0.0:
                z = o.add(Ct2(z, sq.scale), o.mul_scalar(ct, b / a, ct.scale)).data
            e_b, e_a = o.key_switch_acc(sq.data[2], 0)
            outs.append(divide_by_p_and_last(o, e_b, e_a, z, ct.limbs, sq.scale))
            continue
        acc = o.mul(ct, ct)
        if b != 0.0:
            acc = o.add(acc, o.mul_scalar(ct, b / a, ct.scale))
        outs.append(o.rescale(acc))
    return replace(t, cts=outs)


def Ct2(data, scale):
    from .ckks import Ct
    return Ct(np.ascontiguousarray(data), scale)


def rot_steps_conv(o: Oracle, t: OTensor, fh, fw, pad_same=False):
    ph, pw = (fh // 2, fw // 2) if pad_same else (0, 0)
    return sorted({((fy - ph) * t.h_stride + (fx - pw) * t.w_stride) % o.slots for fy in range(fh) for fx in range(fw)} - {0})


def mask_tensor(o: Oracle, t: OTensor):
    """The masking multiply of Sec. "Homomorphic Tensor Operations" (SAME-padding paragraph) as a layer of its own:
    one mulPlain by the 0/1 vector of the element slots (at the scale of the last modulus, so that the divScalar that
    follows leaves the ciphertext scale unchanged) per ciphertext.  Returns (clean tensor, the integers used)."""
    l = t.cts[0].limbs
    per = cts_per_image(t)
    mask_scale = float(o.primes[l - 1])
    sl = np.asarray(tensor_slots(t)).reshape(t.c_inner, t.height * t.width)
    masks = np.zeros((per, o.N), dtype=np.int64)
    for j in range(per):
        z = np.zeros(o.slots)
        z[sl[:min(t.c_inner, t.channels - j * t.c_inner)].reshape(-1)] = 1.0
        masks[j] = o.encode_coeffs(z, mask_scale)
    ints = {"mask_coeffs": masks, "mask_scale": mask_scale}
    return mask_tensor_fixed(o, t, ints), ints


def mask_tensor_fixed(o: Oracle, t: OTensor, ints):
    per = cts_per_image(t)
    outs = []
    for i, ct in enumerate(t.cts):
        temp = o.mul_plain(ct, o.pt_from_coeffs(ints["mask_coeffs"][i % per], ints["mask_scale"], ct.limbs))
        outs.append(o.div_scalar(temp, o.max_scalar_div(temp, float("inf"))))
    return replace(t, cts=outs, clean=1)


def add_bias(o: Oracle, t: OTensor, bias):
    """A bias per channel after a linear layer (not part of Algorithm 1; the HISA offers addPlain for it): channel
    c's elements get bias[c], every other slot stays as it is -- one addPlain per ciphertext of the vector that holds
    bias[c] on the element slots of each channel of that ciphertext, encoded at the ciphertext's own scale.  Returns
    (tensor, the encoded integers [ciphertexts per image][N])."""
    per = cts_per_image(t)
    sl = np.asarray(tensor_slots(t)).reshape(t.c_inner, t.height * t.width)
    coeffs = np.zeros((per, o.N), dtype=np.int64)
    for j in range(per):
        z = np.zeros(o.slots)
        for cl in range(min(t.c_inner, t.channels - j * t.c_inner)):
            z[sl[cl]] = bias[j * t.c_inner + cl]
        coeffs[j] = o.encode_coeffs(z, t.cts[j].scale)
    return add_bias_fixed(o, t, coeffs), coeffs


def add_bias_fixed(o: Oracle, t: OTensor, coeffs):
    per = cts_per_image(t)
    return replace(t, cts=[o.add_plain(ct, o.pt_from_coeffs(coeffs[i % per], ct.scale, ct.limbs)) for i, ct in enumerate(t.cts)])


def chw_conv_geometry(o: Oracle, t: OTensor, fh, fw, pad_same=False):
    """CHW-tiled convolution: the c_inner channel blocks of a ciphertext are combined along diagonals, output block b
    reading input block (b + d) mod c_inner for d = 0 .. c_inner-1, so one rotation per (tap, d) brings every needed
    input channel under every output channel.  The wrap-around of the blocks is a cyclic rotation only if the blocks
    fill the slot vector; otherwise one copy of the blocks is first placed behind them (rotRight by `wrap` and add; the
    slots there must be free, and zero because the input is clean).  Returns (wrap or 0, rotLeft amounts
    [fh][fw][c_inner])."""
    ci, cs = t.c_inner, t.c_stride
    assert ci > 1 and t.clean
    if ci * cs == o.slots:
        wrap = 0
    else:
        assert 2 * ci * cs <= o.slots, "no room behind the channel blocks for their copy"
        wrap = ci * cs
    ph, pw = (fh // 2, fw // 2) if pad_same else (0, 0)
    amounts = [[[((fy - ph) * t.h_stride + (fx - pw) * t.w_stride + d * cs) % o.slots for d in range(ci)]
                for fx in range(fw)] for fy in range(fh)]
    return wrap, amounts


def same_tap_inside(t: OTensor, fh, fw, fy, fx, stride):
    """For a SAME convolution: which outputs (row-major over the output plane) read an element inside the input plane
    under tap (fy, fx)."""
    oh, ow = -(-t.height // stride), -(-t.width // stride)
    ys = np.arange(oh) * stride + fy - fh // 2
    xs = np.arange(ow) * stride + fx - fw // 2
    return (((ys >= 0) & (ys < t.height))[:, None] & ((xs >= 0) & (xs < t.width))[None, :]).reshape(-1)


def conv2d_chw(o: Oracle, t: OTensor, w, stride=1, pad_same=False, shared_moddown=False, schedule="in", fused_rescale=False):
    """w[FH][FW][IC][OC] on a clean CHW-tiled tensor -> clean CHW-tiled tensor with the same channel blocks.  The
    plaintext of (tap, d, input ciphertext j, output ciphertext g) holds, on the valid output positions of block b,
    the weight from input channel j c_inner + (b + d) mod c_inner to output channel g c_inner + b (zero where either
    does not exist), encoded at the scale of the last modulus.  Returns (output, the integers used).

    schedule "taps": the other split of the same rotations -- the inputs are rotated by the diagonals only (d blocks),
    the products of each filter tap are summed where the input elements lie (the plaintext holds the weight of output
    position p on slot p + tap amount) and the sums are rotated by the taps and added, again with one division by P.
    schedule "in": the inputs are rotated by (tap, d) and the products summed.  schedule "out" (the reduction over the
    channels of a ciphertext done after the multiplication, Sec. "CHW-tiled Homomorphic Convolution 2-d"): the inputs
    are rotated by the taps only, the products of diagonal d are summed where the input channels lie -- the plaintext
    holds the same weight d blocks further up, under input block b + d -- and the c_inner sums are rotated down by d
    blocks and added, with one division by P for the whole sum (SharedModDown)."""
    assert schedule in ("in", "out", "taps")
    fh, fw, ic_n, oc_n = w.shape
    assert ic_n == t.channels
    ci, cs = t.c_inner, t.c_stride
    l = t.cts[0].limbs
    pt_scale = float(o.primes[l - 1])
    if pad_same:
        oh, ow = -(-t.height // stride), -(-t.width // stride)
    else:
        oh, ow = (t.height - fh) // stride + 1, (t.width - fw) // stride + 1
    per_in, per_out = cts_per_image(t), -(-oc_n // ci)
    plane = np.asarray(plane_slots(oh, ow, t.h_stride * stride, t.w_stride * stride, t.offset))
    coeffs = np.zeros((fh, fw, ci, per_in, per_out, o.N), dtype=np.int64)
    for fy, fx, d, j, g in np.ndindex(fh, fw, ci, per_in, per_out):
        z = np.zeros(o.slots)
        # pad_same == 2 (SAME by masking): the layout has no zero border; the plaintext of a tap is zero on the
        # outputs whose input element under that tap lies outside the plane
        here = plane[same_tap_inside(t, fh, fw, fy, fx, stride)] if pad_same == 2 else plane
        if schedule == "taps":      # under the input elements: the tap's own rotation comes after the multiplication
            ph, pw = (fh // 2, fw // 2) if pad_same else (0, 0)
            here = here + (fy - ph) * t.h_stride + (fx - pw) * t.w_stride
        for b in range(ci):
            ic, oc = j * ci + (b + d) % ci, g * ci + b
            if ic < ic_n and oc < oc_n:
                at = b + d if schedule == "out" else b    # behind the blocks lies their copy (or, cyclically, block 0)
                z[(here + at * cs) % o.slots] = float(w[fy, fx, ic, oc])
        coeffs[fy, fx, d, j, g] = o.encode_coeffs(z, pt_scale)
    ints = {"pt_coeffs": coeffs, "pt_scale": pt_scale}
    return conv2d_chw_fixed(o, t, ints, oc_n, fh, fw, stride, pad_same, shared_moddown, schedule, fused_rescale), ints


def conv2d_chw_fixed(o: Oracle, t: OTensor, ints, oc_n, fh, fw, stride, pad_same, shared_moddown=False, schedule="in",
                     fused_rescale=False):
    """fused_rescale (the schedules that rotate sums): the divScalar is taken together with the sums' division by P."""
    ci = t.c_inner
    wrap, amounts = chw_conv_geometry(o, t, fh, fw, pad_same)
    if pad_same:
        oh, ow = -(-t.height // stride), -(-t.width // stride)
    else:
        oh, ow = (t.height - fh) // stride + 1, (t.width - fw) // stride + 1
    per_in, per_out = cts_per_image(t), -(-oc_n // ci)
    outs = []
    for b in range(t.batch):
        xs = t.cts[b * per_in:(b + 1) * per_in]
        if wrap:
            xs = [o.add(x, o.rot_right(x, wrap)) for x in xs]
        if schedule == "taps":
            by_diag = {(j, d): o.rot_left(xs[j], (d * t.c_stride) % o.slots) for j in range(per_in) for d in range(ci)}
            for g in range(per_out):
                sums, steps = [], []
                for fy in range(fh):
                    for fx in range(fw):
                        acc = None
                        for d in range(ci):
                            for j in range(per_in):
                                pt = o.pt_from_coeffs(ints["pt_coeffs"][fy, fx, d, j, g], ints["pt_scale"], xs[j].limbs)
                                temp = o.mul_plain(by_diag[(j, d)], pt)
                                acc = temp if acc is None else o.add(acc, temp)
                        sums.append(acc)
                        steps.append(amounts[fy][fx][0])
                total = SharedModDown(o, sums).total([(k, steps[k], 1, None) for k in range(len(sums))], sums[0].scale,
                                                     rescale=fused_rescale)
                outs.append(total if fused_rescale else o.div_scalar(total, o.max_scalar_div(total, float("inf"))))
            continue
        if schedule == "out":
            # amounts[fy][fx][0] is the tap's own amount, d * c_stride the diagonal's
            by_tap = {(j, fy, fx): o.rot_left(xs[j], amounts[fy][fx][0])
                      for j in range(per_in) for fy in range(fh) for fx in range(fw)}
            for g in range(per_out):
                sums = []
                for d in range(ci):
                    acc = None
                    for fy in range(fh):
                        for fx in range(fw):
                            for j in range(per_in):
                                pt = o.pt_from_coeffs(ints["pt_coeffs"][fy, fx, d, j, g], ints["pt_scale"], xs[j].limbs)
                                temp = o.mul_plain(by_tap[(j, fy, fx)], pt)
                                acc = temp if acc is None else o.add(acc, temp)
                    sums.append(acc)
                total = SharedModDown(o, sums).total([(d, d * t.c_stride, 1, None) for d in range(ci)], sums[0].scale,
                                                     rescale=fused_rescale)
                outs.append(total if fused_rescale else o.div_scalar(total, o.max_scalar_div(total, float("inf"))))
            continue
        # the rotations do not depend on the output ciphertext: computed once
        shared = SharedModDown(o, xs) if shared_moddown else None
        rotated = {} if shared_moddown else {
            (j, fy, fx, d): o.rot_left(xs[j], amounts[fy][fx][d])
            for j in range(per_in) for fy in range(fh) for fx in range(fw) for d in range(ci)}
        for g in range(per_out):
            if shared is not None:
                terms = [(j, amounts[fy][fx][d], ints["pt_coeffs"][fy, fx, d, j, g], (fy, fx, d, j, g))
                         for fy in range(fh) for fx in range(fw) for d in range(ci) for j in range(per_in)]
                acc = shared.total(terms, xs[0].scale * ints["pt_scale"])
                outs.append(o.div_scalar(acc, o.max_scalar_div(acc, float("inf"))))
                continue
            acc = None
            for fy in range(fh):
                for fx in range(fw):
                    for d in range(ci):
                        for j in range(per_in):
                            pt = o.pt_from_coeffs(ints["pt_coeffs"][fy, fx, d, j, g], ints["pt_scale"], xs[j].limbs)
                            temp = o.mul_plain(rotated[(j, fy, fx, d)], pt)
                            acc = temp if acc is None else o.add(acc, temp)
            outs.append(o.div_scalar(acc, o.max_scalar_div(acc, float("inf"))))
    return OTensor(outs, t.batch, oc_n, oh, ow, t.h_stride * stride, t.w_stride * stride, t.offset, 1, ci, t.c_stride)


def rot_steps_conv_chw(o: Oracle, t: OTensor, fh, fw, pad_same=False, schedule="in"):
    wrap, amounts = chw_conv_geometry(o, t, fh, fw, pad_same)
    if schedule in ("out", "taps"):
        steps = {row[0] for plane in amounts for row in plane} | {(d * t.c_stride) % o.slots for d in range(t.c_inner)}
    else:
        steps = {a for plane in amounts for row in plane for a in row}
    steps |= {o.slots - wrap} if wrap else set()
    return sorted(steps - {0})


def to_chw(o: Oracle, t: OTensor, c_inner, c_stride):
    """Layout switch HW -> CHW (Sec. "Data Layout Selection", the layouts that change tiling around a layer): channel
    g c_inner + b moves b blocks to the right (rotRight by b c_stride) and the c_inner channels of a group are added
    into one ciphertext.  The input must be clean (what lies between the elements would land on other channels); no
    level is used."""
    assert t.c_inner == 1 and t.clean
    assert t.offset + (c_inner - 1) * c_stride + (t.height - 1) * t.h_stride + (t.width - 1) * t.w_stride < o.slots
    per = -(-t.channels // c_inner)
    outs = []
    for b in range(t.batch):
        for g in range(per):
            acc = t.cts[b * t.channels + g * c_inner]
            for k in range(1, min(c_inner, t.channels - g * c_inner)):
                acc = o.add(acc, o.rot_right(t.cts[b * t.channels + g * c_inner + k], k * c_stride))
            outs.append(acc)
    return replace(t, cts=outs, c_inner=c_inner, c_stride=c_stride)


def to_hw(o: Oracle, t: OTensor):
    """Layout switch CHW -> HW: block b of a ciphertext is rotated to the front (rotLeft by b c_stride) and everything
    but the plane is masked away (mulPlain by the 0/1 vector of the plane's slots at the scale of the last modulus,
    divScalar): one level, clean HW-tiled output.  Returns (tensor, the integers used)."""
    l = t.cts[0].limbs
    mask_scale = float(o.primes[l - 1])
    z = np.zeros(o.slots)
    z[plane_slots(t.height, t.width, t.h_stride, t.w_stride, t.offset)] = 1.0
    ints = {"mask_coeffs": o.encode_coeffs(z, mask_scale), "mask_scale": mask_scale}
    return to_hw_fixed(o, t, ints), ints


def to_hw_fixed(o: Oracle, t: OTensor, ints):
    per = cts_per_image(t)
    outs = []
    for b in range(t.batch):
        for c in range(t.channels):
            ct = t.cts[b * per + c // t.c_inner]
            k = c % t.c_inner
            temp = o.rot_left(ct, k * t.c_stride) if k else ct
            temp = o.mul_plain(temp, o.pt_from_coeffs(ints["mask_coeffs"], ints["mask_scale"], ct.limbs))
            outs.append(o.div_scalar(temp, o.max_scalar_div(temp, float("inf"))))
    return replace(t, cts=outs, c_inner=1, c_stride=0, clean=1)
