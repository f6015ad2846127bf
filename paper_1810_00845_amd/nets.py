"""Encrypted inference schedules for the LeNet-shaped benchmark networks: sequences of calls into the tensor
layer of libhisa (conv2d, poly2_act, sum_pool2x2, fc), nothing else.

A network is a list of layer tuples.  The factors the encrypted layers leave to their successor (the `a` of an
activation a x^2 + b x, the 1/4 of an average pool; Sec. "Runtime" of the paper folds such constants into the next
linear layer) are multiplied into the next layer's weights here, on the host, before the call.

    ("conv", w[FH][FW][IC][OC], stride)      VALID convolution, Algorithm 1 with scalar weights
    ("act", a, b)                            a x^2 + b x
    ("pool",)                                2x2 average pool
    ("fc", w[OUT][C][H][W])                  fully connected over the whole tensor (with layout "chw_fc": homomorphic
                                             matmul with replicas, CHW-tiled from there on)
    ("conv_same", w[FH][FW][IC][OC])         SAME convolution with the masking multiply (clean output)
    ("fire", ws, w1, w3, a, b)               SqueezeNet fire module: 1x1 squeeze, activation, 1x1 and 3x3 (SAME)
                                             expand convolutions whose outputs are concatenated along the channels
    ("gap",)                                 global average pool: one value per channel
    ("bias", b[C])                           b[c] added to channel c, directly after a conv / fc layer
"""
import time

import numpy as np

from . import synth


def lenet_small(seed=3):
    """Benchmark configuration 3: N = 2^13, 8 limbs, one 28x28 image (zero border of one pixel: 30x30 encrypted, so that
    the stride-2 5x5 convolution gives 13x13), conv 1->5, square, FC 845->100, square, FC 100->10."""
    layers = [("conv", synth.conv_weights(seed, 5, 5, 1, 5, dist="normal", std=0.1), 2),
              ("act", 1.0, 0.0),
              ("fc", synth.fc_weights(seed + 1, 100, 5, 13, 13, std=0.1)),
              ("act", 1.0, 0.0),
              ("fc", synth.fc_weights(seed + 2, 10, 100, 1, 1, std=0.1))]
    params = dict(log_n=13, q_bits=[50] + [40] * 7, dnum=2, special_bits=50, scale=2.0 ** 40)
    x = np.zeros((1, 1, 30, 30))
    x[0, 0, 1:29, 1:29] = synth.image(seed + 3, 1, 28, 28)[0]
    return params, layers, x


def lenet_medium(seed=4):
    """Benchmark configuration 4: N = 2^14, 12 limbs, conv5x5 1->20, pool, conv5x5 20->50, pool, FC 800->500, FC 500->10,
    a degree-2 activation a x^2 + b x (a, b uniform in [0.1, 0.5]) after each convolution and the first FC.
    The weight spreads are chosen so that every layer's values stay of order one."""
    rng = np.random.default_rng(seed)
    ab = rng.uniform(0.1, 0.5, (3, 2))
    layers = [("conv", synth.conv_weights(seed, 5, 5, 1, 20, dist="normal", std=0.1), 1),
              ("act", ab[0, 0], ab[0, 1]), ("pool",),
              ("conv", synth.conv_weights(seed + 1, 5, 5, 20, 50, dist="normal", std=0.2), 1),
              ("act", ab[1, 0], ab[1, 1]), ("pool",),
              ("fc", synth.fc_weights(seed + 2, 500, 50, 4, 4, std=0.1)),
              ("act", ab[2, 0], ab[2, 1]),
              ("fc", synth.fc_weights(seed + 3, 10, 500, 1, 1, std=0.15))]
    params = dict(log_n=14, q_bits=[50] + [40] * 11, dnum=3, special_bits=50, scale=2.0 ** 40)
    x = synth.image(seed + 4, 1, 28, 28)[None]
    return params, layers, x


SQUEEZENET_PARAMS = dict(log_n=15, q_bits=[50] + [45] * 20, dnum=3, special_bits=50, scale=2.0 ** 45, border=1)


def _squeezenet_layers(seed, conv, ab):
    """conv3x3 3->64, four fire modules (squeeze 16, 16, 32, 32; expand 64+64, 64+64, 128+128, 128+128), 1x1 convolution to
    10 classes, global average pool; a degree-2 activation after the first convolution, inside and after every fire
    module.  conv(k, filter side, inputs, outputs, (a, b) of the activation in front or None) makes layer k's weights."""
    layers = [("conv_same", conv(1, 3, 3, 64, None)), ("act", ab[0, 0], ab[0, 1])]
    prev = ab[0]
    ic, k = 64, 2
    for i, (sq, ex) in enumerate([(16, 64), (16, 64), (32, 128), (32, 128)]):
        inner = ab[1 + 2 * i]
        layers.append(("fire", conv(k, 1, ic, sq, prev), conv(k + 1, 1, sq, ex, inner), conv(k + 2, 3, sq, ex, inner),
                       inner[0], inner[1]))
        layers.append(("act", ab[2 + 2 * i, 0], ab[2 + 2 * i, 1]))
        prev = ab[2 + 2 * i]
        ic, k = 2 * ex, k + 3
    layers += [("conv", conv(k, 1, ic, 10, prev), 1), ("gap",)]
    return layers


def squeezenet_cifar(seed=5, spread=0.2):
    """Benchmark configuration 5: N = 2^15, 21 limbs, 32x32x3 image, the SqueezeNet-style layers above.  The configuration's
    own weight distribution, N(0, 0.05^2) everywhere, makes a degree-2 network collapse (squeezenet_cifar_literal: the
    outputs are of the order 1e-8), so the weights here are normal with a spread that follows from the layer's shape and
    the activation in front of it, not from any data: a linear layer of fan-in F behind a x^2 + b x gets
    std = g / sqrt(F), g = 1 / sqrt(b^2 + 3 a^2 spread^2) -- the gain that brings values of standard deviation `spread`
    back to it after that activation (for normal values); the first layer g = spread / rms of a uniform [0, 1) image.
    With spread 0.2 the values of seeds 5 .. 9 stay within [-1.4, 1.4] in every layer (random degree-2 networks are not
    stable in general: seed 10 grows beyond any scale)."""
    rng = np.random.default_rng(seed)
    ab = rng.uniform(0.1, 0.5, (9, 2))

    def conv(k, fh, ic, oc, act):
        gain = spread * np.sqrt(3.0) if act is None else 1.0 / np.sqrt(act[1] ** 2 + 3.0 * act[0] ** 2 * spread ** 2)
        return synth.conv_weights(seed + k, fh, fh, ic, oc, dist="normal", std=gain / np.sqrt(fh * fh * ic))
    return dict(SQUEEZENET_PARAMS), _squeezenet_layers(seed, conv, ab), synth.image(seed + 40, 3, 32, 32)[None]


def squeezenet_cifar_literal(seed=5):
    """The same layers with the weights exactly as benchmark configuration 5 words them: N(0, 0.05^2) in every layer.  Every
    layer shrinks the values (3e-1 after the first activation, 1e-7 before the pool, 4e-8 at the output for seed 5), so
    an absolute error bound says little here; the test reports the error relative to the output's size as well."""
    rng = np.random.default_rng(seed)
    ab = rng.uniform(0.1, 0.5, (9, 2))
    conv = lambda k, fh, ic, oc, act: synth.conv_weights(seed + k, fh, fh, ic, oc, dist="normal", std=0.05)
    return dict(SQUEEZENET_PARAMS), _squeezenet_layers(seed, conv, ab), synth.image(seed + 40, 3, 32, 32)[None]


def _concat_channels(ctx, a, b):
    """Channel concatenation of two tensors of one image with identical layout, level and scale."""
    from .hisa import CipherTensor
    assert a.batch == 1 and b.batch == 1 and a.meta()[2:] == b.meta()[2:] and a.channels % a.c_inner == 0
    t = CipherTensor(ctx, list(a.cts) + list(b.cts), 1, a.channels + b.channels, a.height, a.width, a.h_stride,
                     a.w_stride, a.offset, a.clean, a.c_inner, a.c_stride)
    a.cts, b.cts = [], []   # the handles now belong to the concatenation
    return t


LAYOUTS = ("hw", "chw_fc", "chw", "hw_conv")


def chw_blocks(slots, plane_slots_needed, layers, chw_convs=True):
    """CHW-tiling of the input: (channels per ciphertext, channel stride).  The stride is the power of two that holds
    a plane with its border; as many blocks as the slots hold, and no more than the convolutions can rotate through
    (taps x blocks rotation amounts per input ciphertext, at most 256)."""
    c_stride = 1 << max(0, plane_slots_needed - 1).bit_length()
    taps = [1]
    for layer in layers if chw_convs else ():
        if layer[0] in ("conv", "conv_same"):
            taps.append(layer[1].shape[0] * layer[1].shape[1])
        elif layer[0] == "fire":
            taps.append(layer[3].shape[0] * layer[3].shape[1])
    c_inner = 1
    while 2 * c_inner * c_stride <= slots and 2 * c_inner * max(taps) <= 256:
        c_inner *= 2
    return c_inner, c_stride


def run_encrypted(ctx, layers, x, scale, limbs, make_keys=False, border=0, plans=None, layout="hw", shared_moddown=True,
                  layer_times=True, rotate_sums=True, merge_doublings=4, fused_rescale=True, client_times=None):
    """Encrypts x, runs the layers, decrypts.  Returns (output array, seconds from encrypt-done to the last
    ciphertext ready, per-layer seconds).  With make_keys the rotation keys each layer asks for are generated
    on the way (set-up pass); otherwise they must be resident.  `plans` (a dict, filled by the set-up pass and
    reused afterwards) holds the layers' weights converted and encoded ahead of time; without it that is done
    inside every call.  layout: "hw" keeps one channel per ciphertext throughout; "chw_fc" (the paper's "CHW-fc and
    HW-before", Sec. "Data Layout Selection") is HW-tiled up to the first fully connected layer, which runs as a
    matmul with as many replicas as the slots hold and leaves a CHW-tiled tensor for the layers after it; "chw" packs
    several channels into every ciphertext from the input on (CHW-tiled convolutions multiply by plaintexts and need
    clean inputs: a masking multiply follows each pool); "hw_conv" (the paper's "HW-conv and CHW-rest") keeps the tensor
    CHW-tiled between the layers but switches to HW-tiling before every convolution and back after it (one level
    for the way to HW, one for the masking multiply that makes Algorithm 1's output clean enough to pack).
    shared_moddown: the convolutions divide by P once per output ciphertext instead of once per rotation (where the
    parameters have the fused key-switch path).  rotate_sums: a CHW-tiled convolution reduces over the channel blocks
    after the multiplication (HISA_CHW_ROTATE_SUMS) where that takes fewer key switches.  merge_doublings: the
    rotate-and-add chains of FC and matmul take up to that many consecutive doublings as one sum of rotations
    (hisa_set_merge_doublings; 0: the chains as they are).  fused_rescale: layers whose division by P is directly
    followed by their divScalar take both in one base conversion (hisa_set_fused_rescale).  layer_times: wait for the GPU after every layer to time it; without,
    the host queues the whole network ahead of the GPU and only the end-to-end latency is measured (per-layer entries
    are then host queueing times).  client_times: a dict that receives the seconds the client side took, "encrypt_s"
    (encode + encrypt of the image) and "decrypt_s" (decrypt + decode of the result), both outside the latency."""
    assert layout in LAYOUTS
    if layout == "chw":
        border = 0      # CHW-tiled convolutions multiply by plaintexts, which carry the SAME padding: planes back to back
    fused = ctx.log_n >= 12 and max(ctx.primes) < 2 ** 50 and ctx.dnum <= 8
    ctx.set_merge_doublings(merge_doublings if fused else 0)
    ctx.set_fused_rescale(bool(fused_rescale and fused))
    replicas = 1 if layout == "hw" else 1 << 30
    tiling = {}
    if layout in ("chw", "hw_conv"):
        hs = x.shape[3] + 2 * border
        ci, cs = chw_blocks(ctx.N // 2, (x.shape[2] + 2 * border) * hs, layers, chw_convs=layout == "chw")
        if layout == "chw":
            tiling = dict(c_inner=ci, c_stride=cs)
    ctx.sync()
    t_client = time.perf_counter()
    if border:   # leave `border` rows and columns of zero slots around every plane (SAME convolutions need them)
        hs = x.shape[3] + 2 * border
        t = ctx.tensor_encrypt(x, scale, limbs, h_stride=hs, offset=border * hs + border, **tiling)
    else:
        t = ctx.tensor_encrypt(x, scale, limbs, **tiling)
    ctx.sync()
    t_start = time.perf_counter()
    if client_times is not None:
        client_times["encrypt_s"] = t_start - t_client
    per_layer = []
    pending = 1.0     # constant factor the previous layers left to the next linear layer
    def fully_connected(idx, t, w, replicas=1):
        if replicas > 1 or t.c_inner > 1:
            if make_keys:
                ctx.gen_rot_keys(ctx.matmul_rot_steps(t, replicas))
            if plans is None:
                return ctx.matmul(t, w, replicas)
            if idx not in plans:
                plans[idx] = ("matmul", ctx.matmul_prepare(t, w, replicas))
            return ctx.matmul_apply(t, plans[idx][1])
        if make_keys and t.height * t.width > 1:
            ctx.gen_rot_keys(ctx.fc_rot_steps(t))
        if plans is None or t.height * t.width == 1:
            return ctx.fc(t, w)
        if idx not in plans:
            plans[idx] = ("fc", ctx.fc_prepare(t, w))
        return ctx.fc_apply(t, plans[idx][1])

    def convolution(key, t, w, fh, fw, **kw):
        if layout == "hw_conv":           # to HW-tiling, Algorithm 1, masking multiply, back to CHW-tiling
            unpacked = None
            if t.c_inner > 1:
                if make_keys:
                    ctx.gen_rot_keys(ctx.tensor_layout_rot_steps(t))
                t = unpacked = ctx.tensor_to_hw(t)
            out = hw_or_chw_convolution(key, t, w, fh, fw, **kw)
            if unpacked is not None:
                unpacked.free()
            if not out.clean:
                dirty, out = out, ctx.tensor_mask(out)
                dirty.free()
            if make_keys:
                ctx.gen_rot_keys(ctx.tensor_layout_rot_steps(out, ci, cs))
            flat, out = out, ctx.tensor_to_chw(out, ci, cs)
            flat.free()
            return out
        return hw_or_chw_convolution(key, t, w, fh, fw, **kw)

    def hw_or_chw_convolution(key, t, w, fh, fw, plan_only=False, **kw):
        cleaned = None
        if t.c_inner > 1:                 # CHW-tiled: plaintext weights on a clean input
            kw["mode"] = 2
            if kw.get("pad_same") and layout == "chw":
                kw["pad_same"] = 2        # no zero border in this layout: the plaintexts mask what the taps reach outside
            if not t.clean:
                t = cleaned = ctx.tensor_mask(t)
            # Where the rotations go: all on the inputs (tap and diagonal), taps on the inputs and diagonals on the
            # sums, or diagonals on the inputs and taps on the sums -- whichever is cheapest, a rotation of an input
            # (shared decomposition) priced at 0.5 and a rotation inside a sum (shared division by P, its own
            # decomposition) at 0.8 of a stand-alone one
            ci, taps = t.c_inner, fh * fw
            per_in, per_out = -(-t.channels // ci), -(-w.shape[3] // ci)
            fused = ctx.log_n >= 12 and max(ctx.primes) < 2 ** 50 and ctx.dnum <= 8
            price = {0: 0.5 * per_in * (taps * ci - 1)}
            if rotate_sums and fused:
                if ci - 1 <= 32:
                    price[1] = 0.5 * per_in * (taps - 1) + 0.8 * per_out * (ci - 1)
                if 1 < taps <= 33:
                    price[2] = 0.5 * per_in * (ci - 1) + 0.8 * per_out * (taps - 1)
            best = min(price, key=lambda k: (price[k], k))
            if best and price[best] < price[0] / 1.2:
                kw["chw_schedule"] = best
        if make_keys:
            ctx.gen_rot_keys(ctx.conv2d_rot_steps(t, fh, fw, stride=kw.get("stride", 1), pad_same=kw.get("pad_same", False),
                                                  chw_schedule=kw.get("chw_schedule", 0)))
        # one division by P per output instead of one per rotation pays when there are clearly more rotations than
        # outputs and the weights are scalars: with plaintext weights the sum on the l + K limbs reads that many more
        # limbs of every accumulator and plaintext, which costs more than the divisions it saves (measured on the
        # CHW-tiled SqueezeNet: 46.5 ms without, 49.9 ms with)
        scalar = t.c_inner == 1 and kw.get("mode", 0) != 2
        rotations = (fh * fw - 1) * t.channels
        kw["shared_moddown"] = (shared_moddown and scalar and ctx.log_n >= 12 and max(ctx.primes) < 2 ** 50 and
                                rotations >= 4 * w.shape[3] and rotations >= 64)
        if plans is None:
            out = ctx.conv2d(t, w, fh, fw, **kw)
        else:
            if key not in plans:
                plans[key] = ("conv", ctx.conv2d_prepare(t, w, fh, fw, **kw))
            if plan_only:                 # the caller applies it together with other plans of the same tensor
                return None
            out = ctx.conv2d_apply(t, plans[key][1])
        if cleaned is not None:
            cleaned.free()
        return out

    for idx, layer in enumerate(layers):
        t0 = time.perf_counter()
        kind = layer[0]
        if kind == "conv":
            w, stride = layer[1] * pending, layer[2]
            pending = 1.0
            fh, fw = w.shape[:2]
            nxt = convolution(idx, t, w, fh, fw, stride=stride)
        elif kind == "act":
            a, b = layer[1], layer[2]
            nxt = ctx.poly2_act(t, a, b)
            pending *= a
        elif kind == "pool":
            if make_keys:
                ctx.gen_rot_keys(ctx.pool_rot_steps(t))
            nxt = ctx.sum_pool2x2(t)
            pending *= 0.25
        elif kind == "conv_same":
            w = layer[1] * pending
            pending = 1.0
            fh, fw = w.shape[:2]
            nxt = convolution(idx, t, w, fh, fw, pad_same=True, mode=1)
        elif kind == "fire":
            ws, w1, w3, a, b = layer[1] * pending, layer[2], layer[3], layer[4], layer[5]
            pending = 1.0
            s0 = convolution((idx, "squeeze"), t, ws, 1, 1)
            s1 = ctx.poly2_act(s0, a, b)
            s0.free()
            if plans is not None and layout != "hw_conv" and s1.c_inner > 1 and s1.clean:
                # CHW-tiled: both branches rotate the squeezed tensor by the channel diagonals -- once for the two
                hw_or_chw_convolution((idx, "expand1"), s1, w1 * a, 1, 1, plan_only=True)
                hw_or_chw_convolution((idx, "expand3"), s1, w3 * a, 3, 3, plan_only=True, pad_same=True, mode=1)
                e1, e3 = ctx.conv2d_apply_multi(s1, [plans[(idx, "expand1")][1], plans[(idx, "expand3")][1]])
            else:
                e1 = convolution((idx, "expand1"), s1, w1 * a, 1, 1)
                e3 = convolution((idx, "expand3"), s1, w3 * a, 3, 3, pad_same=True, mode=1)
            s1.free()
            nxt = _concat_channels(ctx, e1, e3)
        elif kind == "gap" and fused and 1 < t.width <= 33 and 1 < t.height <= 33:
            # the sum over a plane as two sums of rotations of one ciphertext: along the rows, then along the columns
            # (one decomposition and one division by P each; all channels of a ciphertext at once), then the mean's
            # factor, and what the previous layers left, as one scalar multiplication and its division
            from .hisa import CipherTensor
            hw = t.height * t.width
            cur, own = list(t.cts), False
            for count, stride in ((t.width, t.w_stride), (t.height, t.h_stride)):
                amounts = [k * stride for k in range(count)]
                if make_keys:
                    ctx.gen_rot_keys(amounts[1:])
                summed = ctx.rot_left_sum_batch([cur] * count, amounts)
                if own:
                    for ct in cur:
                        ct.free()
                cur, own = summed, True
            for ct in cur:
                ctx.mul_scalar_assign(ct, pending / hw, float(ctx.primes[ct.limbs - 1]))
            ctx.rescale_batch(cur)
            pending = 1.0
            nxt = CipherTensor(ctx, cur, t.batch, t.channels, 1, 1, 1, 1, t.offset, 0, t.c_inner, t.c_stride)
        elif kind == "gap" and t.height == t.width and t.height > 1 and t.height & (t.height - 1) == 0:
            # a square plane with a power-of-two side: halve it by 2x2 sums down to one element per channel (three
            # rotations sharing a decomposition per halving, all channels of a ciphertext at once), then the mean's
            # factor, and what the previous layers left, as one scalar multiplication and its division
            hw = t.height * t.width
            nxt = t
            while nxt.height > 1:
                if make_keys:
                    ctx.gen_rot_keys(ctx.pool_rot_steps(nxt))
                halved = ctx.sum_pool2x2(nxt)
                if nxt is not t:
                    nxt.free()
                nxt = halved
            for ct in nxt.cts:
                ctx.mul_scalar_assign(ct, pending / hw, float(ctx.primes[ct.limbs - 1]))
            ctx.rescale_batch(nxt.cts)
            pending = 1.0
        elif kind == "gap":
            c, hw = t.channels, t.height * t.width
            w = np.zeros((c, c, t.height, t.width))
            for k in range(c):
                w[k, k] = pending / hw
            pending = 1.0
            nxt = fully_connected(idx, t, w)
        elif kind == "fc":
            w = layer[1] * pending
            pending = 1.0
            nxt = fully_connected(idx, t, w, replicas)
        elif kind == "bias":
            # in place; the linear layer in front has taken up every pending factor (an activation or pool between
            # them would leave the bias at the wrong scale)
            assert pending == 1.0, "a bias follows a linear layer directly"
            ctx.tensor_add_bias(t, np.asarray(layer[1], dtype=np.float64))
            nxt = None
        else:
            raise ValueError(kind)
        if nxt is not None:
            t.free()
            t = nxt
        if layer_times:
            ctx.sync()
        per_layer.append((kind, time.perf_counter() - t0))
    ctx.sync()
    latency = time.perf_counter() - t_start
    t_client = time.perf_counter()
    out = ctx.tensor_decrypt(t) * pending
    if client_times is not None:
        client_times["decrypt_s"] = time.perf_counter() - t_client
    t.free()
    return out, latency, per_layer


def free_plans(ctx, plans):
    for kind, plan in plans.values():
        if kind == "fc":
            ctx.fc_plan_free(plan)
        elif kind == "matmul":
            ctx.matmul_plan_free(plan)
        else:
            ctx.conv_plan_free(plan)
    plans.clear()


# ---------------------------------------------------------------------------
# analysis passes of the compiler (Sec. "Compiler"): each is a dry run of the schedule on the library's analysis
# backend, which records what the circuit would do instead of computing it
# ---------------------------------------------------------------------------
def analyse(ctx, layers, x, scale, limbs, border=0, layout="hw"):
    """Dry run: ({operation: count, "min_limbs": lowest level reached}, left-rotation amounts that need keys).  The
    rotation amounts are the rotation-key selection of Sec. "Rotation Keys Selection"; limbs - min_limbs is the
    number of moduli the circuit consumes (the depth the parameter selection has to provide)."""
    ctx.analysis_begin()
    try:
        run_encrypted(ctx, layers, x, scale, limbs, border=border, layout=layout)
    finally:
        counts, steps = ctx.analysis_end()
    return counts, steps


COST_OPS = ("rot_left", "rot_shared", "rot_summed", "relinearize", "mul", "mul_plain", "mul_scalar", "add", "rescale", "mac_plain",
            "mac_scalar", "key_switch_calls")


def measure_costs(ctx, limbs, batch=64, reps=5, levels=None):
    """The cost table of the layout selection (Sec. "Data Layout Selection": the costs may come from micro-benchmarks):
    seconds per ciphertext operation at `limbs` limbs (see measure_costs_at), and -- a circuit spends most of its
    operations below the level it starts at, where a key switch costs a fraction of what it does at the top -- under
    "poly" the coefficients (c0, c1, c2) of each cost as a polynomial c0 + c1 l + c2 l^2 in the level l, through
    the measurements at `levels` (default: the top, the middle and 2 limbs; two levels give a line, one a constant).
    Interpolation only: no circuit runs above the top or below 2 limbs.  estimate_cost uses the polynomial."""
    if levels is None:
        levels = sorted({limbs, (limbs + 2) // 2, min(limbs, 2)}, reverse=True)
    at = {l: measure_costs_at(ctx, l, batch, reps) for l in levels}
    costs = dict(at[limbs], limbs=limbs, levels=at, poly={})
    for op in COST_OPS:
        if op == "key_switch_calls" or len(levels) == 1:          # launch latency per call does not follow the level
            costs["poly"][op] = (costs[op], 0.0, 0.0)
        else:
            fit = np.polyfit([float(l) for l in levels], [at[l][op] for l in levels], min(2, len(levels) - 1))
            costs["poly"][op] = tuple(float(c) for c in fit[::-1]) + (0.0,) * (3 - len(fit))
    return costs


def measure_costs_at(ctx, limbs, batch=64, reps=5):
    """Seconds per ciphertext operation at `limbs` limbs, from timing each primitive on a batch of random ciphertexts.
    A key-switched call of n ciphertexts takes about t0 + n t1: t1 (from the full batch and a batch of one) is the
    operation's cost, t0 -- what a call costs however small its batch: the launches' latency -- is "key_switch_calls".
    "rot_shared" is what a rotation saves when it shares another one's decomposition (a negative cost), "rot_summed"
    what it saves inside a sum of rotations that takes its division by P once; "mac_plain" and "mac_scalar" are the
    terms of the layers' fused multiply-accumulate, timed on 1x1 convolutions (which rotate nothing)."""
    from .hisa import CipherTensor
    cts = ctx.ct_random_batch(batch, limbs, 2.0 ** 40, 900)
    pt = ctx.encode(np.ones(8), float(ctx.primes[limbs - 1]), limbs)
    ctx.gen_rot_keys([1, 2, 3])

    def timed(fn):                     # seconds per call
        fn()
        ctx.sync()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        ctx.sync()
        return (time.perf_counter() - t0) / reps

    def split(fn):                     # fn(first n ciphertexts): (seconds per ciphertext, seconds per call) of t0 + n t1
        full, single = timed(lambda: fn(batch)), timed(lambda: fn(1))
        t1 = max(0.0, (full - single) / (batch - 1))
        return t1, max(0.0, single - t1)

    def free(out):
        for c in out:
            free(c) if isinstance(c, list) else c.free()

    costs = {}
    costs["rot_left"], costs["key_switch_calls"] = split(lambda n: free(ctx.rot_left_batch(cts[:n], 1)))
    rot = costs["rot_left"]
    # Rotations that share work are priced on groups of nine, the size of a 3x3 convolution's taps (short groups
    # understate the sharing: their fixed costs weigh as much as the rotations).  "rot_shared": what each further
    # rotation of a ciphertext saves when it reuses the decomposition -- nine rotations of every ciphertext in one
    # hoisted call cost 9 rot + 8 rot_shared; never more than nine tenths of a rotation saved.
    many = list(range(1, 10))
    ctx.gen_rot_keys(many)

    def hoisted(n):
        for row in ctx.rot_left_hoisted_batch(cts[:n], many):
            free(row)
    costs["rot_shared"] = min(0.0, max((split(hoisted)[0] - 9 * rot) / 8, -0.9 * rot))
    costs["rot_summed"] = 0.0
    if ctx.log_n >= 12 and max(ctx.primes) < 2 ** 50 and ctx.dnum <= 8:
        # "rot_summed": what a rotation saves inside a sum that takes its division by P once -- a sum of nine
        # rotations of one ciphertext costs 9 rot + 8 rot_shared + 9 rot_summed; its inner product stays to be paid
        def summed(n):
            free(ctx.rot_left_sum_batch([cts[:n]] * 9, many))
        saved = (split(summed)[0] - 9 * rot - 8 * costs["rot_shared"]) / 9
        costs["rot_summed"] = min(0.0, max(saved, -0.9 * (rot + costs["rot_shared"])))
    per_ct = lambda fn: timed(fn) / batch
    costs["add"] = per_ct(lambda: free(ctx.add_batch(cts, cts)))
    costs["mul"] = per_ct(lambda: free(ctx.mul_no_relin_batch(cts, cts)))
    costs["mul_plain"] = per_ct(lambda: free(ctx.mul_plain_batch(cts, pt)))
    costs["mul_scalar"] = costs["mul_plain"]          # both stream a ciphertext through one multiply per residue

    def relin(n):
        sq = ctx.mul_no_relin_batch(cts[:n], cts[:n])
        ctx.relinearize_batch(sq)
        free(sq)
    costs["relinearize"] = max(0.0, split(relin)[0] - costs["mul"])

    def rescale():
        cp = ctx.add_batch(cts, cts)
        ctx.rescale_batch(cp)
        free(cp)
    costs["rescale"] = max(0.0, per_ct(rescale) - costs["add"])
    # fused multiply-accumulate: a 1x1 convolution over `batch` channels is batch * outputs terms and one divScalar per output
    t = CipherTensor(ctx, cts, 1, batch, 1, 1, 1, 1, 0, 1)
    w = np.random.default_rng(0).normal(0.0, 0.1, (1, 1, batch, batch))
    for name, mode in (("mac_scalar", 0), ("mac_plain", 2)):
        plan = ctx.conv2d_prepare(t, w, 1, 1, mode=mode)
        conv = per_ct(lambda: free(ctx.conv2d_apply(t, plan).cts))      # seconds per output
        costs[name] = max(0.0, conv - costs["rescale"]) / batch
        ctx.conv_plan_free(plan)
    t.cts = []
    pt.free()
    free(cts)
    return costs


def estimate_cost(counts, costs, level_aware=True):
    """The analyser's figure for a circuit: sum over the operations of occurrences times cost.  With a cost table that
    knows each cost as c0 + c1 l + c2 l^2 in the level l, an occurrence is charged at its own level: the counts carry
    the limbs and their squares summed over the occurrences, so the sum needs no list of the operations."""
    if not level_aware or "poly" not in costs or "limb_sum" not in counts:
        return sum(counts[op] * costs[op] for op in COST_OPS)
    return sum(c[0] * counts[op] + c[1] * counts["limb_sum"][op] + c[2] * counts["limb_sq_sum"][op]
               for op, c in ((op, costs["poly"][op]) for op in COST_OPS))


def select_layout(ctx, layers, x, scale, limbs, costs, border=0, layouts=LAYOUTS):
    """Data layout selection (Sec. "Data Layout Selection"): build the circuit for every layout, let the analyser
    cost it, keep the cheapest.  Returns (layout, {layout: estimated seconds})."""
    est = {lay: estimate_cost(analyse(ctx, layers, x, scale, limbs, border, lay)[0], costs) for lay in layouts}
    return min(est, key=est.get), est


# 128-bit security for ternary secrets: largest log2(Q P) per ring degree (the table of the Homomorphic Encryption
# Standard that the paper's parameter selection consults)
HE_STANDARD_128 = {10: 27, 11: 54, 12: 109, 13: 218, 14: 438, 15: 881}


def select_parameters(layers, x, log_n, scale_bits, first_bits=50, dnum=3, special_bits=50, border=0, layout="hw",
                      probe_limbs=28):
    """Encryption parameter selection (Sec. "Encryption Parameters Selection"): a dry run of the schedule on a context
    with more moduli than any circuit here needs measures the depth (the number of moduli the divScalar calls
    consume); the modulus chain is then one first prime and one prime of the scale's size per level.  Returns the
    parameters for hisa.Context, the rotation amounts that need keys, and whether the ring degree meets the 128-bit
    table for the resulting modulus."""
    from .hisa import Context
    probe = Context(log_n, [first_bits] + [scale_bits] * (probe_limbs - 1), dnum, special_bits, seed=1)
    try:
        counts, steps = analyse(probe, layers, x, 2.0 ** scale_bits, probe_limbs, border=border, layout=layout)
    finally:
        probe.close()
    depth = probe_limbs - counts["min_limbs"]
    q_bits = [first_bits] + [scale_bits] * depth
    k = -(-len(q_bits) // dnum)
    total_bits = sum(q_bits) + k * special_bits
    return {"log_n": log_n, "q_bits": q_bits, "dnum": dnum, "special_bits": special_bits, "scale": 2.0 ** scale_bits,
            "depth": depth, "rot_steps": steps, "modulus_bits": total_bits,
            "secure_128": total_bits <= HE_STANDARD_128.get(log_n, 0)}
