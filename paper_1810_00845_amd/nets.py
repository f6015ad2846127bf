"""Encrypted inference schedules for the LeNet-shaped benchmark networks: sequences of calls into the tensor
layer of libhisa (conv2d, poly2_act, sum_pool2x2, fc), nothing else.

A network is a list of layer tuples.  The factors the encrypted layers leave to their successor (the `a` of an
activation a x^2 + b x, the 1/4 of an average pool; Sec. "Runtime" of the paper folds such constants into the next
linear layer) are multiplied into the next layer's weights here, on the host, before the call.

    ("conv", w[FH][FW][IC][OC], stride)      VALID convolution, Algorithm 1 with scalar weights
    ("act", a, b)                            a x^2 + b x
    ("pool",)                                2x2 average pool
    ("fc", w[OUT][C][H][W])                  fully connected over the whole tensor
"""
import time

import numpy as np

from . import synth


def lenet_small(seed=3):
    """BASELINE config 3: N = 2^13, 8 limbs, one 28x28 image (zero border of one pixel: 30x30 encrypted, so that
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
    """BASELINE config 4: N = 2^14, 12 limbs, conv5x5 1->20, pool, conv5x5 20->50, pool, FC 800->500, FC 500->10,
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


def run_encrypted(ctx, layers, x, scale, limbs, make_keys=False):
    """Encrypts x, runs the layers, decrypts.  Returns (output array, seconds from encrypt-done to the last
    ciphertext ready, per-layer seconds).  With make_keys the rotation keys each layer asks for are generated
    on the way (set-up pass); otherwise they must be resident."""
    t = ctx.tensor_encrypt(x, scale, limbs)
    ctx.sync()
    t_start = time.perf_counter()
    per_layer = []
    pending = 1.0     # constant factor the previous layers left to the next linear layer
    for layer in layers:
        t0 = time.perf_counter()
        kind = layer[0]
        if kind == "conv":
            w, stride = layer[1] * pending, layer[2]
            pending = 1.0
            fh, fw = w.shape[:2]
            if make_keys:
                ctx.gen_rot_keys(ctx.conv2d_rot_steps(t, fh, fw, stride=stride))
            nxt = ctx.conv2d(t, w, fh, fw, stride=stride)
        elif kind == "act":
            a, b = layer[1], layer[2]
            nxt = ctx.poly2_act(t, a, b)
            pending *= a
        elif kind == "pool":
            if make_keys:
                ctx.gen_rot_keys(ctx.pool_rot_steps(t))
            nxt = ctx.sum_pool2x2(t)
            pending *= 0.25
        elif kind == "fc":
            w = layer[1] * pending
            pending = 1.0
            if make_keys and t.height * t.width > 1:
                ctx.gen_rot_keys(ctx.fc_rot_steps(t))
            nxt = ctx.fc(t, w)
        else:
            raise ValueError(kind)
        t.free()
        t = nxt
        ctx.sync()
        per_layer.append((kind, time.perf_counter() - t0))
    latency = time.perf_counter() - t_start
    out = ctx.tensor_decrypt(t) * pending
    t.free()
    return out, latency, per_layer
