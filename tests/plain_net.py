"""fp64 plaintext tensor operations: what the encrypted layers must agree with (<= 1e-3)."""
import numpy as np


def conv2d(x, w, stride=1, pad_same=False):
    """x[B][C][H][W], w[FH][FW][IC][OC]; cross-correlation (no kernel flip)."""
    b, c, h, wd = x.shape
    fh, fw, ic, oc = w.shape
    assert ic == c
    if pad_same:
        ph, pw = fh // 2, fw // 2
        xp = np.zeros((b, c, h + 2 * ph, wd + 2 * pw))
        xp[:, :, ph:ph + h, pw:pw + wd] = x
        oh, ow = -(-h // stride), -(-wd // stride)
    else:
        xp = x
        oh, ow = (h - fh) // stride + 1, (wd - fw) // stride + 1
    out = np.zeros((b, oc, oh, ow))
    for y in range(oh):
        for xx in range(ow):
            patch = xp[:, :, y * stride:y * stride + fh, xx * stride:xx * stride + fw]   # [B][C][FH][FW]
            out[:, :, y, xx] = np.einsum("bcij,ijco->bo", patch, w)
    return out


def fc(x, w):
    """x[B][C][H][W], w[OUT][C][H][W] -> [B][OUT][1][1]."""
    return np.einsum("bchw,ochw->bo", x, w.reshape((w.shape[0],) + x.shape[1:]))[:, :, None, None]


def sum_pool2x2(x):
    h, w = x.shape[2] // 2 * 2, x.shape[3] // 2 * 2
    x = x[:, :, :h, :w]
    return x[:, :, 0::2, 0::2] + x[:, :, 0::2, 1::2] + x[:, :, 1::2, 0::2] + x[:, :, 1::2, 1::2]


def poly2_act_without_a(x, a, b):
    """x^2 + (b/a) x: the encrypted activation leaves the factor a to the next layer."""
    return x * x + (b / a) * x
