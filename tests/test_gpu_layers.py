"""GPU parity of the HW-tiled tensor layers (C ABI) against the oracle's layers and fp64 tensor arithmetic.

Bit-exact: the *_fixed entry points, fed the integers the oracle derived (weights in fixed point, plaintext
coefficients).  Within 1e-3: the float entry points (which encode on the GPU in fp64) against the fp64 layer.
"""
import numpy as np
import pytest

import plain_net

pytestmark = pytest.mark.gpu


def make_pair(log_n, q_bits, dnum, sb, seed):
    from oracle import Oracle
    from paper_1810_00845_amd import hisa
    return hisa.Context(log_n, q_bits, dnum, sb, seed), Oracle(log_n, q_bits, dnum, sb, seed)


def both_tensors(g, o, x, scale, limbs, **layout):
    """The same encrypted tensor on both sides: the oracle encodes, the GPU imports the same coefficients."""
    from oracle import layers
    from paper_1810_00845_amd import hisa
    b, c, h, w = x.shape
    hs = layout.get("h_stride") or w * layout.get("w_stride", 1)
    ws, off = layout.get("w_stride", 1), layout.get("offset", 0)
    g.set_enc_counter(500); o.enc_counter = 500
    ocs, gcs = [], []
    for bi in range(b):
        for ci in range(c):
            z = np.zeros(o.slots)
            z[layers.plane_slots(h, w, hs, ws, off)] = x[bi, ci].reshape(-1)
            co = o.encode_coeffs(z, scale)
            ocs.append(o.encrypt(o.pt_from_coeffs(co, scale, limbs)))
            gcs.append(g.encrypt(g.pt_from_coeffs(co, scale, limbs)))
    ot = layers.OTensor(ocs, b, c, h, w, hs, ws, off, 1)
    gt = hisa.CipherTensor(g, gcs, b, c, h, w, hs, ws, off, 1)
    return gt, ot


def same_tensor(g, o, gt, ot):
    assert gt.meta() == (ot.batch, ot.channels, ot.height, ot.width, ot.h_stride, ot.w_stride, ot.offset, ot.clean)
    for gc, oc in zip(gt.cts, ot.cts):
        assert np.array_equal(g.ct_export(gc), o.export(oc))
        assert abs(gc.scale - oc.scale) <= 1e-12 * oc.scale


def test_config1_conv_bit_exact_and_accurate():
    """BASELINE config 1: 3x3 conv, 1 -> 1 channel, 8x8 image row-major in the slots, N = 2^12, three 30-bit
    primes + one 60-bit special prime, scale 2^25."""
    from oracle import layers
    from paper_1810_00845_amd import synth
    g, o = make_pair(12, [30, 30, 30], 3, 60, 1)
    x = synth.image(1, 1, 8, 8)[None]
    w = synth.conv_weights(2, 3, 3, 1, 1)
    gt, ot = both_tensors(g, o, x, 2.0 ** 25, 3)
    steps = g.conv2d_rot_steps(gt, 3, 3)
    assert steps == layers.rot_steps_conv(o, ot, 3, 3) and len(steps) == 8
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    want = plain_net.conv2d(x, w)
    for mode in (layers.CONV_PLAIN, layers.CONV_SCALAR):
        oout, ints = layers.conv2d(o, ot, w, mode=mode)
        gout = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], ints["pt_coeffs"], ints["pt_scale"], 1, 3, 3, mode=mode)
        same_tensor(g, o, gout, oout)
        assert np.abs(g.tensor_decrypt(gout) - want).max() <= 1e-3
        gfloat = g.conv2d(gt, w, 3, 3, mode=mode)      # encodes on the GPU
        assert gfloat.meta() == gout.meta()
        assert np.abs(g.tensor_decrypt(gfloat) - want).max() <= 1e-3
    # tensor_encrypt / tensor_decrypt round trip on the GPU alone
    gt2 = g.tensor_encrypt(x, 2.0 ** 25, 3)
    assert np.abs(g.tensor_decrypt(gt2) - x).max() <= 1e-4
    g.close()


def test_multichannel_same_strided_masked_conv():
    from oracle import layers
    from paper_1810_00845_amd import synth
    g, o = make_pair(11, [45, 45, 45], 3, 50, 3)
    x = synth.image(3, 2, 6, 6)[None].repeat(2, axis=0) * np.array([1.0, 0.5])[:, None, None, None]  # batch of 2
    w = synth.conv_weights(4, 3, 3, 2, 5)                 # 5 output channels: ragged last block of the MAC kernel
    gt, ot = both_tensors(g, o, x, 2.0 ** 40, 3, h_stride=8, offset=9)
    steps = sorted(set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True)) | set(g.conv2d_rot_steps(gt, 3, 3)))
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    oout, ints = layers.conv2d(o, ot, w, pad_same=True, mode=layers.CONV_MASKED)
    gout = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], ints["pt_coeffs"], ints["pt_scale"], 5, 3, 3, pad_same=True,
                          mode=layers.CONV_MASKED)
    same_tensor(g, o, gout, oout)
    want = plain_net.conv2d(x, w, pad_same=True)
    assert np.abs(g.tensor_decrypt(gout) - want).max() <= 1e-3
    assert np.abs(g.tensor_decrypt(g.conv2d(gt, w, 3, 3, pad_same=True, mode=layers.CONV_MASKED)) - want).max() <= 1e-3
    # VALID stride 2, literal Algorithm 1
    oout, ints = layers.conv2d(o, ot, w, stride=2, mode=layers.CONV_SCALAR)
    gout = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], None, 1.0, 5, 3, 3, stride=2, mode=layers.CONV_SCALAR)
    same_tensor(g, o, gout, oout)
    assert np.abs(g.tensor_decrypt(gout) - plain_net.conv2d(x, w, stride=2)).max() <= 1e-3
    g.close()


def test_long_contraction_conv_bit_exact():
    """A convolution whose sum over (tap, input channel) is long enough for the matrix-core multiply-accumulate
    (36 and 72 terms, ragged against its 64-wide tiles; 5 and 3 outputs against its 64-output blocks), compared bit
    for bit with the oracle, unmasked and masked, at two levels."""
    from oracle import layers
    from paper_1810_00845_amd import synth
    g, o = make_pair(11, [50, 45, 45, 45], 2, 50, 8)
    x = synth.image(5, 4, 6, 6)[None]
    gt, ot = both_tensors(g, o, x, 2.0 ** 40, 4, h_stride=8, offset=9)
    steps = sorted(set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True)) | set(g.conv2d_rot_steps(gt, 3, 3)))
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    w = synth.conv_weights(6, 3, 3, 4, 5)                       # K = 36
    oout, ints = layers.conv2d(o, ot, w, mode=layers.CONV_SCALAR)
    gout = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], None, 1.0, 5, 3, 3, mode=layers.CONV_SCALAR)
    same_tensor(g, o, gout, oout)
    assert np.abs(g.tensor_decrypt(gout) - plain_net.conv2d(x, w)).max() <= 1e-3
    plan = g.conv2d_prepare(gt, w, 3, 3)                        # weights converted ahead of time: the same bits
    ga, gb = g.conv2d(gt, w, 3, 3), g.conv2d_apply(gt, plan)
    for ca, cb in zip(ga.cts, gb.cts):
        assert np.array_equal(g.ct_export(ca), g.ct_export(cb)) and ca.scale == cb.scale
    assert ga.meta() == gb.meta()
    g.conv_plan_free(plan)
    w2 = synth.conv_weights(7, 3, 3, 4, 8)                      # masked SAME convolution, 8 outputs
    omid, ints = layers.conv2d(o, ot, w2, pad_same=True, mode=layers.CONV_MASKED)
    gmid = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], ints["pt_coeffs"], ints["pt_scale"], 8, 3, 3, pad_same=True,
                          mode=layers.CONV_MASKED)
    same_tensor(g, o, gmid, omid)
    w3 = synth.conv_weights(8, 3, 3, 8, 3)                      # K = 72 on the masked result, one level down
    o3, ints = layers.conv2d(o, omid, w3, pad_same=True, mode=layers.CONV_MASKED)
    g3 = g.conv2d_fixed(gmid, ints["w_int"], ints["w_scale"], ints["pt_coeffs"], ints["pt_scale"], 3, 3, 3, pad_same=True,
                        mode=layers.CONV_MASKED)
    same_tensor(g, o, g3, o3)
    want = plain_net.conv2d(plain_net.conv2d(x, w2, pad_same=True), w3, pad_same=True)
    assert np.abs(g.tensor_decrypt(g3) - want).max() <= 1e-3
    g.close()


def test_activation_pool_fc_chain_bit_exact():
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(11, [50, 45, 45, 45, 45], 5, 55, 4)
    g.keygen(); o.keygen()
    x = synth.image(6, 2, 4, 4)[None]
    gt, ot = both_tensors(g, o, x, 2.0 ** 45, 5)
    steps = sorted(set(g.pool_rot_steps(gt)) | {1, 2, 4, 8})
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    gact, oact = g.poly2_act(gt, 0.3, 0.2), layers.poly2_act(o, ot, 0.3, 0.2)
    same_tensor(g, o, gact, oact)
    gpool, opool = g.sum_pool2x2(gact), layers.sum_pool2x2(o, oact)
    same_tensor(g, o, gpool, opool)
    ref = plain_net.sum_pool2x2(plain_net.poly2_act_without_a(x, 0.3, 0.2))
    assert np.abs(g.tensor_decrypt(gpool) - ref).max() <= 1e-3
    w1 = synth.fc_weights(7, 3, 2, 2, 2, std=0.3)
    assert g.fc_rot_steps(gpool) == [2, 8] == layers.fc_reduce_steps(o, opool)
    of1, ints = layers.fc(o, opool, w1)
    gf1 = g.fc_fixed(gpool, ints["pt_coeffs"], ints["pt_scale"])
    same_tensor(g, o, gf1, of1)
    ref1 = plain_net.fc(ref, w1)
    assert np.abs(g.tensor_decrypt(gf1) - ref1).max() <= 1e-3
    assert np.abs(g.tensor_decrypt(g.fc(gpool, w1)) - ref1).max() <= 1e-3
    # weights encoded ahead of time: bit for bit the result of the call that encodes them itself
    plan = g.fc_prepare(gpool, w1)
    gplain, gplan = g.fc(gpool, w1), g.fc_apply(gpool, plan)
    for a, b in zip(gplain.cts, gplan.cts):
        assert np.array_equal(g.ct_export(a), g.ct_export(b)) and a.scale == b.scale
    assert gplan.meta() == gplain.meta()
    with pytest.raises(hisa.HisaError) as e:
        g.fc_apply(gact, plan)                            # another layout
    assert e.value.code == -1
    g.fc_plan_free(plan)
    w2 = synth.fc_weights(8, 2, 3, 1, 1, std=0.5)
    of2, _ = layers.fc(o, of1, w2)
    gf2 = g.fc(gf1, w2)                                   # 1x1 planes: scalar weights, no encodes, bit-exact as is
    same_tensor(g, o, gf2, of2)
    assert np.abs(g.tensor_decrypt(gf2) - plain_net.fc(ref1, w2)).max() <= 1e-3
    # square activation (b = 0)
    same_tensor(g, o, g.poly2_act(gt, 1.0, 0.0), layers.poly2_act(o, ot, 1.0, 0.0))
    g.close()


def test_layer_error_paths():
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(11, [45, 45], 2, 50, 5)
    x = synth.image(1, 1, 4, 4)[None]
    gt = g.tensor_encrypt(x, 2.0 ** 40, 2)
    w = synth.conv_weights(2, 3, 3, 1, 1)
    with pytest.raises(hisa.HisaError) as e:
        g.conv2d(gt, w, 3, 3)                             # rotation keys were never generated
    assert e.value.code == -4
    g.gen_rot_keys(g.conv2d_rot_steps(gt, 3, 3))
    out = g.conv2d(gt, w, 3, 3)
    with pytest.raises(hisa.HisaError) as e:
        g.conv2d(out, w[:2, :2], 2, 2)                    # one limb left: nothing to rescale into
    assert e.value.code == -6
    with pytest.raises(hisa.HisaError) as e:
        g.conv2d(out, w, 3, 3, pad_same=True)             # SAME needs a clean input; SCALAR output is not
    assert e.value.code == -1
    g.close()
