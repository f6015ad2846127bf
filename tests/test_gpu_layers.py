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
    assert gt.meta() == (ot.batch, ot.channels, ot.height, ot.width, ot.h_stride, ot.w_stride, ot.offset, ot.clean,
                         ot.c_inner, ot.c_stride if ot.c_inner > 1 else gt.c_stride)
    assert len(gt.cts) == len(ot.cts)
    for gc, oc in zip(gt.cts, ot.cts):
        assert np.array_equal(g.ct_export(gc), o.export(oc))
        assert abs(gc.scale - oc.scale) <= 1e-12 * oc.scale


def test_config1_conv_bit_exact_and_accurate():
    """Benchmark configuration 1: 3x3 conv, 1 -> 1 channel, 8x8 image row-major in the slots, N = 2^12, three 30-bit
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


def test_matmul_with_replicas_bit_exact():
    """Homomorphic matmul with replicas through the C ABI against the oracle, bit for bit: a batch of two images, a
    pooled (not clean) HW-tiled input that needs the masking multiply, 10 outputs in ragged groups of 4, then the
    activation and a second matmul on the CHW-tiled result; the plan and the float entry point besides."""
    from oracle import layers
    from paper_1810_00845_amd import synth
    g, o = make_pair(11, [50, 45, 45, 45, 45, 45], 3, 55, 12)
    g.keygen(); o.keygen()
    x = synth.image(21, 3, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.5])[:, None, None, None]
    gt, ot = both_tensors(g, o, x, 2.0 ** 45, 6)
    g.gen_rot_keys([1, 4, 5]); o.gen_rot_keys([1, 4, 5])
    gp, op = g.sum_pool2x2(gt), layers.sum_pool2x2(o, ot)
    same_tensor(g, o, gp, op)
    ref = plain_net.sum_pool2x2(x)
    assert g.matmul_geometry(gp, 10, 4) == (16, 4, 2 * 3) and layers.matmul_geometry(o, op, 4)[:2] == (16, 4)
    steps = g.matmul_rot_steps(gp, 4)
    assert steps == sorted([2, 8, o.slots - 16, o.slots - 32])
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    w1 = synth.fc_weights(22, 10, 3, 2, 2, std=0.3)
    om, ints = layers.matmul(o, op, w1, 4)
    gm = g.matmul_fixed(gp, ints["pt_coeffs"], ints["pt_scale"], ints["mask_coeffs"], ints["mask_scale"], 10, 4)
    same_tensor(g, o, gm, om)
    ref1 = plain_net.fc(ref, w1)
    assert np.abs(g.tensor_decrypt(gm) - ref1).max() <= 1e-3
    gfloat = g.matmul(gp, w1, 4)                                # encodes weights and mask on the GPU
    assert gfloat.meta() == gm.meta()
    assert np.abs(g.tensor_decrypt(gfloat) - ref1).max() <= 1e-3
    plan = g.matmul_prepare(gp, w1, 4)
    gplan = g.matmul_apply(gp, plan)
    for ca, cb in zip(gfloat.cts, gplan.cts):
        assert np.array_equal(g.ct_export(ca), g.ct_export(cb)) and ca.scale == cb.scale
    g.matmul_plan_free(plan)
    # without replicas: the FC layer, bit for bit
    g0, gf = g.matmul(gp, w1, 1), g.fc(gp, w1)
    assert g0.c_inner == 1 and len(g0.cts) == 20
    for ca, cb in zip(g0.cts, gf.cts):
        assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
    # activation on the CHW-tiled tensor, then a matmul that reads it
    ga, oa = g.poly2_act(gm, 0.5, 0.25), layers.poly2_act(o, om, 0.5, 0.25)
    same_tensor(g, o, ga, oa)
    steps = g.matmul_rot_steps(ga, 2)
    assert steps == sorted([16, 32, o.slots - 64])
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    w2 = synth.fc_weights(23, 3, 10, 1, 1, std=0.4)
    o2, ints = layers.matmul(o, oa, w2, 2)
    g2 = g.matmul_fixed(ga, ints["pt_coeffs"], ints["pt_scale"], ints["mask_coeffs"], ints["mask_scale"], 3, 2)
    same_tensor(g, o, g2, o2)
    want = plain_net.fc(plain_net.poly2_act_without_a(ref1, 0.5, 0.25), w2)
    assert np.abs(g.tensor_decrypt(g2) - want).max() <= 1e-3
    assert np.abs(g.tensor_decrypt(g.matmul(ga, w2, 2)) - want).max() <= 1e-3
    g.close()


def test_merged_doublings_in_fc_and_matmul_bit_exact():
    """hisa_set_merge_doublings: the rotate-and-add chains of matmul (replicas and reduction) and FC as sums of
    rotations, against the oracle's merge_doublings schedule bit for bit (fp64 key-switch path, N = 2^12), the extra
    rotation amounts, the dry run's counts, and the refusals."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(12, [50, 45, 45, 45, 45], 2, 50, 21)
    g.keygen(); o.keygen()
    x = synth.image(25, 3, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.5])[:, None, None, None]
    gt, ot = both_tensors(g, o, x, 2.0 ** 45, 5)
    w = synth.fc_weights(26, 6, 3, 4, 4, std=0.3)
    ref = plain_net.fc(x, w)
    plain_steps = g.matmul_rot_steps(gt, 4)
    for merge in (4, 2):
        g.set_merge_doublings(merge)
        block, r, replicate, reduce = layers.matmul_geometry(o, ot, 4)
        want_steps = sorted({a for grp in layers.merge_doublings(reduce, merge) for a in grp} |
                            {o.slots - a for grp in layers.merge_doublings(replicate, merge) for a in grp})
        steps = g.matmul_rot_steps(gt, 4)
        assert steps == want_steps and set(plain_steps) <= set(steps) and len(steps) > len(plain_steps)
        assert g.fc_rot_steps(gt) == sorted({a for grp in layers.merge_doublings(layers.fc_reduce_steps(o, ot), merge) for a in grp})
        g.gen_rot_keys(steps); o.gen_rot_keys(steps)
        om, ints = layers.matmul(o, ot, w, 4, merge=merge)
        gm = g.matmul_fixed(gt, ints["pt_coeffs"], ints["pt_scale"], ints["mask_coeffs"], ints["mask_scale"], 6, 4)
        same_tensor(g, o, gm, om)
        assert np.abs(g.tensor_decrypt(gm) - ref).max() <= 1e-3
        plan = g.matmul_prepare(gt, w, 4)
        gplan, gfloat = g.matmul_apply(gt, plan), g.matmul(gt, w, 4)
        for ca, cb in zip(gfloat.cts, gplan.cts):
            assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
        assert np.abs(g.tensor_decrypt(gfloat) - ref).max() <= 1e-3
        g.matmul_plan_free(plan)
        of, fints = layers.fc(o, ot, w, merge=merge)
        gf = g.fc_fixed(gt, fints["pt_coeffs"], fints["pt_scale"])
        same_tensor(g, o, gf, of)
        assert np.abs(g.tensor_decrypt(gf) - ref).max() <= 1e-3
    # the 2x2 pool as one sum over its four corners
    g.gen_rot_keys(g.pool_rot_steps(gt)); o.gen_rot_keys(g.pool_rot_steps(gt))
    gp, op = g.sum_pool2x2(gt), layers.sum_pool2x2(o, ot, merge=2)
    same_tensor(g, o, gp, op)
    assert np.abs(g.tensor_decrypt(gp) - plain_net.sum_pool2x2(x)).max() <= 1e-3
    # dry run with merge = 2: per image 3 inputs x (one sum of 3 rotations), 2 groups x (sums of 3 + 3 rotations)
    g.analysis_begin()
    g.matmul(gt, w, 4)
    counts, dry_steps = g.analysis_end()
    assert counts["rot_summed"] == 2 * (3 * 3 + 2 * 6) and counts["rot_shared"] == 2 * (3 * 2 + 2 * 4)
    assert dry_steps == g.matmul_rot_steps(gt, 4)
    g.set_merge_doublings(0)
    assert g.matmul_rot_steps(gt, 4) == plain_steps
    with pytest.raises(hisa.HisaError) as e:
        g.set_merge_doublings(5)
    assert e.value.code == -1
    g.close()
    g2, _ = make_pair(11, [50, 45, 45], 3, 55, 12)          # no fused key switch
    with pytest.raises(hisa.HisaError) as e:
        g2.set_merge_doublings(4)
    assert e.value.code == -1
    g2.close()


def test_chw_tensor_layers_and_errors():
    """CHW-tiled tensors through encrypt / decrypt / pool / activation / matmul (clean input: no mask, one level),
    a last ciphertext with fewer channels, and the error paths: conv2d and fc refuse CHW tiling, overlapping
    elements and a missing level are reported."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(10, [50, 40, 40], 3, 55, 13)
    x = synth.image(31, 5, 4, 4)[None]
    gt = g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=4, c_inner=2, c_stride=16)
    assert len(gt.cts) == 3 and gt.clean == 1 and (gt.c_inner, gt.c_stride) == (2, 16)
    assert np.abs(g.tensor_decrypt(gt) - x).max() <= 1e-6
    # the same tensor on both sides, from the oracle's encodings
    ot = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 3, 2, 16, h_stride=4)
    gcs = []
    g.set_enc_counter(700); o.enc_counter = 700
    sl = np.asarray(layers.tensor_slots(ot)).reshape(2, 16)
    ocs = []
    for j in range(3):
        z = np.zeros(o.slots)
        for cl in range(min(2, 5 - 2 * j)):
            z[sl[cl]] = x[0, 2 * j + cl].reshape(-1)
        co = o.encode_coeffs(z, 2.0 ** 40)
        ocs.append(o.encrypt(o.pt_from_coeffs(co, 2.0 ** 40, 3)))
        gcs.append(g.encrypt(g.pt_from_coeffs(co, 2.0 ** 40, 3)))
    ot.cts = ocs
    gt2 = hisa.CipherTensor(g, gcs, 1, 5, 4, 4, 4, 1, 0, 1, 2, 16)
    same_tensor(g, o, gt2, ot)
    steps = sorted(set(g.pool_rot_steps(gt2)) | set(g.matmul_rot_steps(gt2, 1 << 20)))
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    w = synth.fc_weights(32, 4, 5, 4, 4, std=0.3)
    om, ints = layers.matmul(o, ot, w, 1 << 20)
    assert ints["mask_coeffs"] is None
    gm = g.matmul_fixed(gt2, ints["pt_coeffs"], ints["pt_scale"], None, 1.0, 4, 1 << 20)
    same_tensor(g, o, gm, om)
    assert gm.cts[0].limbs == 2 and np.abs(g.tensor_decrypt(gm) - plain_net.fc(x, w)).max() <= 1e-3
    gp, op = g.sum_pool2x2(gt2), layers.sum_pool2x2(o, ot)
    same_tensor(g, o, gp, op)
    assert np.abs(g.tensor_decrypt(gp) - plain_net.sum_pool2x2(x)).max() <= 1e-3
    # errors
    with pytest.raises(hisa.HisaError):
        g.conv2d(gt2, synth.conv_weights(1, 3, 3, 5, 2), 3, 3)
    with pytest.raises(hisa.HisaError):
        g.fc(gt2, w)
    with pytest.raises(hisa.HisaError):                          # channels 8 slots apart overlap 4x4 planes
        g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=4, c_inner=2, c_stride=8)
    with pytest.raises(hisa.HisaError):                          # one level left, the masked form needs two
        g.rescale_batch(gp.cts)
        g.matmul(gp, w[:, :, :2, :2], 2)
    g.close()


def chw_pair(g, o, x, scale, limbs, c_inner, c_stride, counter, **layout):
    """The same CHW-tiled encrypted tensor on both sides, from the oracle's encodings."""
    from oracle import layers
    from paper_1810_00845_amd import hisa
    b, c, h, w = x.shape
    ot = layers.tensor_encrypt_chw(o, x, scale, limbs, c_inner, c_stride, **layout)
    sl = np.asarray(layers.tensor_slots(ot)).reshape(c_inner, h * w)
    per = layers.cts_per_image(ot)
    g.set_enc_counter(counter); o.enc_counter = counter
    ocs, gcs = [], []
    for bi in range(b):
        for j in range(per):
            z = np.zeros(o.slots)
            for cl in range(min(c_inner, c - j * c_inner)):
                z[sl[cl]] = x[bi, j * c_inner + cl].reshape(-1)
            co = o.encode_coeffs(z, scale)
            ocs.append(o.encrypt(o.pt_from_coeffs(co, scale, limbs)))
            gcs.append(g.encrypt(g.pt_from_coeffs(co, scale, limbs)))
    ot.cts = ocs
    gt = hisa.CipherTensor(g, gcs, b, c, h, w, ot.h_stride, ot.w_stride, ot.offset, 1, c_inner, c_stride)
    return gt, ot


@pytest.mark.parametrize("log_n,c_stride", [(10, 128), (10, 64), (12, 64), (12, 512)])
def test_chw_conv_bit_exact(log_n, c_stride):
    """CHW-tiled convolution through the C ABI against the oracle, bit for bit: batch of two, 5 -> 6 channels in
    blocks of 4 (ragged last ciphertexts), SAME and VALID, stride 1 and 2; blocks filling the slots (4 x 128 = 512 slots
    at N = 2^10, 4 x 512 at N = 2^12: cyclic for free) and with the copy behind them; both arithmetic paths (N = 2^12:
    fp64); plan and float entry point."""
    from oracle import layers
    from paper_1810_00845_amd import synth
    g, o = make_pair(log_n, [50, 40, 40], 3, 50, 14)
    x = synth.image(41, 5, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.7])[:, None, None, None]
    w = synth.conv_weights(42, 3, 3, 5, 6)
    gt, ot = chw_pair(g, o, x, 2.0 ** 40, 3, 4, c_stride, 900, h_stride=6, offset=7)
    same_tensor(g, o, gt, ot)
    assert (layers.chw_conv_geometry(o, ot, 3, 3)[0] == 0) == (4 * c_stride == o.slots)
    steps = sorted(set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True)) | set(g.conv2d_rot_steps(gt, 3, 3)))
    assert steps == sorted(set(layers.rot_steps_conv_chw(o, ot, 3, 3, True)) | set(layers.rot_steps_conv_chw(o, ot, 3, 3)))
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    for kw, ref in ((dict(pad_same=True), plain_net.conv2d(x, w, pad_same=True)), (dict(), plain_net.conv2d(x, w)),
                    (dict(stride=2, pad_same=True), plain_net.conv2d(x, w, stride=2, pad_same=True))):
        oout, ints = layers.conv2d_chw(o, ot, w, **kw)
        gout = g.conv2d_fixed(gt, None, 1.0, ints["pt_coeffs"], ints["pt_scale"], 6, 3, 3, mode=layers.CONV_PLAIN, **kw)
        same_tensor(g, o, gout, oout)
        assert np.abs(g.tensor_decrypt(gout) - ref).max() <= 1e-3
        gfloat = g.conv2d(gt, w, 3, 3, mode=layers.CONV_PLAIN, **kw)
        assert gfloat.meta() == gout.meta() and np.abs(g.tensor_decrypt(gfloat) - ref).max() <= 1e-3
        plan = g.conv2d_prepare(gt, w, 3, 3, mode=layers.CONV_PLAIN, **kw)
        gplan = g.conv2d_apply(gt, plan)
        for ca, cb in zip(gfloat.cts, gplan.cts):
            assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
        g.conv_plan_free(plan)
    from paper_1810_00845_amd import hisa
    with pytest.raises(hisa.HisaError):                    # scalar weights cannot tell the channels of a ciphertext apart
        g.conv2d(gt, w, 3, 3, mode=layers.CONV_SCALAR)
    g.close()


@pytest.mark.parametrize("q_bits", [[47, 40, 40, 40], [50, 40, 40, 40], [45, 49, 49, 49], [50, 49, 49, 49]])
def test_plan_plaintexts_in_six_bytes_give_the_same_bits(q_bits):
    """A plan keeps its plaintexts with six bytes per residue on the limbs whose primes are below 2^48 (all of them,
    all but the first, the first only, none): its outputs equal those of the direct call, which multiplies by the
    encoder's eight-byte words, bit for bit -- HW-tiled plaintext weights and the three CHW schedules, at the top level
    and one below (a plan is made for its level) -- and both are within 1e-3 of the plaintext convolution."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g = hisa.Context(12, q_bits, 2, 50, 23)
    g.keygen()
    x = synth.image(43, 9, 4, 4)[None]
    w = synth.conv_weights(44, 3, 3, 9, 10)                  # 10 outputs: groups of eight and a ragged group
    ref = plain_net.conv2d(x, w, pad_same=True)
    hw = g.tensor_encrypt(x, 2.0 ** 40, 4, h_stride=6, offset=7)
    chw = g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=6, offset=7, c_inner=4, c_stride=512)
    steps = set(g.conv2d_rot_steps(hw, 3, 3, pad_same=True))
    for sched in (hisa.CHW_ROTATE_INPUTS, hisa.CHW_ROTATE_SUMS, hisa.CHW_ROTATE_SUMS_TAPS):
        steps |= set(g.conv2d_rot_steps(chw, 3, 3, pad_same=True, chw_schedule=sched))
    g.gen_rot_keys(sorted(steps))
    for t, kws in ((hw, [dict()]), (chw, [dict(chw_schedule=s) for s in (0, 1, 2)])):
        for kw in kws:
            direct = g.conv2d(t, w, 3, 3, pad_same=True, mode=layers.CONV_PLAIN, **kw)
            plan = g.conv2d_prepare(t, w, 3, 3, pad_same=True, mode=layers.CONV_PLAIN, **kw)
            for _ in range(2):                                # a plan is applied many times
                planned = g.conv2d_apply(t, plan)
                assert planned.meta() == direct.meta()
                for ca, cb in zip(direct.cts, planned.cts):
                    assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
            assert np.abs(g.tensor_decrypt(planned) - ref).max() <= 1e-3
            g.conv_plan_free(plan)
    g.close()


@pytest.mark.parametrize("c_stride", [64, 512])
def test_plans_applied_together_share_input_rotations(c_stride):
    """Several plans applied to one tensor in one call: every output equals the plan applied alone bit for bit (and so
    the oracle's convolution), the rotations of the inputs that two plans ask for are made once (one inner-product
    launch over the union of the amounts instead of one per plan), an error leaves nothing behind.  A 1x1 convolution
    rotating its inputs by the channel diagonals, a 3x3 one rotating inputs by the diagonals and sums by the taps and a
    3x3 one rotating the inputs by the taps and the sums by the diagonals; blocks filling the slots and with their copy
    behind them."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g = hisa.Context(12, [50, 40, 40], 3, 50, 29)
    g.keygen()
    x = synth.image(45, 7, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.6])[:, None, None, None]
    t = g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=6, offset=7, c_inner=4, c_stride=c_stride)
    w1, w3, w3b = synth.conv_weights(46, 1, 1, 7, 5), synth.conv_weights(47, 3, 3, 7, 6), synth.conv_weights(48, 3, 3, 7, 3)
    specs = [(w1, 1, dict(chw_schedule=hisa.CHW_ROTATE_INPUTS)),
             (w3, 3, dict(chw_schedule=hisa.CHW_ROTATE_SUMS_TAPS, pad_same=True)),
             (w3b, 3, dict(chw_schedule=hisa.CHW_ROTATE_SUMS, pad_same=True))]
    steps = set()
    for w, f, kw in specs:
        steps |= set(g.conv2d_rot_steps(t, f, f, **kw))
    g.gen_rot_keys(sorted(steps))
    plans = [g.conv2d_prepare(t, w, f, f, mode=layers.CONV_PLAIN, **kw) for w, f, kw in specs]
    g.profile_enable(True)
    alone = [g.conv2d_apply(t, p) for p in plans]
    g.sync()
    launches_alone = sum(c for k, (c, _) in g.profile_read().items() if k.startswith("inner_product_steps"))
    g.profile_enable(False); g.profile_enable(True)
    together = g.conv2d_apply_multi(t, plans)
    g.sync()
    launches_together = sum(c for k, (c, _) in g.profile_read().items() if k.startswith("inner_product_steps"))
    g.profile_enable(False)
    assert launches_together < launches_alone
    for (w, f, kw), a, b in zip(specs, alone, together):
        assert a.meta() == b.meta()
        for ca, cb in zip(a.cts, b.cts):
            assert np.array_equal(g.ct_export(ca), g.ct_export(cb)) and ca.scale == cb.scale
        ref = plain_net.conv2d(x, w, pad_same=kw.get("pad_same", False))
        assert np.abs(g.tensor_decrypt(b) - ref).max() <= 1e-3
    one = g.conv2d_apply_multi(t, plans[:1])                     # a single plan: the plain call
    for ca, cb in zip(alone[0].cts, one[0].cts):
        assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
    lower = g.tensor_encrypt(x, 2.0 ** 40, 2, h_stride=6, offset=7, c_inner=4, c_stride=c_stride)
    with pytest.raises(hisa.HisaError):                           # a plan of another level among them
        g.conv2d_apply_multi(lower, plans)
    for p in plans:
        g.conv_plan_free(p)
    g.close()


@pytest.mark.parametrize("c_stride", [64, 512])
def test_chw_conv_rotating_the_sums_bit_exact(c_stride):
    """The CHW-tiled convolution that reduces over the channel blocks after the multiplication, against the oracle
    bit for bit: batch of two, 5 -> 6 channels in blocks of 4 (ragged last ciphertexts), SAME and VALID, stride 1 and
    2; blocks with their copy behind them (4 x 64 slots) and filling the slot vector (4 x 512 at N = 2^12); fixed-point,
    float and plan entry points; the rotation amounts; the dry run's counts; what it refuses."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(12, [50, 40, 40], 3, 50, 14)
    x = synth.image(41, 5, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.7])[:, None, None, None]
    w = synth.conv_weights(42, 3, 3, 5, 6)
    gt, ot = chw_pair(g, o, x, 2.0 ** 40, 3, 4, c_stride, 900, h_stride=6, offset=7)
    S = hisa.CHW_ROTATE_SUMS
    steps = sorted(set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True, chw_schedule=S)) | set(g.conv2d_rot_steps(gt, 3, 3, chw_schedule=S)))
    assert steps == sorted(set(layers.rot_steps_conv_chw(o, ot, 3, 3, True, schedule="out")) |
                           set(layers.rot_steps_conv_chw(o, ot, 3, 3, schedule="out")))
    assert len(steps) < len(g.conv2d_rot_steps(gt, 3, 3, pad_same=True))
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    for kw, ref in ((dict(pad_same=True), plain_net.conv2d(x, w, pad_same=True)), (dict(), plain_net.conv2d(x, w)),
                    (dict(stride=2, pad_same=True), plain_net.conv2d(x, w, stride=2, pad_same=True))):
        oout, ints = layers.conv2d_chw(o, ot, w, schedule="out", **kw)
        gout = g.conv2d_fixed(gt, None, 1.0, ints["pt_coeffs"], ints["pt_scale"], 6, 3, 3, mode=layers.CONV_PLAIN,
                              chw_schedule=S, **kw)
        same_tensor(g, o, gout, oout)
        assert gout.clean == 1 and np.abs(g.tensor_decrypt(gout) - ref).max() <= 1e-3
        gfloat = g.conv2d(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=S, **kw)
        assert gfloat.meta() == gout.meta() and np.abs(g.tensor_decrypt(gfloat) - ref).max() <= 1e-3
        plan = g.conv2d_prepare(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=S, **kw)
        gplan = g.conv2d_apply(gt, plan)
        for ca, cb in zip(gfloat.cts, gplan.cts):
            assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
        g.conv_plan_free(plan)
    # the other split: diagonals on the inputs, taps on the sums (bordered layout, VALID and SAME, stride 2)
    T = hisa.CHW_ROTATE_SUMS_TAPS
    assert set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True, chw_schedule=T)) == set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True, chw_schedule=S))
    for kw, ref in ((dict(pad_same=True), plain_net.conv2d(x, w, pad_same=True)), (dict(), plain_net.conv2d(x, w)),
                    (dict(stride=2, pad_same=True), plain_net.conv2d(x, w, stride=2, pad_same=True))):
        oout, ints = layers.conv2d_chw(o, ot, w, schedule="taps", **kw)
        gout = g.conv2d_fixed(gt, None, 1.0, ints["pt_coeffs"], ints["pt_scale"], 6, 3, 3, mode=layers.CONV_PLAIN,
                              chw_schedule=T, **kw)
        same_tensor(g, o, gout, oout)
        assert gout.clean == 1 and np.abs(g.tensor_decrypt(gout) - ref).max() <= 1e-3
        gfloat = g.conv2d(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=T, **kw)
        assert gfloat.meta() == gout.meta() and np.abs(g.tensor_decrypt(gfloat) - ref).max() <= 1e-3
        plan = g.conv2d_prepare(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=T, **kw)
        gplan = g.conv2d_apply(gt, plan)
        for ca, cb in zip(gfloat.cts, gplan.cts):
            assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
        g.conv_plan_free(plan)
    g.analysis_begin()
    g.conv2d(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=T, pad_same=True)
    counts, _ = g.analysis_end()
    # per image: 2 input ciphertexts x 3 diagonals (+ the copy), 2 output ciphertexts x 8 taps inside sums
    assert counts["rot_summed"] == 2 * 2 * 8 and counts["rot_left"] == 2 * (2 * 3 + 2 * 8 + (2 if 4 * c_stride != g.slots else 0))
    # dry run: per image 2 input ciphertexts x 8 taps shared-decomposition rotations (+ the copy behind the blocks),
    # 2 output ciphertexts x 3 rotations inside sums, 2 x 9 x 4 x 2 multiply-accumulate terms
    g.analysis_begin()
    dry = g.conv2d(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=S, pad_same=True)
    counts, dry_steps = g.analysis_end()
    wrap = 4 * c_stride != g.slots
    assert counts["rot_summed"] == 2 * 2 * 3 and counts["rot_left"] == 2 * (2 * 8 + 2 * 3 + (2 if wrap else 0))
    assert counts["mac_plain"] == 2 * 2 * 9 * 4 * 2 and counts["rescale"] == 4
    assert set(dry_steps) == set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True, chw_schedule=S))
    assert dry.cts[0].limbs == 2
    with pytest.raises(hisa.HisaError) as e:               # the two ways of sharing a division do not combine
        g.conv2d(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=S, shared_moddown=True)
    assert e.value.code == -1
    with pytest.raises(hisa.HisaError) as e:                # 6 x 6 = 36 sums per output: more than one call adds up
        g.conv2d(gt, np.zeros((6, 6, 5, 6)), 6, 6, mode=layers.CONV_PLAIN, chw_schedule=T, pad_same=True)
    assert e.value.code == -1
    with pytest.raises(hisa.HisaError) as e:
        g.conv2d(gt, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=7)
    assert e.value.code == -1
    g.close()
    g2, _ = make_pair(10, [50, 40, 40], 3, 60, 14)         # no fused key switch: refused, not silently re-scheduled
    gt2 = g2.tensor_encrypt(x, 2.0 ** 40, 3, c_inner=4, c_stride=64, h_stride=6, offset=7)
    with pytest.raises(hisa.HisaError) as e:
        g2.conv2d_rot_steps(gt2, 3, 3) and g2.conv2d(gt2, w, 3, 3, mode=layers.CONV_PLAIN, chw_schedule=S)
    assert e.value.code == -1
    g2.close()


@pytest.mark.parametrize("c_stride", [16, 512])
def test_chw_conv_same_by_masking_bit_exact(c_stride):
    """SAME padding carried by the plaintexts (pad_same = 2) on densely packed planes without a border, against the
    oracle bit for bit: both schedules, stride 1 and 2, blocks with their copy behind them (4 x 16 slots) and filling
    the slots (4 x 512); fixed-point, float and plan entry points; refused for HW-tiled tensors and scalar weights."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(12, [50, 40, 40], 3, 50, 14)
    x = synth.image(45, 5, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.7])[:, None, None, None]
    w = synth.conv_weights(46, 3, 3, 5, 6)
    gt, ot = chw_pair(g, o, x, 2.0 ** 40, 3, 4, c_stride, 902, h_stride=4)
    steps = sorted(set(g.conv2d_rot_steps(gt, 3, 3, pad_same=2)) | set(g.conv2d_rot_steps(gt, 3, 3, pad_same=2, chw_schedule=1)))
    assert set(g.conv2d_rot_steps(gt, 3, 3, pad_same=2, chw_schedule=2)) == set(g.conv2d_rot_steps(gt, 3, 3, pad_same=2, chw_schedule=1))
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    for stride in (1, 2):
        ref = plain_net.conv2d(x, w, stride=stride, pad_same=True)
        for sched, name in ((0, "in"), (1, "out"), (2, "taps")):
            oout, ints = layers.conv2d_chw(o, ot, w, stride=stride, pad_same=2, schedule=name)
            gout = g.conv2d_fixed(gt, None, 1.0, ints["pt_coeffs"], ints["pt_scale"], 6, 3, 3, stride=stride, pad_same=2,
                                  mode=layers.CONV_PLAIN, chw_schedule=sched)
            same_tensor(g, o, gout, oout)
            assert np.abs(g.tensor_decrypt(gout) - ref).max() <= 1e-3
            gfloat = g.conv2d(gt, w, 3, 3, stride=stride, pad_same=2, mode=layers.CONV_PLAIN, chw_schedule=sched)
            assert gfloat.meta() == gout.meta() and np.abs(g.tensor_decrypt(gfloat) - ref).max() <= 1e-3
            plan = g.conv2d_prepare(gt, w, 3, 3, stride=stride, pad_same=2, mode=layers.CONV_PLAIN, chw_schedule=sched)
            gplan = g.conv2d_apply(gt, plan)
            for ca, cb in zip(gfloat.cts, gplan.cts):
                assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
            g.conv_plan_free(plan)
    # the sums' division by P and the divScalar in one base conversion (hisa_set_fused_rescale)
    g.set_fused_rescale(True)
    for sched, name in ((1, "out"), (2, "taps")):
        oout, ints = layers.conv2d_chw(o, ot, w, pad_same=2, schedule=name, fused_rescale=True)
        gout = g.conv2d_fixed(gt, None, 1.0, ints["pt_coeffs"], ints["pt_scale"], 6, 3, 3, pad_same=2, mode=layers.CONV_PLAIN,
                              chw_schedule=sched)
        same_tensor(g, o, gout, oout)
        assert gout.cts[0].limbs == 2 and np.abs(g.tensor_decrypt(gout) - plain_net.conv2d(x, w, pad_same=True)).max() <= 1e-3
    unfused, _ = layers.conv2d_chw(o, ot, w, pad_same=2, schedule="in")
    gin = g.conv2d(gt, w, 3, 3, pad_same=2, mode=layers.CONV_PLAIN)              # the schedule without sums is untouched
    assert np.abs(g.tensor_decrypt(gin) - layers.tensor_decrypt(o, unfused)).max() <= 1e-5
    g.set_fused_rescale(False)
    hw = g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=4)
    for kw in (dict(mode=layers.CONV_PLAIN), dict(mode=layers.CONV_SCALAR)):
        with pytest.raises(hisa.HisaError) as e:
            g.conv2d(hw, w, 3, 3, pad_same=2, **kw)
        assert e.value.code == -1
    with pytest.raises(hisa.HisaError) as e:
        g.conv2d(gt, w, 3, 3, pad_same=3, mode=layers.CONV_PLAIN)
    assert e.value.code == -1
    g.close()


def test_activation_with_fused_rescale_bit_exact():
    """hisa_set_fused_rescale on the degree-2 activation (HW- and CHW-tiled, with and without a linear term, two
    levels): against the oracle's one-division schedule bit for bit, against the fp64 activation, and the dry run."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(12, [50, 40, 40, 40], 2, 50, 31)
    g.keygen(); o.keygen()
    x = synth.image(71, 3, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.6])[:, None, None, None]
    g.set_fused_rescale(True)
    for make in (lambda: both_tensors(g, o, x, 2.0 ** 40, 4), lambda: chw_pair(g, o, x, 2.0 ** 40, 4, 2, 32, 903, h_stride=4)):
        gt, ot = make()
        want = x
        for a, b in ((0.4, 0.3), (0.5, 0.0)):
            gt, ot = g.poly2_act(gt, a, b), layers.poly2_act(o, ot, a, b, fused_rescale=True)
            same_tensor(g, o, gt, ot)
            want = plain_net.poly2_act_without_a(want, a, b)
            assert np.abs(g.tensor_decrypt(gt) - want).max() <= 1e-5
        assert gt.cts[0].limbs == 2
    g.analysis_begin()
    dry = g.poly2_act(both_tensors(g, o, x, 2.0 ** 40, 4)[0], 0.4, 0.3)
    counts, _ = g.analysis_end()
    assert counts["relinearize"] == 6 and counts["rescale"] == 6 and counts["mul"] == 6 and dry.cts[0].limbs == 3
    g.close()


def test_mask_layer_then_chw_conv_on_a_pooled_tensor():
    """pool (not clean) -> masking multiply -> CHW convolution, every step bit for bit; the convolution refuses the
    unmasked tensor."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(10, [50, 40, 40, 40], 2, 50, 15)
    x = synth.image(51, 3, 4, 4)[None]
    gt, ot = chw_pair(g, o, x, 2.0 ** 40, 4, 2, 32, 901, h_stride=4)
    g.gen_rot_keys([1, 4, 5]); o.gen_rot_keys([1, 4, 5])
    gp, op = g.sum_pool2x2(gt), layers.sum_pool2x2(o, ot)
    same_tensor(g, o, gp, op)
    w = synth.conv_weights(52, 1, 1, 3, 4)
    with pytest.raises(hisa.HisaError):
        g.conv2d(gp, w, 1, 1, mode=layers.CONV_PLAIN)
    om, ints = layers.mask_tensor(o, op)
    gm = g.tensor_mask_fixed(gp, ints["mask_coeffs"], ints["mask_scale"])
    same_tensor(g, o, gm, om)
    gm2 = g.tensor_mask(gp)
    assert gm2.meta() == gm.meta() and np.abs(g.tensor_decrypt(gm2) - plain_net.sum_pool2x2(x)).max() <= 1e-3
    steps = g.conv2d_rot_steps(gm, 1, 1)
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    oc_, ints = layers.conv2d_chw(o, om, w)
    gc_ = g.conv2d_fixed(gm, None, 1.0, ints["pt_coeffs"], ints["pt_scale"], 4, 1, 1, mode=layers.CONV_PLAIN)
    same_tensor(g, o, gc_, oc_)
    assert np.abs(g.tensor_decrypt(gc_) - plain_net.conv2d(plain_net.sum_pool2x2(x), w)).max() <= 1e-3
    g.close()


def test_layout_switches_bit_exact():
    """HW -> CHW -> pool -> HW through the C ABI against the oracle, bit for bit (batch of two, ragged last group);
    a tensor that is not clean cannot be packed."""
    from oracle import layers
    from paper_1810_00845_amd import hisa
    from paper_1810_00845_amd import synth
    for log_n in (10, 12):
        g, o = make_pair(log_n, [50, 40, 40], 3, 50, 16)
        x = synth.image(61, 5, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, 0.3])[:, None, None, None]
        gt, ot = both_tensors(g, o, x, 2.0 ** 40, 3, h_stride=4)
        steps = g.tensor_layout_rot_steps(gt, 2, 32)
        assert steps == [o.slots - 32]
        g.gen_rot_keys(steps + [1, 4, 5, 32]); o.gen_rot_keys(steps + [1, 4, 5, 32])
        gc, oc = g.tensor_to_chw(gt, 2, 32), layers.to_chw(o, ot, 2, 32)
        same_tensor(g, o, gc, oc)
        assert np.abs(g.tensor_decrypt(gc) - x).max() <= 1e-6
        gp, op = g.sum_pool2x2(gc), layers.sum_pool2x2(o, oc)
        same_tensor(g, o, gp, op)
        assert g.tensor_layout_rot_steps(gp) == [32]
        oh, ints = layers.to_hw(o, op)
        gh = g.tensor_to_hw_fixed(gp, ints["mask_coeffs"], ints["mask_scale"])
        same_tensor(g, o, gh, oh)
        gh2 = g.tensor_to_hw(gp)
        assert gh2.meta() == gh.meta() and np.abs(g.tensor_decrypt(gh2) - plain_net.sum_pool2x2(x)).max() <= 1e-3
        hw_pool = g.sum_pool2x2(gt)
        with pytest.raises(hisa.HisaError):
            g.tensor_to_chw(hw_pool, 2, 32)
        with pytest.raises(hisa.HisaError):
            g.tensor_to_hw(gt)
        g.close()


def test_shared_moddown_convolutions_bit_exact():
    """The convolution with one division by P per output ciphertext through the C ABI against the oracle's
    SharedModDown schedule, bit for bit: HW-tiled with scalar weights (literal and masked; short contraction on the
    fp64 kernel, long one on the matrix cores), HW-tiled with plaintext weights, CHW-tiled (with the copy behind the
    blocks); batch of two; plan and float entry point; and against the fp64 convolution."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(12, [50, 45, 45], 3, 50, 17)
    x = synth.image(71, 4, 4, 4)[None].repeat(2, axis=0) * np.array([1.0, -0.6])[:, None, None, None]
    gt, ot = both_tensors(g, o, x, 2.0 ** 40, 3, h_stride=6, offset=7)
    steps = sorted(set(g.conv2d_rot_steps(gt, 3, 3, pad_same=True)) | set(g.conv2d_rot_steps(gt, 3, 3)))
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    for oc_n, kw, mode in ((5, dict(pad_same=True), layers.CONV_MASKED),      # K = 32 rotated terms: matrix cores
                           (3, dict(), layers.CONV_SCALAR), (2, dict(stride=2, pad_same=True), layers.CONV_PLAIN)):
        w = synth.conv_weights(72 + oc_n, 3, 3, 4, oc_n)
        ref = plain_net.conv2d(x, w, **kw)
        oout, ints = layers.conv2d(o, ot, w, mode=mode, shared_moddown=True, **kw)
        gout = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], ints["pt_coeffs"], ints["pt_scale"], oc_n, 3, 3, mode=mode,
                              shared_moddown=True, **kw)
        same_tensor(g, o, gout, oout)
        assert np.abs(g.tensor_decrypt(gout) - ref).max() <= 1e-3
        gfloat = g.conv2d(gt, w, 3, 3, mode=mode, shared_moddown=True, **kw)
        assert gfloat.meta() == gout.meta() and np.abs(g.tensor_decrypt(gfloat) - ref).max() <= 1e-3
        plan = g.conv2d_prepare(gt, w, 3, 3, mode=mode, shared_moddown=True, **kw)
        gplan = g.conv2d_apply(gt, plan)
        for ca, cb in zip(gfloat.cts, gplan.cts):
            assert np.array_equal(g.ct_export(ca), g.ct_export(cb))
        g.conv_plan_free(plan)
        exact = g.conv2d(gt, w, 3, 3, mode=mode, **kw)              # the term-by-term schedule: other bits, same values
        assert not np.array_equal(g.ct_export(exact.cts[0]), g.ct_export(gfloat.cts[0]))
        assert np.abs(g.tensor_decrypt(exact) - g.tensor_decrypt(gfloat)).max() <= 1e-6
    # scalar weights under hisa_set_fused_rescale: the division by P and the divScalar as one division; the masked
    # mode (a multiplication in between) keeps its two steps
    g.set_fused_rescale(True)
    w = synth.conv_weights(76, 3, 3, 4, 3)
    oout, ints = layers.conv2d(o, ot, w, mode=layers.CONV_SCALAR, shared_moddown=True, fused_rescale=True, pad_same=True)
    gout = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], None, 1.0, 3, 3, 3, mode=layers.CONV_SCALAR, shared_moddown=True,
                          pad_same=True)
    same_tensor(g, o, gout, oout)
    assert gout.cts[0].limbs == 2 and np.abs(g.tensor_decrypt(gout) - plain_net.conv2d(x, w, pad_same=True)).max() <= 1e-3
    oout, ints = layers.conv2d(o, ot, w, mode=layers.CONV_MASKED, shared_moddown=True, pad_same=True)
    gout = g.conv2d_fixed(gt, ints["w_int"], ints["w_scale"], ints["pt_coeffs"], ints["pt_scale"], 3, 3, 3, mode=layers.CONV_MASKED,
                          shared_moddown=True, pad_same=True)
    same_tensor(g, o, gout, oout)
    g.set_fused_rescale(False)
    # CHW-tiled: 5 -> 6 channels in blocks of 4, 64 slots apart (copy behind the blocks)
    xc = synth.image(73, 5, 4, 4)[None]
    wc = synth.conv_weights(74, 3, 3, 5, 6)
    gc, oc = chw_pair(g, o, xc, 2.0 ** 40, 3, 4, 64, 910, h_stride=6, offset=7)
    steps = g.conv2d_rot_steps(gc, 3, 3, pad_same=True)
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    oout, ints = layers.conv2d_chw(o, oc, wc, pad_same=True, shared_moddown=True)
    gout = g.conv2d_fixed(gc, None, 1.0, ints["pt_coeffs"], ints["pt_scale"], 6, 3, 3, pad_same=True, mode=layers.CONV_PLAIN,
                          shared_moddown=True)
    same_tensor(g, o, gout, oout)
    assert np.abs(g.tensor_decrypt(gout) - plain_net.conv2d(xc, wc, pad_same=True)).max() <= 1e-3
    gfloat = g.conv2d(gc, wc, 3, 3, pad_same=True, mode=layers.CONV_PLAIN, shared_moddown=True)
    assert np.abs(g.tensor_decrypt(gfloat) - plain_net.conv2d(xc, wc, pad_same=True)).max() <= 1e-3
    g.close()
    # parameters without the fused key-switch path refuse the request
    g2, _ = make_pair(10, [50, 40, 40], 3, 50, 17)
    t2 = g2.tensor_encrypt(synth.image(1, 1, 4, 4)[None], 2.0 ** 40, 3)
    with pytest.raises(hisa.HisaError):
        g2.conv2d(t2, synth.conv_weights(1, 3, 3, 1, 1), 3, 3, shared_moddown=True)
    g2.close()


def test_new_layer_entry_points_reject_bad_arguments():
    """Error paths of the CHW / matmul / layout entry points: every one is a host-side check that returns an error
    code (nothing reaches a kernel)."""
    from paper_1810_00845_amd import hisa, synth
    g = hisa.Context(12, [50, 40, 40], 3, 50, 21)
    x = synth.image(81, 4, 4, 4)[None]
    t = g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=4)
    with pytest.raises(hisa.HisaError):
        g.matmul_geometry(t, 3, 0)                                   # no replicas at all
    with pytest.raises(hisa.HisaError):
        g.tensor_to_chw(t, 4, 1024)                                  # four blocks of 1024 slots do not fit 2048
    with pytest.raises(hisa.HisaError):
        g.tensor_to_chw(t, 4, 0)                                     # no channel stride
    with pytest.raises(hisa.HisaError):
        g.matmul(t, synth.fc_weights(1, 3, 4, 4, 4), 4)              # no rotation keys yet
    with pytest.raises(hisa.HisaError):
        g.rot_left_hoisted_batch(t.cts, [1, 2, 3])                   # nor here; nothing is queued, nothing leaks
    c = g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=4, c_inner=4, c_stride=16)
    with pytest.raises(hisa.HisaError):                              # 9 x 9 taps x 4 blocks > 256 rotation amounts
        g.conv2d(c, np.zeros((9, 9, 4, 4)), 9, 9, pad_same=True, mode=2)
    with pytest.raises(hisa.HisaError):                              # 4 blocks of 16 slots neither fill 2048 slots ...
        pass_through = g.tensor_encrypt(x, 2.0 ** 40, 3, h_stride=4, c_inner=4, c_stride=300)
        g.conv2d(pass_through, np.zeros((1, 1, 4, 4)), 1, 1, mode=2)  # ... nor leave room for a copy: 2 x 4 x 300 > 2048
    with pytest.raises(hisa.HisaError):
        g.fc_prepare(c, synth.fc_weights(1, 3, 4, 4, 4))             # fc is HW-tiled only
    low = g.tensor_encrypt(x, 2.0 ** 40, 1, h_stride=4)
    with pytest.raises(hisa.HisaError):
        g.tensor_mask(low)                                           # no level to rescale into
    # sums of rotations: 33 rotated terms, terms of different scale or level
    g.keygen()
    g.gen_rot_keys(list(range(1, 34)))
    with pytest.raises(hisa.HisaError) as e:
        g.rot_left_sum_batch([t.cts[:1]] * 34, [0] + list(range(1, 34)))
    assert e.value.code == -1
    other = g.tensor_encrypt(x, 2.0 ** 39, 3, h_stride=4)
    with pytest.raises(hisa.HisaError) as e:
        g.rot_left_sum_batch([t.cts[:1], other.cts[:1]], [0, 1])
    assert e.value.code == -3
    with pytest.raises(hisa.HisaError) as e:
        g.rot_left_sum_batch([t.cts[:1], low.cts[:1]], [0, 1])
    assert e.value.code == -2
    # the convolution that rotates the sums: more than 33 channel blocks
    many = g.tensor_encrypt(synth.image(82, 64, 2, 2)[None], 2.0 ** 40, 3, h_stride=2, c_inner=64, c_stride=32)
    with pytest.raises(hisa.HisaError) as e:
        g.conv2d(many, np.zeros((1, 1, 64, 64)), 1, 1, mode=2, chw_schedule=hisa.CHW_ROTATE_SUMS)
    assert e.value.code == -1
    g.close()


@pytest.mark.parametrize("chw", [False, True])
def test_bias_bit_exact_and_accurate(chw):
    """The per-channel bias after a linear layer: bit for bit with the oracle's addPlain on the oracle's integers
    (HW- and CHW-tiled, two images), the library's own encoding within 1e-6 of x + bias, nothing outside the element
    slots; a bias whose fixed-point form does not fit is refused."""
    from oracle import layers
    from paper_1810_00845_amd import hisa, synth
    g, o = make_pair(10, [50, 40, 40], 2, 50, 16)
    x = synth.image(61, 5, 3, 3)[None]
    x = np.concatenate([x, 0.5 * x])
    bias = np.array([0.5, -1.25, 2.0, 0.0, -0.75])
    if chw:
        gt, ot = chw_pair(g, o, x, 2.0 ** 40, 3, 2, 16, 902, h_stride=4)
    else:
        gt, ot = both_tensors(g, o, x, 2.0 ** 40, 3, h_stride=4)
    ob, coeffs = layers.add_bias(o, ot, bias)
    gb = g.tensor_add_bias_fixed(gt, coeffs)
    same_tensor(g, o, gb, ob)                                   # in place: gt itself now carries the bias
    assert np.abs(g.tensor_decrypt(gt) - (x + bias[None, :, None, None])).max() <= 1e-6
    # the library's own encoding, on top: twice the bias now
    g.tensor_add_bias(gt, bias)
    assert np.abs(g.tensor_decrypt(gt) - (x + 2 * bias[None, :, None, None])).max() <= 1e-6
    ob2, _ = layers.add_bias(o, ob, bias)
    for gc, oc in zip(gt.cts, ob2.cts):                         # other slots: as the oracle has them (zero here)
        assert np.abs(g.decode(g.decrypt(gc)).real - o.decode(o.decrypt(oc)).real).max() <= 1e-6
    with pytest.raises(hisa.HisaError):
        g.tensor_add_bias(gt, bias * 1e8)                       # 2e8 * 2^40 > 2^62
    g.close()


def test_average_pool_bit_exact():
    """hisa_avg_pool2x2 = the sum pool's ciphertexts at four times the scale, on both sides; decrypts to the 2x2 mean;
    a convolution after it works at that scale."""
    from oracle import layers
    from paper_1810_00845_amd import synth
    g, o = make_pair(10, [50, 40, 40], 2, 50, 17)
    x = synth.image(62, 2, 4, 4)[None]
    gt, ot = both_tensors(g, o, x, 2.0 ** 40, 3)
    g.gen_rot_keys([1, 4, 5]); o.gen_rot_keys([1, 4, 5])
    ga, oa = g.avg_pool2x2(gt), layers.avg_pool2x2(o, ot)
    same_tensor(g, o, ga, oa)
    assert ga.cts[0].scale == 4.0 * gt.cts[0].scale
    mean = x.reshape(1, 2, 2, 2, 2, 2).mean(axis=(3, 5))
    assert np.abs(g.tensor_decrypt(ga) - mean).max() <= 1e-6
    w = synth.conv_weights(63, 1, 1, 2, 3)
    gc = g.conv2d(ga, w, 1, 1)
    assert np.abs(g.tensor_decrypt(gc) - plain_net.conv2d(mean, w)).max() <= 1e-3
    g.close()
