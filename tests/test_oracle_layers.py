"""Pins of the oracle's tensor layers against fp64 plaintext tensor arithmetic (no GPU).

The encrypted layer, decrypted, must agree with the plain layer to 1e-3 on the
value ranges of the workloads; the instruction counts must be those of
Algorithm 1.
"""
import numpy as np
import pytest

import plain_net
from oracle import Oracle, layers
from paper_1810_00845_amd import synth


def config1_oracle(seed=1):
    o = Oracle(12, [30, 30, 30], 3, 60, seed)
    return o


# (MASKED splits the last modulus into weight scale x mask scale 2^25: it needs ~50-bit primes, not these 30-bit ones)
@pytest.mark.parametrize("mode", [layers.CONV_PLAIN, layers.CONV_SCALAR])
def test_config1_conv_matches_plain_conv_and_op_counts(mode):
    o = config1_oracle()
    x = synth.image(1, 1, 8, 8)[None]                    # [1][1][8][8], row-major in the slots
    w = synth.conv_weights(2, 3, 3, 1, 1)
    t = layers.tensor_encrypt(o, x, 2.0 ** 25, 3)
    assert (t.h_stride, t.w_stride, t.offset) == (8, 1, 0)
    o.gen_rot_keys(layers.rot_steps_conv(o, t, 3, 3))
    assert len(o.keys) == 8                               # nine taps, the (0,0) tap needs no key
    counts = {"rot": 0, "ks": 0, "mul": 0, "add": 0, "rescale": 0}
    real = {n: getattr(o, n) for n in ("rot_left", "mul_plain", "mul_int", "add", "div_scalar")}
    def wrap(name, key, extra=None):
        def f(*a, **k):
            counts[key] += 1
            if extra:
                extra(*a)
            return real[name](*a, **k)
        setattr(o, name, f)
    wrap("rot_left", "rot", lambda ct, r: counts.__setitem__("ks", counts["ks"] + (r % o.slots != 0)))
    wrap("mul_plain", "mul"); wrap("mul_int", "mul"); wrap("add", "add"); wrap("div_scalar", "rescale")
    out, ints = layers.conv2d(o, t, w, mode=mode)
    assert counts["rot"] == 9 and counts["ks"] == 8 and counts["add"] == 8 and counts["rescale"] == 1
    assert counts["mul"] == 9
    assert (out.height, out.width, out.channels, out.h_stride) == (6, 6, 1, 8)
    assert out.cts[0].limbs == 2 and abs(out.cts[0].scale - 2.0 ** 25) < 1e-6 * 2.0 ** 25
    got = layers.tensor_decrypt(o, out)
    want = plain_net.conv2d(x, w)
    assert np.abs(got - want).max() <= 1e-3
    if mode != layers.CONV_SCALAR:                        # masked modes leave zeros off the valid positions
        z = o.decode(o.decrypt(out.cts[0])).real
        z[layers.plane_slots(6, 6, 8, 1, 0)] = 0
        assert np.abs(z).max() <= 1e-3


def test_strided_same_multichannel_conv():
    o = Oracle(11, [45, 45, 45], 3, 50, seed=3)
    x = synth.image(3, 2, 6, 6)[None]                     # 2 channels, 6x6 planes
    w = synth.conv_weights(4, 3, 3, 2, 3)
    # SAME padding: the plane sits inside a border of one zero slot (row stride 8, first element at slot 9)
    t = layers.tensor_encrypt(o, x, 2.0 ** 40, 3, h_stride=8, w_stride=1, offset=9)
    o.gen_rot_keys(layers.rot_steps_conv(o, t, 3, 3, pad_same=True))
    out, _ = layers.conv2d(o, t, w, stride=1, pad_same=True, mode=layers.CONV_MASKED)
    assert (out.height, out.width, out.clean) == (6, 6, 1)
    assert np.abs(layers.tensor_decrypt(o, out) - plain_net.conv2d(x, w, pad_same=True)).max() <= 1e-3
    # a second SAME conv on the clean output, stride 2
    w2 = synth.conv_weights(5, 3, 3, 3, 2)
    out2, _ = layers.conv2d(o, out, w2, stride=2, pad_same=True, mode=layers.CONV_MASKED)
    want2 = plain_net.conv2d(plain_net.conv2d(x, w, pad_same=True), w2, stride=2, pad_same=True)
    assert (out2.height, out2.width, out2.h_stride, out2.w_stride) == (3, 3, 16, 2)
    assert np.abs(layers.tensor_decrypt(o, out2) - want2).max() <= 1e-3
    # VALID, stride 2, literal Algorithm 1
    o.gen_rot_keys(layers.rot_steps_conv(o, t, 3, 3))
    out3, _ = layers.conv2d(o, t, w, stride=2, mode=layers.CONV_SCALAR)
    assert (out3.height, out3.width, out3.h_stride, out3.w_stride) == (2, 2, 16, 2)
    assert np.abs(layers.tensor_decrypt(o, out3) - plain_net.conv2d(x, w, stride=2)).max() <= 1e-3


def test_fc_pool_activation_chain():
    o = Oracle(11, [50, 45, 45, 45, 45], 5, 55, seed=4)
    o.keygen()
    x = synth.image(6, 2, 4, 4)[None]
    t = layers.tensor_encrypt(o, x, 2.0 ** 45, 5)
    # activation 0.3 x^2 + 0.2 x, without its leading factor
    act = layers.poly2_act(o, t, 0.3, 0.2)
    ref = plain_net.poly2_act_without_a(x, 0.3, 0.2)
    assert act.cts[0].limbs == 4 and np.abs(layers.tensor_decrypt(o, act) - ref).max() <= 1e-3
    # sum pool
    o.gen_rot_keys([1, 4, 5])
    pool = layers.sum_pool2x2(o, act)
    ref = plain_net.sum_pool2x2(ref)
    assert (pool.height, pool.h_stride, pool.w_stride) == (2, 8, 2)
    assert np.abs(layers.tensor_decrypt(o, pool) - ref).max() <= 1e-3
    # fully connected over 2 channels x 2 x 2 elements -> 3 outputs, then 3 -> 2 on 1x1 planes
    w1 = synth.fc_weights(7, 3, 2, 2, 2, std=0.3)
    assert layers.fc_reduce_steps(o, pool) == [2, 8]     # strided log-step sum: one step per dimension of the 2x2 plane
    o.gen_rot_keys([2, 8])
    f1, _ = layers.fc(o, pool, w1)
    ref1 = plain_net.fc(ref, w1)
    assert (f1.channels, f1.height, f1.width) == (3, 1, 1)
    assert np.abs(layers.tensor_decrypt(o, f1) - ref1).max() <= 1e-3
    w2 = synth.fc_weights(8, 2, 3, 1, 1, std=0.5)
    f2, _ = layers.fc(o, f1, w2)
    assert f2.cts[0].limbs == 2
    assert np.abs(layers.tensor_decrypt(o, f2) - plain_net.fc(ref1, w2)).max() <= 1e-3


def test_plain_reference_conv_is_cross_correlation():
    x = np.zeros((1, 1, 4, 4)); x[0, 0, 1, 2] = 1.0
    w = np.arange(9.0).reshape(3, 3, 1, 1)
    out = plain_net.conv2d(x, w)
    # output (y, x) = sum_ij w[i][j] x[y+i][x+j]: the impulse at (1,2) meets w[1-y][2-x]
    assert out[0, 0].tolist() == [[5.0, 4.0], [2.0, 1.0]]
    same = plain_net.conv2d(x, w, pad_same=True)
    assert same.shape == (1, 1, 4, 4) and same[0, 0, 1, 2] == 4.0 and same[0, 0, 2, 3] == 0.0 and same[0, 0, 0, 1] == 8.0


def test_fc_reduction_rule_and_zero_padding():
    """The log-step sum of the FC layer: strided amounts when the padded rows do not overlap (a 3x3 plane summed as
    4x4: the extra positions are zero after the masked multiply), the contiguous window otherwise; both give the
    plaintext FC."""
    from oracle import Oracle, layers
    from paper_1810_00845_amd import synth
    o = Oracle(10, [50, 40], 2, 55, 9)
    o.keygen()
    x = synth.image(3, 2, 3, 3)[None]
    w = synth.fc_weights(4, 2, 2, 3, 3, std=0.4)
    want = plain_net.fc(x, w)
    for hs, off, expect in ((8, 9, [1, 2, 8, 16]), (3, 0, [1, 2, 4, 8])):
        t = layers.tensor_encrypt(o, x, 2.0 ** 40, 2, h_stride=hs, offset=off)
        assert layers.fc_reduce_steps(o, t) == expect
        o.gen_rot_keys(expect)
        f, _ = layers.fc(o, t, w)
        assert np.abs(layers.tensor_decrypt(o, f) - want).max() <= 1e-3


def test_matmul_with_replicas_chw_output_and_op_counts():
    """Homomorphic matmul with replicas (Sec. "Homomorphic Tensor Operations"): the number of mulPlain drops by the
    number of replicas, replicas and reduction take log-many rotations, the output is CHW-tiled (R outputs per
    ciphertext, one block apart), and a CHW-tiled tensor feeds the next matmul.  Values against the fp64 layers."""
    o = Oracle(11, [50, 45, 45, 45, 45, 45], 3, 55, seed=12)
    o.keygen()
    x = synth.image(21, 3, 4, 4)[None]
    t = layers.tensor_encrypt(o, x, 2.0 ** 45, 6)
    o.gen_rot_keys([1, 4, 5])
    pool = layers.sum_pool2x2(o, t)                       # 3 channels of 2x2, strides (8, 2), not clean
    ref = plain_net.sum_pool2x2(x)
    assert pool.clean == 0
    block, r, replicate, reduce = layers.matmul_geometry(o, pool, 64)
    # last element in slot 8 + 2 = 10 -> blocks of 16 slots; 1024 slots hold 64 of them
    assert (block, r, replicate, reduce) == (16, 64, [16, 32, 64, 128, 256, 512], [2, 8])
    assert layers.matmul_geometry(o, pool, 5)[1] == 4     # rounded down to a power of two
    o.gen_rot_keys([o.slots - a for a in replicate[:2]] + reduce)
    counts = {"mul_plain": 0, "rot_left": 0, "rot_right": 0, "div_scalar": 0}
    real = {n: getattr(o, n) for n in counts}
    for name in counts:
        def f(*a, _n=name, **k):
            counts[_n] += 1
            return real[_n](*a, **k)
        setattr(o, name, f)
    w1 = synth.fc_weights(22, 10, 3, 2, 2, std=0.3)
    m1, ints = layers.matmul(o, pool, w1, 4)
    for name in counts:
        setattr(o, name, real[name])
    groups = 3                                            # ceil(10 / 4)
    assert counts["mul_plain"] == 3 + groups * 3          # the mask on each input, then one per (group, input)
    assert counts["rot_right"] == 3 * 2                   # two doubling steps per input ciphertext
    assert counts["rot_left"] - counts["rot_right"] == groups * 2   # (rotRight is a rotLeft by the complement)
    assert counts["div_scalar"] == 3 + groups
    assert (m1.channels, m1.height, m1.width, m1.c_inner, m1.c_stride, m1.offset, m1.clean) == (10, 1, 1, 4, 16, 0, 0)
    assert len(m1.cts) == groups and m1.cts[0].limbs == 4
    assert ints["mask_coeffs"].shape == (3, o.N) and ints["pt_coeffs"].shape == (groups, 3, o.N)
    ref1 = plain_net.fc(ref, w1)
    assert np.abs(layers.tensor_decrypt(o, m1) - ref1).max() <= 1e-3
    # the same layer without replicas is the plain FC layer, bit for bit
    m0, _ = layers.matmul(o, pool, w1, 1)
    f0, _ = layers.fc(o, pool, w1)
    assert m0.c_inner == 1 and len(m0.cts) == 10
    assert all(np.array_equal(a.data, b.data) for a, b in zip(m0.cts, f0.cts))
    # activation on the CHW-tiled tensor, then a matmul that reads it (elements 16 slots apart: strided reduction)
    act = layers.poly2_act(o, m1, 0.5, 0.25)
    ref_act = plain_net.poly2_act_without_a(ref1, 0.5, 0.25)
    assert (act.c_inner, act.c_stride) == (4, 16)
    assert np.abs(layers.tensor_decrypt(o, act) - ref_act).max() <= 1e-3
    assert layers.matmul_geometry(o, act, 8) == (64, 8, [64, 128, 256], [16, 32])
    o.gen_rot_keys([o.slots - 64, 16, 32])
    w2 = synth.fc_weights(23, 3, 10, 1, 1, std=0.4)
    m2, _ = layers.matmul(o, act, w2, 2)
    assert (m2.c_inner, m2.c_stride, len(m2.cts)) == (2, 64, 2)
    assert np.abs(layers.tensor_decrypt(o, m2) - plain_net.fc(ref_act, w2)).max() <= 1e-3


def test_chw_tensor_round_trip_and_clean_input_needs_no_mask():
    o = Oracle(10, [50, 40, 40], 3, 55, seed=13)
    o.keygen()
    x = synth.image(31, 5, 3, 3)[None]
    t = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 3, c_inner=2, c_stride=16, h_stride=4)
    assert len(t.cts) == 3 and t.clean == 1               # channels (0,1), (2,3), (4)
    assert np.abs(layers.tensor_decrypt(o, t) - x).max() <= 1e-6
    z = o.decode(o.decrypt(t.cts[2])).real                # the last ciphertext holds one channel only
    assert np.abs(z[16:]).max() <= 1e-6
    assert layers.matmul_geometry(o, t, 1 << 20) == (32, 16, [32, 64, 128, 256], [1, 2, 4, 8, 16])
    o.gen_rot_keys([o.slots - 32, 1, 2, 4, 8, 16])
    w = synth.fc_weights(32, 4, 5, 3, 3, std=0.3)
    m, ints = layers.matmul(o, t, w, 2)
    assert ints["mask_coeffs"] is None and m.cts[0].limbs == 2
    assert np.abs(layers.tensor_decrypt(o, m) - plain_net.fc(x, w)).max() <= 1e-3


def test_merged_doublings_in_reductions():
    """Rotate-and-add chains taken as sums of rotations: the grouping rule, and FC / matmul values against the fp64
    layers and against the step-by-step chains (same sums up to the noise of the key switches)."""
    assert layers.merge_doublings([2, 4, 8, 16, 60, 120, 240, 480], 4) == [[2 * m for m in range(1, 16)], [60 * m for m in range(1, 16)]]
    assert layers.merge_doublings([1, 2, 4, 8, 16, 32], 4) == [[m for m in range(1, 16)], [16, 32, 48]]
    assert layers.merge_doublings([2, 8], 4) == [[2], [8]] and layers.merge_doublings([1, 2, 4], 0) == [[1], [2], [4]]
    assert layers.merge_doublings([1, 2, 4], 2) == [[1, 2, 3], [4]]
    # what a grouping must preserve, checked on plain vectors (no oracle arithmetic): rotating and adding by the groups
    # gives the sums the doubling chain gives, for every chain and setting; dropping an amount of a group does not
    rng = np.random.default_rng(8)
    z = rng.uniform(-1, 1, 256)
    def chain(v, groups):
        for grp in groups:
            v = v + sum(np.roll(v, -a) for a in grp)
        return v
    for steps in ([1, 2, 4, 8], [3, 6, 12, 40, 80], [2, 4, 8, 16, 60, 120, 240], [5], [1, 2, 16, 32, 64]):
        want = chain(z, [[s] for s in steps])
        for merge in (0, 1, 2, 3, 4):
            groups = layers.merge_doublings(steps, merge)
            assert sorted(a for g in groups for a in g if a in steps) == sorted(steps)
            assert all(len(g) in (1, 3, 7, 15) and len(g) < (1 << max(merge, 1)) for g in groups)
            assert np.abs(chain(z, groups) - want).max() <= 1e-12
            big = [g for g in groups if len(g) > 1]
            if big:
                cut = [g[:-1] if g is big[0] else g for g in groups]
                assert np.abs(chain(z, cut) - want).max() > 1e-3
    o = Oracle(11, [50, 45, 45, 45, 45, 45], 3, 55, seed=12)
    o.keygen()
    x = synth.image(23, 3, 4, 4)[None]
    t = layers.tensor_encrypt(o, x, 2.0 ** 45, 6)
    w = synth.fc_weights(24, 6, 3, 4, 4, std=0.3)
    block, r, replicate, reduce = layers.matmul_geometry(o, t, 4)
    assert (block, r, replicate, reduce) == (16, 4, [16, 32], [1, 2, 4, 8])
    amounts = {a for g in layers.merge_doublings(reduce, 4) for a in g} | \
        {o.slots - a for g in layers.merge_doublings(replicate, 4) for a in g} | set(reduce) | {o.slots - a for a in replicate}
    o.gen_rot_keys(sorted(amounts))
    counts = {"rot_left": 0, "key_switch_acc": 0, "mod_down": 0}
    real = {n: getattr(o, n) for n in counts}
    for name in counts:
        def f(*a, _n=name, **k):
            counts[_n] += 1
            return real[_n](*a, **k)
        setattr(o, name, f)
    m4, _ = layers.matmul(o, t, w, 4, merge=4)
    for name in counts:
        setattr(o, name, real[name])
    groups = 2                                            # ceil(6 / 4)
    # replicas: one sum of 3 rotations per input ciphertext; reduction: one sum of 15 rotations per group
    assert counts["rot_left"] == 0 and counts["key_switch_acc"] == 3 * 3 + groups * 15
    assert counts["mod_down"] == 2 * (3 + groups)
    ref = plain_net.fc(x, w)
    assert np.abs(layers.tensor_decrypt(o, m4) - ref).max() <= 1e-3
    m0, _ = layers.matmul(o, t, w, 4)
    assert np.abs(layers.tensor_decrypt(o, m4) - layers.tensor_decrypt(o, m0)).max() <= 1e-5
    f4, _ = layers.fc(o, t, w, merge=4)
    f0, _ = layers.fc(o, t, w)
    assert np.abs(layers.tensor_decrypt(o, f4) - ref).max() <= 1e-3
    assert np.abs(layers.tensor_decrypt(o, f4) - layers.tensor_decrypt(o, f0)).max() <= 1e-5
    # a planted mistake shows: one amount of a merged group left out
    bad = layers.rotate_and_add(o, t.cts[0], [[1, 2]])
    good = layers.rotate_and_add(o, t.cts[0], [[1, 2, 3]])
    step = layers.rotate_and_add(o, t.cts[0], [[1], [2]])
    assert np.abs(o.decode(o.decrypt(good)) - o.decode(o.decrypt(step))).max() <= 1e-6
    assert np.abs(o.decode(o.decrypt(bad)) - o.decode(o.decrypt(step))).max() > 1e-2


def test_chw_conv_matches_plain_conv_and_op_counts():
    """CHW-tiled convolution against the fp64 convolution: 5 -> 6 channels, 4 channel blocks per ciphertext (ragged
    last ciphertexts on both sides), VALID and SAME (the SAME one reads the zero border the layout provides), once
    with the blocks filling the slot vector (cyclic for free) and once with the copy behind them; clean outputs; the
    multiplication count is OC*IC*taps / c_inner with whole ciphertexts, one rotation per (input ciphertext, tap, d)."""
    x = synth.image(41, 5, 4, 4)[None]
    w = synth.conv_weights(42, 3, 3, 5, 6)
    for log_n, expect_wrap in ((9, 0), (10, 256)):
        o = Oracle(log_n, [50, 40, 40], 3, 55, seed=14)
        # planes of 4x4 inside a 6x6 frame (one zero slot around): row stride 6, first element at slot 7, blocks of 64
        t = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 3, c_inner=4, c_stride=64, h_stride=6, offset=7)
        wrap, amounts = layers.chw_conv_geometry(o, t, 3, 3, pad_same=True)
        assert wrap == expect_wrap and amounts[1][1] == [0, 64, 128, 192] and amounts[0][0][0] == o.slots - 7
        o.gen_rot_keys(sorted(set(layers.rot_steps_conv_chw(o, t, 3, 3, True)) | set(layers.rot_steps_conv_chw(o, t, 3, 3))))
        counts = {"mul_plain": 0, "rot_left": 0, "div_scalar": 0}
        real = {n: getattr(o, n) for n in counts}
        for name in counts:
            def f(*a, _n=name, **k):
                counts[_n] += 1
                return real[_n](*a, **k)
            setattr(o, name, f)
        same, _ = layers.conv2d_chw(o, t, w, pad_same=True)
        for name in counts:
            setattr(o, name, real[name])
        per_in, per_out = 2, 2
        assert counts["mul_plain"] == per_out * per_in * 9 * 4 and counts["div_scalar"] == per_out
        assert counts["rot_left"] == per_in * 9 * 4 + (per_in if wrap else 0)
        assert (same.channels, same.height, same.c_inner, same.c_stride, same.clean, len(same.cts)) == (6, 4, 4, 64, 1, 2)
        assert np.abs(layers.tensor_decrypt(o, same) - plain_net.conv2d(x, w, pad_same=True)).max() <= 1e-3
        z = o.decode(o.decrypt(same.cts[1])).real          # clean: channels 4, 5 in blocks 0, 1; nothing anywhere else
        z[np.asarray(layers.tensor_slots(same)).reshape(4, 16)[:2].reshape(-1)] = 0
        assert np.abs(z).max() <= 1e-3
        valid, _ = layers.conv2d_chw(o, t, w)
        assert (valid.height, valid.width) == (2, 2)
        assert np.abs(layers.tensor_decrypt(o, valid) - plain_net.conv2d(x, w)).max() <= 1e-3


def test_chw_conv_output_side_schedule():
    """The schedule that reduces over the channels of a ciphertext after the multiplication: against the fp64
    convolution (VALID and SAME, cyclic blocks and blocks with their copy behind them, ragged last ciphertexts), clean
    outputs, the same result as the input-side schedule up to noise, and the counts: (taps - 1) rotations per input
    ciphertext, c_inner - 1 key switches per output ciphertext, the same multiplications."""
    x = synth.image(43, 5, 4, 4)[None]
    w = synth.conv_weights(44, 3, 3, 5, 6)
    for log_n, expect_wrap in ((9, 0), (10, 256)):
        o = Oracle(log_n, [50, 40, 40], 3, 55, seed=16)
        t = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 3, c_inner=4, c_stride=64, h_stride=6, offset=7)
        steps_out = layers.rot_steps_conv_chw(o, t, 3, 3, True, schedule="out")
        steps_in = layers.rot_steps_conv_chw(o, t, 3, 3, True)
        assert set(steps_out) < set(steps_in) and len(steps_out) == 8 + 3 + (1 if expect_wrap else 0)
        assert {64, 128, 192} <= set(steps_out)
        o.gen_rot_keys(sorted(set(steps_in) | set(layers.rot_steps_conv_chw(o, t, 3, 3))))
        counts = {"mul_plain": 0, "rot_left": 0, "key_switch_acc": 0, "mod_down": 0, "div_scalar": 0}
        real = {n: getattr(o, n) for n in counts}
        for name in counts:
            def f(*a, _n=name, **k):
                counts[_n] += 1
                return real[_n](*a, **k)
            setattr(o, name, f)
        same, _ = layers.conv2d_chw(o, t, w, pad_same=True, schedule="out")
        for name in counts:
            setattr(o, name, real[name])
        per_in, per_out = 2, 2
        assert counts["mul_plain"] == per_out * per_in * 9 * 4 and counts["div_scalar"] == per_out
        assert counts["rot_left"] == per_in * 9 + (per_in if expect_wrap else 0)      # the centre tap is a copy
        # per output ciphertext: c_inner - 1 key-switch accumulations, one division by P per polynomial
        assert counts["key_switch_acc"] == per_out * 3 and counts["mod_down"] == per_out * 2
        assert (same.channels, same.height, same.c_inner, same.c_stride, same.clean, len(same.cts)) == (6, 4, 4, 64, 1, 2)
        want = plain_net.conv2d(x, w, pad_same=True)
        assert np.abs(layers.tensor_decrypt(o, same) - want).max() <= 1e-3
        z = o.decode(o.decrypt(same.cts[1])).real
        z[np.asarray(layers.tensor_slots(same)).reshape(4, 16)[:2].reshape(-1)] = 0
        assert np.abs(z).max() <= 1e-3
        other, _ = layers.conv2d_chw(o, t, w, pad_same=True)
        assert np.abs(layers.tensor_decrypt(o, same) - layers.tensor_decrypt(o, other)).max() <= 1e-5
        valid, _ = layers.conv2d_chw(o, t, w, schedule="out")
        assert (valid.height, valid.width) == (2, 2)
        assert np.abs(layers.tensor_decrypt(o, valid) - plain_net.conv2d(x, w)).max() <= 1e-3
        # a planted mistake must show: weights one block off
        bad = np.roll(w, 1, axis=2)
        wrong, _ = layers.conv2d_chw(o, t, bad, pad_same=True, schedule="out")
        assert np.abs(layers.tensor_decrypt(o, wrong) - want).max() > 1e-2


def test_chw_conv_same_by_masking_needs_no_border():
    """SAME padding carried by the plaintexts (pad_same = 2): densely packed planes without a zero border, both
    schedules, stride 1 and 2, cyclic blocks and blocks with their copy behind them; against the fp64 convolution.
    With the ordinary SAME flag the same layout gives wrong borders (the planted mistake)."""
    x = synth.image(45, 5, 4, 4)[None]
    w = synth.conv_weights(46, 3, 3, 5, 6)
    assert layers.same_tap_inside(layers.OTensor([], 1, 1, 4, 4, 4, 1, 0, 1), 3, 3, 0, 1, 1).reshape(4, 4).tolist() == \
        [[False] * 4] + [[True] * 4] * 3
    for c_stride in (64, 16):
        o = Oracle(9, [50, 40, 40], 3, 55, seed=17)
        t = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 3, c_inner=4, c_stride=c_stride, h_stride=4)
        o.gen_rot_keys(sorted(set(layers.rot_steps_conv_chw(o, t, 3, 3, True)) |
                              set(layers.rot_steps_conv_chw(o, t, 3, 3, True, schedule="out"))))
        for stride in (1, 2):
            want = plain_net.conv2d(x, w, stride=stride, pad_same=True)
            for schedule in ("in", "out", "taps"):
                got, _ = layers.conv2d_chw(o, t, w, stride=stride, pad_same=2, schedule=schedule)
                assert got.clean == 1 and np.abs(layers.tensor_decrypt(o, got) - want).max() <= 1e-3
        wrong, _ = layers.conv2d_chw(o, t, w, pad_same=True)
        assert np.abs(layers.tensor_decrypt(o, wrong) - plain_net.conv2d(x, w, pad_same=True)).max() > 1e-2


def test_chw_conv_taps_on_the_sums_schedule():
    """The schedule that rotates the inputs by the diagonals and the per-tap sums by the taps: VALID and SAME on a
    bordered layout (cyclic blocks and blocks with their copy), against the fp64 convolution and the other schedules;
    c_inner - 1 rotations per input ciphertext, taps - 1 key-switch accumulations per output ciphertext."""
    x = synth.image(47, 5, 4, 4)[None]
    w = synth.conv_weights(48, 3, 3, 5, 6)
    for log_n, expect_wrap in ((9, 0), (10, 256)):
        o = Oracle(log_n, [50, 40, 40], 3, 55, seed=18)
        t = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 3, c_inner=4, c_stride=64, h_stride=6, offset=7)
        o.gen_rot_keys(sorted(set(layers.rot_steps_conv_chw(o, t, 3, 3, True, schedule="taps")) |
                              set(layers.rot_steps_conv_chw(o, t, 3, 3, schedule="taps"))))
        counts = {"rot_left": 0, "key_switch_acc": 0, "mod_down": 0, "mul_plain": 0}
        real = {n: getattr(o, n) for n in counts}
        for name in counts:
            def f(*a, _n=name, **k):
                counts[_n] += 1
                return real[_n](*a, **k)
            setattr(o, name, f)
        same, _ = layers.conv2d_chw(o, t, w, pad_same=True, schedule="taps")
        for name in counts:
            setattr(o, name, real[name])
        per_in, per_out = 2, 2
        assert counts["rot_left"] == per_in * 4 + (per_in if expect_wrap else 0)       # d = 0 is a copy
        assert counts["key_switch_acc"] == per_out * 8 and counts["mod_down"] == per_out * 2
        assert counts["mul_plain"] == per_out * per_in * 9 * 4
        want = plain_net.conv2d(x, w, pad_same=True)
        assert same.clean == 1 and np.abs(layers.tensor_decrypt(o, same) - want).max() <= 1e-3
        z = o.decode(o.decrypt(same.cts[1])).real
        z[np.asarray(layers.tensor_slots(same)).reshape(4, 16)[:2].reshape(-1)] = 0
        assert np.abs(z).max() <= 1e-3
        valid, _ = layers.conv2d_chw(o, t, w, schedule="taps")
        assert np.abs(layers.tensor_decrypt(o, valid) - plain_net.conv2d(x, w)).max() <= 1e-3
        strided, _ = layers.conv2d_chw(o, t, w, stride=2, pad_same=True, schedule="taps")
        assert np.abs(layers.tensor_decrypt(o, strided) - plain_net.conv2d(x, w, stride=2, pad_same=True)).max() <= 1e-3
        bad = np.roll(w, 1, axis=1)                        # a planted mistake: taps one column off
        wrong, _ = layers.conv2d_chw(o, t, bad, pad_same=True, schedule="taps")
        assert np.abs(layers.tensor_decrypt(o, wrong) - want).max() > 1e-2


def test_division_by_p_and_rescale_in_one():
    """SharedModDown.total(rescale=True): the divScalar by the last modulus taken together with the division by P.
    Against the two divisions one after the other: every coefficient within a few units (the conversion's rounding), so
    the decrypted values agree to the noise; one limb fewer, scale / q_{l-1}; also dnum = 1 and a level with a ragged last digit."""
    for q_bits, dnum, limbs in (([50, 40, 40, 40], 2, 4), ([50, 40, 40, 40, 40], 1, 5), ([50, 40, 40, 40, 40], 3, 4)):
        o = Oracle(10, q_bits, dnum, 55, seed=5)
        o.keygen(); o.gen_rot_keys([1, 3])
        rng = np.random.default_rng(1)
        zs = [rng.uniform(-1, 1, o.slots) for _ in range(3)]
        big = 2.0 ** 40 * float(o.primes[limbs - 1])      # so that 2^40 is left after the division
        cts = [o.mul_scalar(o.encrypt(o.encode(z, 2.0 ** 40, limbs)), 1.0, float(o.primes[limbs - 1])) for z in zs]
        assert abs(cts[0].scale - big) <= 1e-9 * big
        steps = [1, 0, 3]
        terms = [(s, steps[s], 1, None) for s in range(3)]
        two = o.rescale(layers.SharedModDown(o, cts).total(terms, big))
        one = layers.SharedModDown(o, cts).total(terms, big, rescale=True)
        assert one.limbs == two.limbs == limbs - 1 and abs(one.scale - two.scale) <= 1e-9 * two.scale
        diff = o.export(one).astype(np.int64) - o.export(two).astype(np.int64)
        diff = np.where(diff > 2 ** 39, diff - np.asarray(o.primes[:limbs - 1], dtype=np.int64)[None, :, None], diff)
        diff = np.where(diff < -2 ** 39, diff + np.asarray(o.primes[:limbs - 1], dtype=np.int64)[None, :, None], diff)
        # the fast base conversion is off by at most half a unit per source limb, the two-step rounding by a half
        assert np.abs(diff).max() <= (o.K + 1) // 2 + 1
        ref = sum(np.roll(zs[s], -steps[s]) for s in range(3))
        assert np.abs(o.decode(o.decrypt(one)).real - ref).max() <= 1e-6
        # the planted mistake: the unrotated term left out of the accumulators
        bad = layers.SharedModDown(o, cts).total([terms[0], terms[2]], big, rescale=True)
        assert np.abs(o.decode(o.decrypt(bad)).real - ref).max() > 1e-2


def test_activation_with_one_division():
    """poly2_act(fused_rescale=True) against the fp64 activation and against the two-step schedule."""
    o = Oracle(10, [50, 40, 40, 40], 2, 55, seed=6)
    o.keygen()
    x = synth.image(61, 2, 4, 4)[None]
    t = layers.tensor_encrypt(o, x, 2.0 ** 40, 4)
    for a, b in ((0.4, 0.3), (0.5, 0.0)):
        one, two = layers.poly2_act(o, t, a, b, fused_rescale=True), layers.poly2_act(o, t, a, b)
        want = plain_net.poly2_act_without_a(x, a, b)
        assert one.cts[0].limbs == 3 and abs(one.cts[0].scale - two.cts[0].scale) <= 1e-9 * two.cts[0].scale
        assert np.abs(layers.tensor_decrypt(o, one) - want).max() <= 1e-6
        assert np.abs(layers.tensor_decrypt(o, one) - layers.tensor_decrypt(o, two)).max() <= 1e-7


def test_mask_tensor_cleans_a_pooled_tensor():
    o = Oracle(10, [50, 40, 40], 3, 55, seed=15)
    x = synth.image(51, 3, 4, 4)[None]
    t = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 3, c_inner=2, c_stride=32, h_stride=4)
    o.gen_rot_keys([1, 4, 5])
    pool = layers.sum_pool2x2(o, t)
    assert pool.clean == 0
    z = o.decode(o.decrypt(pool.cts[0])).real
    z[layers.tensor_slots(pool)] = 0
    assert np.abs(z).max() > 0.1                           # leftovers between the pooled elements
    m, ints = layers.mask_tensor(o, pool)
    assert m.clean == 1 and m.cts[0].limbs == 2 and abs(m.cts[0].scale - pool.cts[0].scale) < 1e-6 * m.cts[0].scale
    assert ints["mask_coeffs"].shape == (2, o.N)
    assert np.abs(layers.tensor_decrypt(o, m) - plain_net.sum_pool2x2(x)).max() <= 1e-3
    for ct in m.cts:
        z = o.decode(o.decrypt(ct)).real
        z[layers.tensor_slots(m)] = 0
        assert np.abs(z).max() <= 1e-3


def test_layout_switches_round_trip():
    """HW -> CHW -> HW: values unchanged, the CHW tensor is what tensor_encrypt_chw would hold, the way back costs one
    level and leaves a clean tensor even from a pooled (not clean) CHW tensor."""
    o = Oracle(10, [50, 40, 40], 3, 55, seed=16)
    x = synth.image(61, 5, 4, 4)[None]
    t = layers.tensor_encrypt(o, x, 2.0 ** 40, 3, h_stride=4)
    o.gen_rot_keys([o.slots - 32, 32, 33, 1, 4, 5])
    c = layers.to_chw(o, t, 2, 32)
    assert (c.c_inner, c.c_stride, len(c.cts), c.clean, c.cts[0].limbs) == (2, 32, 3, 1, 3)
    assert np.abs(layers.tensor_decrypt(o, c) - x).max() <= 1e-6
    z = o.decode(o.decrypt(c.cts[2])).real                # channel 4 alone in the last ciphertext
    assert np.abs(z[32:]).max() <= 1e-6
    pooled = layers.sum_pool2x2(o, c)
    h, _ = layers.to_hw(o, pooled)
    assert (h.c_inner, len(h.cts), h.clean, h.cts[0].limbs, h.height, h.h_stride) == (1, 5, 1, 2, 2, 8)
    assert np.abs(layers.tensor_decrypt(o, h) - plain_net.sum_pool2x2(x)).max() <= 1e-3
    for ct in h.cts:
        z = o.decode(o.decrypt(ct)).real
        z[layers.plane_slots(2, 2, 8, 2, 0)] = 0
        assert np.abs(z).max() <= 1e-3
    # every channel sits where the metadata says, independently of tensor_decrypt: slot by slot against the image
    for g, ct in enumerate(c.cts):
        z = o.decode(o.decrypt(ct)).real
        for k in range(min(2, 5 - 2 * g)):
            got = z[[k * 32 + y * 4 + xx for y in range(4) for xx in range(4)]].reshape(4, 4)
            assert np.abs(got - x[0, 2 * g + k]).max() <= 1e-6
    # planted mistakes: the blocks moved the wrong way, or by the wrong amount, put the channels elsewhere
    real_right, real_left = o.rot_right, o.rot_left
    o.rot_right = lambda ct, r: real_left(ct, r)
    wrong = layers.to_chw(o, t, 2, 32)
    o.rot_right = real_right
    assert np.abs(layers.tensor_decrypt(o, wrong) - x).max() > 1e-2
    o.rot_left = lambda ct, r: real_left(ct, r + 1 if r else 0)
    wrong, _ = layers.to_hw(o, c)
    o.rot_left = real_left
    assert np.abs(layers.tensor_decrypt(o, wrong) - x).max() > 1e-2
    back, _ = layers.to_hw(o, c)
    assert np.abs(layers.tensor_decrypt(o, back) - x).max() <= 1e-3


def test_shared_moddown_convolutions():
    """The convolution with one division by P per output (SharedModDown): same plaintext result as Algorithm 1 to
    1e-3, ciphertexts that differ from the term-by-term schedule by a few units per coefficient only (the rounding of
    the division), and the halves of the key switch it is built from reproduce the whole.  HW-tiled (scalar and
    masked) and CHW-tiled."""
    o = Oracle(10, [50, 45, 45], 3, 50, seed=17)
    o.keygen()
    rng = np.random.default_rng(0)
    d = np.stack([rng.integers(0, o.primes[i], o.N, dtype=np.uint64) for i in range(3)])
    o.gen_rot_keys([3])
    g = o.galois_elt(3)
    acc_b, acc_a = o.key_switch_acc(d, g)
    ks0, ks1 = o.key_switch(d, g)
    assert np.array_equal(o.mod_down(acc_b, 3), ks0) and np.array_equal(o.mod_down(acc_a, 3), ks1)
    # HW-tiled: 3 -> 4 channels, 3x3, SAME with the mask and VALID literal
    x = synth.image(71, 3, 4, 4)[None]
    w = synth.conv_weights(72, 3, 3, 3, 4)
    t = layers.tensor_encrypt(o, x, 2.0 ** 40, 3, h_stride=6, offset=7)
    o.gen_rot_keys(sorted(set(layers.rot_steps_conv(o, t, 3, 3, True)) | set(layers.rot_steps_conv(o, t, 3, 3))))
    for kw, mode, ref in ((dict(pad_same=True), layers.CONV_MASKED, plain_net.conv2d(x, w, pad_same=True)),
                          (dict(), layers.CONV_SCALAR, plain_net.conv2d(x, w))):
        plain, _ = layers.conv2d(o, t, w, mode=mode, **kw)
        lazy, _ = layers.conv2d(o, t, w, mode=mode, shared_moddown=True, **kw)
        assert lazy.cts[0].limbs == 2 and (lazy.height, lazy.clean) == (plain.height, plain.clean)
        assert np.abs(layers.tensor_decrypt(o, lazy) - ref).max() <= 1e-3
        diff = 0
        for a, b in zip(lazy.cts, plain.cts):
            for i in range(2):
                q = o.primes[i]
                ca, cb = o.export(a), o.export(b)          # coefficient form
                dd = (ca[:, i].astype(object) - cb[:, i].astype(object)) % q
                diff = max(diff, max(min(int(v), q - int(v)) for v in dd.reshape(-1)))
        assert 0 < diff <= 64            # not bit-identical, but only by the rounding of 8 x 3 divisions, rescaled
    # CHW-tiled
    xc = synth.image(73, 5, 4, 4)[None]
    wc = synth.conv_weights(74, 3, 3, 5, 6)
    tc = layers.tensor_encrypt_chw(o, xc, 2.0 ** 40, 3, c_inner=4, c_stride=64, h_stride=6, offset=7)
    o.gen_rot_keys(layers.rot_steps_conv_chw(o, tc, 3, 3, True))
    lazy, _ = layers.conv2d_chw(o, tc, wc, pad_same=True, shared_moddown=True)
    assert (lazy.c_inner, lazy.clean, len(lazy.cts), lazy.cts[0].limbs) == (4, 1, 2, 2)
    assert np.abs(layers.tensor_decrypt(o, lazy) - plain_net.conv2d(xc, wc, pad_same=True)).max() <= 1e-3


@pytest.mark.parametrize("chw", [False, True])
def test_bias_is_added_to_the_elements_of_its_channel_only(chw):
    """addPlain of the per-channel bias vector: element slots move by exactly bias[c], every other slot by nothing
    (a clean tensor stays clean); a bias vector in the wrong channel order fails."""
    o = Oracle(10, [50, 40], 2, 55, seed=14)
    x = synth.image(33, 5, 3, 3)[None]
    bias = np.array([0.5, -1.25, 2.0, 0.0, -0.75])
    if chw:
        t = layers.tensor_encrypt_chw(o, x, 2.0 ** 40, 2, c_inner=2, c_stride=16, h_stride=4)
    else:
        t = layers.tensor_encrypt(o, x, 2.0 ** 40, 2, h_stride=4)
    before = [o.decode(o.decrypt(ct)).real for ct in t.cts]
    out, coeffs = layers.add_bias(o, t, bias)
    assert coeffs.shape == (len(t.cts), o.N) and out.cts[0].scale == t.cts[0].scale and out.cts[0].limbs == 2
    assert np.abs(layers.tensor_decrypt(o, out) - (x + bias[None, :, None, None])).max() <= 1e-6
    elems = np.zeros((len(t.cts), o.slots), dtype=bool)
    sl = np.asarray(layers.tensor_slots(t)).reshape(t.c_inner, -1)
    for j in range(len(t.cts)):
        for cl in range(min(t.c_inner, 5 - j * t.c_inner)):
            elems[j, sl[cl]] = True
    for j, ct in enumerate(out.cts):
        z = o.decode(o.decrypt(ct)).real
        assert np.abs((z - before[j])[~elems[j]]).max() <= 1e-6       # nothing outside the elements
    wrong, _ = layers.add_bias(o, t, bias[::-1])
    assert np.abs(layers.tensor_decrypt(o, wrong) - (x + bias[None, :, None, None])).max() > 0.1
    # a batch of two images takes the same vectors per image
    x2 = np.concatenate([x, 2 * x])
    t2 = layers.tensor_encrypt_chw(o, x2, 2.0 ** 40, 2, c_inner=2, c_stride=16, h_stride=4) if chw else \
        layers.tensor_encrypt(o, x2, 2.0 ** 40, 2, h_stride=4)
    out2, _ = layers.add_bias(o, t2, bias)
    assert np.abs(layers.tensor_decrypt(o, out2) - (x2 + bias[None, :, None, None])).max() <= 1e-6


def test_average_pool_is_the_sum_pool_at_four_times_the_scale():
    """Against the plain 2x2 mean; the ciphertext data are those of the sum pool (nothing is computed for the 1/4)."""
    o = Oracle(10, [50, 40], 2, 55, seed=15)
    x = synth.image(35, 2, 4, 4)[None]
    t = layers.tensor_encrypt(o, x, 2.0 ** 40, 2)
    o.gen_rot_keys([1, 4, 5])
    avg, summed = layers.avg_pool2x2(o, t), layers.sum_pool2x2(o, t)
    assert np.abs(layers.tensor_decrypt(o, avg) - plain_net.sum_pool2x2(x) / 4.0).max() <= 1e-6
    assert np.abs(layers.tensor_decrypt(o, avg) - x.reshape(1, 2, 2, 2, 2, 2).mean(axis=(3, 5))).max() <= 1e-6
    for a, b in zip(avg.cts, summed.cts):
        assert np.array_equal(a.data, b.data) and a.scale == 4.0 * b.scale
    assert (avg.height, avg.width, avg.h_stride, avg.w_stride, avg.clean) == (2, 2, 8, 2, 0)
