"""The analysis backend of the library (dry runs that record rotation amounts, depth and operation counts) and the
compiler passes built on it: rotation-key selection, depth, data layout selection by cost."""
import numpy as np
import pytest

import plain_net

pytestmark = pytest.mark.gpu


def test_analysis_counts_match_the_schedule_and_leave_the_context_usable():
    """The matmul-with-replicas schedule of the oracle's pin test (3 pooled input ciphertexts, 10 outputs, 4
    replicas): the dry run reports the instruction counts that the oracle's loop executes, needs no key, and the
    same context afterwards computes the real layer."""
    from paper_1810_00845_amd import hisa, synth
    g = hisa.Context(12, [50, 45, 45, 45, 45, 45], 3, 50, 12)   # N and primes within the fused fp64 path
    x = synth.image(21, 3, 4, 4)[None]
    w1 = synth.fc_weights(22, 10, 3, 2, 2, std=0.3)
    t = g.tensor_encrypt(x, 2.0 ** 45, 6)
    g.analysis_begin()
    pool = g.sum_pool2x2(t)                      # no rotation key exists yet: recorded, not an error
    m = g.matmul(pool, w1, 4)
    counts, steps = g.analysis_end()
    assert (m.c_inner, m.c_stride, len(m.cts), m.cts[0].limbs) == (4, 16, 3, 4)
    # The independent count: the oracle's own loops run the same schedule under an instruction recorder.
    from oracle import Oracle, layers
    from oracle_record import recording
    o = Oracle(12, [50, 45, 45, 45, 45, 45], 3, 50, 12)
    ot = layers.tensor_encrypt(o, x, 2.0 ** 45, 6)
    o.gen_rot_keys(steps)                        # exactly the amounts the dry run named: anything missing raises below
    with recording(o) as rec:
        layers.matmul(o, layers.sum_pool2x2(o, ot), w1, 4)
    assert steps == sorted(rec["steps"])
    assert counts["rot_left"] == rec["rotations"] == 9 + 6 + 6
    assert counts["mul_plain"] + counts["mac_plain"] == rec["mul_plain"] and counts["rescale"] == rec["rescale"]
    assert counts["mul"] == rec["mul"] == 0 and counts["relinearize"] == rec["relinearize"] == 0
    assert counts["mul_scalar"] + counts["mac_scalar"] == rec["mul_scalar"] == 0
    assert counts["min_limbs"] == rec["min_limbs"] == 4
    # the oracle adds term by term; the library's fused multiply-accumulate hides one addition per term after the first
    groups, terms = 3, 9
    assert counts["add"] == rec["add"] - (terms - groups)
    # how the library groups the work (its own business, no oracle counterpart): of the pool's three rotations per
    # ciphertext two share the first one's decomposition, and they go out as one set of launches
    assert counts["rot_shared"] == 6 and counts["key_switch_calls"] == 1 + 2 + 2
    assert counts["mul_plain"] == 3 and counts["mac_plain"] == 9
    pool.free(); m.free()
    # outside the analysis the same calls compute: the missing keys are now an error, and with them the result is right
    with pytest.raises(hisa.HisaError):
        g.sum_pool2x2(t)
    g.gen_rot_keys(steps)
    pool = g.sum_pool2x2(t)
    m = g.matmul(pool, w1, 4)
    want = plain_net.fc(plain_net.sum_pool2x2(x), w1)
    assert np.abs(g.tensor_decrypt(m) - want).max() <= 1e-3
    g.close()


def test_analysis_mode_errors():
    from paper_1810_00845_amd import hisa, synth
    g = hisa.Context(10, [50, 40, 40], 3, 55, 5)
    with pytest.raises(hisa.HisaError):
        g.analysis_end()                         # not in analysis mode
    g.analysis_begin()
    with pytest.raises(hisa.HisaError):
        g.analysis_begin()                       # not re-entrant
    with pytest.raises(hisa.HisaError):
        g.gen_rot_keys([1])                      # keys made without kernels would be garbage that outlives the analysis
    with pytest.raises(hisa.HisaError):
        g.keygen()
    t = g.tensor_encrypt(synth.image(1, 2, 4, 4)[None], 2.0 ** 40, 3)
    with pytest.raises(hisa.HisaError):
        g.fc_prepare(t, synth.fc_weights(2, 3, 2, 4, 4))
    act = g.poly2_act(t, 0.5, 0.25)              # no relinearisation key either
    counts, steps = g.analysis_end()
    assert counts["mul"] == 2 and counts["relinearize"] == 2 and counts["mul_scalar"] == 2 and counts["rescale"] == 2
    assert steps == [] and counts["min_limbs"] == 2
    g.close()


@pytest.mark.parametrize("layout,levels,masks,mac_plain,mac_scalar,mul", [("hw", 5, 0, 500, 1125, 105),
                                                                          ("chw_fc", 6, 5, 125 + 250, 125, 30)])
def test_rotation_key_selection_and_depth_by_dry_run(layout, levels, masks, mac_plain, mac_scalar, mul):
    """LeNet-small: the keys named by the dry run are exactly enough to run the network (a context that holds only
    those keys computes the right answer), the depth is the number of divScalar levels of the schedule, and the
    multiply counts are those of the layers (conv 25 taps x 5 outputs; FC 845 -> 100 -> 10 per layout)."""
    from paper_1810_00845_amd import hisa, nets
    params, layers, x = nets.lenet_small()
    limbs = len(params["q_bits"])
    ctx = hisa.Context(params["log_n"], params["q_bits"], params["dnum"], params["special_bits"], seed=11)
    counts, steps = nets.analyse(ctx, layers, x, params["scale"], limbs, layout=layout)
    assert limbs - counts["min_limbs"] == levels
    assert (counts["mul_plain"], counts["mac_plain"], counts["mac_scalar"]) == (masks, mac_plain, mac_scalar)
    assert (counts["mul"], counts["relinearize"], counts["mul_scalar"]) == (mul, mul, 0)
    assert counts["rot_left"] >= 24 and len(steps) >= 24
    ctx.keygen()
    ctx.gen_rot_keys(steps)
    got, _, _ = nets.run_encrypted(ctx, layers, x, params["scale"], limbs, layout=layout)   # make_keys off
    from test_gpu_networks import plain_forward
    assert np.abs(got - plain_forward(layers, x)).max() <= 1e-3
    ctx.close()


def test_dry_run_counts_match_the_oracle_on_a_small_network():
    """A network of LeNet-small's layer kinds, cut down so that the oracle runs it in seconds (conv 5x5 stride 2,
    square, FC over planes with merged rotate-and-add chains, square with the fused division, FC over 1x1 planes):
    the dry run's rotation amounts, rotation count, multiplication counts and depth against the oracle's loops under
    the instruction recorder, in the settings nets.run_encrypted uses."""
    from oracle import Oracle, layers
    from oracle_record import recording
    from paper_1810_00845_amd import hisa, nets, synth
    q_bits, dnum = [50] + [40] * 6, 2
    net = [("conv", synth.conv_weights(71, 5, 5, 1, 2, dist="normal", std=0.1), 2), ("act", 1.0, 0.0),
           ("fc", synth.fc_weights(72, 4, 2, 6, 6, std=0.1)), ("act", 0.5, 0.25), ("fc", synth.fc_weights(73, 3, 4, 1, 1, std=0.1))]
    x = synth.image(74, 1, 15, 15)[None]
    g = hisa.Context(12, q_bits, dnum, 50, 11)
    counts, steps = nets.analyse(g, net, x, 2.0 ** 40, len(q_bits), layout="hw")
    g.close()
    o = Oracle(12, q_bits, dnum, 50, 11)
    o.keygen()
    o.gen_rot_keys(steps)                        # only what the dry run asked for
    cur, pending = layers.tensor_encrypt(o, x, 2.0 ** 40, len(q_bits)), 1.0
    with recording(o) as rec:
        for layer in net:
            if layer[0] == "conv":
                cur, _ = layers.conv2d(o, cur, layer[1] * pending, stride=layer[2])
                pending = 1.0
            elif layer[0] == "act":
                cur = layers.poly2_act(o, cur, layer[1], layer[2], fused_rescale=True)
                pending *= layer[1]
            else:
                cur, _ = layers.fc(o, cur, layer[1] * pending, merge=4)
                pending = 1.0
    assert steps == sorted(rec["steps"])
    assert counts["rot_left"] == rec["rotations"]
    assert counts["mul_plain"] + counts["mac_plain"] == rec["mul_plain"]
    assert counts["mul_scalar"] + counts["mac_scalar"] == rec["mul_scalar"]
    assert (counts["mul"], counts["relinearize"]) == (rec["mul"], rec["relinearize"])
    assert counts["rescale"] == rec["rescale"] and counts["min_limbs"] == rec["min_limbs"]
    # the levels the operations ran at, which the level-aware cost model reads: limbs summed over the occurrences
    ls = counts["limb_sum"]
    assert ls["rot_left"] == rec["limb_sum"]["rotations"] and ls["mul"] == rec["limb_sum"]["mul"]
    assert ls["relinearize"] == rec["limb_sum"]["relinearize"] and ls["rescale"] == rec["limb_sum"]["rescale"]
    h = plain_net.fc(np.square(plain_net.conv2d(x, net[0][1], stride=2)), net[2][1])
    want = plain_net.fc(0.5 * np.square(h) + 0.25 * h, net[4][1])
    assert np.abs(layers.tensor_decrypt(o, cur) * pending - want).max() <= 1e-3


def test_layout_selection_by_cost_agrees_with_the_clock():
    """LeNet-medium: the analyser's cost (operation counts x micro-benchmarked unit costs) ranks the two layouts the
    way the measured latencies do, and picks CHW-fc."""
    from paper_1810_00845_amd import hisa, nets
    params, layers, x = nets.lenet_medium()
    limbs = len(params["q_bits"])
    ctx = hisa.Context(params["log_n"], params["q_bits"], params["dnum"], params["special_bits"], seed=11)
    ctx.keygen()
    costs = nets.measure_costs(ctx, limbs)
    assert costs["rot_left"] > costs["add"] > 0 and costs["rot_shared"] <= 0 and costs["key_switch_calls"] > costs["rot_left"]
    best, est = nets.select_layout(ctx, layers, x, params["scale"], limbs, costs)
    flat = {lay: nets.estimate_cost(nets.analyse(ctx, layers, x, params["scale"], limbs, 0, lay)[0], costs, level_aware=False)
            for lay in est}
    print("unit costs (us):", {k: round(v * 1e6, 2) for k, v in costs.items() if isinstance(v, float)},
          "at the other levels (us):", {l: {k: round(v * 1e6, 2) for k, v in c.items()} for l, c in costs["levels"].items() if l != limbs},
          "estimates (ms):", {k: round(v * 1e3, 2) for k, v in est.items()},
          "at the top level's costs throughout (ms):", {k: round(v * 1e3, 2) for k, v in flat.items()}, flush=True)
    assert best == "chw_fc" and est["chw_fc"] < est["hw"] < est["chw"]
    # a key switch gets cheaper with every level the circuit descends: the level-aware figure is the lower one
    low = costs["levels"][2]
    assert low["rot_left"] < costs["rot_left"] and all(est[lay] < flat[lay] for lay in est)
    measured = {}
    for layout in nets.LAYOUTS:
        plans = {}
        nets.run_encrypted(ctx, layers, x, params["scale"], limbs, make_keys=True, plans=plans, layout=layout)
        measured[layout] = min(nets.run_encrypted(ctx, layers, x, params["scale"], limbs, plans=plans, layout=layout)[1]
                               for _ in range(3))
        nets.free_plans(ctx, plans)
    # The clock is printed, not asserted: wall-clock order on a shared machine is a measurement, not a property of the
    # code (bench.py reports the same figures per layout)
    print("measured (ms):", {k: round(v * 1e3, 2) for k, v in measured.items()},
          "ranking agrees:", measured["chw_fc"] < measured["hw"] < measured["chw"], flush=True)
    ctx.close()


def test_parameter_selection_gives_exactly_the_levels_the_network_needs():
    """The depth measured by the dry run is tight: LeNet-small runs (<= 1e-3) on the modulus chain the pass selects
    and runs out of levels with one prime fewer."""
    from paper_1810_00845_amd import hisa, nets
    from test_gpu_networks import plain_forward
    params, layers, x = nets.lenet_small()
    sel = nets.select_parameters(layers, x, params["log_n"], 40, dnum=params["dnum"], layout="chw_fc")
    assert sel["depth"] == 6 and sel["q_bits"] == [50] + [40] * 6 and not sel["secure_128"]   # 2^13 allows 218 bits
    want = plain_forward(layers, x)
    ctx = hisa.Context(sel["log_n"], sel["q_bits"], sel["dnum"], sel["special_bits"], seed=11)
    ctx.keygen()
    ctx.gen_rot_keys(sel["rot_steps"])
    got, _, _ = nets.run_encrypted(ctx, layers, x, sel["scale"], len(sel["q_bits"]), layout="chw_fc")
    assert np.abs(got - want).max() <= 1e-3
    ctx.close()
    short = hisa.Context(sel["log_n"], sel["q_bits"][:-1], sel["dnum"], sel["special_bits"], seed=11)
    short.keygen()
    with pytest.raises(hisa.HisaError):
        nets.run_encrypted(short, layers, x, sel["scale"], len(sel["q_bits"]) - 1, make_keys=True, layout="chw_fc")
    short.close()
