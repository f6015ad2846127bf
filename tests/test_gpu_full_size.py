"""Parity at the benchmark's full size and launch configuration: batch of 64 ciphertexts, N = 2^15, 16 limbs of
50-bit primes, dnum 3 (and dnum 1), the same batched calls bench.py times.  The oracle recomputes a sample of the
outputs one by one; the comparison is bit for bit in coefficient form."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dnum,sample", [(3, (0, 37, 63)), (1, (5,))])
def test_rot_left_batch_at_benchmark_size(dnum, sample):
    from oracle import Oracle
    from paper_1810_00845_amd import hisa, synth
    log_n, L, bits, B, seed = 15, 16, 50, 64, 1
    g = hisa.Context(log_n, [bits] * L, dnum, bits, seed)
    o = Oracle(log_n, [bits] * L, dnum, bits, seed)
    assert g.primes == o.primes
    steps = [1, 64]
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    # synthetic ciphertexts: residues uniform in [0, q_i), imported in coefficient form on both sides
    coeff = synth.uniform_residues(7, (B, 2, L, g.N), g.primes[:L])
    gcts = g.ct_import_batch(coeff, 2.0 ** 50)
    for r in steps:
        print("[case] dnum", dnum, "rotLeft", r, flush=True)
        gout = g.rot_left_batch(gcts, r)
        for i in sample if r == 1 else sample[:1]:
            want = o.export(o.rot_left(o.import_ct(coeff[i], 2.0 ** 50), r))
            assert np.array_equal(g.ct_export(gout[i]), want), "ciphertext %d differs" % i
        for c in gout:
            c.free()
    # a lower level (ragged last digit) in the same launch configuration
    low = g.ct_import_batch(coeff[:, :, :11], 2.0 ** 50)
    gout = g.rot_left_batch(low, 1)
    i = sample[0]
    assert np.array_equal(g.ct_export(gout[i]), o.export(o.rot_left(o.import_ct(coeff[i][:, :11], 2.0 ** 50), 1)))
    g.close()


def test_relinearize_rescale_batch_at_benchmark_size():
    from oracle import Oracle
    from paper_1810_00845_amd import hisa, synth
    log_n, L, bits, B, seed = 15, 16, 50, 64, 1
    g = hisa.Context(log_n, [bits] * L, 3, bits, seed)
    o = Oracle(log_n, [bits] * L, 3, bits, seed)
    g.keygen(); o.keygen()
    coeff = synth.uniform_residues(8, (B, 2, L, g.N), g.primes[:L])
    gcts = g.ct_import_batch(coeff, 2.0 ** 50)
    prod = g.mul_no_relin_batch(gcts, gcts[1:] + gcts[:1])
    g.relinearize_batch(prod)
    g.rescale_batch(prod)
    for i in (0, 63):
        a, b = o.import_ct(coeff[i], 2.0 ** 50), o.import_ct(coeff[(i + 1) % B], 2.0 ** 50)
        want = o.rescale(o.mul(a, b))
        assert np.array_equal(g.ct_export(prod[i]), o.export(want))
        assert abs(prod[i].scale - want.scale) <= 1e-12 * want.scale
    g.close()


def test_rotation_sums_at_benchmark_size():
    """hisa_rot_left_sum_batch on 64 outputs of three terms each at N = 2^15, 16 limbs (the launch that keeps a
    rotation's key rows across sixteen outputs), distinct terms and terms that rotate one ciphertext; sampled outputs
    against the oracle's sum of key-switch accumulators, bit for bit."""
    from oracle import Oracle
    from oracle.layers import SharedModDown
    from paper_1810_00845_amd import hisa, synth
    log_n, L, bits, B, seed = 15, 16, 50, 64, 1
    g = hisa.Context(log_n, [bits] * L, 3, bits, seed)
    o = Oracle(log_n, [bits] * L, 3, bits, seed)
    steps = [1, 0, 64]
    g.gen_rot_keys([1, 64]); o.gen_rot_keys([1, 64])
    coeff = synth.uniform_residues(9, (B, 2, L, g.N), g.primes[:L])
    gcts = g.ct_import_batch(coeff, 2.0 ** 50)
    terms = [gcts, gcts[1:] + gcts[:1], gcts[2:] + gcts[:2]]
    print("[case] distinct terms", flush=True)
    out = g.rot_left_sum_batch(terms, steps)
    for i in (0, 17, 63):
        ins = [o.import_ct(coeff[(i + s) % B], 2.0 ** 50) for s in range(3)]
        want = SharedModDown(o, ins).total([(s, steps[s], 1, None) for s in range(3)], ins[0].scale)
        assert np.array_equal(g.ct_export(out[i]), o.export(want)), "output %d differs" % i
    print("[case] one ciphertext per output", flush=True)
    out = g.rot_left_sum_batch([gcts, gcts, gcts], steps)
    i = 41
    x = o.import_ct(coeff[i], 2.0 ** 50)
    want = SharedModDown(o, [x]).total([(0, r, 1, None) for r in steps], x.scale)
    assert np.array_equal(g.ct_export(out[i]), o.export(want))
    g.close()


def test_other_primitives_at_benchmark_size():
    """The remaining primitives bench.py times under `ops`, in the same batched calls at the same size (64 ciphertexts,
    N = 2^15, 16 limbs, dnum 3): raw forward / inverse transforms of 64 x 2 x 16 limb-polynomials in one call, add,
    mulPlain, mulNoRelin, rescale of the batch, and three rotations of every ciphertext from one decomposition;
    sampled entries against the oracle, bit for bit."""
    import torch
    from oracle import Oracle
    from paper_1810_00845_amd import hisa, synth
    log_n, L, bits, B, seed = 15, 16, 50, 64, 1
    g = hisa.Context(log_n, [bits] * L, 3, bits, seed)
    o = Oracle(log_n, [bits] * L, 3, bits, seed)
    N = g.N
    print("[case] raw transforms", flush=True)
    q0 = g.primes[0]
    polys = synth.uniform_residues(10, (B * 2 * L, 1, N), [q0])[:, 0, :]
    t = torch.from_numpy(polys.view(np.int64)).cuda()
    g.ntt_raw(t, 0)
    got = t.cpu().numpy().view(np.uint64)
    for i in (0, 777, B * 2 * L - 1):
        assert np.array_equal(got[i], o.ntt(polys[i], 0)), "transform %d differs" % i
    g.ntt_raw(t, 0, inverse=True)
    assert np.array_equal(t.cpu().numpy().view(np.uint64), polys)
    del t
    coeff = synth.uniform_residues(11, (B, 2, L, N), g.primes[:L])
    gcts = g.ct_import_batch(coeff, 2.0 ** 50)
    oct_ = lambda i: o.import_ct(coeff[i % B], 2.0 ** 50)
    shifted = gcts[1:] + gcts[:1]
    print("[case] add, mulPlain, mulNoRelin, rescale", flush=True)
    pt_co = synth.plaintext_coeffs(12, N, 40)
    gp, op = g.pt_from_coeffs(pt_co, 2.0 ** 50, L), o.pt_from_coeffs(pt_co, 2.0 ** 50, L)
    gadd, gmp, gmn = g.add_batch(gcts, shifted), g.mul_plain_batch(gcts, gp), g.mul_no_relin_batch(gcts, shifted)
    gres = g.add_batch(gcts, shifted)
    g.rescale_batch(gres)
    for i in (0, 29, 63):
        a, b = oct_(i), oct_(i + 1)
        assert np.array_equal(g.ct_export(gadd[i]), o.export(o.add(a, b)))
        assert np.array_equal(g.ct_export(gmp[i]), o.export(o.mul_plain(a, op)))
        assert np.array_equal(g.ct_export(gmn[i]), o.export(o.mul_no_relin(a, b)))
        assert np.array_equal(g.ct_export(gres[i]), o.export(o.rescale(o.add(a, b))))
    for xs in (gadd, gmp, gmn, gres):
        for c in xs:
            c.free()
    print("[case] three rotations from one decomposition", flush=True)
    steps = [1, 7, 64]
    g.gen_rot_keys(steps); o.gen_rot_keys(steps)
    rows = g.rot_left_hoisted_batch(gcts, steps)
    for s, i in ((0, 3), (1, 40), (2, 63)):
        assert np.array_equal(g.ct_export(rows[s][i]), o.export(o.rot_left(oct_(i), steps[s]))), "rotation %d of %d" % (steps[s], i)
    g.close()
