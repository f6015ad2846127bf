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
