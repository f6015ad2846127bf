"""Parity at the other points of the primitive sweep, in the launch configuration bench.py times there: batches of 64
ciphertexts at N = 2^14 and 2^13 with 16 and 8 limbs, dnum 3 and 1.  The launcher picks other instantiations of the
transform kernel at these sizes than at N = 2^15 (two target limbs per conversion pass or one, by the number of
rounds of workgroups), so the test also reads the per-kernel timing records and checks that the paired form ran
where the rule selects it.  Sampled outputs are compared bit for bit with the oracle."""
import re

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

# (log_n, limbs, dnum, modes whose conversions must have run two targets per pass)
POINTS = [
    (14, 16, 3, {3, 6}),
    (14, 16, 1, {3, 6}),
    (13, 16, 1, {6}),
    (14, 8, 3, {3, 6}),
    (13, 8, 1, set()),
]


@pytest.mark.parametrize("log_n,L,dnum,paired_modes", POINTS)
def test_rot_left_batch_at_sweep_point(log_n, L, dnum, paired_modes):
    from oracle import Oracle
    from paper_1810_00845_amd import hisa, synth
    bits, B, seed = 50, 64, 3
    print("[case] N=2^%d L=%d dnum=%d batch %d" % (log_n, L, dnum, B), flush=True)
    g = hisa.Context(log_n, [bits] * L, dnum, bits, seed)
    o = Oracle(log_n, [bits] * L, dnum, bits, seed)
    try:
        assert g.primes == o.primes
        g.keygen(); o.keygen()
        g.gen_rot_keys([7]); o.gen_rot_keys([7])
        coeff = synth.uniform_residues(40 + log_n + L + dnum, (B, 2, L, g.N), g.primes[:L])
        gcts = g.ct_import_batch(coeff, 2.0 ** 50)
        g.profile_enable(True)
        gout = g.rot_left_batch(gcts, 7)
        names = set(g.profile_read())
        g.profile_enable(False)
        # which instantiations ran: "ntt_fp_kernel<log2 N - 10, mode, two targets per pass>"
        ran = {(int(m.group(2)), m.group(3) == "true") for m in (re.match(r"ntt_fp_kernel<(\d+), (\d+), (true|false)>", n)
                                                                for n in names) if m}
        assert {m for m, _ in ran} == {2, 3, 5, 6}, names
        for mode in paired_modes:
            assert (mode, True) in ran, (mode, names)
        for i in (0, 41):
            want = o.export(o.rot_left(o.import_ct(coeff[i], 2.0 ** 50), 7))
            assert np.array_equal(g.ct_export(gout[i]), want), "ciphertext %d differs" % i
        # relinearize + rescale through the same kernels (mode 4 of the rescale included)
        prod = g.mul_no_relin_batch(gcts, gcts[1:] + gcts[:1])
        g.relinearize_batch(prod)
        g.rescale_batch(prod)
        a, b = o.import_ct(coeff[5], 2.0 ** 50), o.import_ct(coeff[6], 2.0 ** 50)
        want = o.rescale(o.mul(a, b))
        assert np.array_equal(g.ct_export(prod[5]), o.export(want))
    finally:
        g.close()
