"""Host-side bounds of the multiply-accumulate launches of the tensor kernels (Sec. "Runtime": convolution and matrix
multiplication over CipherTensors): the argument sets below never reach a GPU.  The refused ones include the set that
once ran past its buffers: a launch over ciphertexts of l limbs that had kept the l + K limbs (and entry size) of the
key-switch accumulators handled by the launch before it."""
import pytest

from paper_1810_00845_amd import hisa

ERR_ARG = -1          # HISA_ERR_ARG of include/hisa.h
LOG_N, N = 12, 1 << 12
L, K = 4, 2          # limbs of the inputs; special primes of the accumulators
B, IC, OC, TAPS = 2, 3, 5, 4


def good(**over):
    ctw = 2 * L * N
    a = dict(ic=IC, oc=OC, batch=B, log_n=LOG_N, limbs=L, polys=2, lq=0, gap=0, ct_words=ctw,
             out_words=B * OC * ctw, w_stride_t=OC, w_stride_oc=1, w_extent=TAPS * IC * OC * L * N)
    a.update(over)
    taps = a.pop("taps", [B * IC * ctw] * TAPS)
    return hisa.check_mac_extents(taps, **a)


def test_a_launch_that_fits_passes():
    assert good() == 0
    # one-polynomial entries, and the accumulators' layout: l + K limbs with the special primes after a gap
    acc = 2 * (L + K) * N
    assert good(limbs=L + K, lq=L, gap=6, ct_words=acc, taps=[B * IC * acc] * TAPS, out_words=B * OC * acc,
                w_extent=TAPS * IC * OC * (L + K) * N) == 0
    assert good(polys=1, ct_words=L * N, taps=[B * IC * L * N] * TAPS, out_words=B * OC * L * N) == 0


def test_inherited_accumulator_limbs_are_refused():
    """The earlier fault: buffers of l-limb ciphertexts, fields of the (l + K)-limb launch before."""
    acc = 2 * (L + K) * N
    # limbs alone inherited: an entry no longer holds what the kernel walks over
    assert good(limbs=L + K, lq=L, gap=6) != 0
    # limbs and entry size inherited: entries are consistent, the buffers behind them are not
    assert good(limbs=L + K, lq=L, gap=6, ct_words=acc, w_extent=TAPS * IC * OC * (L + K) * N) != 0
    # the same with inputs that are large enough: the output still is not
    assert good(limbs=L + K, lq=L, gap=6, ct_words=acc, taps=[B * IC * acc] * TAPS,
                w_extent=TAPS * IC * OC * (L + K) * N) != 0


@pytest.mark.parametrize("short", ["tap", "last_tap", "out", "w", "x2", "out2", "batch"])
def test_every_buffer_is_checked(short):
    ctw = 2 * L * N
    full = B * IC * ctw
    x2 = dict(lq=L, x2_words=L * N, x2_tap_words=B * IC * L * N, x2_extent=TAPS * B * IC * L * N, out2_extent=B * OC * L * N)
    assert good(**x2) == 0
    if short == "tap":
        assert good(taps=[full - 1] + [full] * (TAPS - 1)) != 0
    elif short == "last_tap":      # a rotated copy that starts inside a larger block: what is left behind it counts
        assert good(taps=[full] * (TAPS - 1) + [full - N]) != 0
    elif short == "out":
        assert good(out_words=B * OC * ctw - 1) != 0
    elif short == "w":
        assert good(w_extent=TAPS * IC * OC * L * N - 1) != 0
    elif short == "x2":
        assert good(**dict(x2, x2_extent=x2["x2_extent"] - 1)) != 0
    elif short == "out2":
        assert good(**dict(x2, out2_extent=x2["out2_extent"] - 1)) != 0
    else:
        assert good(batch=B + 1) != 0


def test_error_code_is_the_argument_error():
    assert good(out_words=1) == ERR_ARG
