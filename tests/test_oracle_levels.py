"""Pins for the oracle's non-default level set (format field `levels` = 1): all 2^m codes,
c in [-2^(m-1), 2^(m-1) - 1] ({-2, -1, 0, +1} at 2 bits), step sized so that neither end clips.
Not the paper's quantizer (Preliminary, Eq. 1 is symmetric and stays the default); pinned against
exact rational arithmetic, the half-step bound, and the symmetric quantizer it must never lose to."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import decoquant_oracle as O
from test_oracle_quantizer import _exact_step


def _exact_code(x32, step16, lo, hi):
    """argmin over every allowed integer of |x - step*c| in exact arithmetic, ties to even."""
    if float(step16) == 0.0:
        return 0
    x, s = Fraction(float(x32)), Fraction(float(step16))
    return min(range(lo, hi + 1), key=lambda c: (abs(x - s * c), c % 2))


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_steps_and_codes_match_exact_rational_brute_force(bits):
    qmax = (1 << (bits - 1)) - 1
    r = np.random.default_rng(300 + bits)
    group = 8
    kp = (r.standard_normal((32, 32)) * 0.05).astype(np.float32)
    kp[0, :8] = np.float32(0.25) * np.array([0.5, 1.5, -0.5, -1.5, -2.5, -(qmax + 1), qmax, 0.0], np.float32)
    kp[1, 8:16] = 0.0                                         # an all-zero group
    kp[2, :8] = -np.abs(kp[2, :8])                            # one-sided groups
    kp[3, :8] = np.abs(kp[3, :8])
    steps = O.group_steps(kp, group, qmax, full_range=True)
    codes = O.quantize_codes(kp, steps, group, qmax, full_range=True)
    for t in range(kp.shape[0]):
        for g in range(kp.shape[1] // group):
            x = kp[t, g * group:(g + 1) * group]
            up = _exact_step(np.float32(max(x.max(), 0.0)), qmax)
            down = _exact_step(np.float32(max((-x).max(), 0.0)), qmax + 1)
            want = max(up, down)
            assert steps[t, g].view(np.uint16) == want.view(np.uint16), (t, g)
            for e in range(g * group, (g + 1) * group):
                assert codes[t, e] == _exact_code(kp[t, e], steps[t, g], -qmax - 1, qmax), (t, e)
    assert (codes[1, 8:16] == 0).all() and steps[1, 1] == 0
    if bits >= 4:
        # the planted group: step 0.25 exactly, both ends reached, ties to even
        assert float(steps[0, 0]) == 0.25
        assert list(codes[0, :8]) == [0, 2, 0, -2, -2, -(qmax + 1), qmax, 0]
    else:
        # 2 bits: max(x) = 0.375 sets the step (0.375 / 1 against 0.625 / 2); -0.625 / 0.375 = -1.67 -> -2
        assert float(steps[0, 0]) == 0.375
        assert list(codes[0, :8]) == [0, 1, 0, -1, -2, -1, 1, 0]
    # a group without positive values gets the finer step max(-x) / 2^(m-1)
    assert float(steps[2, 0]) == float(_exact_step(np.float32((-kp[2, :8]).max()), qmax + 1))


@pytest.mark.parametrize("bits,group", [(4, 128), (2, 64), (8, 32), (2, 128)])
def test_half_step_bound_holds_at_both_ends_and_the_step_never_exceeds_the_symmetric_one(bits, group):
    qmax = (1 << (bits - 1)) - 1
    r = np.random.default_rng(17)
    kp = (r.standard_normal((256, 128)) * 0.04).astype(np.float32)
    kp[:8, ::group] = -1.0                                   # groups whose largest magnitude is negative by far
    steps = O.group_steps(kp, group, qmax, full_range=True)
    codes = O.quantize_codes(kp, steps, group, qmax, full_range=True)
    assert codes.min() == -qmax - 1 and codes.max() == qmax
    deq = O.dequantize(codes, steps, group)
    delta = np.repeat(steps.astype(np.float64), group, axis=1)
    # no clipping at either end: the half-step bound holds for every element (plus the fp16
    # rounding of the step itself at the extreme codes: at most 2^-11 * (qmax + 1) steps)
    slack = delta * (qmax + 1) * 2.0 ** -11
    assert (np.abs(deq - kp.astype(np.float64)) <= delta / 2 + slack).all()
    sym = O.group_steps(kp, group, qmax)
    assert (steps <= sym).all() and (steps < sym).any()
    # where the largest magnitude of a group is negative the step is qmax / (qmax + 1) of the symmetric one
    x = kp.reshape(256, 128 // group, group)
    neg_dominant = (-x).max(axis=2) * qmax > x.max(axis=2) * (qmax + 1)
    assert neg_dominant[:8].all()
    ratio = steps.astype(np.float64)[neg_dominant] / sym.astype(np.float64)[neg_dominant]
    assert np.abs(ratio - qmax / (qmax + 1)).max() <= 2.0 ** -10


def test_quantization_error_is_lower_than_symmetric_at_two_bits():
    """What the extra level buys: mean squared error of a 2-bit group quantizer on Gaussian data."""
    r = np.random.default_rng(23)
    kp = (r.standard_normal((512, 128)) * 0.03).astype(np.float32)
    err = {}
    for full in (False, True):
        steps = O.group_steps(kp, 64, 1, full_range=full)
        codes = O.quantize_codes(kp, steps, 64, 1, full_range=full)
        err[full] = float(((O.dequantize(codes, steps, 64) - kp) ** 2).mean())
    assert err[True] < 0.85 * err[False]


@pytest.mark.parametrize("bits", [2, 4])
def test_block_round_trip_with_all_codes(bits):
    """compress_block / storage / reconstruct with levels = 1: the stored field 0 (code -2^(m-1))
    survives packing, and the reconstruction obeys the same half-step bound as the default."""
    fmt = O.Format(bits, 64, 128, 16, 8, 128, 1, 1)
    r = np.random.default_rng(5)
    x = (r.standard_normal((128, 128)) * np.exp(0.5 * r.standard_normal((128, 1)))).astype(np.float16)
    x[:, [3, 77]] *= 20
    blk = O.compress_block(x, fmt)
    assert blk.codes.min() == -(1 << (bits - 1)) and blk.codes.max() == (1 << (bits - 1)) - 1
    assert np.array_equal(O.unpack_rows(O.pack_rows(blk.codes, bits), bits), blk.codes)
    cache = O.empty_cache(fmt, 1, 1, 1)
    O.compress_sequence(cache, fmt, 0, 0, x, x)
    k_hat, _ = O.reconstruct_sequence(cache, fmt, 0, 0, 128)
    bound = O.reconstruction_bound(blk.small, blk.steps, fmt)
    t_l = np.abs(O.token_major_to_large(blk.large32.astype(np.float64), 16, 8))
    slack = O.unmatricise(2.0 ** -10 * np.abs(blk.small.astype(np.float64)) @ t_l, 128, 128, 1, 16)
    step_slack = O.unmatricise(np.abs(blk.small.astype(np.float64)) @ O.token_major_to_large(
        np.repeat(blk.steps.astype(np.float64), 64, axis=1) * (1 << (bits - 1)) * 2.0 ** -11, 16, 8), 128, 128, 1, 16)
    assert (np.abs(k_hat - x.astype(np.float64)) <= bound + slack + step_slack + 1e-9).all()
    # and it is closer to the block than the symmetric default
    sym = O.compress_block(x, O.Format(bits, 64, 128, 16, 8, 128))
    e_full = np.linalg.norm(O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt) - x.astype(np.float64))
    e_sym = np.linalg.norm(O.reconstruct_block(sym.small, sym.steps, sym.codes, fmt) - x.astype(np.float64))
    assert e_full < e_sym
