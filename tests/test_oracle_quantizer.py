"""Pins for the oracle's quantizer (Preliminary Eq. 1 applied per group) and byte format."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import decoquant_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pack_examples.txt")


def _fp16_candidates_near(x: float):
    c = np.float16(x)
    out = {c}
    for direction in (np.float16(np.inf), np.float16(-np.inf)):
        out.add(np.nextafter(c, direction))
    return [v for v in out if np.isfinite(v)]


def _exact_step(a32: np.float32, qmax: int) -> np.float16:
    """Round the exact rational a/qmax to fp16, ties to even, by exact comparisons."""
    target = Fraction(float(a32)) / qmax
    cands = _fp16_candidates_near(float(target))
    best = None
    for v in cands:
        err = abs(Fraction(float(v)) - target)
        even = (int(np.float16(v).view(np.uint16)) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, v)
    return np.float16(best[1])


def _exact_code(x32: np.float32, step16: np.float16, qmax: int) -> int:
    """argmin over every allowed integer of |x - step*c| in exact arithmetic, ties to even."""
    if float(step16) == 0.0:
        return 0
    x, s = Fraction(float(x32)), Fraction(float(step16))
    best = None
    for c in range(-qmax, qmax + 1):
        key = (abs(x - s * c), c % 2)        # even c wins a tie
        if best is None or key < best[0]:
            best = (key, c)
    return best[1]


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_steps_and_codes_match_exact_rational_brute_force(bits):
    qmax = (1 << (bits - 1)) - 1
    r = np.random.default_rng(100 + bits)
    group = 8
    kp = (r.standard_normal((24, 32)) * 0.05).astype(np.float32)
    # plant exact ties: x = step * (k + 1/2) for a power-of-two step
    kp[0, :8] = np.float32(0.25) * np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, qmax, 0.0], np.float32)
    kp[1, 8:16] = 0.0                                         # an all-zero group
    steps = O.group_steps(kp, group, qmax)
    codes = O.quantize_codes(kp, steps, group, qmax)
    for t in range(kp.shape[0]):
        for g in range(kp.shape[1] // group):
            a = np.abs(kp[t, g * group:(g + 1) * group]).max()
            want = _exact_step(a, qmax)
            assert steps[t, g].view(np.uint16) == want.view(np.uint16)
            for e in range(g * group, (g + 1) * group):
                assert codes[t, e] == _exact_code(kp[t, e], steps[t, g], qmax), (t, e)
    assert (codes[1, 8:16] == 0).all() and steps[1, 1] == 0
    if bits >= 4:
        # the planted ties round to even: 0.5->0, 1.5->2, 2.5->2
        assert list(codes[0, :6]) == [0, 2, 2, 0, -2, -2]


@pytest.mark.parametrize("bits,group", [(4, 128), (2, 64), (8, 32), (4, 64)])
def test_half_step_error_bound_and_code_range(bits, group):
    qmax = (1 << (bits - 1)) - 1
    r = np.random.default_rng(7)
    kp = (r.standard_normal((256, 128)) * 0.04).astype(np.float32)
    steps = O.group_steps(kp, group, qmax)
    codes = O.quantize_codes(kp, steps, group, qmax)
    assert codes.min() >= -qmax and codes.max() <= qmax
    deq = O.dequantize(codes, steps, group)
    delta = np.repeat(steps.astype(np.float64), group, axis=1)
    assert (steps.astype(np.float64) >= 2.0 ** -14).all()       # normal fp16 steps here
    assert (np.abs(deq - kp.astype(np.float64)) <= delta / 2).all()
    # the largest element of every group takes the extreme code
    idx = np.abs(kp).reshape(256, 128 // group, group).argmax(axis=2)
    top = np.take_along_axis(np.abs(codes).reshape(256, 128 // group, group), idx[..., None], axis=2)
    assert (top == qmax).all()


def test_subnormal_step_is_still_within_the_documented_bound():
    qmax = 7
    kp = np.full((1, 8), 3.1e-6, np.float32)
    kp[0, 3] = -2.9e-5
    steps = O.group_steps(kp, 8, qmax)
    assert 0 < float(steps[0, 0]) < 2.0 ** -14
    codes = O.quantize_codes(kp, steps, 8, qmax)
    err = np.abs(O.dequantize(codes, steps, 8) - kp.astype(np.float64))
    assert (err <= float(steps[0, 0]) / 2 + qmax * 2.0 ** -25).all()


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, codes, hexbytes = [p.strip() for p in line.split("|")]
            rows.append((int(bits), [int(c) for c in codes.split()],
                         [int(h, 16) for h in hexbytes.split()]))
    return rows


def test_packing_matches_hand_computed_bytes():
    rows = _golden_rows()
    assert len(rows) >= 4
    for bits, codes, want in rows:
        got = O.pack_rows(np.array([codes], np.int32), bits)[0]
        assert list(got) == want, (bits, codes)
        assert list(O.unpack_rows(np.array([want], np.uint8), bits)[0]) == codes


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_pack_round_trip(bits):
    qmax = (1 << (bits - 1)) - 1
    r = np.random.default_rng(3)
    c = r.integers(-qmax, qmax + 1, size=(5, 7, 64)).astype(np.int32)
    assert np.array_equal(O.unpack_rows(O.pack_rows(c, bits), bits), c)


def test_value_tile_layout_by_explicit_loops():
    j1, j2 = 4, 2
    n_tok = 2 * O.TILE_TOKENS
    c = np.arange(n_tok * j1 * j2, dtype=np.int32).reshape(n_tok, j1 * j2)
    tiles = O.value_codes_to_tiles(c, j1, j2)
    assert tiles.shape == (2, j2, j1, O.TILE_TOKENS)
    for tile in range(2):
        for b2 in range(j2):
            for r in range(j1):
                for tt in (0, 1, 63, 127):
                    assert tiles[tile, b2, r, tt] == c[tile * O.TILE_TOKENS + tt, r * j2 + b2]
    assert np.array_equal(O.value_tiles_to_codes(tiles), c)


def test_compression_ratio_closed_form_and_storage_bytes():
    # Section 3.3 Eq. 4, steps counted at 16 bits each; approximately B/16.
    fmt = O.Format(4, 128, 128, 16, 8, 128)
    mu = O.compression_ratio(fmt)
    assert abs(mu - (65536 + 4096 + 2048) / 262144) < 1e-15
    cache = O.empty_cache(fmt, 1, 1, 1)
    k_bytes = cache["k_codes"].nbytes + cache["k_scales"].nbytes + cache["k_small"].nbytes
    v_bytes = cache["v_codes"].nbytes + cache["v_scales"].nbytes + cache["v_small"].nbytes
    assert k_bytes == v_bytes == O.cache_bytes_per_block(fmt)
    assert abs(k_bytes / (128 * 128 * 2) - mu) < 1e-15
    for bits, group, tb in [(2, 64, 128), (4, 128, 1024), (8, 128, 256)]:
        f = O.Format(bits, group, 128, 16, 8, tb)
        assert abs(O.compression_ratio(f) - bits / 16) < 0.035
    # bytes per cached token per kv head, keys + values (the benchmark's algorithmic bytes)
    assert 2 * O.cache_bytes_per_block(fmt) / 128 == 140
    assert 2 * O.cache_bytes_per_block(O.Format(2, 64, 128, 16, 8, 128)) / 128 == 80


def test_compression_ratio_against_the_sizes_the_paper_prints():
    # Section 4.2, main results table, column "Size (MB)": 46.7 at 16 bits, 23.3 / 11.7 / 5.8 at
    # 8 / 4 / 2 bits, i.e. B/16 of the fp16 cache to the table's rounding.  Eq. 4 adds the small
    # tensor and the steps on top: a few percent of the fp16 size, never less than B/16.
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table_sizes.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                bits, mb = line.split()
                rows[int(bits)] = float(mb)
    for bits in (8, 4, 2):
        printed = rows[bits] / rows[16]
        assert abs(printed - bits / 16) <= 0.06 / rows[16] + 1e-12          # one unit of the last printed digit
        for group in (128, 64):
            mu = O.compression_ratio(O.Format(bits, group, 128, 16, 8, 128))
            overhead = (16 * 16 * 16 + 128 * (128 // group) * 16) / (128 * 128 * 16.0)
            assert abs(mu - (bits / 16 + overhead)) < 1e-15
            assert printed - 0.002 <= mu <= printed + 0.04
