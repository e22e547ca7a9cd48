"""Pins for the 2-bit quantiser and the (index, code) pair format.

The paper names Q() and never defines it (section 2.1; section 3 says its experiments
used no quantisation), so nothing here checks the rule against the paper:
"parity unpinned" for that.  What is pinned is the rule as this repository
reads it -- hand-computed cases with exactly representable numbers, the closed
form for a zero range, the error bound d/4, and the bit layout of a pair.
"""
import json
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def quantise_chunk(x, kappa, chunk=None):
    chunk = chunk or x.size
    e = np.zeros_like(x)
    pairs, scales = oracle.compress([e], kappa, 1.0, delta=[x], chunk=chunk, quant=True)
    return e, pairs, scales


def test_hand_computed_levels_codes_and_residuals():
    # selected magnitudes {1, 2, 3, 5}: amin 1, amax 5, d 4 -> lo = 2, tau = 3, hi = 4
    x = np.array([0.5, -1.0, 0.25, 2.0, -3.0, 0.0, 5.0, 0.75], np.float32)
    e, pairs, scales = quantise_chunk(x, 4)
    assert scales.tolist() == [2.0, 4.0]
    # idx 1: -1 -> sign 1, low  -> code 2, q = -2, residual  1
    # idx 3: +2 -> sign 0, low  -> code 0, q = +2, residual  0
    # idx 4: -3 -> sign 1, high (3 >= tau) -> code 3, q = -4, residual 1
    # idx 6: +5 -> sign 0, high -> code 1, q = +4, residual 1
    assert pairs.tolist() == [1 | 2 << 12, 3 | 0 << 12, 4 | 3 << 12, 6 | 1 << 12]
    assert e.tolist() == [0.5, 1.0, 0.25, 0.0, 1.0, 0.0, 1.0, 0.75]
    dense = oracle.decode([8], pairs, scales, 4, chunk=8)[0]
    assert dense.tolist() == [0, -2.0, 0, 2.0, -4.0, 0, 4.0, 0]


def test_zero_range_sends_the_values_exactly():
    x = np.array([0.1, -0.7, 0.7, 0.2, -0.7, 0.3], np.float32)
    e, pairs, scales = quantise_chunk(x, 3)
    a = np.float32(0.7)
    assert scales[0] == a and scales[1] == a
    idx, code, valid = oracle.unpack(pairs)
    assert idx.tolist() == [1, 2, 4] and code.tolist() == [3, 1, 3]      # a >= tau holds with equality
    assert e[[1, 2, 4]].tolist() == [0.0, 0.0, 0.0]
    # kappa_c = 1 is the same closed form
    e, pairs, scales = quantise_chunk(x, 1)
    assert scales.tolist() == [a, a] and e[1] == 0.0 and e[2] == a


def test_all_zero_chunk():
    x = np.zeros(16, np.float32)
    x[3] = -0.0
    e, pairs, scales = quantise_chunk(x, 4)
    assert scales.tolist() == [0.0, 0.0]
    idx, code, valid = oracle.unpack(pairs)
    assert idx.tolist() == [0, 1, 2, 3]
    assert code.tolist() == [1, 1, 1, 1]       # 1*0 + (-0) = +0 before selection, so no sign bit survives
    assert not e.any()


@pytest.mark.parametrize("seed", range(4))
def test_quantisation_error_bound_sign_and_level_order(seed):
    rng = np.random.default_rng(seed)
    chunk, kappa, n = 256, 16, 256 * 9 + 40
    x = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    e, pairs, scales = quantise_chunk(x, kappa, chunk)
    dense = oracle.decode([n], pairs, scales, kappa, chunk=chunk)[0]
    idx, code, valid = oracle.unpack(pairs)
    for c in range((n + chunk - 1) // chunk):
        lo, hi = scales[2 * c], scales[2 * c + 1]
        assert 0 <= lo <= hi
        sl = slice(c * chunk, min((c + 1) * chunk, n))
        sel = idx[c * kappa:(c + 1) * kappa][valid[c * kappa:(c + 1) * kappa]]
        xs = x[sl][sel]
        q = dense[sl][sel]
        amin, amax = np.abs(xs).min(), np.abs(xs).max()
        d = np.float64(amax) - np.float64(amin)
        assert np.all(np.signbit(q) == np.signbit(xs))
        assert np.all((np.abs(q) == lo) | (np.abs(q) == hi))
        ulp = np.spacing(np.float32(amax)).astype(np.float64)
        assert np.all(np.abs(xs.astype(np.float64) - q) <= d / 4 + 2 * ulp)
        # residual plus what was sent gives back the folded value (one rounding)
        assert np.all(np.abs((e[sl][sel].astype(np.float64) + q) - xs) <= ulp)
        # levels sit at the quarter points of the selected range
        assert abs(lo - (amin + d / 4)) <= 2 * ulp and abs(hi - (amin + 3 * d / 4)) <= 2 * ulp


def test_pair_bit_layout_exhaustive_round_trip():
    """All 4096 x 4 (index, code) combinations: index in bits 0-11, code in bits
    12-13 (bit 13 = sign, bit 12 = high level), bits 14-15 zero."""
    chunk, lo, hi = 4096, np.float32(0.5), np.float32(2.0)
    level = {0: lo, 1: hi, 2: -lo, 3: -hi}
    for code in range(4):
        pairs = (np.arange(4096, dtype=np.uint32) | (code << 12)).astype(np.uint16)
        assert not (pairs >> 14).any()
        # one pair per chunk, kappa = 1, 4096 chunks
        scales = np.tile(np.array([lo, hi], np.float32), 4096)
        dense = oracle.decode([4096 * chunk], pairs, scales, 1, chunk=chunk)[0].reshape(4096, chunk)
        rows = np.arange(4096)
        assert np.all(dense[rows, rows] == level[code])
        dense[rows, rows] = 0
        assert not dense.any()
        i2, c2, v2 = oracle.unpack(pairs)
        assert np.array_equal(i2, rows) and np.all(c2 == code) and v2.all()


def test_compress_emits_those_bits():
    x = np.zeros(4096, np.float32)
    x[4095] = -3.0
    x[0] = 1.0
    e, pairs, scales = quantise_chunk(x, 2)
    assert pairs.tolist() == [0x0000, 0x3FFF]            # +1 low -> code 0; -3 high -> code 3 at index 4095
    assert scales.tolist() == [1.5, 2.5]


def test_padding_only_after_kappa_c():
    chunk, kappa = 16, 5
    x = np.arange(1, 16 + 3 + 1, dtype=np.float32)         # second chunk has 3 elements
    e, pairs, scales = quantise_chunk(x, kappa, chunk)
    assert np.all(pairs[:5] != 0xFFFF) and np.all(pairs[5:8] != 0xFFFF) and np.all(pairs[8:] == 0xFFFF)
    assert (pairs[5:8] & 0xFFF).tolist() == [0, 1, 2]


def test_worked_example_fixture():
    """A two-replica, one-chunk example (chunk 8, kappa 3) worked through by hand
    from the update equations of section 2.1 under this repository's readings;
    inputs and expected bit patterns live in tests/golden/worked_example.json."""
    with open(os.path.join(HERE, "golden", "worked_example.json")) as f:
        g = json.load(f)
    hx = lambda xs: np.array([int(s, 16) for s in xs], np.uint32)
    theta_o = np.array(g["theta_outer"], np.float32)
    pairs, scales = [], []
    for rep in g["replicas"]:
        dec = np.array(rep["delta_decimal"], np.float32)
        theta_l = (theta_o - dec).astype(np.float32)
        e = np.array(rep["ef"], np.float32)
        p, s = oracle.compress([e], g["kappa"], g["beta"], theta_outer=[theta_o], theta_local=[theta_l],
                               chunk=g["chunk"])
        assert np.array_equal(p.astype(np.uint32), hx(rep["pairs"]))
        assert np.array_equal(s.view(np.uint32), hx(rep["scales_bits"]))
        assert np.array_equal(e.view(np.uint32), hx(rep["ef_after_bits"]))
        pairs.append(p), scales.append(s)
    dbar = oracle.aggregate([8], pairs, scales, g["kappa"], chunk=g["chunk"])[0]
    assert np.array_equal(dbar.view(np.uint32), hx(g["delta_bar_bits"]))
    th = theta_o.copy()
    oracle.outer_update([th], [dbar], g["outer_lr"])
    assert np.array_equal(th.view(np.uint32), hx(g["theta_after_bits"]))
    # tie checks on replica 0: index 0 beats index 4 at equal magnitude
    rep = g["replicas"][0]
    theta_l = (theta_o - np.array(rep["delta_decimal"], np.float32)).astype(np.float32)
    for kappa, want in ((1, [0]), (2, [0, 4])):
        e = np.array(rep["ef"], np.float32)
        p, _ = oracle.compress([e], kappa, g["beta"], theta_outer=[theta_o], theta_local=[theta_l], chunk=8)
        assert (p & 0xFFF).tolist() == want
