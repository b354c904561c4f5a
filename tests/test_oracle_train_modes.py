"""Pins for the oracle's alternative pulse-train generators: a train length chosen per update
vector and trains without randomness, both of which arXiv 2104.02184 Sec. 3 names beside the
stochastic fixed-length trains without giving their rules.  Expected values: exact integer/rational closed forms, the
Hammersley discrepancy bound, and the unchanged mean update."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import DETERMINISTIC, STOCHASTIC, TAG_D, TAG_X, DeviceParams

BITS = (1 << 63) - 1


def popcount(v):
    return bin(int(v) & BITS).count("1")


# ------------------------------------------------------------------ variable length
def test_dynamic_train_length_is_the_shortest_that_keeps_probabilities_below_one():
    g = np.random.default_rng(0)
    lr, dw_min, BL = 0.1, 0.001, 63
    x = g.normal(size=(40, 50)).astype(np.float32)
    d = (g.normal(size=(40, 30)) * g.uniform(0.0005, 0.2, size=(40, 1))).astype(np.float32)
    a_x, a_d, bl = oracle.line_scale_ex(x, d, lr, dw_min, BL, True, True)
    for b in range(40):
        mx, md = float(np.abs(x[b]).max()), float(np.abs(d[b]).max())
        need = Fraction(np.float32(lr).item()) * Fraction(mx) * Fraction(md) / Fraction(np.float32(dw_min).item())
        want = min(BL, max(1, math.ceil(need)))
        assert abs(int(bl[b]) - want) <= (1 if abs(need - round(need)) < 1e-9 else 0)
        A2 = np.float32(lr).item() / (np.float32(dw_min).item() * int(bl[b]))
        assert a_x[b] * a_d[b] == pytest.approx(A2, rel=1e-12)
        assert a_x[b] * mx == pytest.approx(a_d[b] * md, rel=1e-12)
        if want < BL:
            assert a_x[b] * mx <= 1.0 + 1e-12                  # no probability saturates
            if want > 1:                                        # and one pulse fewer would not do
                assert math.sqrt(A2 * int(bl[b]) / (int(bl[b]) - 1) * mx * md) > 1.0 - 1e-12
    assert bl.min() < BL and bl.max() == BL                     # the inputs exercise both regimes
    # fixed length: every sample gets BL
    _, _, bl_fixed = oracle.line_scale_ex(x, d, lr, dw_min, BL, True, False)
    assert (bl_fixed == BL).all()


def test_dynamic_length_words_have_no_pulses_beyond_their_length_and_keep_the_mean():
    lr, dw_min, BL = 0.1, 0.01, 31
    x = np.array([[0.3, -0.2, 0.1]], dtype=np.float32)
    d = np.array([[0.4, -0.25]], dtype=np.float32)
    _, _, bl = oracle.line_scale_ex(x, d, lr, dw_min, BL, True, True)
    assert 1 <= bl[0] < BL
    B = 20000
    xs, ds = np.tile(x, (B, 1)), np.tile(d, (B, 1))
    xw, dw = oracle.pulse_words(xs, ds, lr, dw_min, BL, True, 3, 0, dynamic_bl=True)
    high = np.uint64(((1 << 63) - 1) ^ ((1 << int(bl[0])) - 1))
    assert not (xw & high).any() and not (dw & high).any()
    # mean signed count * dw_min = -lr * d_i * x_j, as with the fixed length
    mask = np.uint64((1 << BL) - 1)
    for i in range(2):
        for j in range(3):
            n = np.array([popcount(v) for v in (xw[:, j] & dw[:, i] & mask)], dtype=float)
            mean = n.mean() * dw_min
            want = lr * abs(float(x[0, j]) * float(d[0, i]))
            p = want / (dw_min * int(bl[0]))
            sd = dw_min * math.sqrt(int(bl[0]) * p * (1 - p) / B)
            assert abs(mean - want) < 4.5 * sd + 1e-7


# ------------------------------------------------------------------ deterministic trains
def test_deterministic_column_train_is_evenly_spaced():
    for BL in (1, 7, 31, 63):
        for p in (0.0, 0.01, 0.2, 0.5, 0.77, 0.999, 1.0):
            T = oracle.threshold(p, 1.0)
            word = oracle.pulse_word_deterministic(TAG_X, p, 1.0, BL)
            want = sum(1 << n for n in range(BL) if Fraction(2 * n + 1, 2 * BL) < Fraction(T, 2**32))
            assert word == want
            assert abs(popcount(word) - BL * T / 2**32) <= 0.5 + 1e-9      # rounding of BL*p
            if popcount(word) > 1:                                          # evenly spaced: a prefix
                assert word == (1 << popcount(word)) - 1
    assert oracle.pulse_word_deterministic(TAG_X, 0.5, -1.0, 8) == 0b1111 | (1 << 63)


def test_deterministic_row_train_follows_the_bit_reversed_sequence():
    BL = 63
    # u_n = reversed bits of n as a binary fraction with every other digit flipped (0.101010..):
    # threshold 1/2: exactly the odd pulse numbers; 1/4: n % 4 == 1; 3/4: all but n % 4 == 2
    assert oracle.pulse_word_deterministic(TAG_D, 0.5, 1.0, BL) == sum(1 << n for n in range(BL) if n % 2 == 1)
    assert oracle.pulse_word_deterministic(TAG_D, 0.25, 1.0, BL) == sum(1 << n for n in range(BL) if n % 4 == 1)
    assert oracle.pulse_word_deterministic(TAG_D, 0.75, 1.0, BL) == sum(1 << n for n in range(BL) if n % 4 != 2)
    assert oracle.pulse_word_deterministic(TAG_D, 1.0, -2.0, BL) == ((1 << BL) - 1) | (1 << 63)
    assert oracle.pulse_word_deterministic(TAG_D, 0.3, 0.0, BL) == 0
    for BL2 in (5, 31, 63):
        for p in (0.1, 0.33, 0.9):
            T = oracle.threshold(p, 1.0)
            word = oracle.pulse_word_deterministic(TAG_D, p, 1.0, BL2)
            want = sum(1 << n for n in range(BL2) if (int(f"{n:032b}"[::-1], 2) ^ 0xAAAAAAAA) < T)
            assert word == want
            assert abs(popcount(word) - BL2 * p) <= 1.5


def test_deterministic_coincidences_track_BL_px_pd_within_the_discrepancy():
    BL = 63
    worst, bias, cnt = 0.0, 0.0, 0
    for px in np.linspace(0.02, 1.0, 29):
        for pd in np.linspace(0.02, 1.0, 31):
            xw = oracle.pulse_word_deterministic(TAG_X, float(px), 1.0, BL)
            dw = oracle.pulse_word_deterministic(TAG_D, float(pd), 1.0, BL)
            err = popcount(xw & dw) - BL * float(px) * float(pd)
            worst = max(worst, abs(err))
            bias += err
            cnt += 1
    assert worst <= 2.0                        # within the discrepancy of the 64-point shifted Hammersley set
    assert abs(bias / cnt) < 0.15              # and without the log2(N)/8 mean error of the unshifted one


def test_deterministic_words_do_not_depend_on_seed_step_or_position():
    g = np.random.default_rng(2)
    x = g.normal(size=(3, 6)).astype(np.float32)
    d = g.normal(size=(3, 4)).astype(np.float32)
    a = oracle.pulse_words(x, d, 0.1, 0.01, 31, False, 1, 0, train_kind=DETERMINISTIC)
    b = oracle.pulse_words(x, d, 0.1, 0.01, 31, False, 99, 7, train_kind=DETERMINISTIC)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
    s = oracle.pulse_words(x, d, 0.1, 0.01, 31, False, 1, 0, train_kind=STOCHASTIC)
    assert not (a[0] == s[0]).all()
    # equal line values give equal words wherever they sit
    x2 = np.full((2, 5), 0.37, dtype=np.float32)
    d2 = np.full((2, 3), -0.21, dtype=np.float32)
    xw, dw = oracle.pulse_words(x2, d2, 0.1, 0.01, 31, False, 1, 0, train_kind=DETERMINISTIC)
    assert (xw == xw[0, 0]).all() and (dw == dw[0, 0]).all()


def test_deterministic_update_approximates_the_rank_update():
    R, C, BL, lr, dw_min = 6, 7, 63, 0.1, 0.001
    g = np.random.default_rng(5)
    x = g.uniform(-1, 1, size=(1, C)).astype(np.float32)
    d = g.uniform(-0.05, 0.05, size=(1, R)).astype(np.float32)
    p = DeviceParams(dw_min=dw_min, w_max=1e6, w_min=-1e6)
    planes = oracle.device_planes(p, 1, R, C)
    W = np.zeros((R, C), dtype=np.float32)
    oracle.pulsed_update(W, planes, p, BL, True, x, d, lr, 1, 0, train_kind=DETERMINISTIC, dynamic_bl=False)
    want = -lr * np.outer(d[0].astype(float), x[0].astype(float))
    assert np.abs(W - want).max() <= dw_min * 2.0
