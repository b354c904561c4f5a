"""Pins for the oracle's device response, sequential application and planes.

Expected values come from closed forms of the three response curves, from
hand-computed tiny cases with injected pulse words, and from properties the
paper states (Sec. 3: finite step per coincidence, device-to-device and
up/down variation, non-linear dependence on the weight, pulse-to-pulse
variation, sequential application, analog (not digital) accumulation over a
mini-batch) together with this build's readings R1, R7, R9, R10.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import CONSTANT_STEP, LINEAR_STEP, SOFT_BOUNDS, DeviceParams

SIGN = np.uint64(1 << 63)
f32 = np.float32


def flat_planes(R, C, s_up, s_dn, bmax, bmin, slope_up=0.0, slope_dn=0.0):
    vals = dict(dw_up=s_up, dw_down=s_dn, b_max=bmax, b_min=bmin, slope_up=slope_up, slope_down=slope_dn)
    return {k: np.full((R, C), v, dtype=np.float32) for k, v in vals.items()}


def words_for_counts(n_x_bits, n_d_bits, x_neg=False, d_neg=False):
    xw = np.uint64((1 << n_x_bits) - 1) | (SIGN if x_neg else np.uint64(0))
    dw = np.uint64((1 << n_d_bits) - 1) | (SIGN if d_neg else np.uint64(0))
    return xw, dw


# ------------------------------------------------- P3: injected words by hand
def test_injected_words_constant_step_by_hand():
    # R=2, C=3, B=2, BL=5.  Words written by hand (bit n = pulse n, bit 63 = negative line).
    BL = 5
    xw = np.array([[0b10110, 0b00001 | (1 << 63), 0b11111],
                   [0b00000, 0b11111, 0b01010 | (1 << 63)]], dtype=np.uint64)
    dw = np.array([[0b00111, 0b11000 | (1 << 63)],
                   [0b11111 | (1 << 63), 0b00100]], dtype=np.uint64)
    # sample 0 coincidences (x&d):  row0: 10110&00111=00110 ->2, 00001&00111 ->1, 11111&00111 ->3
    #                               row1: 10110&11000=10000 ->1, 00001&11000 ->0, 11111&11000 ->2
    # signs sample 0: x=(+,-,+), d=(+,-): product>0 -> DOWN(-), product<0 -> UP(+)
    want0 = np.array([[-2, +1, -3], [+1, 0, +2]])
    # sample 1: row0 (d neg, 11111): x0=0 ->0, x1=11111 ->5 (x+,d-: UP), x2=01010 ->2 (x-,d-: DOWN)
    #           row1 (d pos, 00100): 0, 1 (DOWN), 0
    want1 = np.array([[0, +5, -2], [0, -1, 0]])
    assert (oracle.counts(xw, dw, 0, BL) == want0).all()
    assert (oracle.counts(xw, dw, 1, BL) == want1).all()
    # constant step: up 0.25, down 0.125 (exact in binary), wide bounds
    W = np.zeros((2, 3), dtype=np.float32)
    planes = flat_planes(2, 3, 0.25, 0.125, 100.0, -100.0)
    n = oracle.apply_words(W, planes, CONSTANT_STEP, 0.0, xw, dw, BL, seed=1, t=0)
    step = lambda c: np.where(c > 0, c * 0.25, c * 0.125)
    assert n == np.abs(want0).sum() + np.abs(want1).sum()
    assert (W == (step(want0) + step(want1)).astype(np.float32)).all()


def test_bits_at_or_above_BL_are_ignored_by_the_count():
    xw = np.array([[0xFFFFFFFFFFFFFFFF]], dtype=np.uint64)
    dw = np.array([[0x7FFFFFFFFFFFFFFF]], dtype=np.uint64)
    assert oracle.counts(xw, dw, 0, 7)[0, 0] == 7          # x neg, d pos -> UP


# ------------------------------------------------------ P8: closed forms
@pytest.mark.parametrize("up", [True, False])
def test_closed_forms_of_the_three_curves(up):
    s, bmax, bmin = 0.01, 0.8, -0.5
    b = bmax if up else bmin
    sgn = 1.0 if up else -1.0
    w0 = 0.1
    for k in (1, 7, 40, 300):
        xw, dw = words_for_counts(63, 63, x_neg=up, d_neg=False)     # up <=> product negative
        reps = k // 63
        rest = k % 63
        XW = np.array([[xw]] * reps + [[np.uint64((1 << rest) - 1) | (SIGN if up else np.uint64(0))]], dtype=np.uint64)
        DW = np.array([[dw]] * reps + [[np.uint64((1 << 63) - 1)]], dtype=np.uint64)
        # constant step: w0 +- k s, clipped
        W = np.full((1, 1), w0, dtype=np.float32)
        oracle.apply_words(W, flat_planes(1, 1, s, s, bmax, bmin), CONSTANT_STEP, 0.0, XW, DW, 63, 1, 0)
        want = min(max(w0 + sgn * k * s, bmin), bmax)
        assert W[0, 0] == pytest.approx(want, abs=2e-6)
        # soft bounds: w_k = b - (b - w0)(1 - s/|b|)^k
        W = np.full((1, 1), w0, dtype=np.float32)
        pl = flat_planes(1, 1, s, s, bmax, bmin, 1.0 / bmax, 1.0 / bmin)
        oracle.apply_words(W, pl, SOFT_BOUNDS, 0.0, XW, DW, 63, 1, 0)
        want = b - (b - w0) * (1.0 - s / abs(b)) ** k
        assert W[0, 0] == pytest.approx(want, abs=5e-6)
        # linear step, gamma = 0.3: w_k = b/g - (b/g - w0)(1 - g s/|b|)^k until clipped at b
        gam = 0.3
        W = np.full((1, 1), w0, dtype=np.float32)
        pl = flat_planes(1, 1, s, s, bmax, bmin, gam / bmax, gam / bmin)
        oracle.apply_words(W, pl, LINEAR_STEP, 0.0, XW, DW, 63, 1, 0)
        free = b / gam - (b / gam - w0) * (1.0 - gam * s / abs(b)) ** k
        want = min(free, bmax) if up else max(free, bmin)
        assert W[0, 0] == pytest.approx(want, abs=5e-6)


def test_linear_step_special_cases_are_bit_identical():
    g = np.random.default_rng(2)
    R, C, B, BL = 6, 5, 9, 31
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    xw, dw = oracle.pulse_words(x, d, 0.1, 0.001, BL, False, 11, 0)
    W0 = (g.uniform(-0.3, 0.3, size=(R, C))).astype(np.float32)
    bmax = g.uniform(0.4, 0.8, size=(R, C)).astype(np.float32)
    bmin = -g.uniform(0.4, 0.8, size=(R, C)).astype(np.float32)
    base = dict(dw_up=np.full((R, C), 0.0011, f32), dw_down=np.full((R, C), 0.0009, f32), b_max=bmax, b_min=bmin)
    zero = np.zeros((R, C), f32)
    # gamma = 0  <=>  constant step
    Wc, Wl = W0.copy(), W0.copy()
    oracle.apply_words(Wc, dict(base, slope_up=zero, slope_down=zero), CONSTANT_STEP, 0.3, xw, dw, BL, 5, 2)
    oracle.apply_words(Wl, dict(base, slope_up=zero, slope_down=zero), LINEAR_STEP, 0.3, xw, dw, BL, 5, 2)
    assert (Wc == Wl).all()
    # gamma = 1  <=>  soft bounds
    su, sd = (f32(1.0) / bmax).astype(f32), (f32(1.0) / bmin).astype(f32)
    Ws, Wl = W0.copy(), W0.copy()
    oracle.apply_words(Ws, dict(base, slope_up=su, slope_down=sd), SOFT_BOUNDS, 0.3, xw, dw, BL, 5, 2)
    oracle.apply_words(Wl, dict(base, slope_up=su, slope_down=sd), LINEAR_STEP, 0.3, xw, dw, BL, 5, 2)
    assert (Ws == Wl).all()
    assert not (Ws == Wc).all()


def test_single_step_formula_values():
    # UP uses (dw_up, slope_up, b_max); DOWN uses (dw_down, slope_down, b_min); noise multiplies the step
    st = oracle.device_step
    assert st(CONSTANT_STEP, 0.5, 1, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0) == 0.75
    assert st(CONSTANT_STEP, 0.5, 0, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0) == 0.375
    assert st(CONSTANT_STEP, 0.5, 1, 2.0, 0.5, 0.25, 0.125, 2.0, -2.0) == 1.0      # 0.25*(1+0.5*2)
    assert st(CONSTANT_STEP, 0.5, 1, -4.0, 0.5, 0.25, 0.125, 2.0, -2.0) == 0.25    # noise reverses the step
    assert st(CONSTANT_STEP, 1.9, 1, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0) == 2.0      # clipped at b_max
    assert st(CONSTANT_STEP, -1.9, 0, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0) == -2.0    # clipped at b_min
    # linear: f_up = 1 - slope_up*w ; f_down = 1 - slope_down*w (slope_down < 0)
    assert st(LINEAR_STEP, 0.5, 1, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0, 0.5, -0.25) == 0.5 + 0.25 * 0.75
    assert st(LINEAR_STEP, 0.5, 0, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0, 0.5, -0.25) == 0.5 - 0.125 * 1.125
    assert st(LINEAR_STEP, -1.0, 0, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0, 0.5, -0.25) == -1.0 - 0.125 * 0.75
    # the slope factor never goes negative (a pulse cannot reverse because of the slope)
    assert st(LINEAR_STEP, 1.5, 1, 0.0, 0.0, 0.25, 0.125, 2.0, -2.0, 1.0, -1.0) == 1.5


# ------------------------------------------- P9: analog, not digital, accumulation
def test_batch_is_applied_sequentially_not_as_one_digital_sum():
    # cell near its upper bound: 6 UP pulses (sample 0) clip at b_max, then 4 DOWN pulses (sample 1)
    BL = 31
    XW = np.array([[(1 << 6) - 1 | (1 << 63)], [(1 << 4) - 1]], dtype=np.uint64)
    DW = np.array([[(1 << 31) - 1], [(1 << 31) - 1]], dtype=np.uint64)
    W = np.full((1, 1), 0.9, dtype=np.float32)
    oracle.apply_words(W, flat_planes(1, 1, 0.05, 0.05, 1.0, -1.0), CONSTANT_STEP, 0.0, XW, DW, BL, 1, 0)
    sequential = 1.0 - 4 * 0.05            # clipped at 1.0 after two pulses, then four down
    digital = min(0.9 + (6 - 4) * 0.05, 1.0)
    assert W[0, 0] == pytest.approx(sequential, abs=1e-6)
    assert abs(W[0, 0] - digital) > 0.1
    # and the order of the samples matters
    W2 = np.full((1, 1), 0.9, dtype=np.float32)
    oracle.apply_words(W2, flat_planes(1, 1, 0.05, 0.05, 1.0, -1.0), CONSTANT_STEP, 0.0, XW[::-1].copy(), DW, BL, 1, 0)
    assert W2[0, 0] == pytest.approx(min(0.9 - 0.2 + 0.3, 1.0), abs=1e-6)


# ------------------------------------------------------------ P6: bounds
@pytest.mark.parametrize("kind", [CONSTANT_STEP, LINEAR_STEP, SOFT_BOUNDS])
def test_weights_never_leave_per_cell_bounds(kind):
    g = np.random.default_rng(10 + kind)
    R, C, B, BL = 16, 12, 20, 63
    p = DeviceParams(kind=kind, dw_min=0.05, dw_min_dtod=0.5, dw_min_std=1.0, up_down=0.1, up_down_dtod=0.2,
                     w_max=0.5, w_max_dtod=0.6, w_min=-0.4, w_min_dtod=0.6, gamma_up=0.7, gamma_down=0.4,
                     gamma_dtod=0.5)
    planes = oracle.device_planes(p, seed=77, R=R, C=C)
    assert (planes["b_max"] >= 0).all() and (planes["b_min"] <= 0).all()
    assert (planes["b_max"] == 0).any() or True
    W = np.clip(g.uniform(-0.2, 0.2, size=(R, C)), planes["b_min"], planes["b_max"]).astype(np.float32)
    for t in range(6):
        x = (g.normal(size=(B, C)) * 3).astype(np.float32)
        d = (g.normal(size=(B, R)) * 3).astype(np.float32)
        oracle.pulsed_update(W, planes, p, BL, t % 2 == 0, x, d, lr=5.0, seed=77, t=t)
        assert (W <= planes["b_max"]).all() and (W >= planes["b_min"]).all()
        assert np.isfinite(W).all()


# ------------------------------------------------ P12: weights prove the counts
def test_integer_step_weights_equal_summed_signed_counts():
    g = np.random.default_rng(12)
    R, C, B, BL = 9, 11, 13, 63
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    p = DeviceParams(kind=CONSTANT_STEP, dw_min=1.0, w_max=2.0**20, w_min=-2.0**20)
    planes = oracle.device_planes(p, 1, R, C)
    assert (planes["dw_up"] == 1).all() and (planes["dw_down"] == 1).all()
    W = np.zeros((R, C), dtype=np.float32)
    n = oracle.pulsed_update(W, planes, p, BL, False, x, d, lr=20.0, seed=3, t=9)
    xw, dw = oracle.pulse_words(x, d, 20.0, 1.0, BL, False, 3, 9)
    tot = sum(oracle.counts(xw, dw, b, BL).astype(np.int64) for b in range(B))
    assert (W == tot).all()
    assert n == sum(np.abs(oracle.counts(xw, dw, b, BL).astype(np.int64)).sum() for b in range(B))
    assert n > 1000


# -------------------------------------------- P7: the mean realises the rank update
def test_mean_update_is_minus_lr_d_xT():
    R, C, BL, lr, dw_min = 4, 5, 31, 0.1, 0.01
    g = np.random.default_rng(8)
    x = g.uniform(-0.5, 0.5, size=(1, C)).astype(np.float32)
    d = g.uniform(-0.5, 0.5, size=(1, R)).astype(np.float32)
    p = DeviceParams(kind=CONSTANT_STEP, dw_min=dw_min, w_max=1e6, w_min=-1e6)
    planes = oracle.device_planes(p, 1, R, C)
    N = 6000
    acc = np.zeros((R, C))
    for t in range(N):
        W = np.zeros((R, C), dtype=np.float32)
        oracle.pulsed_update(W, planes, p, BL, False, x, d, lr, seed=21, t=t)
        acc += W
    mean = acc / N
    want = -lr * np.outer(d[0].astype(float), x[0].astype(float))
    A2 = lr / (dw_min * BL)
    pq = A2 * np.abs(np.outer(d[0], x[0]))
    sd = dw_min * np.sqrt(BL * pq * (1 - pq) / N)
    assert (np.abs(mean - want) < 4.5 * sd + 1e-7).all()


# ------------------------------------------ P10: pulse-to-pulse noise statistics
def test_c2c_noise_variance_of_k_pulses():
    # k noisy constant-step pulses: mean k s, variance k s^2 c2c^2 (bounds far away)
    k, s, c2c = 40, 0.01, 0.3
    R, C = 64, 64
    XW = np.full((1, C), (1 << k) - 1, dtype=np.uint64) | SIGN          # x negative -> UP
    DW = np.full((1, R), (1 << 63) - 1, dtype=np.uint64)
    W = np.zeros((R, C), dtype=np.float32)
    n = oracle.apply_words(W, flat_planes(R, C, s, s, 1e3, -1e3), CONSTANT_STEP, c2c, XW, DW, 63, seed=4, t=1)
    assert n == k * R * C
    m = R * C
    assert abs(W.mean() - k * s) < 4 * s * c2c * math.sqrt(k / m)
    var_want = k * s * s * c2c * c2c
    assert abs(W.var() - var_want) < 4 * var_want * math.sqrt(2.0 / m)


def test_noise_stream_is_indexed_by_the_cells_pulse_counter_within_the_call():
    # Two samples with 3 and 2 coincidences: the pulses use Gaussians 0..4 of stream (cell, t, tag 3)
    seed, t, c2c, s = 31, 6, 0.5, 0.125
    R, C = 2, 3
    XW = np.array([[0b111] * C, [0b11] * C], dtype=np.uint64) | SIGN
    DW = np.array([[0b111111] * R] * 2, dtype=np.uint64)
    W = np.zeros((R, C), dtype=np.float32)
    oracle.apply_words(W, flat_planes(R, C, s, s, 1e3, -1e3), CONSTANT_STEP, c2c, XW, DW, 31, seed, t)
    for i in range(R):
        for j in range(C):
            w = f32(0)
            for q in range(5):
                xi = f32(oracle.gauss(seed, i * C + j, t, q, oracle.TAG_C2C))
                w = f32(w + f32(f32(s) * f32(f32(1) + f32(f32(c2c) * xi))))
            assert W[i, j] == w
    # a different step index gives a different stream
    W2 = np.zeros((R, C), dtype=np.float32)
    oracle.apply_words(W2, flat_planes(R, C, s, s, 1e3, -1e3), CONSTANT_STEP, c2c, XW, DW, 31, seed, t + 1)
    assert not (W2 == W).any()


# ---------------------------------------------------- device-to-device planes
def test_device_planes_statistics_and_degenerate_draws():
    R, C = 200, 200
    p = DeviceParams(kind=LINEAR_STEP, dw_min=0.002, dw_min_dtod=0.3, up_down=0.05, up_down_dtod=0.1,
                     w_max=0.6, w_max_dtod=0.3, w_min=-0.5, w_min_dtod=0.2, gamma_up=0.2, gamma_down=0.4,
                     gamma_dtod=0.25)
    pl = oracle.device_planes(p, seed=9, R=R, C=C)
    n = R * C
    dw = (pl["dw_up"].astype(float) + pl["dw_down"]) / 2          # = dw_min |1 + 0.3 g|
    assert (dw >= 0).all()
    assert abs(dw.mean() / 0.002 - 1.0) < 0.01                     # folding at 0 is a 3.3 sigma event
    assert abs(dw.std() / 0.002 - 0.3) < 0.01
    a = (pl["dw_up"].astype(float) - pl["dw_down"]) / (2 * dw)     # asymmetry
    assert abs(a.mean() - 0.05) < 4 * 0.1 / math.sqrt(n)
    assert abs(a.std() - 0.1) < 0.002
    assert abs(pl["b_max"].mean() / 0.6 - 1.0) < 4 * 0.3 / math.sqrt(n) + 1e-3
    assert abs(pl["b_max"].std() / 0.6 - 0.3) < 0.01
    assert abs(pl["b_min"].mean() / -0.5 - 1.0) < 4 * 0.2 / math.sqrt(n)
    assert (pl["b_max"] >= 0).all() and (pl["b_min"] <= 0).all()
    gu = pl["slope_up"].astype(float) * pl["b_max"]
    gd = pl["slope_down"].astype(float) * pl["b_min"]
    ok = pl["b_max"] > 0
    assert abs(gu[ok].mean() - 0.2) < 4 * 0.05 / math.sqrt(n) and abs(gu[ok].std() - 0.05) < 0.002
    assert abs(gd.mean() - 0.4) < 4 * 0.1 / math.sqrt(n) and abs(gd.std() - 0.1) < 0.003
    # the six planes use six different Gaussians of each cell
    cc = np.corrcoef([dw.ravel(), a.ravel(), pl["b_max"].ravel(), pl["b_min"].ravel(), gu.ravel(), gd.ravel()])
    assert (np.abs(cc - np.eye(6)) < 0.03).all()
    # no variation -> exact nominal values; soft bounds slopes are 1/bound; constant step has none
    q = DeviceParams(kind=SOFT_BOUNDS, dw_min=0.001, w_max=0.6, w_min=-0.6)
    ps = oracle.device_planes(q, 1, 3, 4)
    assert (ps["dw_up"] == f32(0.001)).all() and (ps["dw_down"] == f32(0.001)).all()
    assert (ps["slope_up"] == f32(1) / f32(0.6)).all() and (ps["slope_down"] == f32(1) / f32(-0.6)).all()
    pc = oracle.device_planes(DeviceParams(kind=CONSTANT_STEP), 1, 3, 4)
    assert (pc["slope_up"] == 0).all() and (pc["slope_down"] == 0).all()
    # huge bound variation: clipped one-sidedly at 0, slope 0 there
    pz = oracle.device_planes(DeviceParams(kind=SOFT_BOUNDS, w_max=0.5, w_max_dtod=3.0), 2, 50, 50)
    assert (pz["b_max"] == 0).any() and (pz["slope_up"][pz["b_max"] == 0] == 0).all()


def test_selected_cells_equal_the_full_update_on_those_cells():
    g = np.random.default_rng(14)
    R, C, B, BL = 12, 10, 7, 31
    p = DeviceParams(kind=SOFT_BOUNDS, dw_min=0.01, dw_min_std=0.3, w_max=0.6, w_min=-0.6)
    planes = oracle.device_planes(p, 5, R, C)
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    W0 = g.uniform(-0.2, 0.2, size=(R, C)).astype(np.float32)
    Wf, Ws = W0.copy(), W0.copy()
    oracle.pulsed_update(Wf, planes, p, BL, False, x, d, 0.1, 5, 0)
    cells = np.array([0, 7, 55, R * C - 1], dtype=np.int64)
    oracle.pulsed_update(Ws, planes, p, BL, False, x, d, 0.1, 5, 0, cells=cells)
    assert (Ws.ravel()[cells] == Wf.ravel()[cells]).all()
    rest = np.setdiff1d(np.arange(R * C), cells)
    assert (Ws.ravel()[rest] == W0.ravel()[rest]).all()


def test_thread_count_does_not_change_results():
    g = np.random.default_rng(15)
    R, C, B, BL = 40, 33, 11, 63
    p = DeviceParams(kind=LINEAR_STEP, dw_min=0.01, dw_min_dtod=0.3, dw_min_std=0.3, w_max=0.6, w_min=-0.6,
                     gamma_up=0.1, gamma_down=0.1, gamma_dtod=0.3)
    planes = oracle.device_planes(p, 5, R, C)
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    res = []
    n0 = oracle.num_threads()
    for nt in (1, 3, n0):
        oracle.set_num_threads(nt)
        W = np.zeros((R, C), dtype=np.float32)
        oracle.pulsed_update(W, planes, p, BL, True, x, d, 0.1, 5, 3)
        res.append(W)
    oracle.set_num_threads(n0)
    assert (res[0] == res[1]).all() and (res[0] == res[2]).all()
