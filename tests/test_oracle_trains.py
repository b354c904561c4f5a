"""Pins for the oracle's pulse trains and coincidence counts.

What fixes the expected values here is the paper's description (Sec. 3, after
Eq. (2)): independent Bernoulli pulses on every line with probability
proportional to |x_j|, |d_i|, coincidences counted per cross-point; plus this
build's readings R1..R6 (probability resolution 2^-32, saturation, zero
inputs, update management).  The 2x2 joint law is obtained by brute-force
enumeration of every possible set of pulse trains.
"""
import itertools
import math

import numpy as np
import pytest
from scipy import stats

import oracle

SIGN = 1 << 63
BITS = np.uint64((1 << 63) - 1)      # the 63 pulse bits of a word


def popcount(v):
    return bin(int(v)).count("1")


# ---------------------------------------------------------------- thresholds
def test_threshold_is_floor_of_probability_times_2_32():
    g = np.random.default_rng(1)
    for _ in range(2000):
        a = float(g.uniform(0.0, 3.0))
        v = np.float32(g.normal())
        want = int(math.floor(min(1.0, a * abs(float(v))) * 2.0**32)) if v != 0 else 0
        assert oracle.threshold(a, v) == want
    assert oracle.threshold(1.0, 1.0) == 2**32           # saturation is 2^32, not 2^32-1
    assert oracle.threshold(5.0, -7.0) == 2**32
    assert oracle.threshold(1e300, 1e30) == 2**32        # product overflows to +inf
    assert oracle.threshold(0.5, 0.5) == 2**30
    assert oracle.threshold(1.0, 0.0) == 0
    assert oracle.threshold(1.0, float("nan")) == 0
    assert oracle.threshold(1.0, float("inf")) == 0
    assert oracle.threshold(1.0, float("-inf")) == 0


def test_pulse_word_bits_are_the_keyed_philox_words_below_threshold():
    seed, t, b, idx, BL = 0xABCDEF0123456789, 11, 5, 77, 63
    a, v = 0.37, np.float32(-1.3)
    T = oracle.threshold(a, v)
    word = oracle.pulse_word(seed, t, oracle.TAG_D, idx, b, a, v, BL)
    assert word >> 63 == 1                                # negative line value
    for n in range(BL):
        r = oracle.philox4x32_10([idx, b, t, (oracle.TAG_D << 24) | (n >> 2)],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        assert ((word >> n) & 1) == (1 if int(r[n & 3]) < T else 0)
    # bits at and above BL (below the sign bit) are never set
    w31 = oracle.pulse_word(seed, t, oracle.TAG_X, idx, b, 10.0, np.float32(1.0), 31)
    assert w31 == (1 << 31) - 1


def test_bit_frequency_equals_threshold_over_2_32():
    # 63 bits x 4000 samples x 3 probabilities; binomial z-test per probability
    seed = 42
    for a, v in [(0.25, 1.0), (0.9, -0.77), (0.01, 3.0)]:
        T = oracle.threshold(a, np.float32(v))
        p = T / 2.0**32
        ones = 0
        N = 4000
        for b in range(N):
            ones += popcount(oracle.pulse_word(seed, 0, oracle.TAG_X, 3, b, a, np.float32(v), 63) & ~SIGN)
        n = 63 * N
        z = (ones - n * p) / math.sqrt(n * p * (1 - p))
        assert abs(z) < 4.0, (a, v, z)


# ------------------------------------------------------- P2: 2x2 brute force
def _exact_joint_pmf(px, pd, BL):
    """Enumerate every (x0,x1,d0,d1) train tuple of length BL: pmf of (n00,n01,n10,n11)."""
    pmf = {}
    trains = list(itertools.product([0, 1], repeat=BL))

    def weight(tr, p):
        w = 1.0
        for bit in tr:
            w *= p if bit else (1.0 - p)
        return w

    for x0 in trains:
        for x1 in trains:
            wx = weight(x0, px[0]) * weight(x1, px[1])
            for d0 in trains:
                for d1 in trains:
                    w = wx * weight(d0, pd[0]) * weight(d1, pd[1])
                    key = (sum(a & b for a, b in zip(x0, d0)), sum(a & b for a, b in zip(x1, d0)),
                           sum(a & b for a, b in zip(x0, d1)), sum(a & b for a, b in zip(x1, d1)))
                    pmf[key] = pmf.get(key, 0.0) + w
    return pmf


@pytest.mark.parametrize("BL", [1, 2, 3])
def test_2x2_joint_count_law_matches_brute_force(BL):
    lr, dw_min = 0.04 * BL, 0.05          # a = sqrt(lr/(dw_min*BL)) ~ 0.894 for every BL
    x = np.array([0.45, -0.8], dtype=np.float32)
    d = np.array([-0.6, 0.3], dtype=np.float32)
    B = 20000
    xs = np.tile(x, (B, 1))
    ds = np.tile(d, (B, 1))
    a_x, a_d = oracle.line_scale(xs[:1], ds[:1], lr, dw_min, BL, False)
    px = [oracle.threshold(a_x[0], v) / 2.0**32 for v in x]
    pd = [oracle.threshold(a_d[0], v) / 2.0**32 for v in d]
    assert all(0.05 < p < 0.95 for p in px + pd)
    pmf = _exact_joint_pmf(px, pd, BL)
    assert sum(pmf.values()) == pytest.approx(1.0, abs=1e-12)

    observed = {}
    n_total = 0
    n00, n01 = [], []
    for seed, t in [(1, 0), (1, 1), (2, 0), (3, 7), (2**40 + 5, 2)]:
        xw, dw = oracle.pulse_words(xs, ds, lr, dw_min, BL, False, seed, t)
        for b in range(B):
            c = oracle_counts_2x2(xw[b], dw[b], BL)
            observed[c] = observed.get(c, 0) + 1
            n00.append(c[0])
            n01.append(c[1])
        n_total += B
    # chi-square on outcomes with expected >= 5, the rest pooled
    keys = sorted(pmf)
    exp = np.array([pmf[k] * n_total for k in keys])
    obs = np.array([observed.get(k, 0) for k in keys], dtype=float)
    assert set(observed) <= set(keys)
    big = exp >= 5
    e = np.append(exp[big], exp[~big].sum())
    o = np.append(obs[big], obs[~big].sum())
    if e[-1] == 0:
        e, o = e[:-1], o[:-1]
    chi = stats.chisquare(o, e * o.sum() / e.sum())
    assert chi.pvalue > 1e-3, chi
    # shared row line d0 correlates the two cells of row 0:
    cov = np.cov(np.array(n00, float), np.array(n01, float))[0, 1]
    want = BL * pd[0] * (1 - pd[0]) * px[0] * px[1]
    sd = math.sqrt(BL) / math.sqrt(n_total)            # generous bound on the estimator's std
    assert abs(cov - want) < 4 * sd


def oracle_counts_2x2(xrow, drow, BL):
    mask = (1 << BL) - 1
    return tuple(popcount(int(xrow[j]) & int(drow[i]) & mask) for i in range(2) for j in range(2))


def test_counts_function_matches_popcount_and_sign_rule():
    g = np.random.default_rng(3)
    B, R, C, BL = 3, 5, 7, 63
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    xw, dw = oracle.pulse_words(x, d, 0.1, 0.001, BL, False, 9, 4)
    mask = (1 << BL) - 1
    for b in range(B):
        sc = oracle.counts(xw, dw, b, BL)
        for i in range(R):
            for j in range(C):
                n = popcount(int(xw[b, j]) & int(dw[b, i]) & mask)
                up = (x[b, j] * d[b, i]) < 0          # W -= lr d x^T: negative product moves w up
                assert sc[i, j] == (n if up else -n)


# ------------------------------------------------- P4: range and saturation
def test_counts_in_range_and_full_on_double_saturation():
    g = np.random.default_rng(4)
    for BL in (1, 31, 32, 63):
        x = g.normal(size=(4, 9)).astype(np.float32)
        d = g.normal(size=(4, 6)).astype(np.float32)
        xw, dw = oracle.pulse_words(x, d, 0.1, 0.001, BL, False, 1, 0)
        for b in range(4):
            sc = oracle.counts(xw, dw, b, BL).astype(int)
            assert np.abs(sc).max() <= BL
        xs = np.full((2, 5), 1e3, dtype=np.float32)
        ds = np.full((2, 4), -1e3, dtype=np.float32)
        xw, dw = oracle.pulse_words(xs, ds, 0.1, 0.001, BL, False, 1, 0)
        assert (xw == ((1 << BL) - 1)).all()
        assert (dw == (((1 << BL) - 1) | SIGN)).all()
        assert (oracle.counts(xw, dw, 1, BL) == BL).all()      # x*d<0 -> +BL (UP)


# ------------------------------------------------------- P5: zero input
@pytest.mark.parametrize("um", [False, True])
def test_zero_or_nonfinite_lines_give_zero_words(um):
    g = np.random.default_rng(5)
    x = g.normal(size=(3, 8)).astype(np.float32)
    d = g.normal(size=(3, 6)).astype(np.float32)
    x[0, :] = 0.0                   # whole sample zero
    d[1, :] = 0.0
    x[2, 3] = np.nan
    x[2, 4] = np.inf
    d[2, 1] = -np.inf
    d[2, 2] = -0.0
    xw, dw = oracle.pulse_words(x, d, 0.1, 0.001, 31, um, 3, 3)
    assert (xw[0] == 0).all()
    assert (dw[1] == 0).all()
    assert xw[2, 3] == 0 and xw[2, 4] == 0 and dw[2, 1] == 0 and dw[2, 2] == 0
    if um:
        # a sample whose x (or d) is entirely zero is skipped altogether
        assert (dw[0] == 0).all() and (xw[1] == 0).all()
    else:
        assert (dw[0] & BITS).any() and (xw[1] & BITS).any()
    # the non-finite entries do not poison the rest of sample 2
    assert (xw[2, [0, 1, 2, 5, 6, 7]] & BITS).any()


# ---------------------------------------------- P7: expected count and mean
def test_expected_count_is_BL_Tx_Td_over_2_64():
    lr, dw_min, BL = 0.1, 0.01, 31
    x = np.array([[0.3, -0.9, 0.05]], dtype=np.float32)
    d = np.array([[0.5, -0.2]], dtype=np.float32)
    B = 30000
    xs, ds = np.tile(x, (B, 1)), np.tile(d, (B, 1))
    a_x, a_d = oracle.line_scale(x, d, lr, dw_min, BL, False)
    xw, dw = oracle.pulse_words(xs, ds, lr, dw_min, BL, False, 8, 1)
    mask = (1 << BL) - 1
    for i in range(2):
        for j in range(3):
            Tx = oracle.threshold(a_x[0], x[0, j])
            Td = oracle.threshold(a_d[0], d[0, i])
            p = Tx * Td / 2.0**64
            both = xw[:, j] & dw[:, i] & np.uint64(mask)
            n = np.array([popcount(v) for v in both], dtype=float)
            want = BL * p
            sd = math.sqrt(BL * p * (1 - p) / B)
            assert abs(n.mean() - want) < 4 * sd
            # and the probability constant: BL*dw_min*p_x*p_d = lr*|x||d| (up to 2^-32 flooring)
            assert BL * dw_min * p == pytest.approx(lr * abs(x[0, j] * d[0, i]), rel=1e-6)


# ------------------------------------------------------ P11: update management
def test_update_management_balances_probabilities_and_keeps_product():
    g = np.random.default_rng(6)
    lr, dw_min, BL = 0.1, 0.001, 63
    x = g.normal(size=(5, 40)).astype(np.float32)
    d = (g.normal(size=(5, 30)) * 0.01).astype(np.float32)
    a0x, a0d = oracle.line_scale(x, d, lr, dw_min, BL, False)
    a1x, a1d = oracle.line_scale(x, d, lr, dw_min, BL, True)
    A = math.sqrt(float(np.float32(lr)) / (float(np.float32(dw_min)) * BL))
    assert np.allclose(a0x, A, rtol=1e-15) and np.allclose(a0d, A, rtol=1e-15)
    for b in range(5):
        mx, md = float(np.abs(x[b]).max()), float(np.abs(d[b]).max())
        assert a1x[b] * mx == pytest.approx(a1d[b] * md, rel=1e-12)        # equal largest probability
        assert a1x[b] * a1d[b] == pytest.approx(A * A, rel=1e-12)          # product unchanged
        assert a1x[b] == pytest.approx(A * math.sqrt(md / mx), rel=1e-14)


def test_bit_is_set_iff_random_word_strictly_below_threshold():
    # choose the threshold equal to the very random word that decides bit n
    seed, t, b, idx = 77, 2, 1, 9
    for n in (0, 5, 30):
        r = int(oracle.philox4x32_10([idx, b, t, (oracle.TAG_X << 24) | (n >> 2)],
                                     [seed & 0xFFFFFFFF, seed >> 32])[n & 3])
        a_eq = (r + 0.5) / 2.0**32            # T == r      -> bit clear
        a_gt = (r + 1.5) / 2.0**32            # T == r + 1  -> bit set
        assert oracle.threshold(a_eq, 1.0) == r and oracle.threshold(a_gt, 1.0) == r + 1
        assert (oracle.pulse_word(seed, t, oracle.TAG_X, idx, b, a_eq, 1.0, 31) >> n) & 1 == 0
        assert (oracle.pulse_word(seed, t, oracle.TAG_X, idx, b, a_gt, 1.0, 31) >> n) & 1 == 1
