"""Pins of the oracle's unit-cell composition (several devices per cross-point, Sec. 4 of the
paper) against what the reading fixes: shared pulse trains, own response per device, weighted sum."""
import numpy as np

import oracle


def _setup(n, R=12, C=20, B=9, c2c=0.0, d2d=0.0, kinds=None, seed0=11):
    g = np.random.default_rng(5)
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    kinds = kinds or [oracle.SOFT_BOUNDS] * n
    params = [oracle.DeviceParams(kind=k, dw_min=0.01, dw_min_dtod=d2d, dw_min_std=c2c, w_max=0.6, w_min=-0.6)
              for k in kinds]
    seeds = [seed0 + 7 * k for k in range(n)]
    planes = [oracle.device_planes(p, s, R, C) for p, s in zip(params, seeds)]
    Ws = [np.zeros((R, C), dtype=np.float32) for _ in range(n)]
    return x, d, params, seeds, planes, Ws


def test_identical_noise_free_devices_updated_together_stay_identical_and_match_a_single_tile():
    x, d, params, seeds, planes, Ws = _setup(3)
    counts = oracle.unit_cell_update(Ws, planes, params, seeds, 31, False, x, d, 0.3, t=4)
    single = np.zeros_like(Ws[0])
    n1 = oracle.pulsed_update(single, planes[0], params[0], 31, False, x, d, 0.3, seeds[0], 4)
    assert counts == [n1] * 3 and n1 > 0
    for W in Ws:
        assert (W == single).all()
    # equal shares: the cell's weight is the single tile's weight
    eff = oracle.unit_cell_weights(Ws, [0.25, 0.5, 0.25])
    assert np.abs(eff - single).max() <= 1e-7


def test_one_by_one_touches_only_the_chosen_device():
    x, d, params, seeds, planes, Ws = _setup(3, c2c=0.3, d2d=0.2)
    Ws[0][:] = 0.1
    Ws[2][:] = -0.2
    before = [W.copy() for W in Ws]
    counts = oracle.unit_cell_update(Ws, planes, params, seeds, 31, True, x, d, 0.3, t=0, which=1)
    assert counts[0] == 0 and counts[2] == 0 and counts[1] > 0
    assert (Ws[0] == before[0]).all() and (Ws[2] == before[2]).all()
    assert (Ws[1] != before[1]).any()


def test_devices_of_a_cell_see_the_same_coincidences_but_their_own_noise():
    x, d, params, seeds, planes, Ws = _setup(2, c2c=0.3, kinds=[oracle.CONSTANT_STEP, oracle.CONSTANT_STEP])
    counts = oracle.unit_cell_update(Ws, planes, params, seeds, 31, False, x, d, 0.3, t=2)
    assert counts[0] == counts[1] > 0                  # same words, same number of pulses
    assert (Ws[0] != Ws[1]).any()                      # different noise streams
    # without noise the two ConstantStep devices agree exactly
    x, d, params, seeds, planes, Ws = _setup(2, c2c=0.0, kinds=[oracle.CONSTANT_STEP, oracle.CONSTANT_STEP])
    oracle.unit_cell_update(Ws, planes, params, seeds, 31, False, x, d, 0.3, t=2)
    assert (Ws[0] == Ws[1]).all()
    # the direction of every changed cell follows -d_i x_j summed over the batch in the mean:
    # a cell that moved up in one device did not move down in the other (same pulses, same signs)
    assert (np.sign(Ws[0]) * np.sign(Ws[1]) >= 0).all()


def test_effective_weight_is_the_weighted_sum():
    g = np.random.default_rng(1)
    Ws = [g.normal(size=(7, 5)).astype(np.float32) for _ in range(4)]
    gamma = [1.0, -0.5, 0.25, 2.0]                     # powers of two: every product is exact
    eff = oracle.unit_cell_weights(Ws, gamma)
    ref = sum(np.float64(gm) * W.astype(np.float64) for gm, W in zip(gamma, Ws))
    assert eff.dtype == np.float32 and np.abs(eff - ref).max() <= 4 * 2.0**-23 * np.abs(ref).max()
    assert (oracle.unit_cell_weights(Ws[:1], [1.0]) == Ws[0]).all()
    assert (oracle.unit_cell_weights(Ws[:2], [1.0, 0.0]) == Ws[0]).all()
