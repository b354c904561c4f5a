"""Pins for the oracle's once-per-mini-batch temporal processes (decay, diffusion, reset with
device-to-device variability; arXiv 2104.02184, Sec. 4, last paragraph).  Expected values are
closed forms and distribution facts, not re-typed formulas."""
import math

import numpy as np
import pytest

import oracle
from oracle import DeviceParams, TemporalParams

f32 = np.float32


def wide_planes(R, C, bound=1e6):
    z = np.zeros((R, C), f32)
    return dict(dw_up=z, dw_down=z, b_max=np.full((R, C), bound, f32), b_min=np.full((R, C), -bound, f32),
                slope_up=z, slope_down=z)


def test_decay_is_geometric_and_diffusion_free_when_off():
    R, C = 6, 9
    tp = TemporalParams(decay_rate=0.125)                      # exact in binary
    tpl = oracle.temporal_planes(tp, 1, R, C)
    assert (tpl["decay"] == f32(0.125)).all() and (tpl["diffusion"] == 0).all()
    W = np.full((R, C), 0.5, f32)
    for k in range(1, 6):
        oracle.decay_diffuse(W, tpl, wide_planes(R, C), 1, k)
        assert (W == f32(0.5 * 0.875**k)).all()                # powers of 7/8 of 0.5 are exact in fp32 here


def test_zero_parameters_change_nothing():
    g = np.random.default_rng(0)
    W0 = g.normal(size=(5, 7)).astype(f32)
    W = W0.copy()
    oracle.decay_diffuse(W, oracle.temporal_planes(TemporalParams(), 3, 5, 7), wide_planes(5, 7), 3, 0)
    assert (W == W0).all()


def test_diffusion_is_a_gaussian_random_walk():
    R, C, sd = 128, 128, 0.01
    tp = TemporalParams(diffusion=sd)
    tpl = oracle.temporal_planes(tp, 5, R, C)
    W = np.zeros((R, C), f32)
    K = 16
    prev = W.copy()
    incs = []
    for tau in range(K):
        oracle.decay_diffuse(W, tpl, wide_planes(R, C), 5, tau)
        incs.append((W - prev).astype(np.float64) / sd)
        prev = W.copy()
    n = R * C
    assert abs(W.mean()) < 4 * sd * math.sqrt(K / n)
    assert abs(W.var() / (K * sd * sd) - 1) < 4 * math.sqrt(2.0 / n)
    # increments of different steps and of neighbouring cells (numbers of one block) are uncorrelated
    a, b = incs[0].ravel(), incs[1].ravel()
    assert abs(np.corrcoef(a, b)[0, 1]) < 4 / math.sqrt(n)
    assert abs(np.corrcoef(a[0::4], a[1::4])[0, 1]) < 4 / math.sqrt(n / 4)
    assert abs(np.corrcoef(a[0::4], a[3::4])[0, 1]) < 4 / math.sqrt(n / 4)
    # and each increment is Gaussian number `cell` of the step's stream (index 0, t = tau, tag 5)
    for cell in (0, 1, 2, 3, 4, 77, n - 1):
        z = oracle.gauss(5, 0, 3, cell, 5)
        assert incs[3].ravel()[cell] == pytest.approx(float(f32(z)), abs=1e-5)
        assert z == float(f32(oracle.gauss_block_f64(5, 0, 3, cell >> 2, 5)[cell & 3]))


def test_clipping_after_diffusion_and_bounds_hold():
    R, C = 32, 32
    p = DeviceParams(w_max=0.02, w_min=-0.01)
    planes = oracle.device_planes(p, 2, R, C)
    tpl = oracle.temporal_planes(TemporalParams(diffusion=0.05), 2, R, C)
    W = np.zeros((R, C), f32)
    for tau in range(4):
        oracle.decay_diffuse(W, tpl, planes, 2, tau)
        assert (W <= f32(0.02)).all() and (W >= f32(-0.01)).all()
    assert (W == f32(0.02)).any() and (W == f32(-0.01)).any()


def test_temporal_planes_device_to_device_statistics():
    R, C = 200, 200
    tp = TemporalParams(decay_rate=0.01, decay_rate_dtod=0.2, diffusion=0.004, diffusion_dtod=0.3, reset=0.1,
                        reset_dtod=0.02)
    tpl = oracle.temporal_planes(tp, 9, R, C)
    n = R * C
    assert abs(tpl["decay"].mean() / 0.01 - 1) < 4 * 0.2 / math.sqrt(n)
    assert abs(tpl["decay"].std() / 0.01 - 0.2) < 0.005
    assert (tpl["decay"] >= 0).all() and (tpl["decay"] <= 1).all()
    assert abs(tpl["diffusion"].mean() / 0.004 - 1) < 0.01 and abs(tpl["diffusion"].std() / 0.004 - 0.3) < 0.01
    assert (tpl["diffusion"] >= 0).all()
    assert abs(tpl["reset"].mean() - 0.1) < 4 * 0.02 / math.sqrt(n) and abs(tpl["reset"].std() - 0.02) < 0.0005
    dp = oracle.device_planes(DeviceParams(dw_min_dtod=0.3, w_max_dtod=0.3, w_min_dtod=0.3, up_down_dtod=0.1), 9, R, C)
    cc = np.corrcoef([tpl["decay"].ravel(), tpl["diffusion"].ravel(), tpl["reset"].ravel(),
                      dp["dw_up"].ravel(), dp["b_max"].ravel(), dp["b_min"].ravel()])
    assert (np.abs(cc - np.eye(6))[:3] < 0.03).all()           # new planes use Gaussians of their own
    # huge variation: the decay rate stays in [0, 1]
    wild = oracle.temporal_planes(TemporalParams(decay_rate=0.5, decay_rate_dtod=3.0), 9, 50, 50)
    assert (wild["decay"] == 0).any() and (wild["decay"] == 1).any()


def test_reset_touches_only_the_selected_columns():
    R, C = 20, 30
    tp = TemporalParams(reset=0.05, reset_dtod=0.01, reset_std=0.002)
    tpl = oracle.temporal_planes(tp, 4, R, C)
    g = np.random.default_rng(1)
    W0 = g.normal(size=(R, C)).astype(f32)
    W = W0.copy()
    oracle.reset_columns(W, tpl, tp.reset_std, wide_planes(R, C), 4, 7, 5, 10)
    assert (W[:, :5] == W0[:, :5]).all() and (W[:, 15:] == W0[:, 15:]).all()
    dev = (W[:, 5:15].astype(np.float64) - tpl["reset"][:, 5:15]) / 0.002
    assert abs(dev.mean()) < 4 / math.sqrt(dev.size) and abs(dev.std() - 1) < 0.2
    # every reset value is the plane plus Gaussian number `cell` of stream (index 0, t = tau, tag 6)
    for i, j in ((0, 5), (3, 9), (R - 1, 14)):
        want = float(tpl["reset"][i, j]) + float(f32(0.002)) * oracle.gauss(4, 0, 7, i * C + j, 6)
        assert W[i, j] == pytest.approx(want, abs=1e-7)
    # without noise the reset value is the plane itself
    W2 = W0.copy()
    oracle.reset_columns(W2, tpl, 0.0, wide_planes(R, C), 4, 7, 0, C)
    assert (W2 == tpl["reset"]).all()
    # columns beyond the tile are ignored
    W3 = W0.copy()
    oracle.reset_columns(W3, tpl, 0.0, wide_planes(R, C), 4, 7, C - 2, 10)
    assert (W3[:, :C - 2] == W0[:, :C - 2]).all() and (W3[:, C - 2:] == tpl["reset"][:, C - 2:]).all()
