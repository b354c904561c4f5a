"""GPU parity of the once-per-mini-batch temporal processes (decay, diffusion, reset) against
the oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht

from common import gpu_params, gpu_planes, oracle_params, to_dev

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.mark.parametrize("R,C", [(64, 64), (37, 129), (5, 3), (512, 1024)])
def test_decay_diffuse_and_reset_match_oracle(R, C):
    dev = dict(kind=aht.SOFT_BOUNDS, dw_min=0.001, dw_min_dtod=0.3, w_max=0.6, w_max_dtod=0.3, w_min=-0.6, w_min_dtod=0.3)
    tp = oracle.TemporalParams(decay_rate=0.01, decay_rate_dtod=0.2, diffusion=0.004, diffusion_dtod=0.3, reset=0.02,
                               reset_dtod=0.01, reset_std=0.003)
    seed = 21
    oplanes = oracle.device_planes(oracle_params(dev), seed, R, C)
    otp = oracle.temporal_planes(tp, seed, R, C)
    g = np.random.default_rng(3)
    W0 = np.clip(g.uniform(-0.5, 0.5, size=(R, C)), oplanes["b_min"], oplanes["b_max"]).astype(np.float32)
    with aht.Tile(R, C, gpu_params(dev), 31, False, seed) as tile:
        tile.set_temporal(**tp.__dict__)
        for name in aht.binding.TEMPORAL_PLANE_NAMES:
            got = tile.get_temporal_plane(name).cpu().numpy()
            assert np.allclose(got, otp[name], rtol=1e-6, atol=1e-9), name
            assert (got == otp[name]).mean() > 0.999
        tile.set_weights(to_dev(W0))
        Wo = W0.copy()
        for tau in range(5):
            assert tile.temporal_step == tau
            if tau == 2:                                  # reset uses the current step and does not advance it
                tile.reset_columns(1, 2)
                oracle.reset_columns(Wo, otp, tp.reset_std, oplanes, seed, tau, 1, 2)
                tile.reset_columns(C - 1, 100)            # clipped to the tile
                oracle.reset_columns(Wo, otp, tp.reset_std, oplanes, seed, tau, C - 1, 100)
            tile.decay_diffuse()
            oracle.decay_diffuse(Wo, otp, oplanes, seed, tau)
        Wg = tile.get_weights().cpu().numpy()
    err = np.abs(Wg.astype(np.float64) - Wo).max() / 0.6
    print(R, C, "max |dw|/w_max", err)
    assert err <= TOL
    assert (Wg <= oplanes["b_max"]).all() and (Wg >= oplanes["b_min"]).all()


def test_decay_only_is_bit_identical_and_errors_are_reported():
    import torch
    R, C = 33, 65
    dev = dict(kind=aht.CONSTANT_STEP, w_max=1.0, w_min=-1.0)
    with aht.Tile(R, C, gpu_params(dev), 31, False, 1) as tile:
        with pytest.raises(aht.AhtError):
            tile.decay_diffuse()                          # before aht_set_temporal
        with pytest.raises(aht.AhtError):
            tile.set_temporal(decay_rate=1.5)
        with pytest.raises(aht.AhtError):
            tile.set_temporal(diffusion=-1.0)
        tile.set_temporal(decay_rate=0.03, decay_rate_dtod=0.5)
        g = np.random.default_rng(0)
        W0 = g.uniform(-0.9, 0.9, size=(R, C)).astype(np.float32)
        tile.set_weights(to_dev(W0))
        for _ in range(3):
            tile.decay_diffuse()
        with pytest.raises(aht.AhtError):
            tile.reset_columns(-1, 2)
        Wg = tile.get_weights().cpu().numpy()
        planes = gpu_planes(tile)
    otp = oracle.temporal_planes(oracle.TemporalParams(decay_rate=0.03, decay_rate_dtod=0.5), 1, R, C)
    Wo = W0.copy()
    for tau in range(3):
        oracle.decay_diffuse(Wo, otp, planes, 1, tau)
    assert (Wg == Wo).all()
