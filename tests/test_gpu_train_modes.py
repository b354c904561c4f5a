"""GPU parity of the alternative pulse-train generators (deterministic trains, per-sample train
length) against the oracle: pulse words bit for bit, weights within tolerance."""
import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht
from paper_2104_02184_amd import workloads as wl

from common import gpu_params, make_tile, oracle_params, to_dev, words_to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("deterministic", [False, True])
@pytest.mark.parametrize("dynamic_bl", [False, True])
@pytest.mark.parametrize("um", [False, True])
@pytest.mark.parametrize("bl", [7, 31, 63])
def test_pulse_words_bit_exact_in_every_mode(deterministic, dynamic_bl, um, bl):
    g = np.random.default_rng(bl + 2 * um)
    R, C, B = 40, 150, 24
    dev = dict(kind=aht.CONSTANT_STEP, dw_min=0.001, w_max=1.0, w_min=-1.0)
    x = g.normal(size=(B, C)).astype(np.float32)
    d = (g.normal(size=(B, R)) * g.uniform(0.0005, 0.2, size=(B, 1))).astype(np.float32)
    x[3] = 0.0                       # skipped sample
    d[5, 2] = np.nan
    x[7] *= 1e3                      # saturating sample
    with aht.Tile(R, C, gpu_params(dev), bl, um, seed=9) as tile:
        tile.set_pulse_mode(deterministic, dynamic_bl)
        tile.step = 4
        xw, dw = tile.debug_pulse_words(to_dev(x), to_dev(d), 0.1)
        oxw, odw = oracle.pulse_words(x, d, 0.1, 0.001, bl, um, 9, 4, train_kind=int(deterministic), dynamic_bl=dynamic_bl)
        assert (words_to_np(xw) == oxw).all()
        assert (words_to_np(dw) == odw).all()
        if dynamic_bl:
            _, _, blb = oracle.line_scale_ex(x, d, 0.1, 0.001, bl, um, True)
            assert blb.min() < bl


@pytest.mark.parametrize("deterministic,dynamic_bl", [(True, False), (False, True), (True, True)])
def test_weights_in_the_alternative_modes(deterministic, dynamic_bl):
    w = wl.scaled(wl.WORKLOADS["cfg5_4096x4096_linearstep"], rows=70, cols=130, batch=64, steps=4)
    tile = make_tile(w)
    tile.set_pulse_mode(deterministic, dynamic_bl)
    planes = oracle.device_planes(oracle_params(w.device), w.seed, w.rows, w.cols)
    W0 = np.clip(wl.initial_weights(w), planes["b_min"], planes["b_max"]).astype(np.float32)
    tile.set_weights(to_dev(W0))
    Wo = W0.copy()
    po = 0
    for t, x, d in wl.input_stream(w):
        tile.pulsed_update(to_dev(x), to_dev(d), w.lr)
        po += oracle.pulsed_update(Wo, planes, oracle_params(w.device), w.bl, w.update_management, x, d, w.lr,
                                   w.seed, t, train_kind=int(deterministic), dynamic_bl=dynamic_bl)
    Wg = tile.get_weights().cpu().numpy()
    assert tile.pulse_count() == po and po > 0
    tile.close()
    assert np.abs(Wg.astype(np.float64) - Wo).max() / w.device["w_max"] <= 1e-5


def test_unknown_mode_is_rejected():
    with aht.Tile(4, 4, aht.DeviceParams(), 31) as tile:
        L = aht.load_library()
        assert L.aht_set_pulse_mode(tile._h, 7, 0) == 1
