"""GPU parity of the convolution-layer update (patches gathered inside the pulse-train kernel)
against the oracle applied to the explicitly written-out update vectors."""
import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht
from paper_2104_02184_amd import workloads as wl

from common import gpu_params, oracle_params, to_dev, words_to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,Cin,H,W,kh,kw,stride,pad,Cout,um", [
    (2, 3, 6, 7, 3, 3, 1, 1, 5, False), (1, 2, 8, 8, 3, 2, 2, 0, 4, True), (3, 1, 5, 5, 5, 5, 1, 2, 7, False),
    (4, 16, 14, 14, 3, 3, 1, 1, 24, True),
])
def test_conv_update_matches_oracle_on_explicit_patches(N, Cin, H, W, kh, kw, stride, pad, Cout, um):
    g = np.random.default_rng(N + Cin + H)
    dev = dict(wl.WORKLOADS["cfg4_conv_256x2304"].device)
    cols = Cin * kh * kw
    OH, OW = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    img = np.maximum(g.normal(size=(N, Cin, H, W)), 0).astype(np.float32)
    grad = (g.normal(size=(N, Cout, OH, OW)) * 0.05).astype(np.float32)
    x, d = oracle.conv_update_vectors(img, grad, kh, kw, stride, pad)
    seed, lr, bl = 17, 0.1, 31
    planes = oracle.device_planes(oracle_params(dev), seed, Cout, cols)
    Wo = np.zeros((Cout, cols), dtype=np.float32)
    with aht.Tile(Cout, cols, gpu_params(dev), bl, um, seed) as tile:
        xw, dw = tile.debug_pulse_words_conv2d(to_dev(img), to_dev(grad), kh, kw, stride, pad, lr)
        oxw, odw = oracle.pulse_words(x, d, lr, dev["dw_min"], bl, um, seed, 0)
        assert (words_to_np(xw) == oxw).all() and (words_to_np(dw) == odw).all()
        po = 0
        for t in range(2):
            tile.pulsed_update_conv2d(to_dev(img), to_dev(grad), kh, kw, stride, pad, lr)
            po += oracle.pulsed_update(Wo, planes, oracle_params(dev), bl, um, x, d, lr, seed, t)
        Wg = tile.get_weights().cpu().numpy()
        assert tile.pulse_count() == po and tile.step == 2
    assert np.abs(Wg.astype(np.float64) - Wo).max() / dev["w_max"] <= 1e-5


def test_conv_geometry_is_checked():
    import torch
    with aht.Tile(4, 18, aht.DeviceParams(), 31) as tile:
        img = torch.zeros((1, 2, 5, 5), device="cuda")
        with pytest.raises(aht.AhtError):                 # 2*2*2 = 8 columns, tile has 18
            tile.pulsed_update_conv2d(img, torch.zeros((1, 4, 4, 4), device="cuda"), 2, 2, 1, 0, 0.1)
        with pytest.raises(aht.AhtError):                 # kernel larger than the image
            tile.pulsed_update_conv2d(torch.zeros((1, 2, 2, 2), device="cuda"), torch.zeros((1, 4, 0, 0), device="cuda"),
                                      3, 3, 1, 0, 0.1)
        tile.pulsed_update_conv2d(img, torch.zeros((1, 4, 3, 3), device="cuda"), 3, 3, 1, 0, 0.1)
        assert tile.step == 1
