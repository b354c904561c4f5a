"""GPU parity at the full sizes of the five workloads, in the launch configuration the
benchmark uses.  The GPU runs the whole tile for the full number of update calls; the oracle
draws all pulse words of every call but applies them to a sample of cells only (cells are
independent given the words): 4096 random cells, the first and last row, the first and last
column.  Pulse words of the first call are compared bit for bit on the whole tile."""
import time

import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht
from paper_2104_02184_amd import workloads as wl

from common import gpu_planes, make_tile, oracle_params, to_dev, words_to_np

pytestmark = pytest.mark.gpu
WEIGHT_TOL = 1e-5


def _sample_cells(w, n_random=4096):
    g = np.random.default_rng(12345)
    R, C = w.rows, w.cols
    cells = set(int(v) for v in g.integers(0, R * C, size=n_random))
    cells.update(range(0, C))                              # first row
    cells.update(range((R - 1) * C, R * C))                # last row
    cells.update(range(0, R * C, C))                       # first column
    cells.update(range(C - 1, R * C, C))                   # last column
    return np.array(sorted(cells), dtype=np.int64)


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_full_size_workload_matches_oracle_on_sampled_cells(name):
    import torch
    w = wl.WORKLOADS[name]
    t0 = time.time()
    tile = make_tile(w)
    cells = _sample_cells(w)
    # planes: oracle's own, compared with the library's on the sampled cells
    oplanes = oracle.device_planes(oracle_params(w.device), w.seed, w.rows, w.cols)
    gplanes = gpu_planes(tile)
    for n in aht.PLANE_NAMES:
        a, b = gplanes[n].ravel()[cells].astype(np.float64), oplanes[n].ravel()[cells].astype(np.float64)
        assert np.all(np.abs(a - b) <= 1e-6 * np.abs(b)), n
    del gplanes
    W0 = np.clip(wl.initial_weights(w), oplanes["b_min"], oplanes["b_max"]).astype(np.float32)
    tile.set_weights(to_dev(W0))
    Wo = W0.copy()
    p = oracle_params(w.device)
    for t, x, d in wl.input_stream(w):
        xd, dd = to_dev(x), to_dev(d)
        if t == 0:                                         # whole-tile pulse words of the first call
            xw, dw = tile.debug_pulse_words(xd, dd, w.lr)
            oxw, odw = oracle.pulse_words(x, d, w.lr, w.device["dw_min"], w.bl, w.update_management, w.seed, 0)
            assert (words_to_np(xw) == oxw).all() and (words_to_np(dw) == odw).all()
            del xw, dw, oxw, odw
        tile.pulsed_update(xd, dd, w.lr)
        oracle.pulsed_update(Wo, oplanes, p, w.bl, w.update_management, x, d, w.lr, w.seed, t, cells=cells)
        print(f"{name}: step {t + 1}/{w.steps} ({time.time() - t0:.0f} s)", flush=True)
    assert tile.step == w.steps
    Wg = tile.get_weights().cpu().numpy()
    torch.cuda.synchronize()
    tile.close()
    err = np.abs(Wg.ravel()[cells].astype(np.float64) - Wo.ravel()[cells].astype(np.float64)) / w.device["w_max"]
    moved = np.abs(Wo.ravel()[cells] - W0.ravel()[cells]).mean()
    print(f"{name}: {cells.size} sampled cells, max |dw|/w_max = {err.max():.3e}, mean |w - w0| = {moved:.3e}")
    assert err.max() <= WEIGHT_TOL
    assert moved > 0                                       # the update did something
    # properties that hold for every cell: inside the per-cell bounds, finite
    assert np.isfinite(Wg).all()
    assert (Wg <= oplanes["b_max"] * (1 + 1e-6) + 1e-12).all() and (Wg >= oplanes["b_min"] * (1 + 1e-6) - 1e-12).all()


@pytest.mark.parametrize("transposed", [False, True])
def test_full_size_analog_product_matches_oracle(transposed):
    """The analog product of the side benchmark (headline tile, B = 256, the benchmark's noise
    settings plus quantisation) against the oracle's full result."""
    w = wl.WORKLOADS[wl.HEADLINE]
    io_kw = dict(inp_res=1.0 / 126.0, inp_bound=1.0, inp_noise=0.01, w_noise=0.02, out_noise=0.06,
                 out_res=12.0 / 254.0, out_bound=12.0, noise_management=True)
    tile = make_tile(w)
    W = wl.initial_weights(w)
    tile.set_weights(to_dev(W))
    g = wl.rng_for(w, 3)
    n_in = w.rows if transposed else w.cols
    x = g.standard_normal((w.batch, n_in), dtype="float32")
    fn = tile.backward if transposed else tile.forward
    y, pre = fn(to_dev(x), aht.IOParams(**io_kw), with_pre=True)
    y, pre = y.cpu().numpy(), pre.cpu().numpy()
    yo, po = oracle.analog_mvm(W, x, oracle.IOParams(**io_kw), w.seed, 0, transposed=transposed, return_pre=True)
    tol = 2e-5 * max(1.0, float(np.abs(po).max())) * max(1.0, np.sqrt(n_in) / 16)
    assert np.abs(pre.astype(np.float64) - po).max() <= tol
    step_out = io_kw["out_res"] * np.abs(x).max(axis=1, keepdims=True)
    diff = np.abs(y.astype(np.float64) - yo)
    same = diff <= 1e-6 * np.maximum(1.0, np.abs(yo))
    assert (diff <= step_out * (1 + 1e-5) + 1e-9).all() and same.mean() > 0.999
    tile.close()
