"""GPU parity at the full sizes of the five workloads, in the launch configuration the
benchmark uses, on EVERY cell of the tile and for EVERY update call of the workload.

Per workload the GPU runs the whole sequence of calls once (weights and the device's pulse
counter are read back after every call, the pulse words of every call are compared bit for
bit with the oracle's).  The oracle then repeats the sequence on all cells; since cells are
independent given the pulse words, the large tiles are cut into slabs of rows, one test per
slab, so that no single test is silent for long.  Compared: weights after every call within
1e-5 w_max on every cell, and the number of coincidence pulses applied by every call, which
must be equal (a dropped or doubled tile of cells changes it).
"""
import time

import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht
from paper_2104_02184_amd import workloads as wl

from common import gpu_planes, make_tile, oracle_params, to_dev, words_to_np

pytestmark = pytest.mark.gpu
WEIGHT_TOL = 1e-5

# slabs of rows per workload: the oracle needs about 35 s per slab on 16 host threads
SLABS = {"cfg1_64x64_constant": 1, "cfg2_512x512_constant_d2d": 1, "cfg3_1024x1024_softbounds": 1,
         "cfg4_conv_256x2304": 2, "cfg5_4096x4096_linearstep": 4}
_CASES = [(name, k) for name in wl.WORKLOADS for k in range(SLABS[name])]

_runs = {}            # workload name -> what the GPU produced (freed when the module is done)
_oracle_pulses = {}   # (workload name, slab) -> applied pulses per call on that slab


@pytest.fixture(scope="module", autouse=True)
def _free_runs():
    yield
    _runs.clear()
    _oracle_pulses.clear()


def _say(capsys, msg):
    with capsys.disabled():
        print(msg, flush=True)


def _gpu_run(name, capsys):
    """All update calls of the workload on the GPU; weights and pulse counter after every call."""
    if name in _runs:
        return _runs[name]
    import torch
    w = wl.WORKLOADS[name]
    t0 = time.time()
    tile = make_tile(w)
    oplanes = oracle.device_planes(oracle_params(w.device), w.seed, w.rows, w.cols)
    gplanes = gpu_planes(tile)
    for n in aht.PLANE_NAMES:                              # every cell of every plane
        a, b = gplanes[n].astype(np.float64), oplanes[n].astype(np.float64)
        assert np.all(np.abs(a - b) <= 1e-6 * np.abs(b)), n
    del gplanes
    W0 = np.clip(wl.initial_weights(w), oplanes["b_min"], oplanes["b_max"]).astype(np.float32)
    tile.set_weights(to_dev(W0))
    after, pulses, seen = [], [], 0
    for t, x, d in wl.input_stream(w):
        xd, dd = to_dev(x), to_dev(d)
        xw, dw = tile.debug_pulse_words(xd, dd, w.lr)      # whole-tile pulse words of this call
        oxw, odw = oracle.pulse_words(x, d, w.lr, w.device["dw_min"], w.bl, w.update_management, w.seed, t)
        assert (words_to_np(xw) == oxw).all() and (words_to_np(dw) == odw).all(), f"pulse words of call {t}"
        del xw, dw, oxw, odw
        tile.pulsed_update(xd, dd, w.lr)
        after.append(tile.get_weights().cpu().numpy())
        torch.cuda.synchronize()
        total = tile.pulse_count()
        pulses.append(total - seen)
        seen = total
        if (t + 1) % 10 == 0 or w.steps <= 20:
            _say(capsys, f"  {name}: GPU call {t + 1}/{w.steps} ({time.time() - t0:.0f} s)")
    assert tile.step == w.steps
    tile.close()
    _runs[name] = dict(W0=W0, planes=oplanes, after=after, pulses=pulses)
    return _runs[name]


@pytest.mark.parametrize("name,slab", _CASES, ids=[f"{n}-slab{k}" for n, k in _CASES])
def test_full_size_workload_matches_oracle_on_every_cell(name, slab, capsys):
    w = wl.WORKLOADS[name]
    run = _gpu_run(name, capsys)
    nslabs = SLABS[name]
    r0, r1 = w.rows * slab // nslabs, w.rows * (slab + 1) // nslabs
    cells = np.arange(r0 * w.cols, r1 * w.cols, dtype=np.int64)
    p = oracle_params(w.device)
    Wo = run["W0"].copy()
    t0 = time.time()
    worst, counts = 0.0, []
    for t, x, d in wl.input_stream(w):
        counts.append(oracle.pulsed_update(Wo, run["planes"], p, w.bl, w.update_management, x, d, w.lr,
                                           w.seed, t, cells=cells))
        err = np.abs(run["after"][t][r0:r1].astype(np.float64) - Wo[r0:r1].astype(np.float64)).max() / w.device["w_max"]
        worst = max(worst, float(err))
        assert err <= WEIGHT_TOL, f"{name} rows {r0}..{r1 - 1} after call {t}: {err:.3e}"
        if (t + 1) % 10 == 0 or w.steps <= 20:
            _say(capsys, f"  {name} rows {r0}..{r1 - 1}: oracle call {t + 1}/{w.steps} ({time.time() - t0:.0f} s)")
    _oracle_pulses[(name, slab)] = counts
    Wg = run["after"][-1][r0:r1]
    moved = np.abs(Wo[r0:r1] - run["W0"][r0:r1]).mean()
    _say(capsys, f"  {name} rows {r0}..{r1 - 1}: every cell, {w.steps} calls, max |dw|/w_max = {worst:.3e}, "
                 f"mean |w - w0| = {moved:.3e}")
    assert moved > 0                                       # the update did something
    bmax, bmin = run["planes"]["b_max"][r0:r1], run["planes"]["b_min"][r0:r1]
    assert np.isfinite(Wg).all()
    assert (Wg <= bmax * (1 + 1e-6) + 1e-12).all() and (Wg >= bmin * (1 + 1e-6) - 1e-12).all()
    if nslabs == 1:
        assert run["pulses"] == counts


@pytest.mark.parametrize("name", [n for n in wl.WORKLOADS if SLABS[n] > 1])
def test_full_size_pulse_totals_equal_oracle(name, capsys):
    """Applied pulses of every call: the device's counter against the oracle's count summed over
    the slabs (which the slab tests above have left behind; a slab not yet run is run here)."""
    w = wl.WORKLOADS[name]
    run = _gpu_run(name, capsys)
    for k in range(SLABS[name]):
        if (name, k) not in _oracle_pulses:
            test_full_size_workload_matches_oracle_on_every_cell(name, k, capsys)
    per_call = [sum(_oracle_pulses[(name, k)][t] for k in range(SLABS[name])) for t in range(w.steps)]
    _say(capsys, f"  {name}: pulses per call, first and last: GPU {run['pulses'][0]}, {run['pulses'][-1]}; "
                 f"oracle {per_call[0]}, {per_call[-1]}")
    assert run["pulses"] == per_call


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
