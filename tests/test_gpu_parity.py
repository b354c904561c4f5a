"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Bar: bit-exact for everything integer (Philox words, pulse words, counts, signs,
number of applied pulses, integer-step weights); fp32 weights within
1e-5 * w_max absolute after the full number of update calls.
"""
import os

import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht
from paper_2104_02184_amd import workloads as wl

from common import (gpu_params, gpu_planes, make_tile, oracle_params, run_gpu, run_oracle, to_dev,
                    words_to_np)

pytestmark = pytest.mark.gpu
WEIGHT_TOL = 1e-5          # absolute, in units of w_max


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    aht.load_library()
    yield


@pytest.fixture()
def env():
    """set AHT_* launch overrides for one test and restore them afterwards"""
    saved = {k: os.environ.get(k) for k in ("AHT_RPL", "AHT_QWORDS")}

    def setter(**kw):
        for k, v in kw.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = str(v)
    yield setter
    for k, v in saved.items():
        if v is None:
            os.environ.pop(k, None)
        else:
            os.environ[k] = v


# ------------------------------------------------------------------ random streams
def test_philox_bit_exact_on_random_counters():
    import torch
    g = np.random.default_rng(0)
    n = 200_000
    ctr = g.integers(0, 2**32, size=(n, 4), dtype=np.uint64).astype(np.uint32)
    key = g.integers(0, 2**32, size=(n, 2), dtype=np.uint64).astype(np.uint32)
    ctr[0] = 0
    key[0] = 0
    ctr[1] = 0xFFFFFFFF
    key[1] = 0xFFFFFFFF
    got = aht.debug_philox(to_dev(ctr.view(np.int32)), to_dev(key.view(np.int32))).cpu().numpy().view(np.uint32)
    assert [f"{v:08x}" for v in got[0]] == ["6627e8d5", "e169c58d", "bc57ac4c", "9b00dbd8"]
    idx = np.concatenate([np.arange(64), g.integers(0, n, size=4000)])
    for k in idx:
        assert (got[k] == oracle.philox4x32_10(ctr[k], key[k])).all()


def test_gaussians_fast_and_accurate_against_oracle():
    seed, index, t = 0x1234ABCD5678, 4242, 17
    n = 40_000
    want = np.array([oracle.gauss(seed, index, t, q, oracle.TAG_C2C) for q in range(n)], dtype=np.float32)
    acc = aht.debug_gauss(seed, index, t, oracle.TAG_C2C, 0, n, fast=False).cpu().numpy()
    fast = aht.debug_gauss(seed, index, t, oracle.TAG_C2C, 0, n, fast=True).cpu().numpy()
    # creation-time variant: fp64 evaluation, one rounding -> at most one fp32 ulp away, almost always equal
    ulp = np.spacing(np.abs(want))
    assert (np.abs(acc - want) <= ulp).all()
    assert (acc == want).mean() > 0.999
    # hot-path variant on the transcendental unit: the tolerance budget allows 7e-5, demand 2e-5
    err = np.abs(fast.astype(np.float64) - want.astype(np.float64))
    print("fast gauss max abs err", err.max(), "mean", err.mean())
    assert err.max() < 2e-5
    assert err.mean() < 2e-6


def test_device_planes_match_oracle():
    for kind, kw in [(aht.CONSTANT_STEP, {}), (aht.LINEAR_STEP, dict(gamma_up=0.1, gamma_down=0.2, gamma_dtod=0.3)),
                     (aht.SOFT_BOUNDS, {})]:
        dev = dict(kind=kind, dw_min=0.001, dw_min_dtod=0.3, dw_min_std=0.3, up_down=0.02, up_down_dtod=0.01,
                   w_max=0.6, w_max_dtod=0.3, w_min=-0.6, w_min_dtod=0.3, gamma_up=0.0, gamma_down=0.0,
                   gamma_dtod=0.0)
        dev.update(kw)
        R, C, seed = 70, 130, 99
        want = oracle.device_planes(oracle_params(dev), seed, R, C)
        with aht.Tile(R, C, gpu_params(dev), 31, False, seed) as tile:
            got = gpu_planes(tile)
        for name in aht.PLANE_NAMES:
            a, b = got[name].astype(np.float64), want[name].astype(np.float64)
            rel = np.abs(a - b) / np.maximum(np.abs(b), 1e-30)
            assert (rel[b != 0] <= 1e-6).all(), name
            assert (a[b == 0] == 0).all(), name
            assert (got[name] == want[name]).mean() > 0.999, name


# ------------------------------------------------------------------ pulse words, counts
def _edge_inputs(w, x, d):
    x, d = x.copy(), d.copy()
    x[0, 0] = 0.0
    x[0, 1] = np.nan
    x[0, 2] = np.inf
    x[0, 3] = -1e30          # saturates
    d[0, 0] = -0.0
    d[0, 1] = -np.inf
    d[0, 2] = 1e30
    if x.shape[0] > 1:
        x[1, :] = 0.0        # whole sample without x pulses (skipped under update management)
    if x.shape[0] > 2:
        d[2, :] = 0.0
    return x, d


SMALL_CASES = [
    ("cfg1_64x64_constant", dict()),
    ("cfg2_512x512_constant_d2d", dict(rows=96, cols=200, batch=9)),
    ("cfg3_1024x1024_softbounds", dict(rows=130, cols=70, batch=17)),
    ("cfg4_conv_256x2304", dict(rows=37, cols=300, batch=203)),
    ("cfg5_4096x4096_linearstep", dict(rows=150, cols=333, batch=21)),
]


@pytest.mark.parametrize("name,shape", SMALL_CASES)
def test_pulse_words_and_counts_bit_exact(name, shape):
    w = wl.scaled(wl.WORKLOADS[name], **shape) if shape else wl.WORKLOADS[name]
    tile = make_tile(w)
    for t, x, d in wl.input_stream(w):
        if t >= 3:
            break
        if t == 1:
            x, d = _edge_inputs(w, x, d)
        tile.step = t
        xw, dw = tile.debug_pulse_words(to_dev(x), to_dev(d), w.lr)
        oxw, odw = oracle.pulse_words(x, d, w.lr, w.device["dw_min"], w.bl, w.update_management, w.seed, t)
        assert (words_to_np(xw) == oxw).all()
        assert (words_to_np(dw) == odw).all()
        for b in {0, w.batch - 1}:
            got = tile.debug_counts(xw, dw, b).cpu().numpy()
            assert (got == oracle.counts(oxw, odw, b, w.bl)).all()
    tile.close()


@pytest.mark.parametrize("bl", [1, 5, 31, 32, 63])
def test_pulse_words_every_length_and_saturation(bl):
    g = np.random.default_rng(bl)
    R, C, B = 20, 70, 6
    dev = dict(kind=aht.CONSTANT_STEP, dw_min=0.001, w_max=1.0, w_min=-1.0)
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    x[0] = 1e3
    d[0] = -1e3
    for um in (False, True):
        with aht.Tile(R, C, aht.DeviceParams(**dev), bl, um, seed=5) as tile:
            tile.step = 7
            xw, dw = tile.debug_pulse_words(to_dev(x), to_dev(d), 0.01)
            oxw, odw = oracle.pulse_words(x, d, 0.01, 0.001, bl, um, 5, 7)
            assert (words_to_np(xw) == oxw).all() and (words_to_np(dw) == odw).all()
            if not um:
                assert (tile.debug_counts(xw, dw, 0).cpu().numpy() == bl).all()


@pytest.mark.parametrize("bl", [1, 4, 13, 31, 32, 47, 63])
@pytest.mark.parametrize("um", [False, True])
def test_pulse_words_with_few_to_all_lines_needing_random_numbers(bl, um):
    """Waves in which 0, 1, a few, most or all line values lie strictly between zero and
    saturation (the library shares the random blocks of sparse waves among all lanes), ragged
    tails in both directions, zeros after a rectifier, saturated and negative values."""
    g = np.random.default_rng(100 + bl)
    R, C, B = 150, 333, 12
    dev = dict(kind=aht.CONSTANT_STEP, dw_min=0.001, w_max=1.0, w_min=-1.0)
    lr = 0.02
    x = np.zeros((B, C), dtype=np.float32)
    d = np.zeros((B, R), dtype=np.float32)
    fractions = [0.0, 0.01, 0.05, 0.2, 0.4, 0.6, 0.63, 0.7, 0.9, 1.0, 0.3, 0.5]
    for b, f in enumerate(fractions):
        for arr, n in ((x, C), (d, R)):
            v = g.normal(size=n).astype(np.float32) * 0.05          # partial probabilities
            kind = g.random(n)
            v[kind > f] = 0.0                                        # zeros
            sat = (kind > f) & (g.random(n) < 0.3)
            v[sat] = np.where(g.random(sat.sum()) < 0.5, 50.0, -50.0)   # saturated, both signs
            arr[b] = v
    x[10, :64] = g.normal(size=64).astype(np.float32) * 0.05         # one full wave beside sparse ones
    with aht.Tile(R, C, aht.DeviceParams(**dev), bl, um, seed=11) as tile:
        for t in (0, 3):
            tile.step = t
            xw, dw = tile.debug_pulse_words(to_dev(x), to_dev(d), lr)
            oxw, odw = oracle.pulse_words(x, d, lr, 0.001, bl, um, 11, t)
            assert (words_to_np(xw) == oxw).all()
            assert (words_to_np(dw) == odw).all()
    # the inputs do span the cases: a sample without, with few and with only partial line values
    partial = (np.abs(x) > 0) & (np.abs(x) < 1)
    assert partial[0].sum() == 0 and 0 < partial[1].sum() < 10 and partial[9].sum() == C


# ------------------------------------------------------------------ integer-exact weights
@pytest.mark.parametrize("rpl", [1, 2, 4])
@pytest.mark.parametrize("bl,R,C,B", [(31, 45, 77, 13), (63, 70, 130, 22), (63, 16, 64, 4)])
def test_integer_step_weights_prove_counts_signs_and_order(env, rpl, bl, R, C, B):
    env(AHT_RPL=rpl)
    g = np.random.default_rng(100 + bl + R)
    dev = dict(kind=aht.CONSTANT_STEP, dw_min=1.0, w_max=2.0**20, w_min=-2.0**20)
    x = g.normal(size=(B, C)).astype(np.float32)
    d = g.normal(size=(B, R)).astype(np.float32)
    lr, seed, t = 20.0, 3, 9
    with aht.Tile(R, C, aht.DeviceParams(**dev), bl, False, seed) as tile:
        tile.step = t
        tile.pulsed_update(to_dev(x), to_dev(d), lr)
        W = tile.get_weights().cpu().numpy()
        pulses = tile.pulse_count()
        assert tile.step == t + 1
    xw, dw = oracle.pulse_words(x, d, lr, 1.0, bl, False, seed, t)
    tot = sum(oracle.counts(xw, dw, b, bl).astype(np.int64) for b in range(B))
    assert (W == tot).all()
    assert pulses == sum(np.abs(oracle.counts(xw, dw, b, bl).astype(np.int64)).sum() for b in range(B))


def test_sequential_clipping_through_injected_words():
    # 6 UP pulses clip at the bound, then 4 DOWN pulses: sequential result, not the digital sum
    import torch
    R, C = 3, 5
    dev = dict(kind=aht.CONSTANT_STEP, dw_min=0.05, w_max=1.0, w_min=-1.0)
    XW = np.zeros((2, C), dtype=np.uint64)
    DW = np.zeros((2, R), dtype=np.uint64)
    XW[0, :] = ((1 << 6) - 1) | (1 << 63)
    XW[1, :] = (1 << 4) - 1
    DW[:, :] = (1 << 31) - 1
    with aht.Tile(R, C, aht.DeviceParams(**dev), 31, False, 1) as tile:
        tile.set_weights(to_dev(np.full((R, C), 0.9, dtype=np.float32)))
        tile.debug_apply_words(to_dev(XW.view(np.int64)), to_dev(DW.view(np.int64)), 0)
        W = tile.get_weights().cpu().numpy()
        planes = gpu_planes(tile)
    Wo = np.full((R, C), 0.9, dtype=np.float32)
    oracle.apply_words(Wo, planes, oracle.CONSTANT_STEP, 0.0, XW, DW, 31, 1, 0)
    assert (W == Wo).all()
    assert np.allclose(W, 0.8, atol=1e-6)


# ------------------------------------------------------------------ weights, small shapes
def _weight_parity(w, steps, env_kw=None, tol=WEIGHT_TOL):
    tile = make_tile(w)
    planes = gpu_planes(tile)
    oplanes = oracle.device_planes(oracle_params(w.device), w.seed, w.rows, w.cols)
    for n in aht.PLANE_NAMES:
        assert np.allclose(planes[n], oplanes[n], rtol=1e-6, atol=0), n
    W0 = wl.initial_weights(w)
    W0 = np.clip(W0, oplanes["b_min"], oplanes["b_max"]).astype(np.float32)
    Wg, pg = run_gpu(w, W0, steps=steps, tile=tile)
    tile.close()
    Wo, po = run_oracle(w, W0, oplanes, steps=steps)
    assert pg == po                                    # number of applied coincidences: exact
    err = np.abs(Wg.astype(np.float64) - Wo.astype(np.float64)).max() / w.device["w_max"]
    print(w.name, "steps", steps, "pulses", pg, "max |dw|/w_max", err)
    assert err <= tol
    assert (Wg <= oplanes["b_max"]).all() and (Wg >= oplanes["b_min"]).all()
    return Wg


@pytest.mark.parametrize("name,shape,steps", [
    ("cfg1_64x64_constant", dict(), 10),
    ("cfg2_512x512_constant_d2d", dict(rows=96, cols=200, batch=64), 12),
    ("cfg3_1024x1024_softbounds", dict(rows=130, cols=70, batch=128), 12),
    ("cfg4_conv_256x2304", dict(rows=37, cols=300, batch=1003), 3),
    ("cfg5_4096x4096_linearstep", dict(rows=150, cols=333, batch=256), 6),
])
@pytest.mark.parametrize("rpl", [1, 4])
def test_weights_small_shapes_every_workload(env, name, shape, steps, rpl):
    env(AHT_RPL=rpl)
    w = wl.scaled(wl.WORKLOADS[name], **shape) if shape else wl.WORKLOADS[name]
    _weight_parity(w, steps)


def test_cfg1_noiseless_constant_step_is_bit_identical():
    w = wl.WORKLOADS["cfg1_64x64_constant"]
    tile = make_tile(w)
    oplanes = oracle.device_planes(oracle_params(w.device), w.seed, w.rows, w.cols)
    W0 = wl.initial_weights(w)
    Wg, pg = run_gpu(w, W0, tile=tile)
    Wo, po = run_oracle(w, W0, oplanes)
    assert pg == po and (Wg == Wo).all()


@pytest.mark.parametrize("qwords", [5, 7, 40])
def test_small_and_large_streams_give_identical_bits(env, qwords):
    # tiny stream storage forces many early drains (streams restart at q & 31 != 0)
    w = wl.scaled(wl.WORKLOADS["cfg5_4096x4096_linearstep"], rows=64, cols=128, batch=250, steps=2)
    W0 = wl.initial_weights(w)
    env(AHT_RPL=4, AHT_QWORDS=None)
    ref, pr = run_gpu(w, W0)
    for rpl in (1, 2, 4):
        env(AHT_RPL=rpl, AHT_QWORDS=qwords)
        got, pg = run_gpu(w, W0)
        assert pg == pr and (got == ref).all(), (rpl, qwords)


def test_launch_shape_chosen_from_the_pulse_rate_changes_no_bit(env):
    # from 400 k cells on the library picks rows per lane from the tile's own pulse rate, which
    # it learns over the first calls: a sequence that starts with the static choice and changes
    # it on the way gives the bits of a sequence run with a fixed shape
    w = wl.scaled(wl.WORKLOADS["cfg3_1024x1024_softbounds"], rows=640, cols=704, batch=24, steps=7)
    W0 = wl.initial_weights(w)
    env(AHT_RPL=2, AHT_QWORDS=None)
    ref, pr = run_gpu(w, W0)
    env(AHT_RPL=None, AHT_QWORDS=None)
    got, pg = run_gpu(w, W0)
    assert pg == pr and (got == ref).all()
    env(AHT_RPL=4, AHT_QWORDS=None)
    got4, p4 = run_gpu(w, W0)
    assert p4 == pr and (got4 == ref).all()


@pytest.mark.parametrize("R,C,B,bl,kind,c2c,deterministic", [
    (64, 64, 1, 31, aht.CONSTANT_STEP, 0.0, False),        # the smallest workload's shape
    (64, 64, 1, 31, aht.CONSTANT_STEP, 0.3, False),
    (37, 70, 3, 31, aht.SOFT_BOUNDS, 0.3, False),          # ragged rows and columns
    (20, 130, 8, 63, aht.LINEAR_STEP, 0.3, False),         # 64-bit words, the most vectors one launch takes
    (16, 64, 2, 17, aht.LINEAR_STEP, 0.0, True),           # deterministic trains
])
def test_whole_call_in_one_launch_changes_no_bit(R, C, B, bl, kind, c2c, deterministic, monkeypatch):
    """Tiny tiles with a few update vectors take the whole call in one launch, every workgroup drawing the
    pulse words it needs.  Same weights, pulse counts and step counter, bit for bit, as the two-kernel path,
    call after call; and the oracle's result."""
    dev = dict(kind=kind, dw_min=0.004, dw_min_dtod=0.3, dw_min_std=c2c, w_max=0.6, w_max_dtod=0.2, w_min=-0.6,
               w_min_dtod=0.2, gamma_up=0.4, gamma_down=0.6, gamma_dtod=0.1)
    g = np.random.default_rng(R * C + B)
    W0 = g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)
    calls = 4
    xs = [g.normal(size=(B, C)).astype(np.float32) for _ in range(calls)]
    ds = [g.normal(size=(B, R)).astype(np.float32) * np.float32(0.7) for _ in range(calls)]
    xs[1][0, :5] = [0.0, np.nan, np.inf, 50.0, -50.0]                   # zero, non-finite and saturated lines
    out = {}
    for mode in ("0", "1"):
        monkeypatch.setenv("AHT_FUSED", mode)
        tile = aht.Tile(R, C, gpu_params(dev), bl, False, 9)
        if deterministic:
            tile.set_pulse_mode(deterministic=True)
        tile.set_weights(to_dev(W0))
        steps = []
        for x, d in zip(xs, ds):
            tile.pulsed_update(to_dev(x), to_dev(d), 0.2)
            steps.append((tile.get_weights().cpu().numpy(), tile.pulse_count(), tile.step, tile.sync_step()))
        assert tile.launch_info()["stream_words"] == (0 if mode == "1" else 12)      # the path that was asked for
        tile.close()
        out[mode] = steps
    for k, ((w0, p0, s0, d0), (w1, p1, s1, d1)) in enumerate(zip(out["0"], out["1"])):
        assert p0 == p1 and s0 == s1 == d0 == d1 == k + 1
        assert (w0.view(np.uint32) == w1.view(np.uint32)).all()
    assert out["1"][-1][1] > 0
    planes = oracle.device_planes(oracle.DeviceParams(**dev), 9, R, C)
    Wo, po = W0.copy(), 0
    for t, (x, d) in enumerate(zip(xs, ds)):
        po += oracle.pulsed_update(Wo, planes, oracle.DeviceParams(**dev), bl, False, x, d, 0.2, 9, t,
                                   train_kind=oracle.DETERMINISTIC if deterministic else oracle.STOCHASTIC)
    assert po == out["1"][-1][1]
    assert np.abs(out["1"][-1][0].astype(np.float64) - Wo).max() / 0.6 <= WEIGHT_TOL


@pytest.mark.parametrize("R,C,B,d_std,x_scale,lr,kind,c2c,qwords", [
    (64, 320, 1500, 0.01, 1.0, 0.1, aht.CONSTANT_STEP, 0.3, None),    # the conv workload's law: most row trains empty
    (37, 150, 1203, 0.01, 1.0, 0.1, aht.SOFT_BOUNDS, 0.3, None),      # ragged rows, columns and batch
    (23, 70, 999, 0.004, 1.0, 0.1, aht.LINEAR_STEP, 0.0, 6),          # very sparse, no noise, short streams: many drains
    (16, 128, 515, 0.3, 3.0, 0.5, aht.CONSTANT_STEP, 0.3, 7),         # dense and partly saturated: groups with large
                                                                      # counts take the sample-by-sample path
    (8, 64, 3, 0.05, 1.0, 0.1, aht.CONSTANT_STEP, 0.3, None),         # fewer samples than one group
])
def test_walking_row_lists_changes_no_bit(R, C, B, d_std, x_scale, lr, kind, c2c, qwords, monkeypatch):
    """Long batches whose row trains are mostly empty walk, per row, a list of the samples that have
    a pulse instead of all samples.  Same weights and pulse counts, bit for bit, call after call, whether
    the lists are forced on or off; and the oracle's pulse total."""
    dev = dict(kind=kind, dw_min=0.002, dw_min_dtod=0.3, dw_min_std=c2c, w_max=0.6, w_max_dtod=0.2, w_min=-0.6,
               w_min_dtod=0.2, gamma_up=0.4, gamma_down=0.6, gamma_dtod=0.1)
    g = np.random.default_rng(R + C)
    W0 = g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)
    calls = 2
    xs = [(np.maximum(g.normal(size=(B, C)), 0) * x_scale).astype(np.float32) for _ in range(calls)]
    ds = [(g.normal(size=(B, R)) * d_std).astype(np.float32) for _ in range(calls)]
    if qwords:
        monkeypatch.setenv("AHT_QWORDS", str(qwords))
    out = {}
    for mode in ("0", "1"):
        monkeypatch.setenv("AHT_ROWLISTS", mode)
        tile = aht.Tile(R, C, gpu_params(dev), 31, False, 5)
        tile.set_weights(to_dev(W0))
        steps = []
        for x, d in zip(xs, ds):
            tile.pulsed_update(to_dev(x), to_dev(d), lr)
            steps.append((tile.get_weights().cpu().numpy(), tile.pulse_count()))
        tile.close()
        out[mode] = steps
    for (w0, p0), (w1, p1) in zip(out["0"], out["1"]):
        assert p0 == p1 and p0 > 0
        assert (w0.view(np.uint32) == w1.view(np.uint32)).all()
    # and against the oracle: applied pulses equal, weights within the tolerance
    planes = oracle.device_planes(oracle.DeviceParams(**dev), 5, R, C)
    Wo, po = W0.copy(), 0
    for t, (x, d) in enumerate(zip(xs, ds)):
        po += oracle.pulsed_update(Wo, planes, oracle.DeviceParams(**dev), 31, False, x, d, lr, 5, t)
    assert po == out["1"][-1][1]
    assert np.abs(out["1"][-1][0].astype(np.float64) - Wo).max() / 0.6 <= WEIGHT_TOL


@pytest.mark.parametrize("R,C,B,lr,calls,kind,bl", [
    (256, 2304, 48, 0.1, 3, aht.CONSTANT_STEP, 31),      # two rows per lane on 32 strips, one on 4
    (256, 2304, 48, 0.1, 3, aht.SOFT_BOUNDS, 63),
    (500, 784, 24, 0.1, 3, aht.SOFT_BOUNDS, 31),         # ragged in both directions
    (1024, 576, 16, 0.02, 6, aht.LINEAR_STEP, 31),       # few pulses: four rows per lane on 8 strips once the
])                                                       # tile has seen its pulse rate, one row on the ninth
def test_two_shapes_in_one_launch_change_no_bit(R, C, B, lr, calls, kind, bl, monkeypatch):
    """A tile whose waves do not fill the SIMDs a whole number of times (256 x 2304 at two rows per lane:
    4.5 waves per SIMD) runs most column strips at the chosen rows per lane and a few at fewer, in one
    launch of two shapes.  Same weights and pulse counts, bit for bit, as the single shape, call after
    call."""
    dev = dict(kind=kind, dw_min=0.002, dw_min_dtod=0.3, dw_min_std=0.3, w_max=0.6, w_max_dtod=0.2, w_min=-0.6,
               w_min_dtod=0.2, gamma_up=0.4, gamma_down=0.6, gamma_dtod=0.1)
    g = np.random.default_rng(bl + R)
    W0 = g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)
    xs = [g.normal(size=(B, C)).astype(np.float32) for _ in range(calls)]
    ds = [g.normal(size=(B, R)).astype(np.float32) for _ in range(calls)]
    out = {}
    for mode in ("0", "2"):
        monkeypatch.setenv("AHT_EVEN_ROUND", mode)
        tile = aht.Tile(R, C, gpu_params(dev), bl, True, 77)
        tile.set_weights(to_dev(W0))
        steps = []
        for x, d in zip(xs, ds):
            tile.pulsed_update(to_dev(x), to_dev(d), lr)
            steps.append(tile.get_weights().cpu().numpy())
        out[mode] = (steps, tile.pulse_count())
        tile.close()
    assert out["0"][1] == out["2"][1] > 0
    for a, b in zip(out["0"][0], out["2"][0]):
        assert (a.view(np.uint32) == b.view(np.uint32)).all()
    assert (out["0"][0][0] != W0).any()


def test_saturated_lines_fill_whole_trains(env):
    # every sample has 63 coincidences per cell: queues overflow often, counts are maximal
    R, C, B, bl = 33, 65, 40, 63
    dev = dict(kind=aht.SOFT_BOUNDS, dw_min=0.002, dw_min_std=0.3, w_max=0.6, w_min=-0.6)
    g = np.random.default_rng(1)
    x = (g.choice([-1.0, 1.0], size=(B, C)) * 1e3).astype(np.float32)
    d = (g.choice([-1.0, 1.0], size=(B, R)) * 1e3).astype(np.float32)
    oplanes = oracle.device_planes(oracle_params(dev), 4, R, C)
    Wo = np.zeros((R, C), dtype=np.float32)
    n = oracle.pulsed_update(Wo, oplanes, oracle_params(dev), bl, False, x, d, 0.1, 4, 0)
    assert n == R * C * B * bl
    for rpl in (1, 4):
        env(AHT_RPL=rpl)
        with aht.Tile(R, C, gpu_params(dev), bl, False, 4) as tile:
            tile.pulsed_update(to_dev(x), to_dev(d), 0.1)
            Wg = tile.get_weights().cpu().numpy()
            assert tile.pulse_count() == n
        assert np.abs(Wg - Wo).max() / 0.6 <= WEIGHT_TOL


# ------------------------------------------------------------------ degenerate calls
def test_zero_inputs_empty_batch_and_zero_lr_change_nothing():
    import torch
    w = wl.scaled(wl.WORKLOADS["cfg5_4096x4096_linearstep"], rows=40, cols=70, batch=5)
    tile = make_tile(w)
    W0 = wl.initial_weights(w)
    tile.set_weights(to_dev(W0))
    g = np.random.default_rng(0)
    x = g.normal(size=(5, 70)).astype(np.float32)
    d = g.normal(size=(5, 40)).astype(np.float32)
    tile.pulsed_update(to_dev(np.zeros_like(x)), to_dev(d), 0.1)
    tile.pulsed_update(to_dev(x), to_dev(np.zeros_like(d)), 0.1)
    tile.pulsed_update(to_dev(x), to_dev(d), 0.0)
    tile.pulsed_update(torch.empty((0, 70), device="cuda"), torch.empty((0, 40), device="cuda"), 0.1)
    assert tile.step == 4
    assert (tile.get_weights().cpu().numpy() == W0).all()
    assert tile.pulse_count() == 0
    with pytest.raises(aht.AhtError):
        tile.pulsed_update(to_dev(x), to_dev(d), -1.0)
    with pytest.raises(aht.AhtError):
        tile.pulsed_update(to_dev(x), to_dev(d), float("nan"))
    with pytest.raises(ValueError):
        tile.pulsed_update(to_dev(x[:, :5].copy()), to_dev(d), 0.1)
    assert tile.step == 4
    tile.close()


def test_resume_from_saved_state_is_bit_identical():
    w = wl.scaled(wl.WORKLOADS["cfg2_512x512_constant_d2d"], rows=64, cols=96, batch=16, steps=4)
    W0 = wl.initial_weights(w)
    full, _ = run_gpu(w, W0, steps=4)
    inputs = list(wl.input_stream(w))
    a = make_tile(w)
    a.set_weights(to_dev(W0))
    for t, x, d in inputs[:2]:
        a.pulsed_update(to_dev(x), to_dev(d), w.lr)
    saved_w, saved_step = a.get_weights().clone(), a.step
    a.close()
    b = make_tile(w)
    b.set_weights(saved_w)
    b.step = saved_step
    for t, x, d in inputs[2:4]:
        b.pulsed_update(to_dev(x), to_dev(d), w.lr)
    assert (b.get_weights().cpu().numpy() == full).all()
    b.close()


def test_setting_planes_overrides_the_drawn_ones():
    import torch
    w = wl.scaled(wl.WORKLOADS["cfg5_4096x4096_linearstep"], rows=32, cols=64, batch=8, steps=2)
    tile = make_tile(w)
    g = np.random.default_rng(2)
    planes = {
        "dw_up": g.uniform(0.0005, 0.002, (32, 64)), "dw_down": g.uniform(0.0005, 0.002, (32, 64)),
        "b_max": g.uniform(0.3, 0.8, (32, 64)), "b_min": -g.uniform(0.3, 0.8, (32, 64)),
        "slope_up": g.uniform(0.0, 0.5, (32, 64)), "slope_down": -g.uniform(0.0, 0.5, (32, 64)),
    }
    planes = {k: v.astype(np.float32) for k, v in planes.items()}
    for k, v in planes.items():
        tile.set_plane(k, to_dev(v))
    W0 = wl.initial_weights(w)
    Wg, pg = run_gpu(w, W0, tile=tile)
    Wo, po = run_oracle(w, W0, planes)
    tile.close()
    assert pg == po
    assert np.abs(Wg - Wo).max() / 0.6 <= WEIGHT_TOL
    # slope planes are derived, not settable, unless the device is LINEAR_STEP
    with aht.Tile(8, 8, aht.DeviceParams(kind=aht.SOFT_BOUNDS, w_max=0.5, w_min=-0.25), 31) as sb:
        assert np.allclose(sb.get_plane("slope_up").cpu().numpy(), 2.0)
        assert np.allclose(sb.get_plane("slope_down").cpu().numpy(), -4.0)
        with pytest.raises(aht.AhtError):
            sb.set_plane("slope_up", torch.zeros((8, 8), device="cuda"))


def test_more_samples_than_one_grid_dimension_holds():
    # B above 32768 makes the pulse-word kernel loop over samples inside one launch
    R, C, B, bl = 5, 70, 40_000, 31
    dev = dict(kind=aht.CONSTANT_STEP, dw_min=0.0005, dw_min_std=0.3, w_max=0.6, w_min=-0.6)
    g = np.random.default_rng(7)
    x = g.normal(size=(B, C)).astype(np.float32)
    d = (g.normal(size=(B, R)) * 0.05).astype(np.float32)
    oplanes = oracle.device_planes(oracle_params(dev), 11, R, C)
    Wo = np.zeros((R, C), dtype=np.float32)
    po = oracle.pulsed_update(Wo, oplanes, oracle_params(dev), bl, False, x, d, 0.01, 11, 0)
    with aht.Tile(R, C, gpu_params(dev), bl, False, 11) as tile:
        xw, dw = tile.debug_pulse_words(to_dev(x), to_dev(d), 0.01)
        oxw, odw = oracle.pulse_words(x, d, 0.01, 0.0005, bl, False, 11, 0)
        assert (words_to_np(xw) == oxw).all() and (words_to_np(dw) == odw).all()
        tile.pulsed_update(to_dev(x), to_dev(d), 0.01)
        Wg = tile.get_weights().cpu().numpy()
        assert tile.pulse_count() == po
    assert np.abs(Wg - Wo).max() / 0.6 <= WEIGHT_TOL


def test_two_tiles_on_two_streams():
    import torch
    w = wl.scaled(wl.WORKLOADS["cfg3_1024x1024_softbounds"], rows=128, cols=192, batch=32, steps=3)
    W0 = wl.initial_weights(w)
    ref, _ = run_gpu(w, W0)
    tiles = [make_tile(w), make_tile(w)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    inputs = [(to_dev(x), to_dev(d)) for _, x, d in wl.input_stream(w)]
    torch.cuda.synchronize()
    for tile, s in zip(tiles, streams):
        with torch.cuda.stream(s):
            tile.set_weights(to_dev(W0))
    for xd, dd in inputs:
        for tile, s in zip(tiles, streams):
            with torch.cuda.stream(s):
                tile.pulsed_update(xd, dd, w.lr)
    torch.cuda.synchronize()
    for tile in tiles:
        assert (tile.get_weights().cpu().numpy() == ref).all()
        tile.close()
