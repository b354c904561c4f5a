"""GPU parity of unit cells of several devices against the oracle's composition: shared pulse
trains, per-device response and noise, weighted sum, analog product on the effective weight."""
import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht

from common import gpu_params, oracle_params, to_dev
from test_gpu_mvm import IDEAL, NOISY

pytestmark = pytest.mark.gpu

DEVS = [
    dict(kind=aht.SOFT_BOUNDS, dw_min=0.002, dw_min_dtod=0.3, dw_min_std=0.3, w_max=0.6, w_max_dtod=0.2, w_min=-0.6,
         w_min_dtod=0.2),
    dict(kind=aht.LINEAR_STEP, dw_min=0.004, dw_min_dtod=0.1, dw_min_std=0.2, up_down=0.05, up_down_dtod=0.01,
         w_max=0.8, w_max_dtod=0.1, w_min=-0.8, w_min_dtod=0.1, gamma_up=0.4, gamma_down=0.6, gamma_dtod=0.1),
    dict(kind=aht.CONSTANT_STEP, dw_min=0.003, dw_min_std=0.0, w_max=0.5, w_min=-0.5),
]


@pytest.mark.parametrize("R,C,B,bl,um", [(70, 131, 24, 31, True), (64, 128, 40, 63, False)])
def test_unit_cell_updates_weights_and_products_match_the_oracle(R, C, B, bl, um):
    n = len(DEVS)
    seeds = [21, 22, 23]
    gamma = [1.0, 0.5, -0.25]
    g = np.random.default_rng(R + bl)
    tiles = [aht.Tile(R, C, gpu_params(dv), bl, um, s) for dv, s in zip(DEVS, seeds)]
    params = [oracle_params(dv) for dv in DEVS]
    planes = [oracle.device_planes(p, s, R, C) for p, s in zip(params, seeds)]
    Ws = [g.uniform(-0.2, 0.2, size=(R, C)).astype(np.float32) for _ in range(n)]
    for t_, W in zip(tiles, Ws):
        t_.set_weights(to_dev(W))
    cell = aht.UnitCell(tiles, gamma)
    totals = [0] * n
    for step, which in enumerate([-1, 1, -1, 2, 0]):
        x = g.normal(size=(B, C)).astype(np.float32)
        d = (g.normal(size=(B, R)) * 0.5).astype(np.float32)
        cell.pulsed_update(to_dev(x), to_dev(d), 0.05, which)
        counts = oracle.unit_cell_update(Ws, planes, params, seeds, bl, um, x, d, 0.05, step, which)
        totals = [a + b for a, b in zip(totals, counts)]
    for k, t_ in enumerate(tiles):
        Wg = t_.get_weights().cpu().numpy()
        assert t_.pulse_count() == totals[k] and totals[k] > 0
        assert t_.step == 5
        assert np.abs(Wg.astype(np.float64) - Ws[k]).max() / DEVS[k]["w_max"] <= 1e-5, k
    # effective weight: same fp32 operations in the same order
    eff_o = oracle.unit_cell_weights([t_.get_weights().cpu().numpy() for t_ in tiles], gamma)
    eff_g = cell.weights().cpu().numpy()
    assert (eff_g == eff_o).all()
    # analog product on the effective weight (device 0's seed and call counters)
    io_g, io_o = aht.IOParams(**NOISY), oracle.IOParams(**NOISY)
    xin = g.normal(size=(17, C)).astype(np.float32)
    y = cell.forward(to_dev(xin), io_g).cpu().numpy()
    yo = oracle.analog_mvm(eff_o, xin, io_o, seeds[0], 0)
    step_out = NOISY["out_res"] * np.abs(xin).max(axis=1, keepdims=True)
    diff = np.abs(y.astype(np.float64) - yo)
    assert (diff <= step_out * (1 + 1e-5) + 1e-9).all() and (diff <= 1e-6 * np.maximum(1, np.abs(yo))).mean() > 0.99
    din = g.normal(size=(9, R)).astype(np.float32)
    yb = cell.backward(to_dev(din), io_g).cpu().numpy()
    ybo = oracle.analog_mvm(eff_o, din, io_o, seeds[0], 0, transposed=True)
    step_out = NOISY["out_res"] * np.abs(din).max(axis=1, keepdims=True)
    diff = np.abs(yb.astype(np.float64) - ybo)
    assert (diff <= step_out * (1 + 1e-5) + 1e-9).all() and (diff <= 1e-6 * np.maximum(1, np.abs(ybo))).mean() > 0.99
    assert tiles[0].mvm_steps == (1, 1)
    for t_ in tiles:
        t_.close()


def test_unit_cell_product_follows_every_change_of_its_devices():
    """The product of a unit cell uses the devices' weights as they are at the call: between two
    products a device is updated, overwritten, decayed, reset, the factors change, another tile takes
    a device's place; a product with nothing changed in between gives the same result again."""
    R, C, bl = 48, 128, 31
    g = np.random.default_rng(5)
    seeds = [31, 32, 33]
    tiles = [aht.Tile(R, C, gpu_params(dv), bl, True, s) for dv, s in zip(DEVS, seeds)]
    spare = aht.Tile(R, C, gpu_params(DEVS[2]), bl, True, 34)
    for t_ in tiles + [spare]:
        t_.set_weights(to_dev(g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)))
    tiles[1].set_temporal(decay_rate=0.1, reset=0.05, reset_std=0.02)
    cell = aht.UnitCell(tiles, [1.0, 0.5, -0.25])
    io_g, io_o = aht.IOParams(**IDEAL), oracle.IOParams(**IDEAL)
    xin = g.normal(size=(8, C)).astype(np.float32)
    din = g.normal(size=(8, R)).astype(np.float32)
    calls = [0, 0]

    def check(what):
        eff = oracle.unit_cell_weights([t_.get_weights().cpu().numpy() for t_ in cell.devices], cell.gamma)
        for transposed, inp in ((False, xin), (True, din)):
            y = (cell.backward if transposed else cell.forward)(to_dev(inp), io_g).cpu().numpy()
            yo = oracle.analog_mvm(eff, inp, io_o, seeds[0], calls[transposed], transposed=transposed)
            calls[transposed] += 1
            assert np.abs(y - yo).max() <= 1e-5 * np.abs(yo).max(), (what, transposed)
        return eff

    e0 = check("first")
    assert (check("nothing changed") == e0).all()
    x = g.normal(size=(16, C)).astype(np.float32)
    d = g.normal(size=(16, R)).astype(np.float32)
    cell.pulsed_update(to_dev(x), to_dev(d), 0.1, 1)
    e1 = check("one device updated through the cell")
    assert (e1 != e0).any()
    tiles[2].pulsed_update(to_dev(x), to_dev(d), 0.1)
    e2 = check("a device updated on its own")
    assert (e2 != e1).any()
    tiles[0].set_weights(to_dev(g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)))
    e3 = check("weights of the leading device overwritten")
    assert (e3 != e2).any()
    tiles[1].decay_diffuse()
    e4 = check("a device decayed")
    assert (e4 != e3).any()
    tiles[1].reset_columns(3, 2)
    e5 = check("columns of a device reset")
    assert (e5 != e4).any()
    cell.gamma = [1.0, 0.5, 0.75]
    e6 = check("factors changed")
    assert (e6 != e5).any()
    src = aht.Tile(R, C, gpu_params(DEVS[0]), bl, True, 35)
    src.set_weights(to_dev(g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)))
    src.transfer_column_to(tiles[2], 7, 0.5, io_g)
    e7 = check("a device received a transferred column")
    assert (e7 != e6).any()
    cell.devices[2] = spare
    e8 = check("another tile in a device's place")
    assert (e8 != e7).any()
    assert (check("nothing changed again") == e8).all()
    for t_ in tiles + [spare, src]:
        t_.close()


def test_unit_cell_devices_beside_each_other_and_in_two_shapes_change_no_bit(monkeypatch):
    """All devices updated: those after the first run on streams of their own tiles, and a 256 x 768 tile
    (1.5 waves per SIMD at two rows per lane) takes some strips at one row per lane.  Same bits as one
    device after the other in a single shape."""
    R, C, B, bl = 256, 768, 20, 31
    g = np.random.default_rng(8)
    W0 = [g.uniform(-0.2, 0.2, size=(R, C)).astype(np.float32) for _ in DEVS]
    xs = [g.normal(size=(B, C)).astype(np.float32) for _ in range(3)]
    ds = [g.normal(size=(B, R)).astype(np.float32) for _ in range(3)]
    out = {}
    for mode in ("0", "2"):
        monkeypatch.setenv("AHT_EVEN_ROUND", mode)
        tiles = [aht.Tile(R, C, gpu_params(dv), bl, True, 40 + k) for k, dv in enumerate(DEVS)]
        for t_, W in zip(tiles, W0):
            t_.set_weights(to_dev(W))
        cell = aht.UnitCell(tiles, [1.0, 0.5, -0.25])
        for x, d, which in zip(xs, ds, (-1, 2, -1)):
            cell.pulsed_update(to_dev(x), to_dev(d), 0.1, which)
        out[mode] = ([t_.get_weights().cpu().numpy() for t_ in tiles], [t_.pulse_count() for t_ in tiles])
        for t_ in tiles:
            t_.close()
    assert out["0"][1] == out["2"][1] and all(p > 0 for p in out["0"][1])
    for a, b in zip(out["0"][0], out["2"][0]):
        assert (a.view(np.uint32) == b.view(np.uint32)).all()


def test_unit_cell_rejects_mismatched_devices():
    a = aht.Tile(64, 64, aht.DeviceParams(), 31, False, 1)
    b = aht.Tile(64, 128, aht.DeviceParams(), 31, False, 2)
    c = aht.Tile(64, 64, aht.DeviceParams(), 63, False, 3)
    x, d = to_dev(np.zeros((1, 64), np.float32)), to_dev(np.zeros((1, 64), np.float32))
    for devices in ([a, b], [a, c], [a, a]):
        with pytest.raises(aht.AhtError):
            aht.UnitCell(devices).pulsed_update(x, d, 0.1)
    with pytest.raises(aht.AhtError):
        aht.UnitCell([a]).pulsed_update(x, d, 0.1, which=1)
    for t_ in (a, b, c):
        t_.close()
