"""GPU parity of the analog matrix-vector product (forward and transposed) against the oracle.
Continuous values (the value entering the ADC) must agree within fp32 accumulation error; ADC
codes must be equal except where the oracle's value sits within that error of a rounding
boundary, and then differ by one step at most."""
import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht

from common import gpu_params, to_dev

pytestmark = pytest.mark.gpu

IDEAL = dict(inp_res=0.0, inp_bound=1e30, inp_noise=0.0, w_noise=0.0, out_noise=0.0, out_res=0.0, out_bound=1e30,
             noise_management=False)
NOISY = dict(inp_res=1.0 / 126.0, inp_bound=1.0, inp_noise=0.01, w_noise=0.02, out_noise=0.06, out_res=12.0 / 254.0,
             out_bound=12.0, noise_management=True)


def _tile_with_weights(R, C, seed=3):
    g = np.random.default_rng(seed)
    W = g.uniform(-0.6, 0.6, size=(R, C)).astype(np.float32)
    tile = aht.Tile(R, C, aht.DeviceParams(w_max=1.0, w_min=-1.0), 31, False, seed)
    tile.set_weights(to_dev(W))
    return tile, W


def _check(tile, W, x, io_kw, transposed, step):
    io_g, io_o = aht.IOParams(**io_kw), oracle.IOParams(**io_kw)
    tile.mvm_steps = (step, step)
    fn = tile.backward if transposed else tile.forward
    y, pre = fn(to_dev(x), io_g, with_pre=True)
    y, pre = y.cpu().numpy(), pre.cpu().numpy()
    yo, po = oracle.analog_mvm(W, x, io_o, tile_seed(tile), step, transposed=transposed, return_pre=True)
    scale = max(1.0, float(np.abs(po).max()))
    tol = 2e-5 * scale * max(1.0, np.sqrt(x.shape[1]) / 16)
    assert np.abs(pre.astype(np.float64) - po).max() <= tol, (np.abs(pre - po).max(), tol)
    if io_kw["out_res"] == 0.0:
        assert np.abs(y.astype(np.float64) - yo).max() <= tol * max(1.0, float(np.abs(x).max()))
        return
    # ADC codes: equal, or one step apart where the oracle's value is at a rounding boundary
    alpha = np.abs(np.where(np.isfinite(x), x, 0)).max(axis=1, keepdims=True) if io_kw["noise_management"] else 1.0
    step_out = io_kw["out_res"] * alpha
    diff = np.abs(y.astype(np.float64) - yo)
    same = diff <= 1e-6 * np.maximum(1.0, np.abs(yo))
    frac = np.abs(po / io_kw["out_res"] - np.floor(po / io_kw["out_res"]) - 0.5)      # distance to a boundary, in steps
    near = frac <= 2 * tol / io_kw["out_res"]
    assert (same | near).all()
    assert (diff <= step_out * (1 + 1e-5) + 1e-9)[~same].all()
    assert same.mean() > 0.99


def tile_seed(tile):
    return 3


@pytest.mark.parametrize("R,C,B", [(64, 64, 64), (96, 160, 33), (37, 300, 5), (130, 67, 70), (512, 1024, 256)])
@pytest.mark.parametrize("transposed", [False, True])
def test_ideal_product_matches(R, C, B, transposed):
    tile, W = _tile_with_weights(R, C)
    g = np.random.default_rng(R + C + B)
    x = g.normal(size=(B, R if transposed else C)).astype(np.float32)
    _check(tile, W, x, IDEAL, transposed, step=0)
    tile.close()


@pytest.mark.parametrize("R,C,B", [(64, 64, 64), (130, 67, 70), (256, 512, 128)])
@pytest.mark.parametrize("transposed", [False, True])
def test_noisy_quantised_product_matches(R, C, B, transposed):
    tile, W = _tile_with_weights(R, C)
    g = np.random.default_rng(R + C + B + 1)
    x = g.normal(size=(B, R if transposed else C)).astype(np.float32)
    x[1] = 0.0                                   # zero vector
    x[2, 3] = np.nan                             # ignored entries
    x[2, 4] = -np.inf
    x[3] *= 1e-3                                 # dynamic scaling
    _check(tile, W, x, NOISY, transposed, step=5)
    # counters advance per direction
    f, b = tile.mvm_steps
    assert (f, b) == ((5, 6) if transposed else (6, 5))
    tile.close()


@pytest.mark.parametrize("bm,splits", [(64, 1), (64, 3), (128, 1), (128, 2), (128, 16)])
@pytest.mark.parametrize("R,C,B", [(130, 268, 70), (192, 256, 130)])
@pytest.mark.parametrize("transposed", [False, True])
def test_block_height_and_inner_split_do_not_change_the_result(R, C, B, transposed, bm, splits, monkeypatch):
    """Every block height and every number of slices of the inner dimension (partial sums added
    in a second pass) gives the oracle's product; ragged and whole tiles, both directions."""
    monkeypatch.setenv("AHT_MVM_BM", str(bm))
    monkeypatch.setenv("AHT_MVM_SPLITS", str(splits))
    tile, W = _tile_with_weights(R, C)
    g = np.random.default_rng(R + C + B + bm + splits)
    x = g.normal(size=(B, R if transposed else C)).astype(np.float32)
    _check(tile, W, x, NOISY, transposed, step=2)
    tile.close()


# quantised inputs without input noise: the forward product takes the integer DAC codes through the
# bf16 matrix cores (weights cut into three bf16 terms) when the shape allows, else the fp32 path
QUANT = dict(inp_res=1.0 / 126.0, inp_bound=1.0, inp_noise=0.0, w_noise=0.02, out_noise=0.06, out_res=12.0 / 254.0,
             out_bound=12.0, noise_management=True)
QUANT_EXACT = dict(inp_res=1.0 / 126.0, inp_bound=1.0, inp_noise=0.0, w_noise=0.0, out_noise=0.0, out_res=0.0,
                   out_bound=1e30, noise_management=True)


@pytest.mark.parametrize("R,C,B", [(32, 16, 1), (64, 64, 20), (96, 160, 33), (160, 272, 70), (128, 512, 130),
                                   (512, 1024, 256), (64, 1024, 300), (37, 304, 5), (96, 300, 40), (1024, 48, 17)])
@pytest.mark.parametrize("io_kw", [QUANT, QUANT_EXACT])
def test_quantised_forward_product_matches(R, C, B, io_kw):
    tile, W = _tile_with_weights(R, C)
    g = np.random.default_rng(R + C + B + 7)
    x = g.normal(size=(B, C)).astype(np.float32)
    if B > 4:
        x[1] = 0.0
        x[2, 3] = np.nan
        x[3] *= 1e-3
    _check(tile, W, x, io_kw, False, step=4)
    xt = g.normal(size=(B, R)).astype(np.float32)
    _check(tile, W, xt, io_kw, True, step=4)      # the transposed product: same path when R % 32 == 0 and C % 16 == 0
    tile.close()


@pytest.mark.parametrize("splits", [1, 2, 4, 5, 16])
@pytest.mark.parametrize("B", [7, 40, 100, 200])
@pytest.mark.parametrize("transposed", [False, True])
@pytest.mark.parametrize("shape", [(96, 512), (128, 608)])
def test_quantised_product_every_split_and_both_paths_agree(B, splits, transposed, shape, monkeypatch):
    """(96, 512): 16 steps of the inner dimension, outputs not in whole groups of 64; (128, 608): 19
    steps (slices that end inside a turn of the load ring, and empty ones), whole groups of 64
    outputs, so that from 65 vectors on the kernel that shares the codes in LDS runs."""
    R, C = shape[::-1] if transposed else shape
    K = R if transposed else C
    tile, W = _tile_with_weights(R, C)
    g = np.random.default_rng(B + splits)
    x = g.normal(size=(B, K)).astype(np.float32)
    fn = tile.backward if transposed else tile.forward
    monkeypatch.setenv("AHT_MVM_SPLITS", str(splits))
    _check(tile, W, x, QUANT_EXACT, transposed, step=1)
    y_codes = fn(to_dev(x), aht.IOParams(**QUANT_EXACT)).cpu().numpy()
    if splits == 4:                               # four slices are added up and finished inside the kernel:
        monkeypatch.setenv("AHT_MVM_FUSED", "0")  # the same bits as partial sums and a second kernel
        y_two = fn(to_dev(x), aht.IOParams(**QUANT_EXACT)).cpu().numpy()
        assert (y_two == y_codes).all()
        tile.mvm_steps = (3, 3)
        y_two = fn(to_dev(x), aht.IOParams(**QUANT)).cpu().numpy()
        monkeypatch.setenv("AHT_MVM_FUSED", "1")
        tile.mvm_steps = (3, 3)
        y_one = fn(to_dev(x), aht.IOParams(**QUANT)).cpu().numpy()
        assert (y_two == y_one).all()
    # sharing the codes inside a workgroup changes no bit either
    monkeypatch.setenv("AHT_MVM_SHARED", "0")
    monkeypatch.setenv("AHT_MVM_FUSED", "0")
    tile.mvm_steps = (5, 5)
    y_plain = fn(to_dev(x), aht.IOParams(**QUANT)).cpu().numpy()
    monkeypatch.setenv("AHT_MVM_SHARED", "1")
    monkeypatch.setenv("AHT_MVM_FUSED", "1")
    tile.mvm_steps = (5, 5)
    y_shared = fn(to_dev(x), aht.IOParams(**QUANT)).cpu().numpy()
    assert (y_plain == y_shared).all()
    monkeypatch.setenv("AHT_MVM_CODES", "0")
    y_fp32 = fn(to_dev(x), aht.IOParams(**QUANT_EXACT)).cpu().numpy()
    scale = max(1.0, float(np.abs(y_fp32).max()))
    assert np.abs(y_codes.astype(np.float64) - y_fp32).max() <= 2e-5 * scale * max(1.0, np.sqrt(K) / 16)
    tile.close()


@pytest.mark.parametrize("B", [3, 64, 130, 300])
@pytest.mark.parametrize("transposed", [False, True])
@pytest.mark.parametrize("io_kw", [IDEAL, NOISY], ids=["ideal", "noisy"])
def test_three_plane_product_matches_oracle_and_the_fp32_cores(B, transposed, io_kw, monkeypatch):
    """Inputs that are no 8-bit DAC codes (no DAC at all, or input noise) go to the bf16 matrix cores
    as three bf16 planes when the shape allows (inner dimension in steps of 32, outputs in groups of
    64): same tolerance against the oracle as the fp32 cores, and the two agree with each other."""
    R, C = (608, 128) if transposed else (128, 608)
    K = R if transposed else C
    tile, W = _tile_with_weights(R, C)
    g = np.random.default_rng(B)
    x = g.normal(size=(B, K)).astype(np.float32)
    x[0, :5] = [0.0, -0.0, 1e-30, -3.5, 7.25]
    for splits in (0, 1, 3, 16):
        monkeypatch.setenv("AHT_MVM_SPLITS", str(splits))
        _check(tile, W, x, io_kw, transposed, step=2)
    monkeypatch.setenv("AHT_MVM_SPLITS", "0")
    fn = tile.backward if transposed else tile.forward
    tile.mvm_steps = (4, 4)
    _, pre_planes = fn(to_dev(x), aht.IOParams(**io_kw), with_pre=True)
    monkeypatch.setenv("AHT_MVM_PLANES", "0")
    tile.mvm_steps = (4, 4)
    _, pre_fp32 = fn(to_dev(x), aht.IOParams(**io_kw), with_pre=True)
    pre_planes, pre_fp32 = pre_planes.cpu().numpy().astype(np.float64), pre_fp32.cpu().numpy().astype(np.float64)
    scale = max(1.0, float(np.abs(pre_fp32).max()))
    assert np.abs(pre_planes - pre_fp32).max() <= 5e-6 * scale * max(1.0, np.sqrt(K) / 16)
    assert (pre_planes != pre_fp32).any()          # (two different kernels did run)
    tile.close()


def test_bad_io_parameters_are_rejected():
    import torch
    tile, W = _tile_with_weights(8, 8)
    x = torch.zeros((2, 8), device="cuda")
    with pytest.raises(aht.AhtError):
        tile.forward(x, aht.IOParams(out_noise=-1.0))
    with pytest.raises(aht.AhtError):
        tile.forward(x, aht.IOParams(out_bound=0.0))
    tile.close()
