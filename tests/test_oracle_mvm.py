"""Pins for the oracle's analog matrix-vector product (Eq. (1) of arXiv 2104.02184 and its
transposed form): reduction to the plain product, exact DAC/ADC grids, clipping, scaling
invariance, and the variances of the three noise sources."""
import math

import numpy as np
import pytest

import oracle
from oracle import IOParams

f32 = np.float32
IDEAL = IOParams(inp_res=0.0, inp_bound=1e30, inp_noise=0.0, w_noise=0.0, out_noise=0.0, out_res=0.0,
                 out_bound=1e30, noise_management=False)


def data(R=24, C=40, B=6, seed=0):
    g = np.random.default_rng(seed)
    return (g.uniform(-0.6, 0.6, size=(R, C)).astype(f32), g.normal(size=(B, C)).astype(f32),
            g.normal(size=(B, R)).astype(f32))


def test_without_non_idealities_it_is_the_matrix_product():
    W, x, d = data()
    y = oracle.analog_mvm(W, x, IDEAL, 1, 0)
    assert np.allclose(y, x.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-6, atol=1e-6)
    g = oracle.analog_mvm(W, d, IDEAL, 1, 0, transposed=True)
    assert np.allclose(g, d.astype(np.float64) @ W.astype(np.float64), rtol=1e-6, atol=1e-6)
    # dynamic scaling alone changes nothing but rounding
    nm = IOParams(**{**IDEAL.__dict__, "noise_management": True})
    assert np.allclose(oracle.analog_mvm(W, x, nm, 1, 0), y, rtol=1e-5, atol=1e-5)


def test_dac_grid_clipping_and_scaling():
    W = np.eye(8, dtype=f32)                        # y = f(x) element-wise
    io = IOParams(inp_res=0.25, inp_bound=1.0, out_noise=0.0, out_res=0.0, out_bound=1e30, noise_management=False)
    x = np.array([[0.0, 0.1, 0.13, 0.374, 0.376, -0.62, 0.9, 7.0]], dtype=f32)
    y = oracle.analog_mvm(W, x, io, 1, 0)
    assert (y[0] == np.array([0.0, 0.0, 0.25, 0.25, 0.5, -0.5, 1.0, 1.0], dtype=f32)).all()
    # ties go to the even grid point
    t = np.array([[0.125, 0.375, -0.125, 0.625, 0, 0, 0, 0]], dtype=f32)
    assert (oracle.analog_mvm(W, t, io, 1, 0)[0, :4] == np.array([0.0, 0.5, -0.0, 0.5], dtype=f32)).all()
    # with dynamic scaling the grid follows max|x|, and scaling the input by 2^k scales the output exactly
    io2 = IOParams(inp_res=0.25, out_noise=0.0, out_res=0.0, out_bound=1e30, noise_management=True)
    xs = np.array([[0.5, -2.0, 1.1, 0.2, 0, 0, 0, 0]], dtype=f32)
    y2 = oracle.analog_mvm(W, xs, io2, 1, 0)
    assert (y2[0, :4] == np.array([0.5, -2.0, 1.0, 0.0], dtype=f32)).all()
    assert (oracle.analog_mvm(W, xs * 8, io2, 1, 0) == y2 * 8).all()
    # zero vector, NaN and Inf entries
    z = oracle.analog_mvm(W, np.zeros((1, 8), f32), io2, 1, 0)
    assert (z == 0).all()
    bad = xs.copy()
    bad[0, 2] = np.nan
    bad[0, 3] = np.inf
    yb = oracle.analog_mvm(W, bad, io2, 1, 0)
    assert (yb[0, :4] == np.array([0.5, -2.0, 0.0, 0.0], dtype=f32)).all()


def test_adc_grid_and_clipping():
    W = np.eye(6, dtype=f32) * f32(3.0)
    io = IOParams(inp_res=0.0, out_noise=0.0, out_res=0.5, out_bound=2.0, noise_management=False, inp_bound=1e30)
    x = np.array([[0.1, 0.26, -0.4, 0.6, 0.7, -5.0]], dtype=f32)        # 3x = 0.3 0.78 -1.2 1.8 2.1 -15
    y = oracle.analog_mvm(W, x, io, 1, 0)
    assert (y[0] == np.array([0.5, 1.0, -1.0, 2.0, 2.0, -2.0], dtype=f32)).all()
    y, pre = oracle.analog_mvm(W, x, io, 1, 0, return_pre=True)
    assert np.allclose(pre[0], 3.0 * x[0], rtol=1e-6)


def _many(io, W, x, n, transposed=False):
    return np.stack([oracle.analog_mvm(W, x, io, 5, t, transposed=transposed, return_pre=True)[1] for t in range(n)])


def test_output_weight_and_input_noise_variances():
    W, x, d = data(R=16, C=32, B=3, seed=2)
    base = IOParams(inp_res=0.0, inp_bound=1e30, out_res=0.0, out_bound=1e30, out_noise=0.0, noise_management=False)
    clean = oracle.analog_mvm(W, x, base, 5, 0)
    N = 4000
    # output noise: N(0, s_out^2) on every output
    pre = _many(IOParams(**{**base.__dict__, "out_noise": 0.05}), W, x, N) - clean
    assert abs(pre.mean()) < 4 * 0.05 / math.sqrt(pre.size)
    assert abs(pre.std() / 0.05 - 1) < 0.02
    # weight noise: N(0, s_w^2 |x|^2) per output, independent across outputs
    pre = _many(IOParams(**{**base.__dict__, "w_noise": 0.02}), W, x, N) - clean
    want = 0.02 * np.linalg.norm(x.astype(np.float64), axis=1)
    assert np.allclose(pre.std(axis=(0, 2)), want, rtol=0.03)
    assert abs(np.corrcoef(pre[:, 0, 0], pre[:, 0, 1])[0, 1]) < 4 / math.sqrt(N)
    # input noise: propagates through the weights, variance s_inp^2 sum_j w_ij^2
    pre = _many(IOParams(**{**base.__dict__, "inp_noise": 0.1}), W, x, N) - clean
    want = 0.1 * np.linalg.norm(W.astype(np.float64), axis=1)
    assert np.allclose(pre.std(axis=0)[0], want, rtol=0.1)
    # the three sources and the two directions use different random streams
    a = _many(IOParams(**{**base.__dict__, "out_noise": 1.0}), W, x, 50) - clean
    b = _many(IOParams(**{**base.__dict__, "w_noise": 1.0}), W, x, 50) - clean
    assert abs(np.corrcoef(a.ravel(), b.ravel())[0, 1]) < 0.1
    Wsq = W[:, :16].copy()
    f = _many(IOParams(**{**base.__dict__, "out_noise": 1.0}), Wsq, x[:, :16], 50)
    r = _many(IOParams(**{**base.__dict__, "out_noise": 1.0}), Wsq, x[:, :16], 50, transposed=True)
    f -= oracle.analog_mvm(Wsq, x[:, :16], base, 5, 0)
    r -= oracle.analog_mvm(Wsq, x[:, :16], base, 5, 0, transposed=True)
    assert abs(np.corrcoef(f.ravel(), r.ravel())[0, 1]) < 0.1


def test_noise_is_keyed_by_output_sample_and_call():
    W, x, _ = data(R=8, C=12, B=2, seed=3)
    io = IOParams(inp_res=0.0, inp_bound=1e30, out_res=0.0, out_bound=1e30, out_noise=0.5, noise_management=False)
    clean = oracle.analog_mvm(W, x, IDEAL, 9, 0)
    pre = oracle.analog_mvm(W, x, io, 9, 4, return_pre=True)[1]
    for b in range(2):
        for i in range(8):
            z = oracle.gauss_block_f64(9, i >> 1, 4, b, 8)[2 * (i & 1)]
            assert pre[b, i] - clean[b, i] == pytest.approx(0.5 * z, abs=2e-6)


def test_output_referred_weight_noise_has_the_law_of_a_fresh_gaussian_per_cell():
    """Eq. (1) puts a Gaussian on every weight of every product.  The oracle's (and the kernels')
    product draws the sum of those terms directly, one Gaussian per output (reading F4); here it is
    held against the equation as printed, orc_analog_mvm_cellwise, in law: mean, variance per vector
    and output, independence across outputs and vectors, and the whole distribution (two-sample KS)."""
    from scipy import stats
    W, x, d = data(R=10, C=24, B=3, seed=4)
    x[1] *= f32(3.0)                                   # vectors of different norm
    base = IOParams(inp_res=0.0, inp_bound=1e30, out_res=0.0, out_bound=1e30, out_noise=0.0, noise_management=False)
    io = IOParams(**{**base.__dict__, "w_noise": 0.05})
    for transposed, inp in ((False, x), (True, d)):
        clean = oracle.analog_mvm(W, inp, base, 7, 0, transposed=transposed, return_pre=True)[1]
        # without weight noise the two forms are the same function
        assert (oracle.analog_mvm(W, inp, base, 7, 0, transposed=transposed, cellwise_weight_noise=True) ==
                oracle.analog_mvm(W, inp, base, 7, 0, transposed=transposed)).all()
        N = 1500
        ref = np.stack([oracle.analog_mvm(W, inp, io, 7, t, transposed=transposed, return_pre=True)[1]
                        for t in range(N)]) - clean
        cel = np.stack([oracle.analog_mvm(W, inp, io, 7, t, transposed=transposed, return_pre=True,
                                          cellwise_weight_noise=True)[1] for t in range(N)]) - clean
        want = 0.05 * np.linalg.norm(inp.astype(np.float64), axis=1)          # std per vector
        for r in (ref, cel):
            assert np.abs(r.mean(axis=0)).max() < 5 * want.max() / math.sqrt(N)
            assert np.allclose(r.std(axis=0), want[:, None], rtol=0.12)       # every (vector, output)
            assert np.allclose(r.std(axis=(0, 2)), want, rtol=0.03)
            assert abs(np.corrcoef(r[:, 0, 0], r[:, 0, 1])[0, 1]) < 4.5 / math.sqrt(N)     # across outputs
            assert abs(np.corrcoef(r[:, 0, 2], r[:, 1, 2])[0, 1]) < 4.5 / math.sqrt(N)     # across vectors
        for b in range(inp.shape[0]):
            assert stats.ks_2samp(ref[:, b, :].ravel(), cel[:, b, :].ravel()).pvalue > 1e-3
            assert stats.kstest(cel[:, b, :].ravel() / want[b], "norm").pvalue > 1e-3
        # the two forms use different random numbers (the cellwise one its own streams)
        assert abs(np.corrcoef(ref.ravel(), cel.ravel())[0, 1]) < 0.02


def test_cellwise_weight_noise_is_keyed_by_cell_vector_and_call():
    W, x, d = data(R=3, C=5, B=2, seed=6)
    base = IOParams(inp_res=0.0, inp_bound=1e30, out_res=0.0, out_bound=1e30, out_noise=0.0, noise_management=False)
    io = IOParams(**{**base.__dict__, "w_noise": 0.25})
    pre = oracle.analog_mvm(W, x, io, 3, 9, return_pre=True, cellwise_weight_noise=True)[1]
    for b in range(2):
        for i in range(3):
            acc = sum((float(W[i, j]) + float(f32(0.25)) * oracle.gauss_block_f64(3, i * 5 + j, 9, b, 11)[0]) * float(x[b, j])
                      for j in range(5))
            assert pre[b, i] == pytest.approx(acc, rel=1e-6, abs=1e-6)
    pre = oracle.analog_mvm(W, d, io, 3, 9, transposed=True, return_pre=True, cellwise_weight_noise=True)[1]
    for b in range(2):
        for j in range(5):
            acc = sum((float(W[i, j]) + float(f32(0.25)) * oracle.gauss_block_f64(3, i * 5 + j, 9, b, 12)[0]) * float(d[b, i])
                      for i in range(3))
            assert pre[b, j] == pytest.approx(acc, rel=1e-6, abs=1e-6)


def test_input_noise_enters_after_the_dac_and_is_keyed_by_input_vector_and_call():
    """F2/F3: the DAC rounds first, the input noise rides on the rounded value (it is not rounded
    away), one Gaussian per input line, vector and call."""
    W = np.eye(8, dtype=f32)
    io = IOParams(inp_res=0.25, inp_bound=1.0, inp_noise=0.01, out_noise=0.0, out_res=0.0, out_bound=1e30,
                  noise_management=False)
    x = np.array([[0.0, 0.1, 0.13, 0.374, 0.376, -0.62, 0.9, 7.0],
                  [0.5, -0.3, 0.2, 0.8, -0.9, 0.01, 0.49, -0.26]], dtype=f32)
    grid = np.clip(np.round(np.clip(x.astype(np.float64), -1, 1) / 0.25) * 0.25, -1, 1)
    pre = oracle.analog_mvm(W, x, io, 21, 6, return_pre=True)[1]
    for b in range(2):
        for j in range(8):
            z = oracle.gauss_block_f64(21, j >> 2, 6, b, 7)[j & 3]
            assert pre[b, j] == pytest.approx(grid[b, j] + float(f32(0.01)) * z, abs=1e-6)
    assert (np.abs(pre - grid) > 1e-5).mean() > 0.9      # off the grid: the noise was not rounded away
    # backward: its own tag
    pre = oracle.analog_mvm(W, x, io, 21, 6, transposed=True, return_pre=True)[1]
    z = oracle.gauss_block_f64(21, 1, 6, 1, 9)[2]
    assert pre[1, 6] == pytest.approx(grid[1, 6] + float(f32(0.01)) * z, abs=1e-6)
