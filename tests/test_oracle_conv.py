"""Pins for the oracle's convolution update vectors: the patch matrix against PyTorch's unfold
(a library routine), the row vectors against a plain permutation, and the fact the paper
stresses: the update of a convolution is the sequence of its positions' rank-1 updates."""
import numpy as np
import pytest
import torch

import oracle
from oracle import DeviceParams


@pytest.mark.parametrize("N,Cin,H,W,kh,kw,stride,pad", [(2, 3, 6, 7, 3, 3, 1, 1), (1, 2, 8, 8, 3, 2, 2, 0),
                                                        (3, 1, 5, 5, 5, 5, 1, 2), (2, 4, 9, 6, 1, 1, 1, 0)])
def test_patches_match_unfold(N, Cin, H, W, kh, kw, stride, pad):
    g = np.random.default_rng(0)
    img = g.normal(size=(N, Cin, H, W)).astype(np.float32)
    OH, OW = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    Cout = 5
    dgrad = g.normal(size=(N, Cout, OH, OW)).astype(np.float32)
    x, d = oracle.conv_update_vectors(img, dgrad, kh, kw, stride, pad)
    unf = torch.nn.functional.unfold(torch.from_numpy(img), (kh, kw), padding=pad, stride=stride)   # [N][J][L]
    want_x = unf.permute(0, 2, 1).reshape(N * OH * OW, Cin * kh * kw).numpy()
    assert (x == want_x).all()
    want_d = torch.from_numpy(dgrad).permute(0, 2, 3, 1).reshape(N * OH * OW, Cout).numpy()
    assert (d == want_d).all()


def test_mean_conv_update_is_the_weight_gradient():
    # noiseless constant step far from the bounds: the mean update equals -lr * dL/dW of conv2d
    N, Cin, H, W, kh, kw, Cout = 2, 2, 5, 5, 3, 3, 3
    g = np.random.default_rng(1)
    img = g.uniform(-0.5, 0.5, size=(N, Cin, H, W)).astype(np.float32)
    dgrad = g.uniform(-0.3, 0.3, size=(N, Cout, 3, 3)).astype(np.float32)
    x, d = oracle.conv_update_vectors(img, dgrad, kh, kw, 1, 0)
    ti = torch.from_numpy(img)
    wt = torch.zeros((Cout, Cin, kh, kw), requires_grad=True)
    torch.nn.functional.conv2d(ti, wt).backward(torch.from_numpy(dgrad))
    want = -0.1 * wt.grad.reshape(Cout, Cin * kh * kw).numpy().astype(np.float64)
    assert np.allclose(-0.1 * d.astype(np.float64).T @ x.astype(np.float64), want, atol=1e-6)
    p = DeviceParams(dw_min=0.002, w_max=1e6, w_min=-1e6)
    planes = oracle.device_planes(p, 1, Cout, Cin * kh * kw)
    acc = np.zeros_like(want)
    T = 3000
    for t in range(T):
        Wt = np.zeros(want.shape, dtype=np.float32)
        oracle.pulsed_update(Wt, planes, p, 31, False, x, d, 0.1, 3, t)
        acc += Wt
    sd = 0.002 * np.sqrt(31 * x.shape[0] * 0.25 / T)               # generous bound per cell
    assert np.abs(acc / T - want).max() < 4.5 * sd
