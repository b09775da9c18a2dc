"""Pins for the oracle's depthwise convolution and data gradients (CPU only)."""
import numpy as np
import pytest
from scipy.signal import correlate2d

import dk_inputs
import oracle


@pytest.mark.parametrize("C,H,W,k,stride,pad", [(3, 7, 6, 3, 1, 1), (4, 9, 9, 3, 2, 1), (2, 6, 8, 5, 1, 2), (5, 4, 4, 1, 1, 0)])
def test_depthwise_is_the_block_diagonal_convolution(C, H, W, k, stride, pad):
    rng = np.random.default_rng([C, H, k, stride])
    Wd = rng.normal(size=(C, k, k))
    X = rng.normal(size=(2, C, H, W))
    Y = oracle.dwconv_fwd(Wd, X, stride, pad)
    full = np.zeros((C, C, k, k))
    full[np.arange(C), np.arange(C)] = Wd
    assert np.abs(Y - oracle.conv_fwd(full, X, stride, pad)).max() < 1e-12
    # and scipy per channel
    Xp = np.pad(X, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    for c in range(C):
        assert np.abs(Y[1, c] - correlate2d(Xp[1, c], Wd[c], mode="valid")[::stride, ::stride]).max() < 1e-12
    D = rng.normal(size=Y.shape)
    dW = oracle.dwconv_wgrad(D, X, k, k, stride, pad)
    dfull = oracle.conv_wgrad(D, X, k, k, stride, pad)
    assert np.abs(dW - dfull[np.arange(C), np.arange(C)]).max() < 1e-12


@pytest.mark.parametrize("Ci,Co,H,W,k,stride,pad", [(3, 4, 6, 5, 3, 1, 1), (2, 3, 9, 8, 3, 2, 1), (4, 2, 5, 5, 1, 1, 0), (2, 2, 7, 7, 5, 2, 2)])
def test_data_gradients_are_the_adjoints_of_the_forward_maps(Ci, Co, H, W, k, stride, pad):
    """<conv(W, x), d> = <x, dgrad(W, d)> for all x, d: the defining property of
    the transpose, which a wrong flip, shift or stride handling breaks."""
    rng = np.random.default_rng([Ci, Co, H, k, stride, 3])
    Wt = rng.normal(size=(Co, Ci, k, k))
    X = rng.normal(size=(2, Ci, H, W))
    Y = oracle.conv_fwd(Wt, X, stride, pad)
    D = rng.normal(size=Y.shape)
    dX = oracle.conv_dgrad(D, Wt, H, W, stride, pad)
    assert abs((Y * D).sum() - (X * dX).sum()) < 1e-10 * abs((Y * D).sum()) + 1e-10
    # a unit impulse in d reads the filter back, shifted to its place
    E = np.zeros_like(D)
    E[0, 1, 1, 1] = 1.0
    dX1 = oracle.conv_dgrad(E, Wt, H, W, stride, pad)
    for a in range(k):
        for b in range(k):
            i, j = stride + a - pad, stride + b - pad
            if 0 <= i < H and 0 <= j < W:
                assert np.allclose(dX1[0, :, i, j], Wt[1, :, a, b])
    # depthwise
    Wd = rng.normal(size=(Ci, k, k))
    Yd = oracle.dwconv_fwd(Wd, X, stride, pad)
    Dd = rng.normal(size=Yd.shape)
    dXd = oracle.dwconv_dgrad(Dd, Wd, H, W, stride, pad)
    assert abs((Yd * Dd).sum() - (X * dXd).sum()) < 1e-10 * abs((Yd * Dd).sum()) + 1e-10


def test_dense_data_gradient_is_a_matmul():
    rng = np.random.default_rng(9)
    D, W = rng.normal(size=(5, 7)), rng.normal(size=(7, 11))
    assert np.abs(oracle.dense_dgrad(D, W) - D @ W).max() < 1e-12


def test_masked_depthwise_layer_decodes_to_the_plain_layer():
    rng = np.random.default_rng(10)
    K, G, C, H = 3, 2, 4, 6
    L = dk_inputs.conv(C, C, H, H, 3)
    d = dk_inputs.masked_layer_inputs(rng, L, K=K, batch=G * K, delta_std=1.0)
    Wd = rng.normal(size=(C, 3, 3)).astype(np.float32)
    o = oracle.masked_dw_layer(Wd, d["X"], d["r"], d["delta"], d["A"], d["gamma"], 1, 1)
    Y = oracle.dwconv_fwd(Wd, d["X"], 1, 1)
    dW = oracle.dwconv_wgrad(d["delta"], d["X"], 3, 3, 1, 1)
    assert np.abs(o["Y"] - Y).max() < 1e-9 * np.abs(Y).max() * 100
    assert np.abs(o["dW"] - dW).max() < 1e-9 * np.abs(dW).max() * 100
    assert not o["verdict"].any()
