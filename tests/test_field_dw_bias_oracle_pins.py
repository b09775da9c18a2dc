"""Pins for the field oracle's depthwise convolution and bias (CPU only)."""
import numpy as np
import scipy.signal

import dk_inputs
from oracle import field as F

P = F.P


def _lift(v, p=P):
    v = np.asarray(v).astype(np.int64)
    return np.where(v > p // 2, v - p, v)


def test_depthwise_equals_the_block_diagonal_full_convolution():
    rng = np.random.default_rng(0)
    C, kh, kw = 3, 3, 2
    W = rng.integers(0, P, size=(C, kh, kw), dtype=np.uint32)
    X = rng.integers(0, P, size=(2, C, 6, 5), dtype=np.uint32)
    full = np.zeros((C, C, kh, kw), dtype=np.uint32)
    for c in range(C):
        full[c, c] = W[c]
    for stride, pad in ((1, 1), (2, 0), (2, 1)):
        assert np.array_equal(F.dwconv_fwd(W, X, stride, pad), F.conv_fwd(full, X, stride, pad))
        Ho, Wo = F.conv_out_hw(6, 5, kh, kw, stride, pad)
        D = rng.integers(0, P, size=(2, C, Ho, Wo), dtype=np.uint32)
        g_full = F.conv_wgrad(D, X, kh, kw, stride, pad)
        g_dw = F.dwconv_wgrad(D, X, kh, kw, stride, pad)
        for c in range(C):
            assert np.array_equal(g_dw[c], g_full[c, c])


def test_depthwise_on_small_integers_is_the_integer_correlation():
    rng = np.random.default_rng(1)
    W = rng.integers(-50, 50, size=(2, 3, 3))
    X = rng.integers(-300, 300, size=(1, 2, 7, 6))
    got = _lift(F.dwconv_fwd((W % P).astype(np.uint32), (X % P).astype(np.uint32), 1, 1))
    for c in range(2):
        assert np.array_equal(got[0, c], scipy.signal.correlate2d(X[0, c], W[c], mode="same"))


def test_masked_depthwise_layer_equals_the_integer_layer():
    L = dk_inputs.dwconv(3, 6, 5, 3)
    d = dk_inputs.field_layer_inputs(np.random.default_rng(2), L, K=2, batch=4, delta_std=1.0)
    o = F.masked_dw_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=1, pad=1)
    Wq, Xq, Dq = _lift(o["Wq"]), _lift(o["Xq"]), _lift(o["Dq"])
    for s in range(4):
        for c in range(3):
            assert np.array_equal(_lift(o["Yq"])[s, c], scipy.signal.correlate2d(Xq[s, c], Wq[c], mode="same"))
    # dW[c][a][b] = sum_{s,h,w} D[s][c][h][w] X[s][c][h+a-1][w+b-1]
    Xp = np.pad(Xq, ((0, 0), (0, 0), (1, 1), (1, 1)))
    want = np.zeros((3, 3, 3), dtype=np.int64)
    for a in range(3):
        for b in range(3):
            want[:, a, b] = (Dq * Xp[:, :, a:a + 6, b:b + 5]).sum(axis=(0, 2, 3))
    assert np.array_equal(_lift(o["dWq"]), want)
    assert not o["verdict"].any()


def test_bias_hand_values_and_layer():
    # l = 1: b_q = Round(4 b); entries of a row take bias[e // per]
    yq = np.array([[0, 1, 2, 3], [P - 1, 5, 6, 7]], dtype=np.uint32)
    out = F.add_bias(yq, np.array([0.25, -0.6], dtype=np.float32), per=2, l=1)
    # 4*0.25 = 1 -> 1;  4*(-0.6) = -2.4 -> Round -> -2
    assert out.tolist() == [[1, 2, 0, 1], [0, 6, 4, 5]]
    # a dense layer with bias: the de-quantised result is W x + b within the fixed-point bound
    rng = np.random.default_rng(3)
    W = rng.normal(0, 0.3, size=(5, 7)).astype(np.float32)
    X = rng.normal(size=(4, 7)).astype(np.float32)
    b = rng.normal(size=5).astype(np.float32)
    d = dk_inputs.field_layer_inputs(np.random.default_rng(4), dk_inputs.linear(5, 7), K=2, batch=4)
    o = F.masked_dense_layer(W, X, d["r"], d["delta"], d["A"], d["gamma"])
    y = F.dequantize(F.add_bias(o["Yq"], b, per=1))
    ref = X.astype(np.float64) @ W.astype(np.float64).T + b
    # quantisation of W, X (2^-9 each, times the operand sizes), of b (2^-17) and of the result (2^-9)
    bound = 2.0**-9 * (np.abs(W).sum(1).max() + np.abs(X).sum(1).max()) + 7 * 2.0**-18 + 2.0**-9 + 2.0**-17
    assert np.abs(y - ref).max() <= bound
    # exactly: lift(Y_q + b_q) = X_q W_q^T + Round(b 2^16)
    want = _lift(o["Xq"]) @ _lift(o["Wq"]).T + np.floor(b.astype(np.float64) * 65536 + 0.5).astype(np.int64)
    assert np.array_equal(_lift(F.add_bias(o["Yq"], b, per=1)), want)
