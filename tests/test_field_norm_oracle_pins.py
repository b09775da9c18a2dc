"""Pins for the dynamic-normalisation part of the finite-field oracle (CPU only).

Section "Privacy Guarantee", paragraph "Quantization": for networks without
normalisation layers a vector whose values pass the limits is divided by its
largest absolute entry before quantisation.  The checks use exact rationals,
hand values and the real layer in fp64, never the oracle's own formulas.
"""
from fractions import Fraction

import numpy as np
import pytest

import dk_inputs
from oracle import field as F

P = F.P


def _lift(v):
    v = v.astype(np.int64)
    return np.where(v > P // 2, v - P, v)


def _round_fraction(q):
    # floor below one half, floor + 1 otherwise (procedure Round)
    fl = q.numerator // q.denominator
    return fl + 1 if q - fl >= Fraction(1, 2) else fl


def test_scales_hand_values():
    x = np.array([[0.5, -0.25, 0.125],       # inside the limit: untouched
                  [4.0, -8.0, 2.0],          # 1/8
                  [1.0, 1.0, -1.0],          # exactly at the limit: untouched
                  [np.nan, -16.0, 3.0],      # NaN skipped: 1/16
                  [np.inf, 2.0, 1.0],        # infinite maximum: untouched
                  [0.0, 0.0, 0.0]], dtype=np.float32)
    s = F.norm_scales(x, 1.0)
    assert s.dtype == np.float32
    assert s.tolist() == [1.0, 0.125, 1.0, 0.0625, 1.0, 1.0]
    # a maximum that is no power of two: the factor is the fp32 nearest to 1/m
    s = F.norm_scales(np.array([[3.0, -1.0]], dtype=np.float32), 2.0)
    assert s[0] == np.float32(1.0 / 3.0)
    # the limit is a threshold on the maximum, not a target
    assert F.norm_scales(np.array([[3.0, -1.0]], dtype=np.float32), 3.0)[0] == 1.0


def test_rows_inside_the_limit_quantise_as_before():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((5, 37)).astype(np.float32)
    s = F.norm_scales(x, 100.0)
    assert (s == 1.0).all()
    assert np.array_equal(F.quantize_scaled(x, s, 8), F.quantize(x, 8))


def test_scaled_quantisation_against_exact_rationals():
    rng = np.random.default_rng(12)
    x = (rng.standard_normal((4, 29)) * np.array([[3.0], [1e3], [0.01], [77.0]])).astype(np.float32)
    # make some products land exactly on a half
    x[0, 0], x[0, 1] = 3.0, 3.0 / 512
    s = F.norm_scales(x, 2.0)
    s[0] = np.float32(1.0)
    for l in (0, 5, 8):
        got = _lift(F.quantize_scaled(x, s, l))
        for i in range(x.shape[0]):
            for e in range(x.shape[1]):
                want = _round_fraction(Fraction(float(x[i, e])) * Fraction(float(s[i])) * (1 << l))
                assert got[i, e] == want, (l, i, e)


def test_normalised_rows_stay_inside_one_and_peak_at_two_to_the_l():
    rng = np.random.default_rng(13)
    x = (rng.standard_normal((6, 200)) * 10.0 ** rng.integers(1, 6, size=(6, 1))).astype(np.float32)
    s = F.norm_scales(x, 1.0)
    q = _lift(F.quantize_scaled(x, s, 8))
    assert np.abs(q).max(axis=1).tolist() == [256] * 6
    assert (np.abs(q) <= 256).all()
    # the position of the peak is the position of the largest entry, with its sign
    j = np.abs(x).argmax(axis=1)
    assert np.array_equal(q[np.arange(6), j], 256 * np.sign(x[np.arange(6), j]).astype(np.int64))


def test_unscale_and_delta_quantisation_hand_values():
    y = np.array([[1.0, -3.0], [0.5, 2.0]], dtype=np.float32)
    out = F.unscale(y, np.array([0.5, 0.25], dtype=np.float32), 0.125)
    assert out.tolist() == [[16.0, -48.0], [16.0, 64.0]]
    d = np.array([[0.25, -1.0 / 512], [1.0, 3.0]], dtype=np.float32)
    q = _lift(F.quantize_unscaled_delta(d, np.array([0.5, 1.0], dtype=np.float32), 8))
    # row 0 doubled: 0.5 -> 128, -1/256 -> -1; row 1 as it is
    assert q.tolist() == [[128, -1], [256, 768]]


@pytest.mark.parametrize("K,G,M,N,seed", [(1, 2, 5, 9, 0), (2, 2, 8, 16, 1), (4, 3, 7, 33, 2)])
def test_normalised_dense_layer_tracks_the_real_layer(K, G, M, N, seed):
    """Inputs and weights far outside the fixed-point range: the plain field
    layer wraps around the modulus, the normalised one reproduces X W^T and
    sum_i delta_i (x) x_i up to the fixed-point error, scaled back."""
    rng = np.random.default_rng([seed, 21])
    d = dk_inputs.field_layer_inputs(rng, dk_inputs.linear(M, N), K=K, batch=G * K, w_std=40.0,
                                     delta_std=1e-3)
    X = (d["X"] * (50.0 * (1 + np.arange(G * K)))[:, None]).astype(np.float32)
    W, delta = d["W"], d["delta"]
    l = 8
    o = F.masked_layer_normalized(W, X, d["r"], delta, d["A"], d["gamma"], limit=1.0, l=l)
    assert not o["verdict"].any()
    mx = np.abs(X).max(axis=1).astype(np.float64)
    mw = float(np.abs(W).max())
    assert np.allclose(o["xscale"], 1.0 / mx, rtol=1e-6) and np.isclose(o["wscale"][0], 1.0 / mw, rtol=1e-6)
    # the field values are the integer layer of the normalised, rounded operands
    Wi, Xi = _lift(o["Wq"]), _lift(o["Xq"])
    assert np.array_equal(_lift(o["Yq"]), Xi @ Wi.T)
    assert np.array_equal(_lift(o["dWq"]), _lift(o["Dq"]).T @ Xi)
    # forward: each normalised operand is off by at most 2^-(l+1) per entry
    h = 2.0 ** -(l + 1)
    Y = X.astype(np.float64) @ W.astype(np.float64).T
    Xn, Wn = np.abs(X) / mx[:, None], np.abs(W) / mw
    err = h * (Xn.sum(1)[:, None] + Wn.sum(1)[None, :] + N * h) + h
    assert (np.abs(o["Y"] - Y) <= err * (mx[:, None] * mw) * 1.001).all()
    # the plain path is useless on these inputs
    o0 = F.masked_dense_layer(W, X, d["r"], delta, d["A"], d["gamma"], l=l)
    assert np.abs(o0["Y"] - Y).max() > 100 * np.abs(o["Y"] - Y).max()
    # weight gradient, no factor afterwards
    dW = delta.astype(np.float64).T @ X.astype(np.float64)
    Dn = np.abs(delta) * mx[:, None]          # magnitudes after the division by the factor
    errw = h * (Dn.sum(0)[:, None] + Xn.sum(0)[None, :] + G * K * h) + h
    assert (np.abs(o["dW"] - dW) <= errw * 1.001 + 1e-6 * np.abs(dW)).all()


def test_normalised_conv_layer_tracks_the_real_layer():
    rng = np.random.default_rng(31)
    lay = dk_inputs.conv(3, 4, 6, 5, 3, stride=1, pad=1)
    d = dk_inputs.field_layer_inputs(rng, lay, K=2, batch=4, w_std=9.0, delta_std=1e-2)
    X = (d["X"] * np.array([30.0, 0.2, 700.0, 5.0])[:, None, None, None]).astype(np.float32)
    o = F.masked_layer_normalized(d["W"], X, d["r"], d["delta"], d["A"], d["gamma"], limit=1.0,
                                  stride=1, pad=1)
    assert not o["verdict"].any()
    assert o["xscale"][1] == 1.0 and (o["xscale"][[0, 2, 3]] < 1.0).all()
    # real convolution in fp64, written out
    Xp = np.pad(X.astype(np.float64), ((0, 0), (0, 0), (1, 1), (1, 1)))
    Y = np.zeros((4, 4, 6, 5))
    for a in range(3):
        for b in range(3):
            Y += np.einsum("oc,nchw->nohw", d["W"][:, :, a, b].astype(np.float64), Xp[:, :, a:a + 6, b:b + 5])
    mx = np.maximum(np.abs(X).reshape(4, -1).max(1), 1.0)
    mw = float(np.abs(d["W"]).max())
    h = 2.0 ** -9
    bound = (h * (2 * 27 + 27 * h) + h) * mx[:, None, None, None] * mw
    assert (np.abs(o["Y"] - Y) <= bound).all()
    dW = np.zeros(d["W"].shape)
    for a in range(3):
        for b in range(3):
            dW[:, :, a, b] = np.einsum("nohw,nchw->oc", d["delta"].astype(np.float64), Xp[:, :, a:a + 6, b:b + 5])
    nterms = 4 * 30
    dmax = np.abs(d["delta"]).reshape(4, -1).max(1) * mx
    boundw = h * nterms * (1.0 + dmax.max() + h) + h
    assert np.abs(o["dW"] - dW).max() <= boundw


def test_planted_mistakes_in_normalisation_are_caught():
    """Each plausible slip changes a value that the exact checks above fix."""
    x = np.array([[4.0, -8.0, 2.0], [1.0, 0.5, 0.25]], dtype=np.float32)
    s = F.norm_scales(x, 1.0)
    good = _lift(F.quantize_scaled(x, s, 8)).tolist()
    assert good == [[128, -256, 64], [256, 128, 64]]
    # factor taken from the wrong row
    assert _lift(F.quantize_scaled(x, s[::-1], 8)).tolist() != good
    # signed maximum instead of the absolute one would give 1/4 for row 0
    assert s[0] != np.float32(0.25)
    # multiplying instead of dividing when scaling back
    y = np.array([[1.0], [1.0]], dtype=np.float32)
    assert F.unscale(y, s, 1.0).tolist() == [[8.0], [1.0]]
