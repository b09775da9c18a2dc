"""Pins for the fp64 CPU oracle: it is checked against things other than
itself -- library routines (numpy matmul, scipy correlate2d), a hand-worked
example, closed forms and the invariants the paper states -- so that a dropped
term, a wrong sign/index or a transposed operand anywhere in it fails here.
No GPU needed.
"""
import json
import os

import numpy as np
import pytest
from scipy.signal import correlate2d

import dk_inputs
import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def rel(a, b):
    den = np.max(np.abs(b))
    return np.max(np.abs(np.asarray(a) - np.asarray(b))) / (den if den else 1.0)


# ----------------------------------------------------------------------
# plain layer definitions vs library routines
# ----------------------------------------------------------------------

def test_dense_fwd_is_matmul():
    rng = np.random.default_rng(10)
    W, X = rng.standard_normal((7, 5)), rng.standard_normal((3, 5))
    assert rel(oracle.dense_fwd(W, X), X @ W.T) < 1e-14


def test_dense_wgrad_is_matmul():
    rng = np.random.default_rng(11)
    D, X = rng.standard_normal((6, 4)), rng.standard_normal((6, 9))
    assert rel(oracle.dense_wgrad(D, X, scale=0.25), 0.25 * D.T @ X) < 1e-14


def _conv_via_scipy(W, X, stride, pad):
    """Independent formulation: zero-pad, scipy 2-D 'valid' cross-correlation
    per (co, ci) pair, sum over ci, subsample by the stride."""
    Co, Ci, kh, kw = W.shape
    R = X.shape[0]
    Xp = np.pad(X, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    out = None
    for s in range(R):
        for co in range(Co):
            acc = sum(correlate2d(Xp[s, ci], W[co, ci], mode="valid") for ci in range(Ci))
            acc = acc[::stride, ::stride]
            if out is None:
                out = np.zeros((R, Co) + acc.shape)
            out[s, co] = acc
    return out


@pytest.mark.parametrize("kh,kw,stride,pad,H,Wd", [
    (3, 3, 1, 1, 6, 7), (3, 3, 2, 1, 7, 8), (1, 1, 1, 0, 5, 4), (1, 1, 2, 0, 6, 6),
    (7, 7, 2, 3, 12, 11), (3, 2, 1, 0, 5, 6), (3, 3, 1, 2, 4, 4)])
def test_conv_fwd_vs_scipy(kh, kw, stride, pad, H, Wd):
    rng = np.random.default_rng(12)
    W = rng.standard_normal((3, 2, kh, kw))
    X = rng.standard_normal((2, 2, H, Wd))
    got = oracle.conv_fwd(W, X, stride, pad)
    ref = _conv_via_scipy(W, X, stride, pad)
    assert got.shape == ref.shape
    assert rel(got, ref) < 1e-13


def test_conv_1x1_is_matmul_over_pixels():
    rng = np.random.default_rng(13)
    W = rng.standard_normal((4, 3, 1, 1))
    X = rng.standard_normal((2, 3, 5, 6))
    ref = np.einsum("oc,schw->sohw", W[:, :, 0, 0], X)
    assert rel(oracle.conv_fwd(W, X, 1, 0), ref) < 1e-14


def test_conv_centre_delta_kernel_is_identity():
    rng = np.random.default_rng(14)
    X = rng.standard_normal((2, 3, 6, 5))
    W = np.zeros((3, 3, 3, 3))
    for c in range(3):
        W[c, c, 1, 1] = 1.0
    assert np.array_equal(oracle.conv_fwd(W, X, 1, 1), X)


def test_conv_not_flipped():
    """A kernel with a single 1 at (a,b)=(0,2) must read the input pixel up
    one row and right one column (cross-correlation, not convolution)."""
    X = np.arange(25, dtype=np.float64).reshape(1, 1, 5, 5)
    W = np.zeros((1, 1, 3, 3))
    W[0, 0, 0, 2] = 1.0
    Y = oracle.conv_fwd(W, X, 1, 1)
    assert Y[0, 0, 2, 2] == X[0, 0, 1, 3]
    assert Y[0, 0, 0, 0] == 0.0          # reads above the image
    assert Y[0, 0, 4, 4] == 0.0          # reads right of the image


def test_conv_is_bilinear():
    rng = np.random.default_rng(15)
    W = rng.standard_normal((3, 2, 3, 3))
    X1, X2 = rng.standard_normal((2, 1, 2, 5, 5))
    lhs = oracle.conv_fwd(W, 2.5 * X1 - 1.5 * X2, 1, 1)
    rhs = 2.5 * oracle.conv_fwd(W, X1, 1, 1) - 1.5 * oracle.conv_fwd(W, X2, 1, 1)
    assert rel(lhs, rhs) < 1e-13


@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (3, 2, 1), (1, 1, 0), (1, 2, 0), (5, 2, 2)])
def test_conv_wgrad_is_derivative_of_the_forward(k, stride, pad):
    """L(W) = sum(delta * conv(W, x)) is linear in W, so dL/dW[e] = L(unit_e)
    exactly; the forward used here is the one pinned against scipy above."""
    rng = np.random.default_rng(16)
    Ci, Co, H, Wd, R = 2, 3, 6, 7, 2
    X = rng.standard_normal((R, Ci, H, Wd))
    Ho, Wo = oracle.conv_out_hw(H, Wd, k, k, stride, pad)
    D = rng.standard_normal((R, Co, Ho, Wo))
    dW = oracle.conv_wgrad(D, X, k, k, stride, pad, scale=1.0)
    ref = np.zeros_like(dW)
    for idx in np.ndindex(*dW.shape):
        E = np.zeros_like(dW)
        E[idx] = 1.0
        ref[idx] = np.sum(D * _conv_via_scipy(E, X, stride, pad))
    assert rel(dW, ref) < 1e-13
    assert rel(oracle.conv_wgrad(D, X, k, k, stride, pad, scale=0.5), 0.5 * ref) < 1e-13


def test_point_evaluators_match_full_tensors():
    rng = np.random.default_rng(17)
    W = rng.standard_normal((5, 3, 3, 3)).astype(np.float32)
    X = rng.standard_normal((4, 3, 6, 6)).astype(np.float32)
    Y = oracle.conv_fwd(W, X, 2, 1)
    pts = np.array([[s, co, h, w] for s in range(4) for co in (0, 4) for h in (0, 2) for w in (1, 2)])
    assert rel(oracle.conv_fwd_points(W, X, pts, 2, 1), Y[tuple(pts.T)]) < 1e-14
    D = rng.standard_normal(Y.shape).astype(np.float32)
    dW = oracle.conv_wgrad(D, X, 3, 3, 2, 1, scale=2.0)
    pts = np.array([[co, ci, a, b] for co in range(5) for ci in range(3) for a in (0, 2) for b in (1,)])
    assert rel(oracle.conv_wgrad_points(D, X, 3, 3, pts, 2, 1, scale=2.0), dW[tuple(pts.T)]) < 1e-14
    Wd = rng.standard_normal((6, 8)).astype(np.float32)
    Xd = rng.standard_normal((5, 8)).astype(np.float32)
    Dd = rng.standard_normal((5, 6)).astype(np.float32)
    pts = np.array([[s, o] for s in range(5) for o in range(6)])
    assert rel(oracle.dense_fwd_points(Wd, Xd, pts),
               (Xd.astype(np.float64) @ Wd.astype(np.float64).T)[tuple(pts.T)]) < 1e-14
    pts = np.array([[o, k] for o in range(6) for k in range(8)])
    assert rel(oracle.dense_wgrad_points(Dd, Xd, pts, scale=3.0),
               3.0 * (Dd.astype(np.float64).T @ Xd.astype(np.float64))[tuple(pts.T)]) < 1e-14


# ----------------------------------------------------------------------
# hand-worked example (index conventions of A, Ainv, B, nvec)
# ----------------------------------------------------------------------

def test_hand_worked_example():
    ex = json.load(open(os.path.join(HERE, "golden", "hand_example_K1.json")))
    e = ex["expect"]
    A, gamma = np.array(ex["A"]), np.array(ex["gamma"])
    Ainv, nvec, B = oracle.coefficients(A, gamma)
    assert np.allclose(Ainv, e["Ainv"], atol=1e-14)
    assert np.allclose(nvec, e["nvec"], atol=1e-14)
    assert np.allclose(B, e["B"], atol=1e-14)
    xbar = oracle.encode(ex["x"], ex["r"], A)
    assert np.allclose(xbar, e["xbar"], atol=1e-14)
    ybar = oracle.dense_fwd(ex["W"], xbar)
    assert np.allclose(ybar, e["ybar"], atol=1e-13)
    full = oracle.decode(ybar, Ainv, ncols=3)
    assert np.allclose(full[0], e["y"][0], atol=1e-13)
    assert np.allclose(full[1], e["Wr"][0], atol=1e-13)
    assert np.allclose(full[2], 0.0, atol=1e-13)
    assert np.allclose(oracle.decode(ybar, Ainv), e["y"], atol=1e-13)
    verdict, rho = oracle.verify(ybar, nvec, 1e-3)
    assert verdict.tolist() == [0] and rho[0] < 1e-14
    dW = oracle.masked_dense_wgrad(ex["delta"], B, gamma, xbar, scale=1.0)
    assert np.allclose(dW, e["dW"], atol=1e-13)
    dt = oracle.delta_mix(ex["delta"], B, gamma)
    # gamma_j beta_j delta = Ainv[j][0] * delta
    assert np.allclose(dt, np.outer(np.array(e["Ainv"])[0][:, 0], ex["delta"][0]), atol=1e-14)


# ----------------------------------------------------------------------
# coefficient relations (Backward Propagation matrix relation, integrity)
# ----------------------------------------------------------------------

@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_coefficient_relations(K):
    rng = np.random.default_rng(20 + K)
    G, S = 5, K + 2
    A, gamma = dk_inputs.sample_coeff_draws(rng, G, K)
    assert A.dtype == np.float32 and gamma.dtype == np.float32
    Ainv, nvec, B = oracle.coefficients(A, gamma)
    A64 = A.astype(np.float64)
    for g in range(G):
        assert np.linalg.cond(A64[g], 2) < 101
        assert np.max(np.abs(A64[g] @ Ainv[g] - np.eye(S))) < 1e-12
        A_ext = A64[g][:K + 1]                       # (K+1) x (K+2) encoding matrix
        assert np.max(np.abs(A_ext @ nvec[g])) < 1e-12
        lhs = B[g].T @ np.diag(gamma[g].astype(np.float64)) @ A_ext.T
        ref = np.hstack([np.eye(K), np.zeros((K, 1))])
        assert np.max(np.abs(lhs - ref)) < 1e-12
        assert np.all(np.abs(gamma[g]) >= 0.5) and np.all(np.abs(gamma[g]) <= 1.5)


# ----------------------------------------------------------------------
# encode / decode / mixing: library-matmul form and special cases
# ----------------------------------------------------------------------

def _case(K=3, G=4, n=11, m=7, seed=30):
    rng = np.random.default_rng(seed)
    d = dk_inputs.masked_layer_inputs(rng, dk_inputs.linear(m, n), K=K, batch=G * K)
    return d


def test_encode_is_matrix_product_X_times_A():
    d = _case()
    K, G = d["K"], d["G"]
    Xbar = oracle.encode(d["X"], d["r"], d["A"])
    for g in range(G):
        src = np.vstack([d["X"][g * K:(g + 1) * K], d["r"][g:g + 1]]).astype(np.float64)  # (K+1) x n
        ref = (src.T @ d["A"][g].astype(np.float64)[:K + 1]).T                              # S x n
        assert rel(Xbar[g * (K + 2):(g + 1) * (K + 2)], ref) < 1e-14


def test_encode_identity_and_permutation():
    K, G, n = 2, 1, 5
    rng = np.random.default_rng(31)
    X, r = rng.standard_normal((K, n)), rng.standard_normal((1, n))
    A = np.eye(4)[None]
    Xbar = oracle.encode(X, r, A)
    assert np.array_equal(Xbar[:2], X) and np.array_equal(Xbar[2], r[0]) and not Xbar[3].any()
    P = np.zeros((1, 4, 4))
    for src, dst in enumerate([2, 0, 3, 1]):       # source i lands in encoding dst
        P[0, src, dst] = 1.0
    Xbar = oracle.encode(X, r, P)
    assert np.array_equal(Xbar[2], X[0]) and np.array_equal(Xbar[0], X[1])
    assert np.array_equal(Xbar[3], r[0]) and not Xbar[1].any()


def test_encode_ignores_the_phantom_row_of_A():
    d = _case()
    A2 = d["A"].copy()
    A2[:, -1, :] += 7.0
    assert np.array_equal(oracle.encode(d["X"], d["r"], d["A"]), oracle.encode(d["X"], d["r"], A2))


def test_decode_is_matrix_product_with_Ainv():
    d = _case()
    K, G = d["K"], d["G"]
    S = K + 2
    rng = np.random.default_rng(32)
    Ybar = rng.standard_normal((G * S, 6))
    Ainv, _, _ = oracle.coefficients(d["A"], d["gamma"])
    Y = oracle.decode(Ybar, Ainv, ncols=S)
    for g in range(G):
        ref = (Ybar[g * S:(g + 1) * S].T @ Ainv[g]).T
        assert rel(Y[g * S:(g + 1) * S], ref) < 1e-13


def test_delta_mix_is_matrix_product():
    d = _case()
    K, G = d["K"], d["G"]
    S = K + 2
    _, _, B = oracle.coefficients(d["A"], d["gamma"])
    Dt = oracle.delta_mix(d["delta"], B, d["gamma"])
    for g in range(G):
        ref = np.diag(d["gamma"][g].astype(np.float64)) @ B[g] @ d["delta"][g * K:(g + 1) * K].astype(np.float64)
        assert rel(Dt[g * S:(g + 1) * S], ref) < 1e-13


# ----------------------------------------------------------------------
# the paper's invariants, dense and conv
# ----------------------------------------------------------------------

@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_dense_masked_layer_reproduces_plain_layer(K):
    rng = np.random.default_rng(40 + K)
    d = dk_inputs.masked_layer_inputs(rng, dk_inputs.linear(13, 17), K=K, batch=3 * K)
    out = oracle.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    Yplain = d["X"].astype(np.float64) @ d["W"].astype(np.float64).T
    dWplain = d["delta"].astype(np.float64).T @ d["X"].astype(np.float64)
    assert rel(out["Y"], Yplain) < 1e-9          # decode(W encode(X)) = W X
    assert rel(out["dW"], dWplain) < 1e-9        # sum_j gamma_j Eq_j = sum_i delta_i x_i^T
    assert not out["verdict"].any() and out["rho"].max() < 1e-9
    # the dropped column is <W, r>, the phantom column vanishes
    Ainv, _, _ = oracle.coefficients(d["A"], d["gamma"])
    full = oracle.decode(out["Ybar"], Ainv, ncols=K + 2).reshape(3, K + 2, 13)
    Wr = d["r"].astype(np.float64) @ d["W"].astype(np.float64).T
    assert rel(full[:, K], Wr) < 1e-9
    assert np.max(np.abs(full[:, K + 1])) < 1e-9 * np.max(np.abs(Wr))


@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (1, 1, 0), (3, 2, 1)])
def test_conv_masked_layer_reproduces_plain_layer(k, stride, pad):
    rng = np.random.default_rng(50 + k + stride)
    L = dk_inputs.conv(3, 4, 6, 6, k, stride, pad)
    d = dk_inputs.masked_layer_inputs(rng, L, K=2, batch=4)
    out = oracle.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"],
                              stride=stride, pad=pad, scale=0.5)
    Yplain = _conv_via_scipy(d["W"].astype(np.float64), d["X"].astype(np.float64), stride, pad)
    assert rel(out["Y"], Yplain) < 1e-9
    dWplain = oracle.conv_wgrad(d["delta"], d["X"], k, k, stride, pad, scale=0.5)
    assert rel(out["dW"], dWplain) < 1e-9
    assert not out["verdict"].any()


def test_masked_wgrad_equals_contraction_with_mixed_deltas():
    """sum_j gamma_j Eq_j (Eq_j formed one by one) equals one contraction of
    the gamma-scaled mixed gradients with the encodings."""
    d = _case(K=4, G=3, n=9, m=5)
    _, _, B = oracle.coefficients(d["A"], d["gamma"])
    Xbar = oracle.encode(d["X"], d["r"], d["A"])
    Dt = oracle.delta_mix(d["delta"], B, d["gamma"])
    assert rel(oracle.masked_dense_wgrad(d["delta"], B, d["gamma"], Xbar, scale=0.25),
               0.25 * Dt.T @ Xbar) < 1e-12


# ----------------------------------------------------------------------
# integrity
# ----------------------------------------------------------------------

def _clean_ybar(K=3, G=6, seed=60):
    rng = np.random.default_rng(seed)
    d = dk_inputs.masked_layer_inputs(rng, dk_inputs.linear(19, 23), K=K, batch=G * K)
    Xbar = oracle.encode(d["X"], d["r"], d["A"])
    return d, oracle.dense_fwd(d["W"], Xbar)


def test_verify_fires_on_exactly_the_corrupted_group():
    d, Ybar = _clean_ybar()
    K, G = d["K"], d["G"]
    S = K + 2
    _, nvec, _ = oracle.coefficients(d["A"], d["gamma"])
    v, rho = oracle.verify(Ybar, nvec, 1e-3)
    assert not v.any() and rho.max() < 1e-12
    rng = np.random.default_rng(61)
    for _ in range(20):
        g, j, e = rng.integers(G), rng.integers(S), rng.integers(Ybar.shape[1])
        if abs(nvec[g, j]) < 1e-2:
            continue
        Yc = Ybar.copy()
        Yc[g * S + j, e] += 0.05 * np.max(np.abs(Ybar[g * S + j]))
        v, rho = oracle.verify(Yc, nvec, 1e-3)
        expect = np.zeros(G, dtype=np.int32)
        expect[g] = 1
        assert v.tolist() == expect.tolist()
        v2, _ = oracle.verify_two_subsets(Yc, d["A"], 1e-6)
        assert v2.tolist() == expect.tolist()


def test_two_subset_check_agrees_on_clean_data():
    d, Ybar = _clean_ybar(K=2, G=4, seed=62)
    v2, diff = oracle.verify_two_subsets(Ybar, d["A"], 1e-9)
    assert not v2.any()


def test_verify_detects_tampered_encodings_and_nonfinite():
    d, _ = _clean_ybar(K=2, G=3, seed=63)
    S = 4
    _, nvec, _ = oracle.coefficients(d["A"], d["gamma"])
    Xbar = oracle.encode(d["X"], d["r"], d["A"])
    assert not oracle.verify(Xbar, nvec, 1e-3)[0].any()      # Xbar nvec = 0 too
    Xc = Xbar.copy()
    Xc[1 * S + int(np.argmax(np.abs(nvec[1]))), 3] += 5.0
    assert oracle.verify(Xc, nvec, 1e-3)[0].tolist() == [0, 1, 0]
    for bad in (np.nan, np.inf, -np.inf):
        Xc = Xbar.copy()
        Xc[2 * S + 1, 0] = bad
        assert oracle.verify(Xc, nvec, 1e-3)[0].tolist() == [0, 0, 1]


def test_verify_all_zero_group_is_clean():
    nvec = np.ones((2, 3))
    v, rho = oracle.verify(np.zeros((6, 4)), nvec, 1e-3)
    assert v.tolist() == [0, 0] and rho.tolist() == [0.0, 0.0]


# ----------------------------------------------------------------------
# planted mistakes must be caught by the pins above (run on CPU copies)
# ----------------------------------------------------------------------

def test_transposed_A_breaks_the_round_trip():
    d = _case(K=3, G=2, n=8, m=6, seed=70)
    At = np.ascontiguousarray(np.swapaxes(d["A"], 1, 2))
    Ainv, _, _ = oracle.coefficients(d["A"], d["gamma"])
    Ybar = oracle.dense_fwd(d["W"], oracle.encode(d["X"], d["r"], At))
    Y = oracle.decode(Ybar, Ainv)
    assert rel(Y, d["X"].astype(np.float64) @ d["W"].astype(np.float64).T) > 1e-2
