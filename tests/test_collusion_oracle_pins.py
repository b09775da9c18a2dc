"""Pins for the oracle's M-noise-vector ("colluding accelerators") functions
(CPU only): they must reduce to the single-noise functions at M = 1, decode
to the plain layer for any M, satisfy the section's matrix relation, and hide
the inputs from any M encodings."""
import itertools

import numpy as np
import pytest

import dk_inputs
import oracle


def _case(K, M, G, layer, seed):
    rng = np.random.default_rng([K, M, G, seed])
    return dk_inputs.collusion_layer_inputs(rng, layer, K=K, M=M, batch=G * K, delta_std=1.0)


def test_m_equal_one_reduces_to_the_single_noise_functions():
    d = _case(3, 1, 2, dk_inputs.linear(7, 11), 0)
    a = oracle.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], 3)
    b = oracle.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    for k in ("Xbar", "Ybar", "Y", "rho"):
        assert np.array_equal(a[k], b[k]), k
    # (the single-noise oracle forms every Eq_j explicitly: another summation order)
    assert np.abs(a["dW"] - b["dW"]).max() <= 1e-12 * np.abs(b["dW"]).max()
    assert np.array_equal(a["verdict"], b["verdict"])
    for x, y in zip(oracle.coefficients_m(d["A"], d["gamma"], 3), oracle.coefficients(d["A"], d["gamma"])):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("K,M,G", [(1, 2, 2), (2, 2, 1), (4, 3, 2), (3, 5, 1)])
def test_decoded_results_are_the_plain_layer(K, M, G):
    d = _case(K, M, G, dk_inputs.linear(9, 13), 1)
    o = oracle.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], K)
    Y = d["X"].astype(np.float64) @ d["W"].astype(np.float64).T
    dW = d["delta"].astype(np.float64).T @ d["X"].astype(np.float64)
    assert np.abs(o["Y"] - Y).max() <= 1e-9 * np.abs(Y).max() * 100
    assert np.abs(o["dW"] - dW).max() <= 1e-9 * np.abs(dW).max() * 100
    assert not o["verdict"].any()
    # the columns after the K outputs are <W, r_q> for the M noise vectors, then zero
    Ainv, _, _ = oracle.coefficients_m(d["A"], d["gamma"], K)
    S = K + M + 1
    full = oracle.decode_m(o["Ybar"], Ainv, S).reshape(G, S, -1)
    Wr = (d["r"].astype(np.float64) @ d["W"].astype(np.float64).T).reshape(G, M, -1)
    assert np.abs(full[:, K:K + M] - Wr).max() <= 1e-8 * np.abs(Wr).max()
    assert np.abs(full[:, S - 1]).max() <= 1e-8 * np.abs(Wr).max()


def test_conv_layer_with_two_noise_vectors():
    L = dk_inputs.conv(3, 4, 6, 5, 3)
    d = _case(2, 2, 2, L, 2)
    o = oracle.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], 2, stride=1, pad=1)
    Y = oracle.conv_fwd(d["W"], d["X"], 1, 1)
    dW = oracle.conv_wgrad(d["delta"], d["X"], 3, 3, 1, 1)
    assert np.abs(o["Y"] - Y).max() <= 1e-8 * np.abs(Y).max()
    assert np.abs(o["dW"] - dW).max() <= 1e-8 * np.abs(dW).max()


def test_matrix_relation_and_null_vector():
    K, M = 3, 2
    S = K + M + 1
    d = _case(K, M, 2, dk_inputs.linear(4, 4), 3)
    Ainv, nvec, B = oracle.coefficients_m(d["A"], d["gamma"], K)
    for g in range(2):
        A = d["A"][g].astype(np.float64)
        Gm = np.diag(d["gamma"][g].astype(np.float64))
        rel = B[g].T @ Gm @ A[:K + M].T          # B^T Gamma A_ext^T over the K+M real sources
        want = np.concatenate([np.eye(K), np.zeros((K, M))], 1)
        assert np.abs(rel - want).max() < 1e-10
        assert np.abs(A[:K + M] @ nvec[g]).max() < 1e-10


def test_any_m_encodings_are_masked_by_independent_noise():
    """Section "Privacy Guarantee", colluding case: for any M columns, the
    M x M block of A_2 is non-singular, so M colluders cannot cancel the
    noise.  (A property of the drawn matrices; checked on the generator's draws.)"""
    K, M = 2, 3
    S = K + M + 1
    d = _case(K, M, 1, dk_inputs.linear(4, 4), 4)
    A2 = d["A"][0].astype(np.float64)[K:K + M]
    for cols in itertools.combinations(range(S), M):
        assert abs(np.linalg.det(A2[:, cols])) > 1e-6


def test_verify_with_more_noise_vectors():
    K, M, G = 2, 2, 3
    S = K + M + 1
    d = _case(K, M, G, dk_inputs.linear(6, 8), 5)
    o = oracle.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], K)
    _, nvec, _ = oracle.coefficients_m(d["A"], d["gamma"], K)
    for row in (0, S + 2, 3 * S - 1):
        bad = o["Ybar"].copy()
        g = row // S
        scale = np.abs(nvec[g] * bad[g * S:(g + 1) * S].T).sum(1).max()
        bad[row, 1] += 0.5 * scale / abs(nvec[g, row % S])
        verdict, _ = oracle.verify_m(bad, nvec, 1e-3)
        assert verdict.tolist() == [int(q == g) for q in range(G)]
