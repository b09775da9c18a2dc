"""Pins for the finite-field oracle's functions for several colluding
accelerators (CPU only): M noise vectors per group, uniform over F_p,
S = K + M + 1 encodings (section "Colluding GPUs" and the paragraph of
"Privacy Guarantee" on it).

Checked against things other than the oracle itself: the single-noise
functions at M = 1, exact Python integers, numpy's int64 matmul of the
un-masked quantised operands, the algebraic relations of the coefficient
matrices, exhaustion of a tiny field for the privacy statement, and brute
force over single-element corruptions."""
import itertools

import numpy as np
import pytest

import dk_inputs
from oracle import field as F

P = F.P


def _lift(v, p=P):
    v = np.asarray(v).astype(np.int64)
    return np.where(v > p // 2, v - p, v)


def _case(K, M, G, layer, seed, **kw):
    return dk_inputs.field_collusion_layer_inputs(np.random.default_rng([K, M, G, seed]), layer, K=K, M=M,
                                                  batch=G * K, **kw)


def test_m_equal_one_reduces_bit_for_bit():
    d = _case(3, 1, 2, dk_inputs.linear(7, 11), 0)
    a = F.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], 3)
    b = F.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    for k in b:
        assert np.array_equal(a[k], b[k]), k
    for x, y in zip(F.coefficients_m(d["A"], d["gamma"], 3), F.coefficients(d["A"], d["gamma"])):
        assert np.array_equal(x, y)
    L = dk_inputs.conv(2, 3, 5, 4, 3)
    d = _case(2, 1, 2, L, 1)
    a = F.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], 2, stride=1, pad=1)
    b = F.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=1, pad=1)
    for k in b:
        assert np.array_equal(a[k], b[k]), k


def test_encode_and_mix_against_python_integers():
    K, M, G, n = 2, 3, 2, 5
    S = K + M + 1
    rng = np.random.default_rng(3)
    xq = rng.integers(0, P, size=(G * K, n), dtype=np.uint32)
    r = rng.integers(0, P, size=(G * M, n), dtype=np.uint32)
    A = rng.integers(0, P, size=(G, S, S), dtype=np.uint32)
    got = F.encode_m(xq, r, A, K)
    for g in range(G):
        for j in range(S):
            for e in range(n):
                want = sum(int(A[g, i, j]) * int(xq[g * K + i, e]) for i in range(K))
                want += sum(int(A[g, K + q, j]) * int(r[g * M + q, e]) for q in range(M))
                assert int(got[g * S + j, e]) == want % P
    B = rng.integers(0, P, size=(G, S, K), dtype=np.uint32)
    gamma = rng.integers(1, P, size=(G, S), dtype=np.uint32)
    got = F.delta_mix_m(xq, B, gamma)
    for g in range(G):
        for j in range(S):
            for e in range(n):
                want = int(gamma[g, j]) * sum(int(B[g, j, i]) * int(xq[g * K + i, e]) for i in range(K))
                assert int(got[g * S + j, e]) == want % P


def test_coefficient_relations_over_the_field():
    K, M, G = 3, 2, 3
    S = K + M + 1
    d = _case(K, M, G, dk_inputs.linear(4, 4), 4)
    Ainv, nvec, B = F.coefficients_m(d["A"], d["gamma"], K)
    for g in range(G):
        A = [[int(v) for v in row] for row in d["A"][g]]
        inv = [[int(v) for v in row] for row in Ainv[g]]
        for i in range(S):
            for j in range(S):
                assert sum(A[i][k] * inv[k][j] for k in range(S)) % P == (i == j)
        # the combination nvec vanishes on every real source (inputs and noise)
        for i in range(K + M):
            assert sum(A[i][j] * int(nvec[g, j]) for j in range(S)) % P == 0
        # B^T Gamma A^T = [I_K | 0] over the K + M real sources
        for i in range(K):
            for src in range(K + M):
                v = sum(int(B[g, j, i]) * int(d["gamma"][g, j]) * A[src][j] for j in range(S)) % P
                assert v == (i == src)


@pytest.mark.parametrize("K,M,G", [(1, 2, 2), (2, 2, 1), (4, 3, 2), (3, 4, 1)])
def test_staged_path_equals_integer_matmul_of_the_quantised_operands(K, M, G):
    """No masking, no field: the lifted decoded outputs and weight gradient are
    the int64 products of the quantised operands (values stay far below p/2)."""
    L = dk_inputs.linear(9, 13)
    d = _case(K, M, G, L, 5, delta_std=1.0)
    o = F.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], K)
    Wq, Xq, Dq = _lift(o["Wq"]), _lift(o["Xq"]), _lift(o["Dq"])
    assert np.array_equal(_lift(o["Yq"]), Xq @ Wq.T)
    assert np.array_equal(_lift(o["dWq"]), Dq.T @ Xq)
    assert not o["verdict"].any()
    # the decoded columns after the K outputs: <W_q, r_q> for each noise vector, then zero
    S = K + M + 1
    Ainv, _, _ = F.coefficients_m(d["A"], d["gamma"], K)
    full = F.decode_m(o["Ybar"], Ainv, S).reshape(G, S, -1)
    Wr = (d["r"].astype(object) @ o["Wq"].astype(object).T) % P
    assert np.array_equal(full[:, K:K + M].reshape(G * M, -1), np.asarray(Wr, dtype=np.uint32))
    assert not full[:, S - 1].any()


def test_conv_layer_with_two_noise_vectors():
    import scipy.signal
    L = dk_inputs.conv(2, 3, 6, 5, 3)
    K, M, G = 2, 2, 2
    d = _case(K, M, G, L, 6, delta_std=1.0)
    o = F.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], K, stride=1, pad=1)
    Wq, Xq = _lift(o["Wq"]), _lift(o["Xq"])
    want = np.zeros((G * K, 3, 6, 5), dtype=np.int64)
    for s in range(G * K):
        for co in range(3):
            for ci in range(2):
                want[s, co] += scipy.signal.correlate2d(Xq[s, ci], Wq[co, ci], mode="same")
    assert np.array_equal(_lift(o["Yq"]), want)
    assert not o["verdict"].any()


def test_any_m_encodings_are_uniform_whatever_the_inputs():
    """The privacy statement for M colluders, by exhausting a tiny field: for
    K = 1, M = 2 over F_5, any two encodings whose 2 x 2 block of A_2 is
    non-singular take every pair of values exactly once as the noise runs over
    F_5^2 -- for every input -- so they say nothing about it; a pair with a
    singular block does not."""
    p, K, M = 5, 1, 2
    S = K + M + 1
    A = np.array([[[1, 2, 3, 4], [1, 1, 2, 1], [1, 2, 1, 3], [0, 1, 1, 1]]], dtype=np.uint32)
    A2 = A[0, K:K + M].astype(int)
    seen_good = seen_bad = False
    for cols in itertools.combinations(range(S), M):
        det = int(A2[0, cols[0]] * A2[1, cols[1]] - A2[0, cols[1]] * A2[1, cols[0]]) % p
        tables = []
        for x in range(p):
            xq = np.full((1, p * p), x, dtype=np.uint32)
            r = np.array([[a for a in range(p) for _ in range(p)], [b for _ in range(p) for b in range(p)]],
                         dtype=np.uint32)
            enc = F.encode_m(xq, r, A, K, p=p)
            tables.append(sorted(zip(enc[cols[0]].tolist(), enc[cols[1]].tolist())))
        every_pair_once = [(a, b) for a in range(p) for b in range(p)]
        if det:
            assert all(t == every_pair_once for t in tables), cols
            seen_good = True
        else:
            assert any(t != every_pair_once for t in tables), cols
            seen_bad = True
    assert seen_good and seen_bad


def test_every_noise_block_of_the_drawn_matrices_is_non_singular():
    K, M = 2, 3
    S = K + M + 1
    d = _case(K, M, 4, dk_inputs.linear(4, 4), 7)
    for g in range(4):
        A2 = [[int(v) for v in row] for row in d["A"][g][K:K + M]]
        for cols in itertools.combinations(range(S), M):
            sub = [[A2[q][c] for c in cols] for q in range(M)]
            F.inv_mod_matrix(sub)          # raises if singular


def test_verify_flags_exactly_the_corrupted_group():
    K, M, G = 2, 2, 3
    S = K + M + 1
    d = _case(K, M, G, dk_inputs.linear(3, 4), 8)
    o = F.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], K)
    _, nvec, _ = F.coefficients_m(d["A"], d["gamma"], K)
    assert not F.verify_m(o["Ybar"], nvec).any()
    for row in range(G * S):
        for e in range(3):
            bad = o["Ybar"].copy()
            bad[row, e] = (int(bad[row, e]) + 1) % P
            g = row // S
            want = [int(q == g and int(nvec[g, row % S]) != 0) for q in range(G)]
            assert F.verify_m(bad, nvec).tolist() == want
    bad = o["Ybar"].copy()
    bad[S + 1, 0] = P + 3                  # not a field element
    assert F.verify_m(bad, nvec).tolist() == [0, 1, 0]


def test_planted_mistake_is_caught():
    """Decoding with the noise rows and input rows of A swapped must not give
    the plain product (a check that the pins above can fail)."""
    K, M, G = 2, 2, 1
    d = _case(K, M, G, dk_inputs.linear(5, 6), 9, delta_std=1.0)
    A = d["A"].copy()
    A[0, [0, K]] = A[0, [K, 0]]
    Xq = F.quantize(d["X"])
    Xbar = F.encode_m(Xq, d["r"], A, K)
    Ainv, _, _ = F.coefficients_m(d["A"], d["gamma"], K)
    Ybar = F.dense_fwd(F.quantize(d["W"]), Xbar)
    Yq = F.decode_m(Ybar, Ainv, K)
    assert not np.array_equal(_lift(Yq), _lift(Xq) @ _lift(F.quantize(d["W"])).T)
