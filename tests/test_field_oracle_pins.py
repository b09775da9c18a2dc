"""Pins for the finite-field oracle (CPU only).

Each test checks the oracle against something other than itself: exact Python
integers, numpy's int64 matmul on the un-masked quantised values, hand-worked
roundings, the algebraic relations of the coefficient matrices, and brute
force over every single-element corruption of a tiny case.
"""
import itertools

import numpy as np
import pytest

import dk_inputs
from oracle import field as F

P = F.P


def test_prime_is_the_largest_25_bit_prime():
    # section "Privacy Guarantee": p = 2^25 - 39 is the largest 25-bit prime
    def is_prime(n):
        if n % 2 == 0:
            return False
        d = 3
        while d * d <= n:
            if n % d == 0:
                return False
            d += 2
        return True
    assert P == 33554393 and P < (1 << 25) and is_prime(P)
    assert not any(is_prime(q) for q in range(P + 1, 1 << 25))


def test_round_and_field_hand_values():
    # Round: floor when the fraction is below one half, floor + 1 otherwise
    # (so 2.5 -> 3 and -2.5 -> -2); Field: negative values get p added.
    # With l = 1 the input is doubled first.
    x = np.array([1.25, 1.2, -1.25, -1.3, 0.24, -0.25, -0.26, 0.0, 3.0], dtype=np.float32)
    # 2x = 2.5, 2.4, -2.5, -2.6, 0.48, -0.5, -0.52, 0, 6
    want = [3, 2, -2, -3, 0, 0, -1, 0, 6]
    got = F.quantize(x, l=1)
    assert got.tolist() == [w % P for w in want]
    # l = 8: 1/512 is exactly half a unit
    x = np.array([1 / 512, -1 / 512, 1 / 256, 0.999], dtype=np.float32)
    assert F.quantize(x, l=8).tolist() == [1, 0, 1, 256]


def test_quantize_clamps_and_maps_nan_to_zero():
    x = np.array([1e30, -1e30, np.nan], dtype=np.float32)
    got = F.quantize(x, l=8).tolist()
    assert got == [(2**31 - 1) % P, (-2**31) % P, 0]


def test_dequantize_hand_values():
    # centred lift, then Round(v * 2^-l) * 2^-l, l = 2
    v = np.array([0, 5, 6, P - 5, P - 6, P - 2, 2], dtype=np.uint32)
    # lifted: 0, 5, 6, -5, -6, -2, 2; /4: 0, 1.25, 1.5, -1.25, -1.5, -0.5, 0.5
    # rounded: 0, 1, 2, -1, -1, 0, 1; times 1/4
    assert F.dequantize(v, l=2).tolist() == [0.0, 0.25, 0.5, -0.25, -0.25, 0.0, 0.25]


def test_quantize_dequantize_roundtrip_of_products():
    rng = np.random.default_rng(0)
    a = rng.normal(size=50).astype(np.float32)
    b = rng.normal(size=50).astype(np.float32)
    aq, bq = F.quantize(a), F.quantize(b)
    prod = (aq.astype(np.uint64) * bq.astype(np.uint64) % P).astype(np.uint32)
    back = F.dequantize(prod)
    assert np.abs(back - a.astype(np.float64) * b).max() < 3 * 2.0**-8 * 4


def test_matrix_inverse_over_field():
    rng = np.random.default_rng(1)
    for n in (1, 2, 4, 10):
        A = rng.integers(0, P, size=(n, n)).tolist()
        inv = F.inv_mod_matrix(A)
        for i in range(n):
            for j in range(n):
                assert sum(A[i][k] * inv[k][j] for k in range(n)) % P == (i == j)
    with pytest.raises(ValueError):
        F.inv_mod_matrix([[1, 2], [2, 4]])
    # a hand case: [[2, 1], [1, 1]]^-1 = [[1, -1], [-1, 2]]
    assert F.inv_mod_matrix([[2, 1], [1, 1]]) == [[1, P - 1], [P - 1, 2]]


def test_coefficient_relations():
    rng = np.random.default_rng(2)
    G, K = 3, 4
    S = K + 2
    A = rng.integers(0, P, size=(G, S, S), dtype=np.uint32)
    gamma = rng.integers(1, P, size=(G, S), dtype=np.uint32)
    Ainv, nvec, B = F.coefficients(A, gamma)
    for g in range(G):
        a = A[g].astype(object)
        # the K+1 real sources times the null vector vanish
        for i in range(K + 1):
            assert sum(int(a[i][j]) * int(nvec[g, j]) for j in range(S)) % P == 0
        # B^T Gamma A_ext^T = [I_K | 0] over the K+1 real sources
        for i in range(K):
            for ip in range(K + 1):
                v = sum(int(gamma[g, j]) * int(B[g, j, i]) * int(a[ip][j]) for j in range(S)) % P
                assert v == (i == ip)
        assert np.array_equal(nvec[g], Ainv[g][:, S - 1])


def test_encode_special_cases():
    rng = np.random.default_rng(3)
    K, n = 2, 7
    S = K + 2
    xq = rng.integers(0, P, size=(K, n), dtype=np.uint32)
    r = rng.integers(0, P, size=(1, n), dtype=np.uint32)
    eye = np.eye(S, dtype=np.uint32)[None]
    xb = F.encode(xq, r, eye)
    assert np.array_equal(xb[:K], xq) and np.array_equal(xb[K], r[0]) and not xb[K + 1].any()
    # brute force with Python integers
    A = rng.integers(0, P, size=(1, S, S), dtype=np.uint32)
    xb = F.encode(xq, r, A)
    for j in range(S):
        for e in range(n):
            want = (sum(int(A[0, i, j]) * int(xq[i, e]) for i in range(K)) + int(A[0, K, j]) * int(r[0, e])) % P
            assert int(xb[j, e]) == want


def test_dense_matmul_against_python_integers():
    rng = np.random.default_rng(4)
    R, M, N = 3, 4, 50
    W = rng.integers(0, P, size=(M, N), dtype=np.uint32)
    X = rng.integers(0, P, size=(R, N), dtype=np.uint32)
    Y = F.dense_fwd(W, X)
    want = (X.astype(object) @ W.astype(object).T) % P
    assert np.array_equal(Y.astype(object), want)
    D = rng.integers(0, P, size=(R, M), dtype=np.uint32)
    dW = F.dense_wgrad(D, X)
    assert np.array_equal(dW.astype(object), (D.astype(object).T @ X.astype(object)) % P)
    pts = [(0, 0), (2, 3), (1, 2)]
    assert F.dense_fwd_points(W, X, pts).tolist() == [int(want[s, o]) for s, o in pts]
    wpts = [(0, 0), (3, 49), (2, 17)]
    assert F.dense_wgrad_points(D, X, wpts).tolist() == [int(dW[o, k]) for o, k in wpts]


def _lift(v):
    v = v.astype(np.int64)
    return np.where(v > P // 2, v - P, v)


@pytest.mark.parametrize("K,G,M,N,seed", [(1, 2, 5, 9, 0), (2, 1, 8, 16, 1), (4, 3, 7, 33, 2), (8, 2, 6, 20, 3)])
def test_staged_path_equals_plain_integer_layer(K, G, M, N, seed):
    """Decoding Correctness over the field: the decoded field values, lifted,
    are exactly the integer products of the quantised operands (numpy int64
    matmul, no masking, no field), forward and weight gradient."""
    rng = np.random.default_rng([seed, 7])
    d = dk_inputs.field_layer_inputs(rng, dk_inputs.linear(M, N), K=K, batch=G * K, w_std=0.5, delta_std=1.0)
    o = F.masked_dense_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    Wi, Xi, Di = (np.floor(a.astype(np.float64) * 256 + 0.5).astype(np.int64) for a in (d["W"], d["X"], d["delta"]))
    assert np.array_equal(_lift(o["Wq"]), Wi) and np.array_equal(_lift(o["Xq"]), Xi)
    assert np.array_equal(_lift(o["Yq"]), Xi @ Wi.T)
    assert np.array_equal(_lift(o["dWq"]), Di.T @ Xi)
    assert not o["verdict"].any()
    # the float results are the real layer up to the fixed-point error
    Y = d["X"].astype(np.float64) @ d["W"].astype(np.float64).T
    bound = 2.0**-9 * (np.abs(d["X"]).sum(1).max() + np.abs(d["W"]).sum(1).max() + N * 2.0**-9) + 2.0**-9
    assert np.abs(o["Y"] - Y).max() <= bound * 1.0001


def test_decoded_extra_columns_are_noise_product_and_zero():
    rng = np.random.default_rng(11)
    K, G, M, N = 2, 2, 5, 12
    d = dk_inputs.field_layer_inputs(rng, dk_inputs.linear(M, N), K=K, batch=G * K)
    o = F.masked_dense_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    Ainv, _, _ = F.coefficients(d["A"], d["gamma"])
    full = F.decode(o["Ybar"], Ainv, ncols=K + 2).reshape(G, K + 2, M)
    Wr = F.dense_fwd(o["Wq"], d["r"])
    assert np.array_equal(full[:, K], Wr)            # column K is <W, r>
    assert not full[:, K + 1].any()                  # the phantom source decodes to zero
    assert np.array_equal(full[:, :K].reshape(G * K, M), o["Yq"])


def test_encodings_hide_the_inputs_exactly_like_a_one_time_pad():
    # "Privacy Guarantee": x + uniform noise is uniform.  For fixed A with a
    # non-zero noise weight, running r over the whole of a tiny field makes
    # every encoded value take every field value exactly once.
    p = 13
    K, S = 1, 3
    A = np.array([[[3, 5, 7], [2, 6, 11], [1, 4, 9]]], dtype=np.uint32)
    xq = np.array([[4]], dtype=np.uint32)
    seen = [set() for _ in range(S)]
    for rv in range(p):
        xb = F.encode(xq, np.array([[rv]], dtype=np.uint32), A, p=p)
        for j in range(S):
            seen[j].add(int(xb[j, 0]))
    assert all(len(s) == p for s in seen)


def test_verify_detects_every_single_element_corruption():
    rng = np.random.default_rng(12)
    K, G, M, N = 2, 2, 3, 5
    S = K + 2
    d = dk_inputs.field_layer_inputs(rng, dk_inputs.linear(M, N), K=K, batch=G * K)
    o = F.masked_dense_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    _, nvec, _ = F.coefficients(d["A"], d["gamma"])
    assert nvec.all()     # (a zero entry has probability 1/p; this seed has none)
    assert F.verify(o["Ybar"], nvec).tolist() == [0] * G
    for row, e, add in itertools.product(range(G * S), range(M), (1, 2, P - 1, 12345)):
        bad = o["Ybar"].copy()
        bad[row, e] = (int(bad[row, e]) + add) % P
        want = [int(g == row // S) for g in range(G)]
        assert F.verify(bad, nvec).tolist() == want
    # a value outside the field is a corruption too
    bad = o["Ybar"].copy()
    bad[S, 0] = P
    assert F.verify(bad, nvec).tolist() == [0, 1]


def test_delta_mix_against_python_integers():
    rng = np.random.default_rng(13)
    K, G, m = 2, 2, 4
    S = K + 2
    dq = rng.integers(0, P, size=(G * K, m), dtype=np.uint32)
    B = rng.integers(0, P, size=(G, S, K), dtype=np.uint32)
    gamma = rng.integers(1, P, size=(G, S), dtype=np.uint32)
    out = F.delta_mix(dq, B, gamma)
    for g, j, e in itertools.product(range(G), range(S), range(m)):
        want = int(gamma[g, j]) * sum(int(B[g, j, i]) * int(dq[g * K + i, e]) for i in range(K)) % P
        assert int(out[g * S + j, e]) == want


def test_planted_mistakes_are_caught():
    """A transposed inverse, or the null vector taken from the wrong column,
    breaks the pins above: the decoded values stop matching the plain layer
    and clean data stops verifying."""
    rng = np.random.default_rng(14)
    K, G, M, N = 2, 1, 4, 6
    d = dk_inputs.field_layer_inputs(rng, dk_inputs.linear(M, N), K=K, batch=G * K)
    o = F.masked_dense_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    Ainv, nvec, _ = F.coefficients(d["A"], d["gamma"])
    wrong = np.ascontiguousarray(Ainv.transpose(0, 2, 1))
    assert not np.array_equal(F.decode(o["Ybar"], wrong), o["Yq"])
    assert F.verify(o["Ybar"], np.ascontiguousarray(Ainv[:, :, K])).any()


def _int_corr(Wi, Xi, stride, pad):
    """Cross-correlation of int64 arrays with scipy's correlate2d (valid mode on
    a zero-padded image, then subsampled): an independent library routine."""
    from scipy.signal import correlate2d
    R, Ci, H, W = Xi.shape
    Co, _, kh, kw = Wi.shape
    Xp = np.pad(Xi, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    out = []
    for s in range(R):
        rows = []
        for co in range(Co):
            acc = sum(correlate2d(Xp[s, ci], Wi[co, ci], mode="valid") for ci in range(Ci))
            rows.append(acc[::stride, ::stride])
        out.append(rows)
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("K,G,Ci,Co,H,W,k,stride,pad", [(2, 1, 3, 4, 6, 5, 3, 1, 1), (1, 2, 2, 3, 7, 7, 3, 2, 1),
                                                        (4, 1, 3, 2, 5, 6, 1, 1, 0), (2, 2, 2, 2, 6, 6, 2, 2, 0)])
def test_staged_conv_path_equals_plain_integer_convolution(K, G, Ci, Co, H, W, k, stride, pad):
    rng = np.random.default_rng([K, G, Ci, Co, H, 21])
    L = dk_inputs.conv(Ci, Co, H, W, k, stride, pad)
    d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, w_std=0.5, delta_std=1.0)
    o = F.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=stride, pad=pad)
    Wi, Xi, Di = (np.floor(a.astype(np.float64) * 256 + 0.5).astype(np.int64) for a in (d["W"], d["X"], d["delta"]))
    assert np.array_equal(_lift(o["Yq"]), _int_corr(Wi, Xi, stride, pad))
    assert not o["verdict"].any()
    # weight gradient: dW[co][ci] = sum_s correlate(X[s][ci] padded, D[s][co] dilated by the stride)
    from scipy.signal import correlate2d
    Ho, Wo = F.conv_out_hw(H, W, k, k, stride, pad)
    Xp = np.pad(Xi, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    want = np.zeros((Co, Ci, k, k), dtype=np.int64)
    for s in range(G * K):
        for co in range(Co):
            Dd = np.zeros(((Ho - 1) * stride + 1, (Wo - 1) * stride + 1), dtype=np.int64)
            Dd[::stride, ::stride] = Di[s, co]
            for ci in range(Ci):
                want[co, ci] += correlate2d(Xp[s, ci], Dd, mode="valid")[:k, :k]
    assert np.array_equal(_lift(o["dWq"]), want)
    # sampled evaluators agree with the full ones
    pts = [(0, 0, 0, 0), (G * (K + 2) - 1, Co - 1, Ho - 1, Wo - 1), (1, Co // 2, Ho // 2, 0)]
    assert F.conv_fwd_points(o["Wq"], o["Xbar"], pts, stride, pad).tolist() == [int(o["Ybar"][t]) for t in pts]
    wpts = [(0, 0, 0, 0), (Co - 1, Ci - 1, k - 1, k - 1)]
    assert F.conv_wgrad_points(o["Dtilde"], o["Xbar"], k, k, wpts, stride, pad).tolist() == [int(o["dWq"][t]) for t in wpts]


def test_field_conv_1x1_is_a_matmul_over_pixels():
    rng = np.random.default_rng(31)
    R, Ci, Co, H, W = 2, 5, 3, 4, 3
    X = rng.integers(0, P, size=(R, Ci, H, W), dtype=np.uint32)
    Wq = rng.integers(0, P, size=(Co, Ci, 1, 1), dtype=np.uint32)
    Y = F.conv_fwd(Wq, X)
    flat = F.dense_fwd(Wq.reshape(Co, Ci), np.ascontiguousarray(X.transpose(0, 2, 3, 1).reshape(-1, Ci)))
    assert np.array_equal(Y, flat.reshape(R, H, W, Co).transpose(0, 3, 1, 2))
