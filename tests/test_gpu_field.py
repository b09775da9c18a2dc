"""GPU parity of the finite-field variant against the field oracle, through
the C ABI.  Everything is integer arithmetic modulo p, so every comparison is
exact; the float outputs are exact too (a rounded integer times 2^-l)."""
import numpy as np
import pytest

import dk_inputs
from oracle import field as F

pytestmark = pytest.mark.gpu

P = F.P


@pytest.fixture(scope="module")
def dk():
    import torch
    import paper_2207_00083_amd as m
    m.load()
    assert torch.cuda.is_available()
    return m


def dev(a):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def host(t):
    import torch
    a = t.cpu().numpy()
    return a.view(np.uint32) if a.dtype == np.int32 else a


def test_quantize_and_dequantize(dk):
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 3, 1003), rng.normal(0, 1e5, 50),
                        [0.0, -0.0, 1 / 512, -1 / 512, 1e30, -1e30, np.nan, np.inf, -np.inf,
                         0.49999997, -2.5 / 256, 2.5 / 256]]).astype(np.float32)
    for l in (0, 1, 8, 12):
        assert np.array_equal(host(dk.dkf_quantize(dev(x), l=l)), F.quantize(x, l=l))
    q = rng.integers(0, P, size=4099, dtype=np.uint32)
    q[:4] = [0, P - 1, P // 2, P // 2 + 1]
    for l in (0, 3, 8):
        assert np.array_equal(host(dk.dkf_dequantize(dev(q), l=l)), F.dequantize(q, l=l))


@pytest.mark.parametrize("K,G,n", [(1, 3, 17), (2, 2, 1024), (4, 5, 4100), (8, 3, 2051), (16, 2, 260)])
def test_encode(dk, K, G, n):
    rng = np.random.default_rng([K, G, n])
    d = dk_inputs.field_layer_inputs(rng, dk_inputs.linear(3, n), K=K, batch=G * K)
    got = host(dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K))
    want = F.encode(F.quantize(d["X"]), d["r"], d["A"])
    assert np.array_equal(got, want)


@pytest.mark.parametrize("R,M,N,small", [(5, 7, 9, False), (130, 200, 300, False), (130, 200, 300, True),
                                         (384, 257, 1000, False), (64, 129, 4099, True), (1, 1, 1, False)])
def test_linear_fwd_full(dk, R, M, N, small):
    rng = np.random.default_rng([R, M, N, int(small)])
    X = rng.integers(0, P, size=(R, N), dtype=np.uint32)
    if small:   # field images of small signed integers: only the low digits are non-zero
        W = (rng.integers(-3000, 3000, size=(M, N)) % P).astype(np.uint32)
    else:
        W = rng.integers(0, P, size=(M, N), dtype=np.uint32)
    got = host(dk.dkf_linear_fwd(dev(W), dev(X)))
    assert np.array_equal(got, F.dense_fwd(W, X))


@pytest.mark.parametrize("x_small,w_small", [(True, True), (True, False), (False, True)])
def test_linear_fwd_digit_halves_skipped(dk, x_small, w_small):
    """Operands whose high digit halves are all zero take the short path (the
    device flags switch parts off); every combination must stay exact."""
    rng = np.random.default_rng([int(x_small), int(w_small), 3])
    R, M, N = 150, 140, 260
    small = lambda shape: (rng.integers(-8000, 8000, size=shape) % P).astype(np.uint32)
    big = lambda shape: rng.integers(0, P, size=shape, dtype=np.uint32)
    X = small((R, N)) if x_small else big((R, N))
    W = small((M, N)) if w_small else big((M, N))
    assert np.array_equal(host(dk.dkf_linear_fwd(dev(W), dev(X))), F.dense_fwd(W, X))
    # all-zero operands
    Z = np.zeros((R, N), dtype=np.uint32)
    assert not host(dk.dkf_linear_fwd(dev(W), dev(Z))).any()


@pytest.mark.parametrize("top", [127, 128, 200, 8191])
def test_forward_one_digit_weights(dk, top):
    """Weights whose field images all lie in [-127, 127] occupy one digit plane and take the
    one-plane steps; a single element just outside (128, or -129) must switch them off.  Dense
    product, convolution read in place (16 channels) and through the stored patch matrix."""
    rng = np.random.default_rng([top, 41])
    def weights(shape):
        w = rng.integers(-127, 128, size=shape)
        w.reshape(-1)[:4] = (-127, 127, 64, -65)
        if top > 127:
            w.reshape(-1)[w.size // 2] = top
            w.reshape(-1)[w.size // 3] = -top - 1
        return (w % P).astype(np.uint32)
    for R, M, N in ((150, 140, 260), (70, 64, 1000), (3, 5, 7), (300, 1, 129)):
        X = rng.integers(0, P, size=(R, N), dtype=np.uint32)
        W = weights((M, N))
        assert np.array_equal(host(dk.dkf_linear_fwd(dev(W), dev(X))), F.dense_fwd(W, X))
    # all-zero weights (no plane holds anything) and all-zero encodings next to one-digit weights
    X = rng.integers(0, P, size=(130, 200), dtype=np.uint32)
    assert not host(dk.dkf_linear_fwd(dev(np.zeros((70, 200), dtype=np.uint32)), dev(X))).any()
    assert not host(dk.dkf_linear_fwd(dev(weights((70, 200))), dev(np.zeros_like(X)))).any()
    # (the one-plane steps need more than 64 output channels and a contraction of at least 512)
    for Ci, Co, H, k, stride, pad in ((64, 96, 8, 3, 1, 1), (128, 130, 9, 3, 2, 1), (60, 70, 6, 3, 1, 1),
                                     (512, 65, 5, 1, 1, 0), (16, 96, 12, 3, 1, 1), (16, 40, 12, 3, 1, 1)):
        L = dk_inputs.conv(Ci, Co, H, H, k, stride, pad)
        X = rng.integers(0, P, size=(5, Ci, H, H), dtype=np.uint32)
        W = weights((Co, Ci, k, k))
        got = host(dk.dkf_conv_fwd(L, dev(W), dev(X)))
        assert np.array_equal(got, F.conv_fwd(W, X, stride=stride, pad=pad))


def test_every_field_element_through_the_digit_planes(dk):
    """All p field elements as entries of the encoded operand, against rows of ones and of
    random field elements: a wrong digit of any element changes a sum that the oracle fixes."""
    N, R = 8192, 4096
    X = (np.arange(R * N, dtype=np.int64) % P).astype(np.uint32).reshape(R, N)
    rng = np.random.default_rng(2207)
    W = np.stack([np.ones(N, dtype=np.uint32), rng.integers(0, P, N, dtype=np.uint32),
                  rng.integers(0, 128, N).astype(np.uint32)])
    assert np.array_equal(host(dk.dkf_linear_fwd(dev(W), dev(X))), F.dense_fwd(W, X))


def test_linear_fwd_extreme_digits(dk):
    """Operands at the ends of the centred range and at digit boundaries."""
    vals = np.array([0, 1, P - 1, P // 2, P // 2 + 1, 63, 64, 65, P - 64, P - 65, 127, 128, 129, P - 127,
                     P - 128, P - 129, 8191, 8192, 8256, 8257, P - 8256, P - 8257, 1 << 21, (1 << 24) - 1],
                    dtype=np.uint32)
    X = np.tile(vals, (len(vals), 1))
    W = np.tile(vals[:, None], (1, len(vals)))
    got = host(dk.dkf_linear_fwd(dev(np.ascontiguousarray(W)), dev(X)))
    assert np.array_equal(got, F.dense_fwd(W, X))
    # long rows of the largest digit products (every digit -64) exercise the
    # int32 accumulators close to the longest k slice the plan allows
    N = 1_500_000
    v = P - 64 * (1 + 128 + 128 * 128)
    X = np.full((2, N), v, dtype=np.uint32)
    W = np.full((3, N), v, dtype=np.uint32)
    assert np.array_equal(host(dk.dkf_linear_fwd(dev(W), dev(X))), F.dense_fwd(W, X))
    # the largest single-digit elements (a lift of +-127 is one digit): products of 127^2
    for vx, vw in ((127, 127), (P - 127, 127), (P - 127, P - 127)):
        X = np.full((2, N), vx, dtype=np.uint32)
        W = np.full((3, N), vw, dtype=np.uint32)
        assert np.array_equal(host(dk.dkf_linear_fwd(dev(W), dev(X))), F.dense_fwd(W, X))


@pytest.mark.parametrize("K,G,m", [(1, 2, 33), (2, 3, 512), (4, 4, 1028), (8, 2, 1000), (16, 1, 77)])
def test_decode_verify(dk, K, G, m):
    import torch
    rng = np.random.default_rng([K, G, m, 5])
    S = K + 2
    A = rng.integers(0, P, size=(G, S, S), dtype=np.uint32)
    gamma = rng.integers(1, P, size=(G, S), dtype=np.uint32)
    Ainv, nvec, _ = F.coefficients(A, gamma)
    # consistent results: encodings of random sources with a zero phantom row
    src = rng.integers(0, P, size=(G * S, m), dtype=np.uint32)
    src.reshape(G, S, m)[:, S - 1] = 0
    ybar = np.empty_like(src)
    for g in range(G):
        ybar[g * S:(g + 1) * S] = (A[g].astype(object).T @ src[g * S:(g + 1) * S].astype(object) % P).astype(np.uint32)
    y, yq, verdict = dk.dkf_decode_verify(dev(ybar), dev(Ainv), dev(nvec), K, want_yq=True)
    want_q = F.decode(ybar, Ainv)
    assert np.array_equal(host(yq), want_q)
    assert np.array_equal(host(y), F.dequantize(want_q))
    assert np.array_equal(host(verdict), F.verify(ybar, nvec)) and not host(verdict).any()
    assert np.array_equal(want_q, src.reshape(G, S, m)[:, :K].reshape(G * K, m))
    # corrupt one element of the last group, and put a non-element into group 0
    bad = ybar.copy()
    bad[G * S - 2, m - 1] = (int(bad[G * S - 2, m - 1]) + 1) % P
    if G > 1:
        bad[1, 0] = P + 5
    _, _, verdict = dk.dkf_decode_verify(dev(bad), dev(Ainv), dev(nvec), K)
    want = F.verify(bad, nvec)
    assert np.array_equal(host(verdict), want) and want[G - 1] == 1 and (G == 1 or want[0] == 1)
    # stale verdicts are overwritten
    v = torch.full((G,), 7, dtype=torch.int32, device="cuda")
    dk.dkf_decode_verify(dev(ybar), dev(Ainv), dev(nvec), K, verdict=v)
    assert not host(v).any()


@pytest.mark.parametrize("K,G,M,N", [(2, 1, 512, 256), (4, 3, 70, 130), (8, 4, 257, 300), (1, 5, 33, 129)])
def test_masked_dense_layer(dk, K, G, M, N):
    rng = np.random.default_rng([K, G, M, N, 9])
    L = dk_inputs.linear(M, N)
    d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, delta_std=1.0)
    o = F.masked_dense_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    Wq = dk.dkf_quantize(dev(d["W"]))
    assert np.array_equal(host(Wq), o["Wq"])
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    assert np.array_equal(host(xbar), o["Xbar"])
    ybar = dk.dkf_linear_fwd(Wq, xbar)
    assert np.array_equal(host(ybar), o["Ybar"])
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    assert np.array_equal(host(yq), o["Yq"]) and np.array_equal(host(y), o["Y"])
    assert np.array_equal(host(verdict), o["verdict"])
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True)
    assert np.array_equal(host(dwq), o["dWq"]) and np.array_equal(host(dW), o["dW"])
    # scale and accumulate
    import torch
    base = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, dW=base, scale=0.25, accumulate=True)
    assert np.array_equal(host(base), (0.5 + 0.25 * o["dW"]).astype(np.float32))
    # and the decoded values are the plain integer layer (no masking, no field)
    Wi, Xi = (np.floor(a.astype(np.float64) * 256 + 0.5).astype(np.int64) for a in (d["W"], d["X"]))
    lift = host(yq).astype(np.int64)
    lift = np.where(lift > P // 2, lift - P, lift)
    assert np.array_equal(lift, Xi @ Wi.T)


@pytest.mark.parametrize("va,vb", [(-15736896, -15736896), (-15736896, 15720383), (15720383, 15720383),
                                   (127, 127), (-127, 127), (-127, 15720383)])
def test_wgrad_extreme_digit_sums(dk, va, vb):
    """Operands whose base-128 digits are all at one end (-64, -64, -64, -7 or
    63, 63, 63, 7), on every row: the digit sums of the halves reach -128 and
    126, the largest accumulator growth per term of the weight gradient; and
    the largest single-digit elements (+-127, one digit each)."""
    G, K, M, N = 700, 1, 70, 130
    S = K + 2
    L = dk_inputs.linear(M, N)
    B = np.full((G, S, K), va % P, dtype=np.uint32)        # dtilde = gamma * B * Dq with Dq = 1
    gamma = np.ones((G, S), dtype=np.uint32)
    delta = np.full((G * K, M), 1.0 / 256, dtype=np.float32)
    xbar = np.full((G * S, N), vb % P, dtype=np.uint32)
    rng = np.random.default_rng(3)
    xbar[rng.integers(0, G * S, 50), rng.integers(0, N, 50)] = rng.integers(0, P, 50, dtype=np.uint32)
    dt = F.delta_mix(F.quantize(delta), B, gamma)
    assert (dt == va % P).all()
    _, dwq = dk.dkf_wgrad(L, dev(delta), dev(B), dev(gamma), dev(xbar), K, want_dwq=True)
    assert np.array_equal(host(dwq), F.dense_wgrad(dt, xbar))


def test_config1_field(dk):
    d = dk_inputs.config1_field()
    L, K = d["layer"], d["K"]
    o = F.masked_dense_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"])
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    ybar = dk.dkf_linear_fwd(dk.dkf_quantize(dev(d["W"])), xbar)
    y, _, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K)
    dW, _ = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K)
    assert np.array_equal(host(y), o["Y"]) and np.array_equal(host(dW), o["dW"]) and not host(verdict).any()


@pytest.mark.parametrize("index", [2, 0])
def test_config5_field_sampled(dk, index):
    """Classifier layers at full size; the oracle evaluates sampled outputs of
    the two contractions and the whole of the cheap stages."""
    d = dk_inputs.config5_field(index=index)[0]
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    rng = np.random.default_rng([5, index, 99])
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    Wq_o = F.quantize(d["W"])
    xbar_o = F.encode(F.quantize(d["X"]), d["r"], d["A"])
    Wq = dk.dkf_quantize(dev(d["W"]))
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    assert np.array_equal(host(xbar), xbar_o)
    ybar = dk.dkf_linear_fwd(Wq, xbar)
    yb = host(ybar)
    pts = np.stack([rng.integers(0, G * S, 3000), rng.integers(0, L.M, 3000)], 1)
    assert np.array_equal(yb[pts[:, 0], pts[:, 1]], F.dense_fwd_points(Wq_o, xbar_o, pts))
    # decode and verify the accelerator's own ybar with the oracle: clean, and
    # the decoded values are the plain integer layer at the sampled positions
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    assert not host(verdict).any() and not F.verify(yb, nvec).any()
    assert np.array_equal(host(yq), F.decode(yb, Ainv))
    assert np.array_equal(host(y), F.dequantize(host(yq)))
    Wi = np.floor(d["W"].astype(np.float64) * 256 + 0.5).astype(np.int64)
    Xi = np.floor(d["X"].astype(np.float64) * 256 + 0.5).astype(np.int64)
    spts = np.stack([rng.integers(0, G * K, 500), rng.integers(0, L.M, 500)], 1)
    lift = host(yq).astype(np.int64)
    lift = np.where(lift > P // 2, lift - P, lift)
    assert np.array_equal(lift[spts[:, 0], spts[:, 1]], np.einsum("pk,pk->p", Xi[spts[:, 0]], Wi[spts[:, 1]]))
    # weight gradient
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True)
    dt_o = F.delta_mix(F.quantize(d["delta"]), B, d["gamma"])
    wpts = np.stack([rng.integers(0, L.M, 3000), rng.integers(0, L.N, 3000)], 1)
    got = host(dwq)
    assert np.array_equal(got[wpts[:, 0], wpts[:, 1]], F.dense_wgrad_points(dt_o, xbar_o, wpts))
    assert np.array_equal(host(dW), F.dequantize(got))


@pytest.mark.parametrize("K,G,Ci,Co,H,W,k,stride,pad", [
    (2, 1, 3, 5, 9, 7, 3, 1, 1), (4, 2, 16, 24, 12, 12, 3, 1, 1), (2, 3, 8, 130, 10, 10, 3, 2, 1),
    (8, 1, 20, 12, 7, 7, 1, 1, 0), (1, 2, 6, 9, 11, 8, 5, 2, 2), (4, 1, 64, 64, 16, 16, 3, 1, 1),
    # stride 1 with an output width that is, or nearly is, a multiple of 16
    (2, 2, 5, 7, 16, 16, 3, 1, 1), (3, 1, 6, 9, 9, 30, 3, 1, 0), (2, 1, 4, 6, 12, 16, 5, 1, 2),
    (1, 3, 3, 4, 8, 16, 3, 1, 0), (2, 1, 3, 130, 5, 32, 3, 1, 1), (2, 2, 70, 3, 6, 14, 3, 1, 1),
    # the contraction index (encoded row, output pixel) with Ho*Wo a multiple of 4: the gradient mixing
    # writes the digit planes itself (rows and k beyond the operand zeroed separately)
    (4, 2, 20, 12, 6, 6, 1, 1, 0), (2, 3, 16, 70, 8, 8, 3, 2, 1), (8, 1, 8, 130, 4, 12, 1, 1, 0),
    (16, 1, 4, 6, 4, 4, 1, 1, 0), (3, 2, 64, 128, 4, 8, 1, 1, 0),
    # a long contraction over a small result: the forward is cut into 16 or more k slices, folded by the
    # kernel that spreads the slices over the waves of a workgroup, into the image-major layout
    (2, 1, 256, 40, 4, 4, 3, 1, 1), (1, 1, 300, 7, 3, 5, 3, 1, 1)])
def test_masked_conv_layer(dk, K, G, Ci, Co, H, W, k, stride, pad):
    rng = np.random.default_rng([K, G, Ci, Co, H, k, 17])
    L = dk_inputs.conv(Ci, Co, H, W, k, stride, pad)
    d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, delta_std=1.0)
    o = F.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=stride, pad=pad)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    Wq = dk.dkf_quantize(dev(d["W"]))
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    assert np.array_equal(host(xbar), o["Xbar"])
    ybar = dk.dkf_conv_fwd(L, Wq, xbar)
    assert np.array_equal(host(ybar), o["Ybar"])
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    assert np.array_equal(host(yq), o["Yq"]) and np.array_equal(host(y), o["Y"])
    assert not host(verdict).any()
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True)
    assert np.array_equal(host(dwq), o["dWq"]) and np.array_equal(host(dW), o["dW"])
    # a corrupted encoded result is caught, in its group only
    bad = o["Ybar"].copy()
    bad.reshape(-1)[bad.size - 1] = (int(bad.reshape(-1)[-1]) + 3) % P
    _, _, verdict = dk.dkf_decode_verify(dev(bad), dev(Ainv), dev(nvec), K)
    assert host(verdict).tolist() == [0] * (G - 1) + [1]


def _random_field_conv_shapes(seed, count):
    """Seeded draw of small convolution shapes across the operand forms of the
    field contraction: channel counts that are and are not multiples of 16
    (implicit or materialised forward operand), output widths that do and do
    not take the shifted-rows weight gradient, 1x1 filters, stride 2."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k = int(rng.choice([1, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 1, 2]))
        pad = int(rng.choice([0, k // 2]))
        H = int(rng.choice([3, 5, 8, 9, 14]))
        W = int(rng.choice([4, 7, 14, 16, 18, 30, 32]))
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        Ci = int(rng.choice([1, 5, 16, 32, 40]))
        Co = int(rng.choice([1, 7, 64, 70, 130]))
        K = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2]))
        out.append((K, G, Ci, Co, H, W, k, stride, pad))
    return out


@pytest.mark.parametrize("K,G,Ci,Co,H,W,k,stride,pad", _random_field_conv_shapes(20261, 24))
def test_masked_conv_layer_random_shapes(dk, K, G, Ci, Co, H, W, k, stride, pad):
    rng = np.random.default_rng([K, G, Ci, Co, H, W, k, stride, pad])
    L = dk_inputs.conv(Ci, Co, H, W, k, stride, pad)
    d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, delta_std=1.0)
    o = F.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=stride, pad=pad)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    ybar = dk.dkf_conv_fwd(L, dk.dkf_quantize(dev(d["W"])), xbar)
    assert np.array_equal(host(ybar), o["Ybar"])
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    assert np.array_equal(host(yq), o["Yq"]) and not host(verdict).any()
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True)
    assert np.array_equal(host(dwq), o["dWq"]) and np.array_equal(host(dW), o["dW"])


def test_config2_field_sampled(dk):
    """Config 2 (conv 3x3 64->64 @32x32, batch 256, K=4) over the field at full
    size; the oracle evaluates sampled outputs of the two contractions."""
    d = dk_inputs.config2_field()
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    rng = np.random.default_rng(77)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    Wq_o = F.quantize(d["W"])
    xbar_o = F.encode(F.quantize(d["X"]), d["r"], d["A"])
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    assert np.array_equal(host(xbar), xbar_o)
    ybar = dk.dkf_conv_fwd(L, dk.dkf_quantize(dev(d["W"])), xbar)
    yb = host(ybar)
    pts = np.stack([rng.integers(0, G * S, 4000), rng.integers(0, 64, 4000), rng.integers(0, 32, 4000),
                    rng.integers(0, 32, 4000)], 1)
    pts[:8, 2:] = [[0, 0], [0, 31], [31, 0], [31, 31], [0, 5], [31, 7], [9, 0], [13, 31]]
    assert np.array_equal(yb[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], F.conv_fwd_points(Wq_o, xbar_o, pts, 1, 1))
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    assert not host(verdict).any() and not F.verify(yb, nvec).any()
    assert np.array_equal(host(yq), F.decode(yb, Ainv))
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True)
    dt_o = F.delta_mix(F.quantize(d["delta"]), B, d["gamma"])
    wpts = np.stack([rng.integers(0, 64, 300), rng.integers(0, 64, 300), rng.integers(0, 3, 300),
                     rng.integers(0, 3, 300)], 1)
    got = host(dwq)
    assert np.array_equal(got[wpts[:, 0], wpts[:, 1], wpts[:, 2], wpts[:, 3]],
                          F.conv_wgrad_points(dt_o, xbar_o, 3, 3, wpts, 1, 1))
    assert np.array_equal(host(dW), F.dequantize(got))


@pytest.mark.parametrize("cfg,index", [(3, 3), (3, 8), (4, 11), (4, 13), (4, 16)])
def test_config34_field_layers_sampled(dk, cfg, index):
    """Layers of configs 3 and 4 with more than 64 output channels over the field at full size
    (3x3 at 16x16 and 4x4, 3x3 stride 2, 1x1 256->1024 and 1024->512): the He-initialised
    filters fit one digit plane, so their forward takes the one-plane steps of the contraction,
    except those of the 1x1 256->1024 layer (smallest fan-in: a few weights lie beyond 63/256),
    which takes two planes.
    The oracle evaluates sampled outputs of the two contractions."""
    d = dk_inputs.config3_field(index=index) if cfg == 3 else dk_inputs.config4_field(index=index)[0]
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    rng = np.random.default_rng([cfg, index, 5])
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    Wq_o = F.quantize(d["W"])
    lifted = np.where(Wq_o > P // 2, Wq_o.astype(np.int64) - P, Wq_o.astype(np.int64))
    assert L.Co > 64 and (lifted.min() >= -64 and lifted.max() <= 63) == (index != 13)
    xbar_o = F.encode(F.quantize(d["X"]), d["r"], d["A"])
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    assert np.array_equal(host(xbar), xbar_o)
    ybar = dk.dkf_conv_fwd(L, dk.dkf_quantize(dev(d["W"])), xbar)
    yb = host(ybar)
    n = 3000
    pts = np.stack([rng.integers(0, G * S, n), rng.integers(0, L.Co, n), rng.integers(0, L.Ho, n),
                    rng.integers(0, L.Wo, n)], 1)
    pts[:4, 2:] = [[0, 0], [0, L.Wo - 1], [L.Ho - 1, 0], [L.Ho - 1, L.Wo - 1]]
    pts[:4, :2] = [[0, 0], [G * S - 1, L.Co - 1], [0, L.Co - 1], [G * S - 1, 0]]
    assert np.array_equal(yb[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]],
                          F.conv_fwd_points(Wq_o, xbar_o, pts, L.stride, L.pad))
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    assert not host(verdict).any() and not F.verify(yb, nvec).any()
    assert np.array_equal(host(yq), F.decode(yb, Ainv))
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True)
    dt_o = F.delta_mix(F.quantize(d["delta"]), B, d["gamma"])
    m = 200
    wpts = np.stack([rng.integers(0, L.Co, m), rng.integers(0, L.Ci, m), rng.integers(0, L.kh, m),
                     rng.integers(0, L.kw, m)], 1)
    got = host(dwq)
    assert np.array_equal(got[wpts[:, 0], wpts[:, 1], wpts[:, 2], wpts[:, 3]],
                          F.conv_wgrad_points(dt_o, xbar_o, L.kh, L.kw, wpts, L.stride, L.pad))
    assert np.array_equal(host(dW), F.dequantize(got))


def test_field_arguments_refused(dk):
    import torch
    from paper_2207_00083_amd import DkError
    W = torch.zeros((8, 8), dtype=torch.int32, device="cuda")
    X = torch.zeros((4, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(DkError) as e:
        dk.dkf_linear_fwd(W, X, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 5
    with pytest.raises(DkError) as e:
        dk.dkf_quantize(torch.zeros(4, device="cuda"), l=13)
    assert e.value.status == 2
    conv = dk_inputs.conv(4, 4, 8, 8, 3)
    assert dk.dkf_wgrad_workspace_bytes(conv, 1, 2) > 0 and dk.dkf_conv_fwd_workspace_bytes(conv, 4) > 0
    assert dk.dkf_conv_fwd_workspace_bytes(dk_inputs.linear(4, 4), 4) == 0


@pytest.mark.parametrize("M,N,R,l", [(40, 200, 12, 8), (130, 515, 7, 8), (64, 4096, 20, 3), (16, 33, 5, 12)])
def test_linear_forward_from_real_weights(dk, M, N, R, l):
    """dkf_linear_fwd_w = dkf_quantize + dkf_linear_fwd, bit for bit, and the oracle's product."""
    rng = np.random.default_rng([M, N, R, l])
    W = rng.normal(0, 0.7, size=(M, N)).astype(np.float32)
    W[0, 0] = 2.0 ** -(l + 1)                      # a tie of Round
    W[M - 1, N - 1] = -3.5 * 2.0 ** -l
    xbar = rng.integers(0, F.P, size=(R, N), dtype=np.uint32)
    got = host(dk.dkf_linear_fwd_w(dev(W), dev(xbar), l=l))
    two = host(dk.dkf_linear_fwd(dk.dkf_quantize(dev(W), l=l), dev(xbar)))
    assert np.array_equal(got, two)
    assert np.array_equal(got, F.dense_fwd(F.quantize(W, l=l), xbar))


def test_matrix_rate_probe_runs(dk):
    import torch
    for kind in (0, 1, 2):
        ops = dk.dkf_probe_mfma_rate(kind, 50)
        assert ops == 256 * 4 * 50 * 16 * 65536.0
    torch.cuda.synchronize()
