"""GPU parity of the dynamic normalisation of the finite-field variant (section
"Privacy Guarantee", paragraph "Quantization") against the field oracle,
through the C ABI.  Factors, field values and float outputs are all defined
bit for bit, so every comparison is exact."""
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
    a = t.cpu().numpy()
    return a.view(np.uint32) if a.dtype == np.int32 else a


def same_bits(a, b):
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def wild(rng, rows, n):
    """Rows of very different magnitudes, some inside the limit, with the
    special values the maximum has to cope with."""
    x = rng.standard_normal((rows, n)) * 10.0 ** rng.integers(-3, 6, size=(rows, 1))
    return x.astype(np.float32)


@pytest.mark.parametrize("rows,n", [(1, 1), (3, 17), (8, 1024), (5, 4100), (2, 300001), (300, 129)])
def test_norm_scales(dk, rows, n):
    rng = np.random.default_rng([rows, n])
    x = wild(rng, rows, n)
    if n >= 17:
        x[0, 3] = np.nan
        x[rows - 1, n - 1] = -np.abs(x[rows - 1]).max() * 2      # the maximum in the ragged tail
    if rows >= 3 and n >= 17:
        x[1, 5] = np.inf
        x[2, :] = 0.0
    for limit in (1.0, 50.0):
        got = host(dk.dkf_norm_scales(dev(x), limit))
        assert same_bits(got, F.norm_scales(x, limit)), limit
    # the buffer is reused: a second call must not see the first call's values
    import torch
    s = torch.full((rows,), 7.0, dtype=torch.float32, device="cuda")
    dk.dkf_norm_scales(dev(x), 1.0, scale=s)
    dk.dkf_norm_scales(dev(x * np.float32(0.5)), 1.0, scale=s)
    assert same_bits(host(s), F.norm_scales(x * np.float32(0.5), 1.0))


def test_norm_scales_of_a_weight_tensor_and_off_alignment(dk):
    import torch
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((6, 5, 3, 3)) * 20).astype(np.float32)
    got = host(dk.dkf_norm_scales(dev(W), 1.0, rows=1))
    assert same_bits(got, F.norm_scales(W.reshape(1, -1), 1.0))
    # a base 4 bytes past a 16-byte boundary takes the scalar path
    buf = torch.zeros(4 * 1024 + 1, dtype=torch.float32, device="cuda")
    x = wild(rng, 4, 1024)
    buf[1:].copy_(dev(x).reshape(-1))
    got = host(dk.dkf_norm_scales(buf[1:].view(4, 1024), 1.0))
    assert same_bits(got, F.norm_scales(x, 1.0))


@pytest.mark.parametrize("rows,n,l", [(1, 1003, 8), (4, 1024, 8), (7, 333, 0), (3, 4100, 12)])
def test_quantize_norm(dk, rows, n, l):
    rng = np.random.default_rng([rows, n, l, 1])
    x = wild(rng, rows, n)
    x[0, :4] = [1e30, -1e30, np.nan, 0.0]
    s = F.norm_scales(x, 1.0)
    got = host(dk.dkf_quantize(dev(x), l=l, scale=dev(s)))
    assert np.array_equal(got, F.quantize_scaled(x, s, l))
    # factors of 1 reproduce the plain call
    one = np.ones(rows, dtype=np.float32)
    assert np.array_equal(host(dk.dkf_quantize(dev(x), l=l, scale=dev(one))), F.quantize(x, l=l))


@pytest.mark.parametrize("K,G,n", [(1, 3, 17), (2, 2, 1024), (4, 5, 4100), (8, 3, 2051), (16, 2, 260)])
def test_encode_norm(dk, K, G, n):
    rng = np.random.default_rng([K, G, n, 2])
    d = dk_inputs.field_layer_inputs(rng, dk_inputs.linear(3, n), K=K, batch=G * K)
    X = (d["X"] * 10.0 ** rng.integers(-1, 4, size=(G * K, 1))).astype(np.float32)
    s = F.norm_scales(X, 4.0)
    assert (s < 1).any()
    want = F.encode(F.quantize_scaled(X, s), d["r"], d["A"])
    got = host(dk.dkf_encode(dev(X), dev(d["r"]), dev(d["A"]), K, xscale=dev(s)))
    assert np.array_equal(got, want)
    # noise from the seed: the same encodings as with the noise rows in memory
    r = dk.dkf_noise_rng(G, n, 99)
    got = host(dk.dkf_encode_rng(dev(X), dev(d["A"]), K, 99, xscale=dev(s)))
    assert np.array_equal(got, F.encode(F.quantize_scaled(X, s), host(r), d["A"]))


@pytest.mark.parametrize("K,G,M,N", [(2, 1, 512, 256), (4, 3, 70, 130), (8, 4, 257, 300), (1, 5, 33, 129)])
def test_masked_dense_layer_normalised(dk, K, G, M, N):
    rng = np.random.default_rng([K, G, M, N, 19])
    L = dk_inputs.linear(M, N)
    d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, w_std=30.0, delta_std=1e-3)
    X = (d["X"] * 10.0 ** rng.integers(-1, 4, size=(G * K, 1))).astype(np.float32)
    o = F.masked_layer_normalized(d["W"], X, d["r"], d["delta"], d["A"], d["gamma"], limit=1.0)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    xs = dk.dkf_norm_scales(dev(X), 1.0)
    ws = dk.dkf_norm_scales(dev(d["W"]), 1.0, rows=1)
    assert same_bits(host(xs), o["xscale"]) and same_bits(host(ws), o["wscale"])
    Wq = dk.dkf_quantize(dev(d["W"]), scale=ws)
    assert np.array_equal(host(Wq), o["Wq"])
    xbar = dk.dkf_encode(dev(X), dev(d["r"]), dev(d["A"]), K, xscale=xs)
    assert np.array_equal(host(xbar), o["Xbar"])
    ybar = dk.dkf_linear_fwd(Wq, xbar)
    assert np.array_equal(host(ybar), o["Ybar"])
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True, xscale=xs, wscale=ws)
    assert np.array_equal(host(yq), o["Yq"]) and same_bits(host(y), o["Y"])
    assert not host(verdict).any()
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True, xscale=xs)
    assert np.array_equal(host(dwq), o["dWq"]) and same_bits(host(dW), o["dW"])
    # and the result is the real layer, which the plain field path cannot give here
    Y = X.astype(np.float64) @ d["W"].astype(np.float64).T
    rel = np.abs(host(y) - Y).max() / np.abs(Y).max()
    assert rel < 0.05


@pytest.mark.parametrize("K,G,Ci,Co,H,W,k,stride,pad", [
    (2, 1, 3, 5, 9, 7, 3, 1, 1), (4, 2, 16, 24, 12, 12, 3, 1, 1), (8, 1, 20, 12, 7, 7, 1, 1, 0),
    (1, 2, 6, 9, 11, 8, 5, 2, 2), (4, 2, 20, 12, 6, 6, 1, 1, 0), (2, 1, 8, 10, 6, 16, 3, 1, 1),
    (2, 2, 5, 7, 5, 30, 3, 1, 0)])
def test_masked_conv_layer_normalised(dk, K, G, Ci, Co, H, W, k, stride, pad):
    rng = np.random.default_rng([K, G, Ci, Co, H, k, 23])
    L = dk_inputs.conv(Ci, Co, H, W, k, stride, pad)
    d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, w_std=5.0, delta_std=1e-2)
    X = (d["X"] * 10.0 ** rng.integers(-1, 3, size=(G * K, 1, 1, 1))).astype(np.float32)
    o = F.masked_layer_normalized(d["W"], X, d["r"], d["delta"], d["A"], d["gamma"], limit=2.0,
                                  stride=stride, pad=pad)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    xs = dk.dkf_norm_scales(dev(X), 2.0)
    ws = dk.dkf_norm_scales(dev(d["W"]), 2.0, rows=1)
    assert same_bits(host(xs), o["xscale"]) and same_bits(host(ws), o["wscale"])
    Wq = dk.dkf_quantize(dev(d["W"]), scale=ws)
    xbar = dk.dkf_encode(dev(X), dev(d["r"]), dev(d["A"]), K, xscale=xs)
    assert np.array_equal(host(Wq), o["Wq"]) and np.array_equal(host(xbar), o["Xbar"])
    ybar = dk.dkf_conv_fwd(L, Wq, xbar)
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True, xscale=xs, wscale=ws)
    assert np.array_equal(host(yq), o["Yq"]) and same_bits(host(y), o["Y"])
    assert not host(verdict).any()
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True, xscale=xs)
    assert np.array_equal(host(dwq), o["dWq"]) and same_bits(host(dW), o["dW"])


def test_factors_of_one_reproduce_the_plain_calls(dk):
    import torch
    rng = np.random.default_rng(41)
    K, G, M, N = 4, 2, 40, 96
    L = dk_inputs.linear(M, N)
    d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, delta_std=1.0)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    xs = dk.dkf_norm_scales(dev(d["X"]), 1e6)
    ws = dk.dkf_norm_scales(dev(d["W"]), 1e6, rows=1)
    assert (host(xs) == 1).all() and (host(ws) == 1).all()
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    assert torch.equal(xbar, dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K, xscale=xs))
    ybar = dk.dkf_linear_fwd(dk.dkf_quantize(dev(d["W"])), xbar)
    y0, _, _ = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K)
    y1, _, _ = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, xscale=xs, wscale=ws)
    assert torch.equal(y0, y1)
    w0, _ = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K)
    w1, _ = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, xscale=xs)
    assert torch.equal(w0, w1)


def test_config3_first_layer_normalised_sampled(dk):
    """A VGG-16 convolution (the network the paper normalises dynamically) at
    its full shape, raw-pixel-like inputs in [0, 255]; the oracle evaluates the
    bandwidth-bound steps in full and sampled outputs of the contraction."""
    d = dk_inputs.config3_field(index=0)
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    rng = np.random.default_rng(78)
    X = np.abs(d["X"] * 64.0).clip(0, 255).astype(np.float32)
    xs_o = F.norm_scales(X, 1.0)
    ws_o = F.norm_scales(d["W"].reshape(1, -1), 1.0)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    xs = dk.dkf_norm_scales(dev(X), 1.0)
    ws = dk.dkf_norm_scales(dev(d["W"]), 1.0, rows=1)
    assert same_bits(host(xs), xs_o) and same_bits(host(ws), ws_o)
    Wq_o = F.quantize_scaled(d["W"].reshape(1, -1), ws_o).reshape(d["W"].shape)
    xbar_o = F.encode(F.quantize_scaled(X, xs_o), d["r"], d["A"])
    xbar = dk.dkf_encode(dev(X), dev(d["r"]), dev(d["A"]), K, xscale=xs)
    assert np.array_equal(host(xbar), xbar_o)
    ybar = dk.dkf_conv_fwd(L, dk.dkf_quantize(dev(d["W"]), scale=ws), xbar)
    yb = host(ybar)
    Co, Ho, Wo = yb.shape[1:]
    n = 2000
    pts = np.stack([rng.integers(0, G * S, n), rng.integers(0, Co, n), rng.integers(0, Ho, n),
                    rng.integers(0, Wo, n)], 1)
    assert np.array_equal(yb[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]],
                          F.conv_fwd_points(Wq_o, xbar_o, pts, L.stride, L.pad))
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True, xscale=xs, wscale=ws)
    assert not host(verdict).any()
    yq_o = F.decode(yb, Ainv)
    assert np.array_equal(host(yq), yq_o)
    assert same_bits(host(y), F.unscale(F.dequantize(yq_o), xs_o, ws_o[0]))


def test_norm_arguments_refused(dk):
    import torch
    from paper_2207_00083_amd import DkError
    x = torch.zeros((4, 8), device="cuda")
    for limit in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(DkError) as e:
            dk.dkf_norm_scales(x, limit)
        assert e.value.status == 2
    with pytest.raises(ValueError):
        dk.dkf_norm_scales(x, 1.0, rows=3)
    with pytest.raises(ValueError):
        dk.dkf_quantize(x, scale=torch.ones(3, device="cuda"))
