"""GPU parity of the finite-field entry points for several colluding
accelerators (M noise vectors per group over F_p, S = K + M + 1) against the
field oracle, through the C ABI.  All arithmetic is modulo p: every comparison
is exact, the float outputs included."""
import sys

import numpy as np
import pytest

import dk_inputs
from oracle import field as F

pytestmark = pytest.mark.gpu

P = F.P


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


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
    torch.cuda.synchronize()
    a = t.cpu().numpy()
    return a.view(np.uint32) if a.dtype == np.int32 else a


CASES = [
    # K, M, G, layer
    (1, 2, 3, dk_inputs.linear(40, 50)),
    (2, 2, 2, dk_inputs.linear(130, 257)),
    (4, 3, 2, dk_inputs.linear(64, 1027)),               # ragged rows: scalar path
    (8, 2, 2, dk_inputs.linear(100, 300)),
    (3, 14, 1, dk_inputs.linear(20, 36)),                # K + M - 1 = 16, the limit
    (15, 2, 1, dk_inputs.linear(20, 36)),
    (2, 2, 2, dk_inputs.conv(8, 16, 12, 12, 3)),
    (4, 2, 2, dk_inputs.conv(16, 24, 8, 8, 1, 1, 0)),
    (2, 3, 2, dk_inputs.conv(6, 10, 9, 7, 3, 2, 1)),
]


@pytest.mark.parametrize("K,M,G,L", CASES)
def test_whole_layer_with_m_noise_vectors(dk, K, M, G, L):
    say("field layer, M noise vectors", dict(K=K, M=M, G=G), L)
    d = dk_inputs.field_collusion_layer_inputs(np.random.default_rng([K, M, G, 11]), L, K=K, M=M,
                                               batch=G * K, delta_std=1.0)
    o = F.masked_layer_m(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], K, stride=L.stride, pad=L.pad)
    Ainv, nvec, B = dk.dkf_coeffs_m(d["A"], d["gamma"], K)
    for got, want in zip((Ainv, nvec, B), F.coefficients_m(d["A"], d["gamma"], K)):
        assert np.array_equal(got, want)
    xbar = dk.dkf_encode_m(dev(d["X"]), dev(d["r"]), dev(d["A"]), K, M)
    assert np.array_equal(host(xbar), o["Xbar"])
    Wq = dk.dkf_quantize(dev(d["W"]))
    ybar = dk.dkf_linear_fwd(Wq, xbar) if L.kind == "linear" else dk.dkf_conv_fwd(L, Wq, xbar)
    assert np.array_equal(host(ybar), o["Ybar"])
    y, yq, verdict = dk.dkf_decode_verify_m(ybar, dev(Ainv), dev(nvec), K, M, want_yq=True)
    assert np.array_equal(host(yq), o["Yq"])
    assert np.array_equal(host(y), o["Y"])
    assert host(verdict).tolist() == [0] * G
    dW, dwq = dk.dkf_wgrad_m(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, M, want_dwq=True)
    assert np.array_equal(host(dwq), o["dWq"])
    assert np.array_equal(host(dW), o["dW"])
    # one changed element of the results of group G-1 is flagged, and only there
    bad = o["Ybar"].copy().reshape(G * (K + M + 1), -1)
    j = int(np.argmax(nvec[G - 1] != 0))
    bad[(G - 1) * (K + M + 1) + j, 3] = (int(bad[(G - 1) * (K + M + 1) + j, 3]) + 1) % P
    _, _, v2 = dk.dkf_decode_verify_m(dev(bad.reshape(o["Ybar"].shape)), dev(Ainv), dev(nvec), K, M)
    assert host(v2).tolist() == F.verify_m(bad, nvec).tolist() == [0] * (G - 1) + [1]


def test_one_noise_vector_equals_the_plain_entry_points(dk):
    K, G = 4, 3
    L = dk_inputs.linear(70, 260)
    d = dk_inputs.field_layer_inputs(np.random.default_rng(5), L, K=K, batch=G * K)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    for a, b in zip((Ainv, nvec, B), dk.dkf_coeffs_m(d["A"], d["gamma"], K)):
        assert np.array_equal(a, b)
    x1 = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    x2 = dk.dkf_encode_m(dev(d["X"]), dev(d["r"]), dev(d["A"]), K, 1)
    assert np.array_equal(host(x1), host(x2))
    ybar = dk.dkf_linear_fwd(dk.dkf_quantize(dev(d["W"])), x1)
    a = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    b = dk.dkf_decode_verify_m(ybar, dev(Ainv), dev(nvec), K, 1, want_yq=True)
    for u, v in zip(a, b):
        assert np.array_equal(host(u), host(v))
    a = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), x1, K, want_dwq=True)
    b = dk.dkf_wgrad_m(L, dev(d["delta"]), dev(B), dev(d["gamma"]), x1, K, 1, want_dwq=True)
    for u, v in zip(a, b):
        assert np.array_equal(host(u), host(v))
