"""GPU parity, bit for bit, of the finite-field depthwise layers and of the
quantised bias against the field oracle, through the C ABI."""
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


DW = [(2, 3, dk_inputs.dwconv(12, 16, 16, 3)), (4, 2, dk_inputs.dwconv(24, 15, 13, 3, 2)),
      (1, 2, dk_inputs.dwconv(8, 7, 7, 5, 1, 2)), (8, 1, dk_inputs.dwconv(6, 9, 9, 7, 2, 3)),
      (2, 40, dk_inputs.dwconv(3, 20, 20, 3)), (2, 2, dk_inputs.dwconv(300, 4, 4, 3)),
      # rows of 4 n outputs (four per thread): stride 2, 5x5, 7x7, one strip per row, a single row
      (2, 3, dk_inputs.dwconv(10, 16, 16, 3, 2, 1)), (4, 1, dk_inputs.dwconv(5, 12, 12, 5, 1, 2)),
      (2, 2, dk_inputs.dwconv(4, 16, 16, 7, 2, 3)), (2, 2, dk_inputs.dwconv(7, 8, 8, 5, 2, 2)),
      (2, 2, dk_inputs.dwconv(3, 1, 4, 3, 1, 1)), (1, 2, dk_inputs.dwconv(2, 40, 36, 3, 1, 1))]


@pytest.mark.parametrize("K,G,L", DW)
def test_depthwise_layer_over_the_field(dk, K, G, L):
    say("field depthwise layer", dict(K=K, G=G), L)
    d = dk_inputs.field_layer_inputs(np.random.default_rng([K, G, L.Ci, L.H, L.kh]), L, K=K, batch=G * K,
                                     delta_std=1.0)
    o = F.masked_dw_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=L.stride, pad=L.pad)
    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    xbar = dk.dkf_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    ybar = dk.dkf_conv_fwd(L, dk.dkf_quantize(dev(d["W"])), xbar)
    assert np.array_equal(host(ybar), o["Ybar"])
    y, yq, verdict = dk.dkf_decode_verify(ybar, dev(Ainv), dev(nvec), K, want_yq=True)
    assert np.array_equal(host(yq), o["Yq"]) and np.array_equal(host(y), o["Y"])
    assert host(verdict).tolist() == [0] * G
    dW, dwq = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, want_dwq=True)
    assert np.array_equal(host(dwq), o["dWq"])
    assert np.array_equal(host(dW), o["dW"])
    # accumulate with a scale on top
    dW2, _ = dk.dkf_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, dW=dW.clone(), scale=0.5,
                          accumulate=True)
    assert np.array_equal(host(dW2), (o["dW"] + np.float32(0.5) * o["dW"]).astype(np.float32))


def test_depthwise_with_non_field_entries_is_flagged(dk):
    K, G = 2, 2
    L = dk_inputs.dwconv(4, 6, 6, 3)
    d = dk_inputs.field_layer_inputs(np.random.default_rng(9), L, K=K, batch=G * K)
    o = F.masked_dw_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=1, pad=1)
    _, nvec, _ = dk.dkf_coeffs(d["A"], d["gamma"])
    bad = o["Ybar"].copy()
    bad[5, 1, 2, 3] = (int(bad[5, 1, 2, 3]) + 7) % P
    Ainv = F.coefficients(d["A"], d["gamma"])[0]
    _, _, v = dk.dkf_decode_verify(dev(bad), dev(Ainv), dev(nvec), K)
    assert host(v).tolist() == F.verify(bad, nvec).tolist() == [0, 1]


@pytest.mark.parametrize("rows,m,per,l", [(4, 37, 1, 8), (6, 8 * 25, 25, 8), (3, 1000, 1, 3), (2, 64, 64, 12)])
def test_bias_over_the_field(dk, rows, m, per, l):
    rng = np.random.default_rng([rows, m, per, l])
    yq = rng.integers(0, P, size=(rows, m), dtype=np.uint32)
    bias = rng.normal(0, 3, size=m // per).astype(np.float32)
    bias[0] = -0.5 * 2.0 ** (-2 * l)                     # a tie of Round
    want = F.add_bias(yq, bias, per, l=l)
    got_q, got_y = dk.dkf_add_bias(dev(yq), dev(bias), per, l=l)
    assert np.array_equal(host(got_q), want)
    assert np.array_equal(host(got_y), F.dequantize(want, l=l))
