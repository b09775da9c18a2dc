"""GPU parity of the un-encoded data gradient against the fp64 oracle."""
import numpy as np
import pytest

import dk_inputs
import oracle
from conftest import normwise_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dk():
    import torch
    import paper_2207_00083_amd as m
    m.load()
    assert torch.cuda.is_available()
    return m


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


@pytest.mark.parametrize("R,M,N", [(5, 7, 9), (130, 200, 300), (64, 512, 256), (33, 129, 1027)])
def test_dense_dgrad(dk, R, M, N):
    rng = np.random.default_rng([R, M, N])
    W = rng.normal(size=(M, N)).astype(np.float32)
    D = rng.normal(size=(R, M)).astype(np.float32)
    dx = dk.dk_dgrad(dk_inputs.linear(M, N), dev(W), dev(D))
    assert normwise_err(dx.cpu().numpy(), oracle.dense_dgrad(D, W)) < 1e-5


CONVS = [dk_inputs.conv(16, 24, 12, 12, 3), dk_inputs.conv(64, 64, 16, 16, 3), dk_inputs.conv(8, 130, 10, 10, 3, 2, 1),
         dk_inputs.conv(20, 12, 7, 7, 1), dk_inputs.conv(6, 9, 11, 8, 5, 2, 2), dk_inputs.conv(24, 40, 14, 14, 1, 2, 0),
         dk_inputs.conv(5, 7, 9, 9, 3, 1, 0), dk_inputs.conv(12, 16, 8, 8, 5, 1, 2),
         # strided: one dense sub-convolution per residue class of input pixels
         dk_inputs.conv(70, 130, 15, 13, 3, 2, 1), dk_inputs.conv(16, 24, 14, 14, 3, 2, 0),
         dk_inputs.conv(12, 20, 11, 16, 2, 2, 0), dk_inputs.conv(9, 8, 13, 10, 3, 3, 1),
         dk_inputs.conv(6, 10, 12, 12, 5, 3, 2), dk_inputs.conv(8, 8, 9, 9, 1, 3, 0),
         dk_inputs.conv(3, 16, 30, 30, 7, 2, 3), dk_inputs.conv(130, 64, 8, 8, 1, 2, 0),
         dk_inputs.conv(4, 6, 5, 5, 2, 3, 0)]


@pytest.mark.parametrize("L", CONVS)
def test_conv_dgrad(dk, L):
    rng = np.random.default_rng([L.Ci, L.Co, L.H, L.kh, L.stride])
    R = 6
    W = rng.normal(size=L.w_shape).astype(np.float32)
    D = rng.normal(size=(R,) + L.out_shape).astype(np.float32)
    dx = dk.dk_dgrad(L, dev(W), dev(D))
    assert tuple(dx.shape) == (R,) + L.in_shape
    assert normwise_err(dx.cpu().numpy(), oracle.conv_dgrad(D, W, L.H, L.W, L.stride, L.pad)) < 1e-5


@pytest.mark.parametrize("L", [dk_inputs.dwconv(32, 16, 16, 3), dk_inputs.dwconv(24, 15, 13, 3, 2),
                               dk_inputs.dwconv(8, 7, 7, 5, 1, 2)])
def test_depthwise_dgrad(dk, L):
    rng = np.random.default_rng([L.Ci, L.H, L.stride, 2])
    R = 5
    W = rng.normal(size=L.w_shape).astype(np.float32)
    D = rng.normal(size=(R,) + L.out_shape).astype(np.float32)
    dx = dk.dk_dgrad(L, dev(W), dev(D))
    assert normwise_err(dx.cpu().numpy(), oracle.dwconv_dgrad(D, W, L.H, L.W, L.stride, L.pad)) < 1e-5


def _random_dgrad_convs(seed, count):
    """Seeded draw of convolution shapes for the data gradient: stride-1
    shapes run as a forward convolution with flipped filters, the rest on the
    gather loaders; widths and channel counts on both sides of the tile sizes."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k = int(rng.choice([1, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 2]))
        pad = int(rng.choice([0, k // 2]))
        H = int(rng.choice([2, 4, 7, 8, 14, 16]))
        W = int(rng.choice([2, 4, 7, 8, 14, 16, 32]))
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        out.append(dk_inputs.conv(int(rng.choice([1, 3, 16, 24, 70])), int(rng.choice([1, 8, 33, 64, 130])),
                                  H, W, k, stride, pad))
    return out


@pytest.mark.parametrize("L", _random_dgrad_convs(20264, 24))
def test_conv_dgrad_random_shapes(dk, L):
    rng = np.random.default_rng([L.Ci, L.Co, L.H, L.W, L.kh, L.stride, L.pad])
    R = int(rng.choice([1, 3, 10]))
    W = rng.normal(size=L.w_shape).astype(np.float32)
    D = rng.normal(size=(R,) + L.out_shape).astype(np.float32)
    dx = dk.dk_dgrad(L, dev(W), dev(D))
    assert tuple(dx.shape) == (R,) + L.in_shape
    assert normwise_err(dx.cpu().numpy(), oracle.conv_dgrad(D, W, L.H, L.W, L.stride, L.pad)) < 1e-5
