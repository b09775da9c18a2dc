"""Parity at the workloads' full sizes and through every aggregation path.

  * every layer shape of the VGG-16 stack (13), of the ResNet-50 bottlenecks
    (22 distinct shapes) and of the VGG classifier (3), at the batch sizes and
    K the workloads name, on sampled outputs the oracle evaluates one by one
    from the plain definitions;
  * `accumulate=1` with `scale != 1` -- the sum over virtual batches of the
    parameter-update algorithm -- through every kernel that folds partial
    sums into dW: two calls on two independent batches against the oracle's
    sum;
  * a layer whose weight-gradient plan needs more than 64 KB of LDS in the
    4-byte-read kernel, run before and after a layer of the 16-byte-read
    kernel in the same process.

Tolerance: 1e-3 normwise on decoded outputs and gradients, verdicts exact.
"""
import sys

import numpy as np
import pytest

import dk_inputs
import oracle
from conftest import normwise_err as nerr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL_CONTRACT = 1e-3


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dk():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    import paper_2207_00083_amd as dk
    dk.load()
    return dk


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def _run_masked(dk, d, corrupt=None, scale=1.0):
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    Ainv, nvec, B = dk.dk_coeffs(d["A"], d["gamma"])
    xbar = dk.dk_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    W = dev(d["W"])
    ybar = dk.dk_linear_fwd(W, xbar) if L.kind == "linear" else dk.dk_conv_fwd(L, W, xbar)
    if corrupt:
        flat = ybar.view(G * S, -1)
        for g, j, e, eta in corrupt:
            flat[g * S + j, e] += eta
    y, verdict, resid = dk.dk_decode_verify(ybar, dev(Ainv), dev(nvec), K, tol=1e-3)
    dW = dk.dk_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, scale=scale)
    out = dict(verdict=host(verdict), resid=host(resid), y=host(y), dW=host(dW), nvec=nvec)
    del xbar, ybar, y, dW, W
    torch.cuda.empty_cache()
    return out


def _sampled_conv_check(dk, d, npts, nw, seed):
    L, K, G = d["layer"], d["K"], d["G"]
    out = _run_masked(dk, d)
    rng = np.random.default_rng(seed)
    pts = np.stack([rng.integers(G * K, size=npts), rng.integers(L.Co, size=npts),
                    rng.integers(L.Ho, size=npts), rng.integers(L.Wo, size=npts)], axis=1)
    # image borders, first and last sample, first and last channel are always among the samples
    pts[:50, 2] = 0; pts[50:100, 2] = L.Ho - 1; pts[100:150, 3] = 0; pts[150:200, 3] = L.Wo - 1
    pts[200:225, 0] = 0; pts[225:250, 0] = G * K - 1; pts[250:275, 1] = 0; pts[275:300, 1] = L.Co - 1
    ref = oracle.conv_fwd_points(d["W"], d["X"], pts, L.stride, L.pad)
    got = out["y"][tuple(pts.T)]
    assert np.max(np.abs(got - ref)) / float(np.max(np.abs(out["y"]))) < TOL_CONTRACT
    wpts = np.stack([rng.integers(L.Co, size=nw), rng.integers(L.Ci, size=nw),
                     rng.integers(L.kh, size=nw), rng.integers(L.kw, size=nw)], axis=1)
    wpts[:20, 0] = 0; wpts[20:40, 0] = L.Co - 1; wpts[40:60, 1] = 0; wpts[60:80, 1] = L.Ci - 1
    wref = oracle.conv_wgrad_points(d["delta"], d["X"], L.kh, L.kw, wpts, L.stride, L.pad)
    wgot = out["dW"][tuple(wpts.T)]
    assert np.max(np.abs(wgot - wref)) / float(np.max(np.abs(out["dW"]))) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G
    assert out["resid"].max() < 1e-4


@pytest.mark.parametrize("index", range(len(dk_inputs.VGG16_CONVS)))
def test_config3_every_layer_full_size_sampled(dk, index):
    d = dk_inputs.config3(index=index)[0]
    say("config 3 layer", index, d["layer"], "batch 128, K=4")
    _sampled_conv_check(dk, d, npts=12000, nw=3000, seed=300 + index)


@pytest.mark.parametrize("index", range(len(dk_inputs.resnet50_convs())))
def test_config4_every_shape_full_size_sampled(dk, index):
    (d, count), = list(dk_inputs.config4(index=index))
    say("config 4 shape", index, d["layer"], "x%d, batch 64, K=8" % count)
    _sampled_conv_check(dk, d, npts=6000, nw=1500, seed=400 + index)


def test_config5_first_layer_full_size_sampled(dk):
    """The longest contraction of the five workloads (25088) in fp32: decoded
    outputs and gradient on 2*10^4 sampled points each, one corrupted element
    in groups 0 and 64 ("one per 64 groups"), verdicts exact."""
    say("config 5 layer 1 (dense 25088->4096, batch 1024, K=8), sampled outputs, 2 corrupted groups")
    d = dk_inputs.config5(index=0)[0]
    L, K, G = d["layer"], d["K"], d["G"]
    nv = dk.dk_coeffs(d["A"], d["gamma"])[1]
    corrupt = []
    for g in (0, 64):
        j = int(np.argmax(np.abs(nv[g])))
        corrupt.append((g, j, 1000 + 17 * g, 200.0))
    out = _run_masked(dk, d, corrupt=corrupt)
    expect = np.zeros(G, dtype=np.int32)
    expect[[0, 64]] = 1
    assert out["verdict"].tolist() == expect.tolist()
    assert out["resid"][expect == 0].max() < 1e-4
    assert out["resid"][expect == 1].min() > 1e-2
    rng = np.random.default_rng(50)
    npts = 20000
    clean_rows = np.array([s for s in range(G * K) if s // K not in (0, 64)])
    pts = np.stack([rng.choice(clean_rows, size=npts), rng.integers(L.M, size=npts)], axis=1)
    pts[:40, 1] = 0; pts[40:80, 1] = L.M - 1
    ref = oracle.dense_fwd_points(d["W"], d["X"], pts)
    got = out["y"][tuple(pts.T)]
    assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) < TOL_CONTRACT
    wpts = np.stack([rng.integers(L.M, size=npts), rng.integers(L.N, size=npts)], axis=1)
    wpts[:40, 1] = 0; wpts[40:80, 1] = L.N - 1; wpts[80:120, 0] = 0; wpts[120:160, 0] = L.M - 1
    wref = oracle.dense_wgrad_points(d["delta"], d["X"], wpts)
    wgot = out["dW"][tuple(wpts.T)]
    assert np.max(np.abs(wgot - wref)) / np.max(np.abs(wref)) < TOL_CONTRACT


# ----------------------------------------------------------------------
# dW = dW + scale * (this batch's gradient): every path that writes dW
# ----------------------------------------------------------------------

ACCUMULATE = [
    # label, K, G, layer
    ("3x3, 16-byte-read kernel + its fold", 4, 4, dk_inputs.conv(64, 64, 16, 16, 3)),
    ("3x3, width 4 mod 8 (tile split by rows)", 2, 3, dk_inputs.conv(40, 24, 12, 12, 3)),
    ("3x3, 4-byte-read kernel + its fold", 2, 8, dk_inputs.conv(64, 64, 13, 12, 3)),
    ("3x3, few input channels (gather)", 4, 2, dk_inputs.conv(3, 64, 16, 16, 3)),
    ("3x3 stride 2 (gather)", 2, 3, dk_inputs.conv(24, 40, 15, 13, 3, 2, 1)),
    ("3x3 odd width (gather)", 2, 3, dk_inputs.conv(20, 33, 7, 7, 3)),
    ("1x1", 4, 3, dk_inputs.conv(72, 40, 12, 12, 1, 1, 0)),
    ("1x1, many rows (sliced)", 2, 40, dk_inputs.conv(64, 64, 14, 14, 1, 1, 0)),
    ("1x1 stride 2 (gather)", 2, 3, dk_inputs.conv(16, 72, 14, 14, 1, 2, 0)),
    ("5x5 (gather)", 2, 2, dk_inputs.conv(8, 16, 10, 10, 5, 1, 2)),
    ("2x2-pixel images (refold)", 4, 4, dk_inputs.conv(130, 70, 2, 2, 3)),
    ("1x1-pixel images (refold)", 2, 3, dk_inputs.conv(24, 40, 1, 1, 3)),
    ("dense, one slice (epilogue)", 4, 3, dk_inputs.linear(96, 200)),
    ("dense, >= 64 slices (deep fold, 16 waves)", 2, 700, dk_inputs.linear(40, 50)),
    ("dense, ~10 slices (deep fold, 4 waves)", 2, 40, dk_inputs.linear(40, 50)),
    ("dense, odd output length", 2, 300, dk_inputs.linear(33, 91)),
    ("dense, 64-column tile", 2, 300, dk_inputs.linear(150, 47)),
    ("dense, large output, few slices (wide fold)", 2, 256, dk_inputs.linear(1024, 1024)),
    ("dense, large odd output (scalar wide fold)", 2, 128, dk_inputs.linear(1023, 1025)),
    ("depthwise 3x3", 4, 2, dk_inputs.dwconv(24, 16, 16, 3)),
]


@pytest.mark.parametrize("label,K,G,L", ACCUMULATE, ids=[c[0] for c in ACCUMULATE])
def test_wgrad_accumulates_over_virtual_batches(dk, label, K, G, L):
    say("accumulate:", label, dict(K=K, G=G), L)
    scale = 0.25
    ref = None
    dW = None
    for call, acc in enumerate((False, True, True)):
        d = dk_inputs.masked_layer_inputs(np.random.default_rng([31, call, K, G]), L, K=K, batch=G * K)
        _, _, B = dk.dk_coeffs(d["A"], d["gamma"])
        xbar = dk.dk_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
        if dW is None:
            # a first call without `accumulate` must overwrite whatever dW held
            dW = torch.full(L.w_shape, 1e6, dtype=torch.float32, device="cuda")
        out = dk.dk_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, dW=dW, scale=scale,
                          accumulate=acc)
        assert out.data_ptr() == dW.data_ptr()
        if L.kind == "linear":
            part = oracle.dense_wgrad(d["delta"], d["X"], scale=scale)
        elif L.kind == "dwconv":
            part = scale * oracle.dwconv_wgrad(d["delta"], d["X"], L.kh, L.kw, L.stride, L.pad)
        else:
            part = scale * oracle.conv_wgrad(d["delta"], d["X"], L.kh, L.kw, L.stride, L.pad)
        ref = part if ref is None else ref + part
        assert nerr(host(dW), ref) < TOL_CONTRACT, "after call %d" % call


def test_patch_wgrad_with_large_lds_before_and_after_the_quad_kernel(dk):
    """13x12 images, 64 -> 64 channels, 64 encoded rows: the 4-byte-read
    weight-gradient kernel is planned with a 7-row tile (134 KB of LDS, above
    the 64 KB a kernel may use without being allowed more).  It must work
    whether or not the 16-byte-read kernel, which has the same function type,
    ran first in the process."""
    Lp = dk_inputs.conv(64, 64, 13, 12, 3)
    Lq = dk_inputs.conv(64, 64, 16, 16, 3)
    for L, K, G in ((Lp, 2, 16), (Lq, 4, 4), (Lp, 2, 16)):
        say("large-LDS weight gradient", L, dict(K=K, G=G))
        d = dk_inputs.masked_layer_inputs(np.random.default_rng([77, L.H]), L, K=K, batch=G * K)
        out = _run_masked(dk, d)
        assert nerr(out["dW"], oracle.conv_wgrad(d["delta"], d["X"], 3, 3, 1, 1)) < TOL_CONTRACT
        assert nerr(out["y"], oracle.conv_fwd(d["W"], d["X"], 1, 1)) < TOL_CONTRACT
