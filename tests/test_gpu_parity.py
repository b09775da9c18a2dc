"""Parity of the HIP path (through the C ABI) with the fp64 oracle, element by
element on the same seeded fp32 inputs.  Every test prints its case first so
that a faulting launch can be named from the log.

Tolerances (normwise, max|got-ref| / max|ref|):
  * 1e-3 on decoded outputs and weight gradients against the plain layer
    definitions -- the contract;
  * 2e-5 on single bandwidth-bound kernels and 1e-4 on single contractions
    against the oracle's stage of the same name (fp32 rounding only);
  * integrity verdicts: exact.
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
TOL_MIX = 2e-5
TOL_GEMM = 1e-4


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


def coeffs_dev(dk, d):
    Ainv, nvec, B = dk.dk_coeffs(d["A"], d["gamma"])
    return Ainv, nvec, B


# ----------------------------------------------------------------------
# bandwidth-bound kernels vs the oracle stage of the same name
# ----------------------------------------------------------------------

MIX_CASES = [(1, 1, 1), (1, 3, 7), (2, 1, 256), (2, 5, 1023), (3, 4, 1024), (4, 6, 4100),
             (4, 64, 2048), (5, 2, 333), (8, 3, 5000), (8, 16, 8192), (16, 2, 777), (7, 2, 12)]


@pytest.mark.parametrize("K,G,n", MIX_CASES)
def test_encode_decode_verify_stages(dk, K, G, n):
    say("mix stages", dict(K=K, G=G, n=n))
    rng = np.random.default_rng(1000 + K * 7 + G * 3 + n)
    S = K + 2
    X = rng.standard_normal((G * K, n)).astype(np.float32)
    r = (10 * rng.standard_normal((G, n))).astype(np.float32)
    A, gamma = dk_inputs.sample_coeff_draws(rng, G, K)
    Ainv, nvec, B = dk.dk_coeffs(A, gamma)

    xbar = host(dk.dk_encode(dev(X), dev(r), dev(A), K))
    ref = oracle.encode(X, r, A)
    assert xbar.shape == (G * S, n)
    assert nerr(xbar, ref) < TOL_MIX

    # decode / verify are checked on a synthetic Ybar with the oracle's encodings as data
    ybar = ref.astype(np.float32)
    y = host(dk.dk_decode(dev(ybar), dev(Ainv), K))
    yref = oracle.decode(ybar, Ainv)
    assert y.shape == (G * K, n)
    assert np.max(np.abs(y - yref)) < TOL_MIX * np.max(np.abs(ybar)) * np.max(np.abs(Ainv)) * S

    v, rho = dk.dk_verify(dev(ybar), dev(nvec), K, tol=1e-3)
    vref, rhoref = oracle.verify(ybar, nvec, 1e-3)
    assert host(v).tolist() == vref.tolist() == [0] * G
    # corrupt one element per odd group, where the null vector is largest
    yc = ybar.copy()
    expect = np.zeros(G, dtype=np.int32)
    for g in range(0, G, 2):
        j = int(np.argmax(np.abs(nvec[g])))
        e = int(rng.integers(n))
        yc[g * S + j, e] += 0.5 * max(1.0, float(np.max(np.abs(ybar[g * S:(g + 1) * S]))))
        expect[g] = 1
    v, rho = dk.dk_verify(dev(yc), dev(nvec), K, tol=1e-3)
    vref, rhoref = oracle.verify(yc, nvec, 1e-3)
    assert vref.tolist() == expect.tolist()
    assert host(v).tolist() == vref.tolist()
    assert np.allclose(host(rho)[expect == 1], rhoref[expect == 1], rtol=1e-3)

    # the fused sweep gives what the two calls give
    y2, v2, rho2 = dk.dk_decode_verify(dev(yc), dev(Ainv), dev(nvec), K, tol=1e-3)
    assert host(v2).tolist() == vref.tolist()
    assert np.array_equal(host(rho2), host(rho))
    assert np.array_equal(host(y2), host(dk.dk_decode(dev(yc), dev(Ainv), K)))


def test_verify_nonfinite_and_zero(dk):
    say("verify non-finite / all-zero")
    K, G, n = 2, 4, 600
    S = K + 2
    rng = np.random.default_rng(5)
    ybar = rng.standard_normal((G * S, n)).astype(np.float32)
    nvec = np.ones((G, S), dtype=np.float32)
    ybar[0:S] = 0.0                          # all-zero group: clean by definition
    ybar[1 * S + 1, 17] = np.nan
    ybar[2 * S + 3, 599] = np.inf
    ybar[3 * S:4 * S] = 0.0
    ybar[3 * S + 0, 5] = 1.0
    ybar[3 * S + 1, 5] = -1.0                # consistent: t = 0
    v, rho = dk.dk_verify(dev(ybar), dev(nvec), K, tol=1e-3)
    vref, rhoref = oracle.verify(ybar, nvec, 1e-3)
    assert vref.tolist() == [0, 1, 1, 0]
    assert host(v).tolist() == vref.tolist()
    rho = host(rho)
    assert rho[0] == 0.0 and np.isinf(rho[1]) and np.isinf(rho[2]) and rho[3] == 0.0


def test_verify_workspace_contents_do_not_matter(dk):
    """The integrity check is one launch: workgroups publish their maxima in
    the workspace under a tag drawn per call and the one that finds all slots
    of its group tagged writes the verdict.  Whatever the workspace holds
    beforehand -- garbage, or the slots of an earlier call with another
    partition -- must not matter, and a call must leave it reusable."""
    say("verify workspace: garbage, stale slots, reuse")
    rng = np.random.default_rng(12)
    cases = [(4, 3, 70000), (2, 64, 4100), (8, 2, 1003), (1, 200, 64), (4, 3, 70000)]
    nbytes = max(dk.dk_workspace_bytes(None, dk.DK_OP_VERIFY, G, K) for K, G, _ in cases)
    ws = torch.from_numpy(rng.integers(0, 256, nbytes, dtype=np.uint8)).cuda()
    for rep, (K, G, n) in enumerate(cases):
        S = K + 2
        A, gamma = dk_inputs.sample_coeff_draws(rng, G, K)
        Ainv, nvec, _ = dk.dk_coeffs(A, gamma)
        X = rng.standard_normal((G * K, n)).astype(np.float32)
        r = (10 * rng.standard_normal((G, n))).astype(np.float32)
        ybar = oracle.encode(X, r, A).astype(np.float32)
        expect = np.zeros(G, dtype=np.int32)
        for g in range(rep % 2, G, 2):
            j = int(np.argmax(np.abs(nvec[g])))
            ybar[g * S + j, int(rng.integers(n))] += 0.5 * max(1.0, float(np.max(np.abs(ybar[g * S:(g + 1) * S]))))
            expect[g] = 1
        vref, rhoref = oracle.verify(ybar, nvec, 1e-3)
        assert vref.tolist() == expect.tolist()
        yd = dev(ybar)
        for call in range(2):           # the same workspace twice in a row
            v, rho = dk.dk_verify(yd, dev(nvec), K, tol=1e-3, ws=ws)
            assert host(v).tolist() == vref.tolist(), (rep, call)
            assert np.allclose(host(rho)[expect == 1], rhoref[expect == 1], rtol=1e-3)
            y2, v2, rho2 = dk.dk_decode_verify(yd, dev(Ainv), dev(nvec), K, tol=1e-3, ws=ws)
            assert host(v2).tolist() == vref.tolist(), (rep, call)
            assert np.array_equal(host(rho2), host(rho))


# ----------------------------------------------------------------------
# contractions vs the plain definitions
# ----------------------------------------------------------------------

DENSE_CASES = [(4, 512, 256), (1, 1, 1), (3, 5, 7), (150, 300, 77), (260, 130, 1000),
               (129, 257, 1025), (64, 1000, 4096), (384, 128, 130)]


@pytest.mark.parametrize("R,M,N", DENSE_CASES)
def test_linear_fwd(dk, R, M, N):
    say("linear fwd", dict(R=R, M=M, N=N))
    rng = np.random.default_rng(R * 31 + M * 17 + N)
    W = rng.standard_normal((M, N)).astype(np.float32)
    X = rng.standard_normal((R, N)).astype(np.float32)
    got = host(dk.dk_linear_fwd(dev(W), dev(X)))
    ref = oracle.dense_fwd(W, X)
    assert got.shape == ref.shape
    assert nerr(got, ref) < TOL_GEMM


CONV_CASES = [
    # Ci, Co, H, W, k, stride, pad, R
    (8, 16, 12, 12, 3, 1, 1, 6),
    (3, 64, 32, 32, 3, 1, 1, 6),
    (16, 130, 9, 11, 3, 1, 1, 5),
    (20, 24, 14, 14, 1, 1, 0, 6),
    (24, 136, 7, 7, 1, 1, 0, 5),
    (72, 40, 12, 12, 1, 1, 0, 7),
    (16, 72, 14, 14, 1, 2, 0, 4),
    (8, 8, 15, 13, 3, 2, 1, 3),
    (3, 16, 30, 30, 7, 2, 3, 3),
    (64, 64, 8, 8, 3, 1, 1, 12),
    (5, 7, 6, 6, 3, 1, 0, 2),
    (130, 20, 4, 4, 3, 1, 1, 3),
    (32, 40, 2, 2, 3, 1, 1, 12),
    # pixel tiles that slide over the batch (images of 100, 196, 49 and 99 pixels; ragged last tile)
    (16, 64, 10, 10, 3, 1, 1, 7),
    (24, 136, 14, 14, 3, 1, 1, 5),
    (8, 130, 7, 7, 3, 1, 1, 9),
    (12, 72, 11, 9, 3, 1, 1, 6),
    (10, 48, 13, 13, 3, 1, 0, 4),
]


@pytest.mark.parametrize("Ci,Co,H,W,k,stride,pad,R", CONV_CASES)
def test_conv_fwd(dk, Ci, Co, H, W, k, stride, pad, R):
    L = dk_inputs.conv(Ci, Co, H, W, k, stride, pad)
    say("conv fwd", L, "R=%d" % R)
    rng = np.random.default_rng(Ci * 131 + Co * 17 + H + k + stride)
    Wt = rng.standard_normal(L.w_shape).astype(np.float32)
    X = rng.standard_normal((R,) + L.in_shape).astype(np.float32)
    got = host(dk.dk_conv_fwd(L, dev(Wt), dev(X)))
    ref = oracle.conv_fwd(Wt, X, stride, pad)
    assert got.shape == ref.shape
    assert nerr(got, ref) < TOL_GEMM


def _masked_case(L, K, G, seed, **kw):
    rng = np.random.default_rng(seed)
    return dk_inputs.masked_layer_inputs(rng, L, K=K, batch=G * K, **kw)


def _run_masked(dk, d, tol=1e-3, scale=1.0, corrupt=None):
    """Whole hot path on the GPU: encode -> layer on encodings -> verify ->
    decode -> wgrad.  `corrupt` = list of (g, j, flat index, eta) added to Ybar."""
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
    verdict, resid = dk.dk_verify(ybar, dev(nvec), K, tol=tol)
    y = dk.dk_decode(ybar, dev(Ainv), K)
    dW = dk.dk_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, scale=scale)
    return dict(xbar=host(xbar), ybar=host(ybar), verdict=host(verdict), resid=host(resid),
                y=host(y), dW=host(dW), nvec=nvec)


DENSE_MASKED = [(2, 1, 512, 256), (1, 3, 40, 50), (4, 8, 300, 260), (8, 4, 130, 1030), (3, 5, 37, 91)]


@pytest.mark.parametrize("K,G,M,N", DENSE_MASKED)
def test_dense_masked_layer(dk, K, G, M, N):
    L = dk_inputs.linear(M, N)
    say("dense masked layer", dict(K=K, G=G, M=M, N=N))
    d = _masked_case(L, K, G, seed=K * 1000 + G * 100 + M + N)
    out = _run_masked(dk, d, scale=1.0 / K)
    Y = oracle.dense_fwd(d["W"], d["X"])
    dW = oracle.dense_wgrad(d["delta"], d["X"], scale=1.0 / K)
    assert nerr(out["y"], Y) < TOL_CONTRACT
    assert nerr(out["dW"], dW) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G
    # stage-level diagnostics against the staged oracle
    st = oracle.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], scale=1.0 / K)
    assert nerr(out["xbar"], st["Xbar"]) < TOL_MIX
    assert nerr(out["ybar"], st["Ybar"]) < TOL_GEMM
    assert st["verdict"].tolist() == [0] * G


CONV_MASKED = [
    # K, G, Ci, Co, H, W, k, stride, pad
    (4, 3, 8, 16, 12, 12, 3, 1, 1),
    (2, 4, 3, 64, 16, 16, 3, 1, 1),
    (4, 2, 16, 130, 9, 11, 3, 1, 1),
    (2, 3, 20, 24, 14, 14, 1, 1, 0),
    (3, 2, 24, 136, 7, 7, 1, 1, 0),
    (4, 2, 132, 72, 12, 12, 1, 1, 0),
    (3, 2, 16, 72, 14, 14, 1, 2, 0),
    (2, 2, 8, 8, 15, 13, 3, 2, 1),
    (1, 2, 3, 16, 30, 30, 7, 2, 3),
    (8, 1, 32, 40, 2, 2, 3, 1, 1),
    (4, 2, 70, 20, 4, 4, 3, 1, 1),
    # at most four input channels (direct vector-ALU kernels)
    (4, 3, 1, 5, 9, 8, 3, 1, 1),
    (2, 2, 2, 33, 7, 4, 3, 1, 1),
    (4, 8, 3, 64, 32, 32, 3, 1, 1),
    (3, 2, 4, 70, 5, 12, 3, 1, 1),
    # widths that are 4 mod 8 (weight gradient splits the tile by rows)
    (4, 2, 40, 24, 12, 12, 3, 1, 1),
    (2, 3, 24, 70, 20, 20, 3, 1, 1),
    (2, 2, 32, 32, 28, 28, 3, 1, 1),
    (3, 5, 70, 130, 4, 4, 3, 1, 1),
    # strided 1x1 (ragged sizes, stride 3)
    (2, 2, 20, 24, 9, 7, 1, 2, 0),
    (2, 2, 12, 130, 10, 10, 1, 3, 0),
    # images of at most 2x2 pixels (run as a dense layer on unfolded filters)
    (2, 3, 24, 40, 1, 1, 3, 1, 1),
    (3, 2, 12, 20, 2, 2, 3, 2, 1),
    (2, 2, 16, 8, 2, 2, 2, 1, 0),
    (4, 4, 130, 70, 2, 2, 3, 1, 1),
]


@pytest.mark.parametrize("K,G,Ci,Co,H,W,k,stride,pad", CONV_MASKED)
def test_conv_masked_layer(dk, K, G, Ci, Co, H, W, k, stride, pad):
    L = dk_inputs.conv(Ci, Co, H, W, k, stride, pad)
    say("conv masked layer", dict(K=K, G=G), L)
    d = _masked_case(L, K, G, seed=K * 1000 + G * 100 + Ci + Co + H + k)
    out = _run_masked(dk, d)
    Y = oracle.conv_fwd(d["W"], d["X"], stride, pad)
    dW = oracle.conv_wgrad(d["delta"], d["X"], k, k, stride, pad)
    assert nerr(out["y"], Y) < TOL_CONTRACT
    assert nerr(out["dW"], dW) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G


def _random_conv_shapes(seed, count):
    """Seeded draw of small convolution shapes that between them reach every
    kernel family the planner can pick: widths that are and are not multiples
    of 4 and 8, odd and even heights, 1x1 to 5x5 filters, strides 1 and 2,
    channel counts on both sides of the tile sizes."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k = int(rng.choice([1, 1, 3, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 1, 2]))
        pad = int(rng.choice([0, k // 2]))
        H = int(rng.choice([1, 2, 4, 6, 7, 8, 12, 14, 16, 20]))
        W = int(rng.choice([1, 2, 4, 7, 8, 12, 14, 16, 24, 32]))
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        Ci = int(rng.choice([1, 3, 8, 17, 20, 32, 48, 70]))
        Co = int(rng.choice([1, 5, 16, 33, 64, 72, 130]))
        K = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 3]))
        out.append((K, G, Ci, Co, H, W, k, stride, pad))
    return out


@pytest.mark.parametrize("K,G,Ci,Co,H,W,k,stride,pad", _random_conv_shapes(20260, 40))
def test_conv_masked_layer_random_shapes(dk, K, G, Ci, Co, H, W, k, stride, pad):
    L = dk_inputs.conv(Ci, Co, H, W, k, stride, pad)
    say("conv masked layer, drawn shape", dict(K=K, G=G), L)
    d = _masked_case(L, K, G, seed=[K, G, Ci, Co, H, W, k, stride, pad])
    out = _run_masked(dk, d)
    Y = oracle.conv_fwd(d["W"], d["X"], stride, pad)
    dW = oracle.conv_wgrad(d["delta"], d["X"], k, k, stride, pad)
    assert nerr(out["y"], Y) < TOL_CONTRACT
    assert nerr(out["dW"], dW) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G


def _random_dense_shapes(seed, count):
    rng = np.random.default_rng(seed)
    sizes = [1, 3, 31, 64, 65, 127, 128, 130, 200, 257, 300, 520]
    return [(int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 5])), int(rng.choice(sizes)),
             int(rng.choice(sizes + [1030, 2049]))) for _ in range(count)]


@pytest.mark.parametrize("K,G,M,N", _random_dense_shapes(20263, 24))
def test_dense_masked_layer_random_shapes(dk, K, G, M, N):
    L = dk_inputs.linear(M, N)
    say("dense masked layer, drawn shape", dict(K=K, G=G, M=M, N=N))
    d = _masked_case(L, K, G, seed=[K, G, M, N, 5])
    out = _run_masked(dk, d)
    assert nerr(out["y"], oracle.dense_fwd(d["W"], d["X"])) < TOL_CONTRACT
    assert nerr(out["dW"], oracle.dense_wgrad(d["delta"], d["X"])) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G


def test_wgrad_accumulate_and_scale(dk):
    say("wgrad accumulate")
    L = dk_inputs.linear(96, 200)
    d1 = _masked_case(L, 4, 3, seed=77)
    d2 = _masked_case(L, 4, 3, seed=78)
    ref = np.zeros(L.w_shape)
    dW = None
    for d, acc in ((d1, False), (d2, True)):
        _, _, B = dk.dk_coeffs(d["A"], d["gamma"])
        xbar = dk.dk_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), 4)
        dW = dk.dk_wgrad(L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, 4, dW=dW,
                         scale=0.25, accumulate=acc)
        ref += oracle.dense_wgrad(d["delta"], d["X"], scale=0.25)
    assert nerr(host(dW), ref) < TOL_CONTRACT


# Contractions cut into slices along the contraction axis, one case per fold
# variant and tile shape: (many slices, tiny output), (a few slices, small
# output), (odd output length), (slices over a large output), narrow tiles.
SLICED_WGRAD = [
    # K, G, M, N
    (2, 700, 40, 50),      # contraction 2800 over a 40x50 output: >= 64 slices
    (2, 40, 40, 50),       # ~10 slices
    (2, 300, 33, 91),      # odd output length, 64-row tile
    (2, 300, 150, 47),     # 64-column tile
]


@pytest.mark.parametrize("K,G,M,N", SLICED_WGRAD)
def test_sliced_wgrad_folds(dk, K, G, M, N):
    L = dk_inputs.linear(M, N)
    say("sliced dense wgrad", dict(K=K, G=G, M=M, N=N))
    d = _masked_case(L, K, G, seed=K * 7 + G + M * 3 + N)
    _, _, B = dk.dk_coeffs(d["A"], d["gamma"])
    xbar = dk.dk_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    args = (L, dev(d["delta"]), dev(B), dev(d["gamma"]), xbar, K)
    dW = host(dk.dk_wgrad(*args, scale=0.5))
    ref = oracle.dense_wgrad(d["delta"], d["X"], scale=0.5)
    assert nerr(dW, ref) < TOL_CONTRACT
    # slices are folded in a fixed order: a rerun is bitwise identical
    assert np.array_equal(dW, host(dk.dk_wgrad(*args, scale=0.5)))


def test_sliced_forward_folds(dk):
    # dense: 130 x 257 outputs (odd length) over a contraction of 4096;
    # conv: 1.5 M outputs over 256 input channels (a few slices, vector fold)
    say("sliced dense fwd")
    rng = np.random.default_rng(4242)
    W = rng.standard_normal((257, 4096)).astype(np.float32)
    X = rng.standard_normal((130, 4096)).astype(np.float32)
    assert nerr(host(dk.dk_linear_fwd(dev(W), dev(X))), oracle.dense_fwd(W, X)) < TOL_GEMM
    L = dk_inputs.conv(256, 128, 16, 16, 3, 1, 1)
    say("sliced conv fwd", L)
    Wt = rng.standard_normal(L.w_shape).astype(np.float32)
    Xc = rng.standard_normal((48,) + L.in_shape).astype(np.float32)
    got = host(dk.dk_conv_fwd(L, dev(Wt), dev(Xc)))
    pts = np.stack([rng.integers(0, s, 4000) for s in got.shape], axis=1)
    ref = oracle.conv_fwd_points(Wt, Xc, pts, 1, 1)
    assert np.max(np.abs(got[tuple(pts.T)] - ref)) / np.max(np.abs(ref)) < TOL_GEMM


def test_verdicts_match_oracle_under_corruption(dk):
    say("verdicts under corruption")
    L = dk_inputs.conv(8, 16, 10, 10, 3, 1, 1)
    K, G = 4, 8
    S = K + 2
    d = _masked_case(L, K, G, seed=4242)
    st = oracle.masked_layer(d["W"], d["X"], d["r"], d["delta"], d["A"], d["gamma"], stride=1, pad=1)
    _, nvec, _ = oracle.coefficients(d["A"], d["gamma"])
    rng = np.random.default_rng(9)
    corrupt, expect = [], np.zeros(G, dtype=np.int32)
    ybar_c = st["Ybar"].reshape(G * S, -1).copy()
    for g in (1, 6):
        j = int(np.argmax(np.abs(nvec[g])))
        e = int(rng.integers(ybar_c.shape[1]))
        scale_g = np.max(np.sum(np.abs(nvec[g][:, None] * ybar_c[g * S:(g + 1) * S]), axis=0))
        eta = float(0.5 * scale_g / abs(nvec[g, j]))
        corrupt.append((g, j, e, eta))
        ybar_c[g * S + j, e] += eta
        expect[g] = 1
    vref, rhoref = oracle.verify(ybar_c, nvec, 1e-3)
    assert vref.tolist() == expect.tolist()
    out = _run_masked(dk, d, corrupt=corrupt)
    assert out["verdict"].tolist() == vref.tolist()
    clean = out["resid"][expect == 0]
    assert clean.max() < 1e-4               # honest fp32 residual stays 10x below tol
    assert np.all(out["resid"][expect == 1] > 1e-2)


# ----------------------------------------------------------------------
# the named workloads
# ----------------------------------------------------------------------

def test_config1_full(dk):
    say("config 1 (dense 256->512, K=2, one group)")
    d = dk_inputs.config1()
    out = _run_masked(dk, d)
    assert nerr(out["y"], oracle.dense_fwd(d["W"], d["X"])) < TOL_CONTRACT
    assert nerr(out["dW"], oracle.dense_wgrad(d["delta"], d["X"])) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0]


def test_config2_reduced_full_compare(dk):
    say("config 2 reduced (conv 3x3 64->64 @16x16, batch 16, K=4)")
    d = dk_inputs.config2(batch=16, hw=16)
    out = _run_masked(dk, d)
    assert nerr(out["y"], oracle.conv_fwd(d["W"], d["X"], 1, 1)) < TOL_CONTRACT
    assert nerr(out["dW"], oracle.conv_wgrad(d["delta"], d["X"], 3, 3, 1, 1)) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * d["G"]


def test_config2_full_size_sampled(dk):
    say("config 2 full size (batch 256 @32x32), sampled outputs")
    d = dk_inputs.config2()
    L, K, G = d["layer"], d["K"], d["G"]
    out = _run_masked(dk, d)
    rng = np.random.default_rng(22)
    npts = 20000
    pts = np.stack([rng.integers(G * K, size=npts), rng.integers(L.Co, size=npts),
                    rng.integers(L.Ho, size=npts), rng.integers(L.Wo, size=npts)], axis=1)
    pts[:64, 2] = 0; pts[64:128, 2] = L.Ho - 1; pts[128:192, 3] = 0; pts[192:256, 3] = L.Wo - 1
    ref = oracle.conv_fwd_points(d["W"], d["X"], pts, 1, 1)
    got = out["y"][tuple(pts.T)]
    ymax = float(np.max(np.abs(out["y"])))
    assert np.max(np.abs(got - ref)) / ymax < TOL_CONTRACT
    wpts = np.array([[co, ci, a, b] for co in range(0, L.Co, 3) for ci in range(0, L.Ci, 5)
                     for a in range(3) for b in range(3)])
    wref = oracle.conv_wgrad_points(d["delta"], d["X"], 3, 3, wpts, 1, 1)
    wgot = out["dW"][tuple(wpts.T)]
    assert np.max(np.abs(wgot - wref)) / np.max(np.abs(wref)) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G
    assert out["resid"].max() < 1e-4


def test_config5_layer2_full_size_sampled(dk):
    say("config 5 layer 2 (dense 4096->4096, batch 1024, K=8), sampled outputs, 2 corrupted groups")
    d = dk_inputs.config5(index=1)[0]
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    nv = dk.dk_coeffs(d["A"], d["gamma"])[1]
    corrupt = []
    for g in (0, 64):
        j = int(np.argmax(np.abs(nv[g])))
        corrupt.append((g, j, 123 + g, 50.0))
    out = _run_masked(dk, d, corrupt=corrupt)
    expect = np.zeros(G, dtype=np.int32)
    expect[[0, 64]] = 1
    assert out["verdict"].tolist() == expect.tolist()
    rng = np.random.default_rng(55)
    npts = 20000
    clean_rows = np.array([s for s in range(G * K) if s // K not in (0, 64)])
    pts = np.stack([rng.choice(clean_rows, size=npts), rng.integers(L.M, size=npts)], axis=1)
    ref = oracle.dense_fwd_points(d["W"], d["X"], pts)
    got = out["y"][tuple(pts.T)]
    assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) < TOL_CONTRACT
    wpts = np.stack([rng.integers(L.M, size=npts), rng.integers(L.N, size=npts)], axis=1)
    wref = oracle.dense_wgrad_points(d["delta"], d["X"], wpts)
    wgot = out["dW"][tuple(wpts.T)]
    assert np.max(np.abs(wgot - wref)) / np.max(np.abs(wref)) < TOL_CONTRACT


def _sampled_conv_check(dk, d, npts=20000, seed=1):
    L, K, G = d["layer"], d["K"], d["G"]
    out = _run_masked(dk, d)
    rng = np.random.default_rng(seed)
    pts = np.stack([rng.integers(G * K, size=npts), rng.integers(L.Co, size=npts),
                    rng.integers(L.Ho, size=npts), rng.integers(L.Wo, size=npts)], axis=1)
    pts[:50, 2] = 0; pts[50:100, 2] = L.Ho - 1; pts[100:150, 3] = 0; pts[150:200, 3] = L.Wo - 1
    ref = oracle.conv_fwd_points(d["W"], d["X"], pts, L.stride, L.pad)
    got = out["y"][tuple(pts.T)]
    assert np.max(np.abs(got - ref)) / float(np.max(np.abs(out["y"]))) < TOL_CONTRACT
    nw = min(npts, L.Co * L.Ci * L.kh * L.kw)
    wpts = np.stack([rng.integers(L.Co, size=nw), rng.integers(L.Ci, size=nw),
                     rng.integers(L.kh, size=nw), rng.integers(L.kw, size=nw)], axis=1)[:4000]
    wref = oracle.conv_wgrad_points(d["delta"], d["X"], L.kh, L.kw, wpts, L.stride, L.pad)
    wgot = out["dW"][tuple(wpts.T)]
    assert np.max(np.abs(wgot - wref)) / float(np.max(np.abs(out["dW"]))) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G
    assert out["resid"].max() < 1e-4


def test_config3_layer_full_size_sampled(dk):
    say("config 3 layer 5 (VGG conv 256->256 @8x8, batch 128, K=4), sampled outputs")
    _sampled_conv_check(dk, dk_inputs.config3(index=5)[0])


def test_config3_first_layer_full_size_sampled(dk):
    say("config 3 layer 0 (VGG conv 3->64 @32x32, images ~U[0,1]), sampled outputs")
    _sampled_conv_check(dk, dk_inputs.config3(index=0)[0])


def test_config4_shapes_full_size_sampled(dk):
    for idx in (10, 11):       # 1x1 512->256 @28x28 and 3x3 stride 2 256->256 @28x28, batch 64, K=8
        for k, (d, count) in enumerate(dk_inputs.config4()):
            if k == idx:
                say("config 4 shape", idx, d["layer"], "x%d" % count)
                _sampled_conv_check(dk, d, npts=8000)
                break


def test_config5_last_layer_full_size_sampled(dk):
    say("config 5 layer 3 (dense 4096->1000, batch 1024, K=8), sampled outputs")
    d = dk_inputs.config5(index=2)[0]
    L, K, G = d["layer"], d["K"], d["G"]
    out = _run_masked(dk, d, scale=1.0 / K)
    rng = np.random.default_rng(7)
    npts = 20000
    pts = np.stack([rng.integers(G * K, size=npts), rng.integers(L.M, size=npts)], axis=1)
    ref = oracle.dense_fwd_points(d["W"], d["X"], pts)
    assert np.max(np.abs(out["y"][tuple(pts.T)] - ref)) / np.max(np.abs(ref)) < TOL_CONTRACT
    wpts = np.stack([rng.integers(L.M, size=npts), rng.integers(L.N, size=npts)], axis=1)
    wref = oracle.dense_wgrad_points(d["delta"], d["X"], wpts, scale=1.0 / K)
    assert np.max(np.abs(out["dW"][tuple(wpts.T)] - wref)) / np.max(np.abs(wref)) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G


def _off1(a):
    """Device copy of `a` that starts 4 bytes past a 16-byte boundary."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    buf = torch.empty(a.size + 1, dtype=torch.float32, device="cuda")
    v = buf[1:].view(a.shape)
    v.copy_(torch.from_numpy(a))
    assert v.data_ptr() % 16 == 4
    return v


UNALIGNED = [
    (4, 3, dk_inputs.linear(96, 200)),
    (2, 3, dk_inputs.conv(16, 24, 16, 16, 3, 1, 1)),      # the 16-byte-read kernels must step aside
    (2, 2, dk_inputs.conv(32, 40, 8, 8, 1, 1, 0)),
    (3, 2, dk_inputs.dwconv(12, 16, 16, 3, 1)),
]


@pytest.mark.parametrize("K,G,L", UNALIGNED)
def test_bases_off_16_byte_alignment(dk, K, G, L):
    # every tensor (inputs, outputs, workspaces aside) sits 4 bytes off a 16-byte
    # boundary although its sizes would allow vector accesses
    say("unaligned bases", dict(K=K, G=G), L)
    d = _masked_case(L, K, G, seed=K * 31 + G)
    S = K + 2
    Ainv, nvec, B = dk.dk_coeffs(d["A"], d["gamma"])
    xbar = dk.dk_encode(_off1(d["X"]), _off1(d["r"]), dev(d["A"]), K,
                        xbar=_off1(np.zeros((G * S,) + L.in_shape)))
    W = _off1(d["W"])
    ybar0 = _off1(np.zeros((G * S,) + L.out_shape))
    ybar = dk.dk_linear_fwd(W, xbar, ybar=ybar0) if L.kind == "linear" else dk.dk_conv_fwd(L, W, xbar, ybar=ybar0)
    y, v, rho = dk.dk_decode_verify(ybar, dev(Ainv), dev(nvec), K, y=_off1(np.zeros((G * K,) + L.out_shape)))
    dW = dk.dk_wgrad(L, _off1(d["delta"]), dev(B), dev(d["gamma"]), xbar, K, dW=_off1(np.zeros(L.w_shape)))
    if L.kind == "linear":
        Y, dWr = oracle.dense_fwd(d["W"], d["X"]), oracle.dense_wgrad(d["delta"], d["X"])
    elif L.kind == "dwconv":
        Y = oracle.dwconv_fwd(d["W"], d["X"], L.stride, L.pad)
        dWr = oracle.dwconv_wgrad(d["delta"], d["X"], L.kh, L.kw, L.stride, L.pad)
    else:
        Y = oracle.conv_fwd(d["W"], d["X"], L.stride, L.pad)
        dWr = oracle.conv_wgrad(d["delta"], d["X"], L.kh, L.kw, L.stride, L.pad)
    assert nerr(host(y), Y) < TOL_CONTRACT
    assert nerr(host(dW), dWr) < TOL_CONTRACT
    assert host(v).tolist() == [0] * G


def test_operand_beyond_two_gigabytes(dk):
    # W is 2.56 GB: past the 32-bit byte offsets of the loaders' fast path, which
    # must step aside for it (the encodings, 16 MB, still take it)
    say("dense forward, W of 2.56 GB")
    M, N, R = 640, 1_000_000, 4
    rng = np.random.default_rng(99)
    W = rng.standard_normal((M, N), dtype=np.float32)
    X = rng.standard_normal((R, N), dtype=np.float32)
    got = host(dk.dk_linear_fwd(dev(W), dev(X)))
    pts = np.stack([rng.integers(0, R, 300), rng.integers(0, M, 300)], axis=1)
    pts[:4] = [[0, 0], [R - 1, M - 1], [0, M - 1], [R - 1, 0]]
    ref = oracle.dense_fwd_points(W, X, pts)
    assert np.max(np.abs(got[tuple(pts.T)] - ref)) / np.max(np.abs(ref)) < TOL_GEMM


def test_verify_flags_tampered_stored_encodings(dk):
    # The encodings kept for the backward pass satisfy Xbar . nvec = 0 like the
    # forward results do: the same check, run on them before dk_wgrad, flags a
    # group whose stored encodings were changed after the forward pass.
    say("verify on stored encodings")
    K, G = 4, 5
    L = dk_inputs.conv(6, 10, 9, 9, 3, 1, 1)
    d = _masked_case(L, K, G, seed=2024)
    S = K + 2
    _, nvec, _ = dk.dk_coeffs(d["A"], d["gamma"])
    xbar = dk.dk_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), K)
    v, rho = dk.dk_verify(xbar, dev(nvec), K, tol=1e-3)
    assert host(v).tolist() == [0] * G and float(host(rho).max()) < 1e-4
    xb = host(xbar).reshape(G * S, -1).copy()
    g, j = 3, int(np.argmax(np.abs(nvec[3])))
    xb[g * S + j, 123] += 0.5 * float(np.max(np.abs(xb[g * S:(g + 1) * S])))
    v, rho = dk.dk_verify(dev(xb), dev(nvec), K, tol=1e-3)
    vref, _ = oracle.verify(xb, nvec, 1e-3)
    assert vref.tolist() == [0, 0, 0, 1, 0]
    assert host(v).tolist() == vref.tolist()


@pytest.mark.parametrize("L,K,G", [
    (dk_inputs.conv(64, 64, 32, 32, 3), 4, 4),          # the two 16-byte-read convolution kernels
    (dk_inputs.conv(24, 40, 14, 14, 3), 2, 3),          # patch forward, gather weight gradient
    (dk_inputs.conv(128, 64, 14, 14, 1, 1, 0), 4, 2),   # image-aware 1x1 loaders
    (dk_inputs.conv(32, 48, 2, 2, 3), 2, 2),            # small images on the dense engine
    (dk_inputs.linear(300, 1100), 8, 3),                # dense, sliced contraction
    (dk_inputs.dwconv(24, 16, 16, 3), 4, 2)])
def test_whole_path_is_bitwise_reproducible(dk, L, K, G):
    """No atomics on floating-point data and fixed fold orders: two runs of the
    whole path on the same inputs agree bit for bit."""
    say("rerun", L)
    d = _masked_case(L, K, G, seed=4711)
    a = _run_masked(dk, d)
    b = _run_masked(dk, d)
    for key in ("xbar", "ybar", "y", "dW", "resid"):
        assert np.array_equal(a[key].view(np.uint32), b[key].view(np.uint32)), key
    assert a["verdict"].tolist() == b["verdict"].tolist()


def test_bias_rides_along_as_an_input_feature(dk):
    """The layer's bias needs no entry point of its own: encoding and decoding
    are linear, so a constant-one input feature (dense) or a constant-one
    channel whose filter has the bias on its centre tap (convolution) decodes
    to W x + b, and its weight gradient is the bias gradient sum_i delta_i."""
    say("bias as an input feature")
    K, G, M, N = 4, 3, 37, 50
    rng = np.random.default_rng(77)
    d = _masked_case(dk_inputs.linear(M, N + 1), K, G, seed=78)
    b = rng.standard_normal(M).astype(np.float32)
    d["X"][:, N] = 1.0
    d["W"][:, N] = b
    out = _run_masked(dk, d)
    Y = d["X"][:, :N].astype(np.float64) @ d["W"][:, :N].astype(np.float64).T + b.astype(np.float64)
    assert nerr(out["y"], Y) < TOL_CONTRACT
    assert nerr(out["dW"][:, N], d["delta"].astype(np.float64).sum(0)) < TOL_CONTRACT
    assert out["verdict"].tolist() == [0] * G
    # convolution: 3x3, pad 1; the ones channel sees zero padding, the centre tap never does
    Ci, Co, H, W = 5, 6, 9, 8
    L = dk_inputs.conv(Ci + 1, Co, H, W, 3, 1, 1)
    d = _masked_case(L, 2, 2, seed=79)
    b = rng.standard_normal(Co).astype(np.float32)
    d["X"][:, Ci] = 1.0
    d["W"][:, Ci] = 0.0
    d["W"][:, Ci, 1, 1] = b
    out = _run_masked(dk, d)
    Y = oracle.conv_fwd(d["W"][:, :Ci], d["X"][:, :Ci], 1, 1) + b.astype(np.float64)[None, :, None, None]
    assert nerr(out["y"], Y) < TOL_CONTRACT
    assert nerr(out["dW"][:, Ci, 1, 1], d["delta"].astype(np.float64).sum((0, 2, 3))) < TOL_CONTRACT


# ----------------------------------------------------------------------
# error behaviour through the C ABI
# ----------------------------------------------------------------------

def test_short_workspace_is_refused(dk):
    say("short workspace")
    L = dk_inputs.linear(64, 64)
    d = _masked_case(L, 2, 2, seed=3)
    xbar = dk.dk_encode(dev(d["X"]), dev(d["r"]), dev(d["A"]), 2)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(dk.DkError) as e:
        dk.dk_linear_fwd(dev(d["W"]), xbar, ws=small)
    assert e.value.status == 5
