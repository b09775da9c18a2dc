"""The library enqueues on the caller's stream, allocates nothing and never
synchronises: the whole path gives the same bits on a side stream and when a
captured HIP graph of it is replayed (fp32 and finite-field entry points)."""
import numpy as np
import pytest
import torch

import dk_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dk():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    import paper_2207_00083_amd as m
    m.load()
    return m


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


class Fp32Path:
    """Pre-allocated buffers and one call that runs every step of the path."""

    def __init__(self, dk, L, K, G, seed):
        import ctypes as C
        rng = np.random.default_rng(seed)
        d = dk_inputs.masked_layer_inputs(rng, L, K=K, batch=G * K)
        S = K + 2
        Ainv, nvec, B = dk.dk_coeffs(d["A"], d["gamma"])
        self.dk, self.L, self.K = dk, L, K
        self.X, self.r, self.A, self.W, self.delta = (dev(d[k]) for k in ("X", "r", "A", "W", "delta"))
        self.Ainv, self.nvec, self.B, self.gamma = dev(Ainv), dev(nvec), dev(B), dev(d["gamma"])
        f32 = dict(dtype=torch.float32, device="cuda")
        self.xbar = torch.empty((G * S,) + L.in_shape, **f32)
        self.ybar = torch.empty((G * S,) + L.out_shape, **f32)
        self.y = torch.empty((G * K,) + L.out_shape, **f32)
        self.dW = torch.empty(L.w_shape, **f32)
        self.verdict = torch.empty(G, dtype=torch.int32, device="cuda")
        self.resid = torch.empty(G, **f32)
        lib, lay = dk.load(), dk.DkLayer.of(L)
        u8 = dict(dtype=torch.uint8, device="cuda")
        self.ws_fwd = torch.empty(max(256, lib.dk_fwd_workspace_bytes(C.byref(lay), G * S)), **u8)
        self.ws_wg = torch.empty(max(256, dk.dk_workspace_bytes(L, dk.DK_OP_WGRAD, G, K)), **u8)
        self.ws_vf = torch.empty(max(256, dk.dk_workspace_bytes(None, dk.DK_OP_VERIFY, G, K)), **u8)

    def outputs(self):
        return (self.xbar, self.ybar, self.y, self.dW, self.verdict, self.resid)

    def step(self):
        dk, L, K = self.dk, self.L, self.K
        dk.dk_encode(self.X, self.r, self.A, K, xbar=self.xbar)
        if L.kind == "linear":
            dk.dk_linear_fwd(self.W, self.xbar, ybar=self.ybar, ws=self.ws_fwd)
        else:
            dk.dk_conv_fwd(L, self.W, self.xbar, ybar=self.ybar, ws=self.ws_fwd)
        dk.dk_decode_verify(self.ybar, self.Ainv, self.nvec, K, tol=1e-3, y=self.y, verdict=self.verdict,
                            resid=self.resid, ws=self.ws_vf)
        dk.dk_wgrad(L, self.delta, self.B, self.gamma, self.xbar, K, dW=self.dW, ws=self.ws_wg)


class FieldPath:
    def __init__(self, dk, L, K, G, seed):
        rng = np.random.default_rng(seed)
        d = dk_inputs.field_layer_inputs(rng, L, K=K, batch=G * K, delta_std=1.0)
        S = K + 2
        Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
        self.dk, self.L, self.K = dk, L, K
        self.X, self.r, self.A, self.W, self.delta = (dev(d[k]) for k in ("X", "r", "A", "W", "delta"))
        self.Ainv, self.nvec, self.B, self.gamma = dev(Ainv), dev(nvec), dev(B), dev(d["gamma"])
        i32 = dict(dtype=torch.int32, device="cuda")
        f32 = dict(dtype=torch.float32, device="cuda")
        self.Wq = torch.empty(L.w_shape, **i32)
        self.xbar = torch.empty((G * S,) + L.in_shape, **i32)
        self.ybar = torch.empty((G * S,) + L.out_shape, **i32)
        self.y = torch.empty((G * K,) + L.out_shape, **f32)
        self.dW = torch.empty(L.w_shape, **f32)
        self.verdict = torch.empty(G, **i32)
        u8 = dict(dtype=torch.uint8, device="cuda")
        R = G * S
        fwd = (dk.dkf_fwd_workspace_bytes(L.M, L.N, R) if L.kind == "linear"
               else dk.dkf_conv_fwd_workspace_bytes(L, R))
        self.ws_fwd = torch.empty(fwd, **u8)
        self.ws_wg = torch.empty(dk.dkf_wgrad_workspace_bytes(L, G, K), **u8)

    def outputs(self):
        return (self.Wq, self.xbar, self.ybar, self.y, self.dW, self.verdict)

    def step(self):
        dk, L, K = self.dk, self.L, self.K
        dk.dkf_quantize(self.W, xq=self.Wq)
        dk.dkf_encode(self.X, self.r, self.A, K, xbar=self.xbar)
        if L.kind == "linear":
            dk.dkf_linear_fwd(self.Wq, self.xbar, ybar=self.ybar, ws=self.ws_fwd)
        else:
            dk.dkf_conv_fwd(L, self.Wq, self.xbar, ybar=self.ybar, ws=self.ws_fwd)
        dk.dkf_decode_verify(self.ybar, self.Ainv, self.nvec, K, y=self.y, verdict=self.verdict)
        dk.dkf_wgrad(L, self.delta, self.B, self.gamma, self.xbar, K, dW=self.dW, ws=self.ws_wg)


class FusedPath(Fp32Path):
    """1x1 layers through the fused kernels: forward + decode + verify in one
    kernel (its verdict taken inside the kernel or by a second launch,
    depending on the number of tiles per virtual batch) and the weight gradient
    with the mixing in its loader."""

    def __init__(self, dk, L, K, G, seed):
        super().__init__(dk, L, K, G, seed)
        u8 = dict(dtype=torch.uint8, device="cuda")
        self.ws_fdv = torch.empty(dk.dk_conv_fwd_decode_verify_workspace_bytes(L, G, K), **u8)

    def outputs(self):
        return (self.xbar, self.y, self.dW, self.verdict, self.resid)

    def step(self):
        dk, L, K = self.dk, self.L, self.K
        dk.dk_set_option(dk.DK_OPT_FUSE_FWD, dk.DK_FUSE_ALWAYS)
        dk.dk_set_option(dk.DK_OPT_FUSE_WGRAD, dk.DK_FUSE_ALWAYS)
        try:
            dk.dk_encode(self.X, self.r, self.A, K, xbar=self.xbar)
            dk.dk_conv_fwd_decode_verify(L, self.W, self.xbar, self.Ainv, self.nvec, K, tol=1e-3, y=self.y,
                                         verdict=self.verdict, resid=self.resid, ws=self.ws_fdv)
            dk.dk_wgrad(L, self.delta, self.B, self.gamma, self.xbar, K, dW=self.dW, ws=self.ws_wg)
        finally:
            dk.dk_set_option(dk.DK_OPT_FUSE_FWD, dk.DK_FUSE_AUTO)
            dk.dk_set_option(dk.DK_OPT_FUSE_WGRAD, dk.DK_FUSE_AUTO)


CASES = [(Fp32Path, dk_inputs.conv(64, 64, 16, 16, 3), 4, 3), (Fp32Path, dk_inputs.linear(200, 1100), 8, 2),
         (FusedPath, dk_inputs.conv(64, 128, 16, 16, 1, 1, 0), 8, 2),       # 8 tiles per batch: verdict in the kernel
         (FusedPath, dk_inputs.conv(32, 64, 48, 48, 1, 1, 0), 4, 2),        # 36 tiles per batch: second launch
         (Fp32Path, dk_inputs.conv(3, 16, 16, 16, 3), 2, 3),                # direct small-channel kernels
         (Fp32Path, dk_inputs.conv(24, 40, 14, 14, 3, 2, 1), 2, 2),
         (FieldPath, dk_inputs.conv(32, 64, 16, 16, 3), 4, 2), (FieldPath, dk_inputs.linear(130, 300), 2, 3)]


def _eager_reference(path):
    path.step()
    torch.cuda.synchronize()
    return [t.clone() for t in path.outputs()]


def _scrub(path):
    for t in path.outputs():
        t.fill_(77)
    torch.cuda.synchronize()


@pytest.mark.parametrize("cls,L,K,G", CASES)
def test_side_stream(dk, cls, L, K, G):
    path = cls(dk, L, K, G, seed=31)
    ref = _eager_reference(path)
    _scrub(path)
    side = torch.cuda.Stream()                     # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path.step()
    # nothing was enqueued on the default stream: the results appear only once the side stream is done
    side.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(path.outputs(), ref))


@pytest.mark.parametrize("cls,L,K,G", CASES)
def test_graph_replay(dk, cls, L, K, G):
    path = cls(dk, L, K, G, seed=32)
    ref = _eager_reference(path)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            path.step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # several replays, with the program's own eager work and synchronisations in between
    for _ in range(3):
        _scrub(path)
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(path.outputs(), ref))
        path.step()                                # eager again between replays
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(path.outputs(), ref))


def test_explicit_stream_with_automatic_workspaces(dk):
    """`stream=` given, `ws=` not: the binding takes the temporary workspace
    from that stream's pool, so work queued afterwards on the current stream
    (which reuses freed blocks at once) cannot overwrite it while the side
    stream's kernels still run."""
    L, K, G = dk_inputs.linear(300, 1100), 8, 3           # sliced contraction: the workspace holds partial sums
    path = Fp32Path(dk, L, K, G, seed=33)
    ref = _eager_reference(path)
    _scrub(path)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for _ in range(3):
        dk.dk_encode(path.X, path.r, path.A, K, xbar=path.xbar, stream=side)
        dk.dk_linear_fwd(path.W, path.xbar, ybar=path.ybar, stream=side)
        dk.dk_decode_verify(path.ybar, path.Ainv, path.nvec, K, tol=1e-3, y=path.y, verdict=path.verdict,
                            resid=path.resid, stream=side)
        dk.dk_wgrad(L, path.delta, path.B, path.gamma, path.xbar, K, dW=path.dW, stream=side)
        # current-stream allocations of the workspaces' sizes, filled at once
        junk = [torch.full((n,), 255, dtype=torch.uint8, device="cuda")
                for n in (path.ws_fwd.numel(), path.ws_wg.numel(), path.ws_vf.numel())]
        del junk
    side.synchronize()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(path.outputs(), ref))


def test_fp32_matrix_rate_probe_runs(dk):
    import torch
    for kind in (0, 1):
        assert dk.dk_probe_mfma_rate(kind, 50) == 256 * 4 * 50 * 16 * 4096.0
    torch.cuda.synchronize()
