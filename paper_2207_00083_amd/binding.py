"""ctypes binding of libdarknight.so: marshals torch tensors (device memory)
and numpy arrays (host memory) into the C ABI declared in include/darknight.h.

No arithmetic of the method happens here.  If the library has not been built
the import of any entry point fails loudly; there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libdarknight.so")

DK_OP_FWD, DK_OP_WGRAD, DK_OP_VERIFY = 0, 1, 2
DK_OPT_FUSE_FWD, DK_OPT_FUSE_WGRAD = 0, 1
DK_FUSE_NEVER, DK_FUSE_ALWAYS, DK_FUSE_AUTO = 0, 1, 2
DK_MAX_K = 16

_lib = None


class DkError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, dk_status_str(status), status))


class DkLayer(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("kind", "M", "N", "Ci", "Co", "H", "W", "kh", "kw", "stride", "pad")]

    @classmethod
    def of(cls, layer):
        """Accepts a DkLayer or any object with the same attribute names
        (kind may be 'linear'/'conv'/'dwconv' or 0/1/2)."""
        if isinstance(layer, cls):
            return layer
        kind = layer.kind
        if isinstance(kind, str):
            kind = {"linear": 0, "conv": 1, "dwconv": 2}[kind]
        return cls(kind, *[int(getattr(layer, n)) for n in
                           ("M", "N", "Ci", "Co", "H", "W", "kh", "kw", "stride", "pad")])


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libdarknight.so (built in-tree by paper_2207_00083_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libdarknight.so is not built: run `python -m paper_2207_00083_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, ip, ll, sz, fl = C.c_void_p, C.c_int, C.c_longlong, C.c_size_t, C.c_float
    LP = C.POINTER(DkLayer)
    sig = {
        "dk_status_str": (C.c_char_p, [ip]),
        "dk_version": (ip, []),
        "dk_layer_in_len": (ll, [LP]),
        "dk_layer_out_len": (ll, [LP]),
        "dk_workspace_bytes": (sz, [LP, ip, ip, ip]),
        "dk_fwd_workspace_bytes": (sz, [LP, ll]),
        "dk_coeffs": (ip, [vp, vp, ip, ip, vp, vp, vp]),
        "dk_encode": (ip, [vp, vp, vp, vp, ip, ip, ll, vp]),
        "dk_linear_fwd": (ip, [vp, vp, vp, ip, ip, ip, vp, sz, vp]),
        "dk_conv_fwd": (ip, [LP, vp, vp, vp, ip, vp, sz, vp]),
        "dk_wgrad": (ip, [LP, vp, vp, vp, vp, vp, ip, ip, fl, ip, vp, sz, vp]),
        "dk_decode": (ip, [vp, vp, vp, ip, ip, ll, vp]),
        "dk_verify": (ip, [vp, vp, fl, vp, vp, ip, ip, ll, vp, sz, vp]),
        "dk_decode_verify": (ip, [vp, vp, vp, fl, vp, vp, vp, ip, ip, ll, vp, sz, vp]),
        "dk_conv_fwd_decode_verify": (ip, [LP, vp, vp, vp, vp, fl, vp, vp, vp, ip, ip, vp, sz, vp]),
        "dk_conv_fwd_decode_verify_workspace_bytes": (sz, [LP, ip, ip]),
        "dk_set_option": (ip, [ip, ip]),
        "dk_get_option": (ip, [ip]),
        "dk_decode_verify_static": (ip, [vp, vp, vp, fl, vp, vp, vp, ip, ip, ll, vp]),
        "dk_static_scratch_bytes": (sz, []),
        "dk_coeffs_m": (ip, [vp, vp, ip, ip, ip, vp, vp, vp]),
        "dk_encode_m": (ip, [vp, vp, vp, vp, ip, ip, ip, ll, vp]),
        "dk_decode_verify_m": (ip, [vp, vp, vp, fl, vp, vp, vp, ip, ip, ip, ll, vp, sz, vp]),
        "dk_wgrad_m": (ip, [LP, vp, vp, vp, vp, vp, ip, ip, ip, fl, ip, vp, sz, vp]),
        "dk_workspace_bytes_m": (sz, [LP, ip, ip, ip, ip]),
        "dk_dgrad": (ip, [LP, vp, vp, vp, ip, vp, sz, vp]),
        "dk_dgrad_workspace_bytes": (sz, [LP, ip]),
        "dk_noise_rng": (ip, [vp, ip, ip, ll, C.c_ulonglong, fl, vp]),
        "dk_encode_rng": (ip, [vp, vp, vp, ip, ip, ip, ll, C.c_ulonglong, fl, vp]),
        "dkf_noise_rng": (ip, [vp, ip, ll, C.c_ulonglong, vp]),
        "dkf_encode_rng": (ip, [vp, vp, vp, ip, ip, ll, ip, C.c_ulonglong, vp]),
        "dkf_coeffs": (ip, [vp, vp, ip, ip, vp, vp, vp]),
        "dkf_quantize": (ip, [vp, vp, ll, ip, vp]),
        "dkf_dequantize": (ip, [vp, vp, ll, ip, vp]),
        "dkf_encode": (ip, [vp, vp, vp, vp, ip, ip, ll, ip, vp]),
        "dkf_linear_fwd": (ip, [vp, vp, vp, ip, ip, ip, vp, sz, vp]),
        "dkf_linear_fwd_w": (ip, [vp, ip, vp, vp, ip, ip, ip, vp, sz, vp]),
        "dkf_decode_verify": (ip, [vp, vp, vp, vp, vp, vp, ip, ip, ll, ip, vp]),
        "dkf_wgrad": (ip, [LP, vp, vp, vp, vp, vp, vp, ip, ip, ip, fl, ip, vp, sz, vp]),
        "dkf_conv_fwd": (ip, [LP, vp, vp, vp, ip, vp, sz, vp]),
        "dkf_norm_scales": (ip, [vp, vp, ll, ll, fl, vp]),
        "dkf_quantize_norm": (ip, [vp, vp, vp, ll, ll, ip, vp]),
        "dkf_encode_norm": (ip, [vp, vp, vp, vp, vp, ip, ip, ll, ip, vp]),
        "dkf_encode_rng_norm": (ip, [vp, vp, vp, vp, ip, ip, ll, ip, C.c_ulonglong, vp]),
        "dkf_decode_verify_norm": (ip, [vp, vp, vp, vp, vp, vp, vp, vp, ip, ip, ll, ip, vp]),
        "dkf_wgrad_norm": (ip, [LP, vp, vp, vp, vp, vp, vp, vp, ip, ip, ip, fl, ip, vp, sz, vp]),
        "dkf_conv_fwd_workspace_bytes": (sz, [LP, ip]),
        "dkf_probe_mfma_rate": (ip, [ip, ip, vp, vp]),
        "dk_probe_mfma_rate": (ip, [ip, ip, vp, vp]),
        "dkf_add_bias": (ip, [vp, vp, vp, ll, ll, ll, ip, vp]),
        "dkf_coeffs_m": (ip, [vp, vp, ip, ip, ip, vp, vp, vp]),
        "dkf_encode_m": (ip, [vp, vp, vp, vp, ip, ip, ip, ll, ip, vp]),
        "dkf_decode_verify_m": (ip, [vp, vp, vp, vp, vp, vp, ip, ip, ip, ll, ip, vp]),
        "dkf_wgrad_m": (ip, [LP, vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, fl, ip, vp, sz, vp]),
        "dkf_wgrad_workspace_bytes_m": (sz, [LP, ip, ip, ip]),
        "dkf_fwd_workspace_bytes": (sz, [ip, ip, ip]),
        "dkf_wgrad_workspace_bytes": (sz, [LP, ip, ip]),
        "dk_profile_enable": (ip, [ip]),
        "dk_profile_read": (ip, [ip, C.c_char_p, ip, C.POINTER(C.c_double), C.POINTER(ip)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def dk_status_str(status) -> str:
    return load().dk_status_str(int(status)).decode()


def dk_version() -> int:
    return int(load().dk_version())


def _check(status, where):
    if status != 0:
        raise DkError(status, where)


def _torch():
    import torch
    return torch


def _dev(t, name):
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError("%s must be contiguous float32" % name)
    return t


def _stream(stream):
    if stream is None:
        stream = _torch().cuda.current_stream()
    return C.c_void_p(int(stream.cuda_stream))


def _ptr(t):
    return C.c_void_p(0 if t is None else int(t.data_ptr()))


def _workspace(nbytes, like, stream=None):
    """A temporary workspace for one call.  It is dropped when the call
    returns while its kernels may still be queued, so it has to come from the
    pool of the stream the kernels run on: the caching allocator then hands
    the block only to later work on that same stream."""
    torch = _torch()
    nbytes = max(int(nbytes), 256)
    if stream is None:
        return torch.empty(nbytes, dtype=torch.uint8, device=like.device)
    with torch.cuda.stream(stream):
        return torch.empty(nbytes, dtype=torch.uint8, device=like.device)


def _wshape(lay):
    if lay.kind == 0:
        return (lay.M, lay.N)
    if lay.kind == 2:
        return (lay.Ci, lay.kh, lay.kw)
    return (lay.Co, lay.Ci, lay.kh, lay.kw)


def dk_layer_in_len(layer) -> int:
    return int(load().dk_layer_in_len(C.byref(DkLayer.of(layer))))


def dk_layer_out_len(layer) -> int:
    return int(load().dk_layer_out_len(C.byref(DkLayer.of(layer))))


def dk_workspace_bytes(layer, op, G, K) -> int:
    lp = None if layer is None else C.byref(DkLayer.of(layer))
    return int(load().dk_workspace_bytes(lp, int(op), int(G), int(K)))


def dk_coeffs(A, gamma):
    """Host arrays A[G,S,S], gamma[G,S] (fp32) -> host Ainv[G,S,S], nvec[G,S], B[G,S,K]."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    gamma = np.ascontiguousarray(gamma, dtype=np.float32)
    G, S, _ = A.shape
    K = S - 2
    Ainv = np.empty((G, S, S), dtype=np.float32)
    nvec = np.empty((G, S), dtype=np.float32)
    B = np.empty((G, S, K), dtype=np.float32)
    _check(load().dk_coeffs(A.ctypes.data, gamma.ctypes.data, G, K, Ainv.ctypes.data,
                            nvec.ctypes.data, B.ctypes.data), "dk_coeffs")
    return Ainv, nvec, B


def dk_encode(x, r, A, K, xbar=None, stream=None):
    """x[G*K, ...], r[G, ...], A[G,S,S] (device) -> xbar[G*S, ...] (device)."""
    torch = _torch()
    x, r, A = _dev(x, "x"), _dev(r, "r"), _dev(A, "A")
    G = r.shape[0]
    S = K + 2
    n = x[0].numel()
    if x.shape[0] != G * K or A.shape != (G, S, S) or r[0].numel() != n:
        raise ValueError("dk_encode: inconsistent shapes")
    if xbar is None:
        xbar = torch.empty((G * S,) + tuple(x.shape[1:]), dtype=torch.float32, device=x.device)
    _dev(xbar, "xbar")
    if xbar.numel() != G * S * n:
        raise ValueError("dk_encode: xbar has the wrong size")
    _check(load().dk_encode(_ptr(x), _ptr(r), _ptr(A), _ptr(xbar), G, K, n, _stream(stream)),
           "dk_encode")
    return xbar


def dk_linear_fwd(W, xbar, ybar=None, ws=None, stream=None):
    """W[M,N], xbar[R,N] (device) -> ybar[R,M] (device)."""
    torch = _torch()
    W, xbar = _dev(W, "W"), _dev(xbar, "xbar")
    M, N = W.shape
    R = xbar.shape[0]
    if xbar[0].numel() != N:
        raise ValueError("dk_linear_fwd: inconsistent shapes")
    if ybar is None:
        ybar = torch.empty((R, M), dtype=torch.float32, device=W.device)
    _dev(ybar, "ybar")
    if ybar.numel() != R * M:
        raise ValueError("dk_linear_fwd: ybar has the wrong size")
    if ws is None:
        lay = DkLayer(0, M, N, 0, 0, 0, 0, 1, 1, 1, 0)
        ws = _workspace(_fwd_ws_bytes(lay, R), W, stream)
    _check(load().dk_linear_fwd(_ptr(W), _ptr(xbar), _ptr(ybar), M, N, R, _ptr(ws), ws.numel(),
                                _stream(stream)), "dk_linear_fwd")
    return ybar


def _fwd_ws_bytes(lay, R):
    return load().dk_fwd_workspace_bytes(C.byref(lay), R)


def dk_conv_fwd(layer, W, xbar, ybar=None, ws=None, stream=None):
    """W[Co,Ci,kh,kw], xbar[R,Ci,H,W] (device) -> ybar[R,Co,Ho,Wo] (device)."""
    torch = _torch()
    lay = DkLayer.of(layer)
    W, xbar = _dev(W, "W"), _dev(xbar, "xbar")
    R = xbar.shape[0]
    n, m = dk_layer_in_len(lay), dk_layer_out_len(lay)
    if n == 0:
        raise DkError(2, "dk_conv_fwd")
    if xbar[0].numel() != n or W.numel() != int(np.prod(_wshape(lay))):
        raise ValueError("dk_conv_fwd: inconsistent shapes")
    if ybar is None:
        Ho = (lay.H + 2 * lay.pad - lay.kh) // lay.stride + 1
        Wo = (lay.W + 2 * lay.pad - lay.kw) // lay.stride + 1
        ybar = torch.empty((R, lay.Co, Ho, Wo), dtype=torch.float32, device=W.device)
    _dev(ybar, "ybar")
    if ybar.numel() != R * m:
        raise ValueError("dk_conv_fwd: ybar has the wrong size")
    if ws is None:
        ws = _workspace(_fwd_ws_bytes(lay, R), W, stream)
    _check(load().dk_conv_fwd(C.byref(lay), _ptr(W), _ptr(xbar), _ptr(ybar), R, _ptr(ws),
                              ws.numel(), _stream(stream)), "dk_conv_fwd")
    return ybar


def dk_wgrad(layer, delta, B, gamma, xbar, K, dW=None, scale=1.0, accumulate=False, ws=None,
             stream=None):
    """delta[G*K, ...], B[G,S,K], gamma[G,S], xbar[G*S, ...] (device) -> dW (device)."""
    torch = _torch()
    lay = DkLayer.of(layer)
    delta, B, gamma, xbar = _dev(delta, "delta"), _dev(B, "B"), _dev(gamma, "gamma"), _dev(xbar, "xbar")
    G, S = gamma.shape
    n, m = dk_layer_in_len(lay), dk_layer_out_len(lay)
    if n == 0:
        raise DkError(2, "dk_wgrad")
    if (S != K + 2 or B.shape != (G, S, K) or delta.numel() != G * K * m
            or xbar.numel() != G * S * n):
        raise ValueError("dk_wgrad: inconsistent shapes")
    wshape = _wshape(lay)
    if dW is None:
        if accumulate:
            raise ValueError("dk_wgrad: accumulate needs an existing dW")
        dW = torch.empty(wshape, dtype=torch.float32, device=delta.device)
    _dev(dW, "dW")
    if dW.numel() != int(np.prod(wshape)):
        raise ValueError("dk_wgrad: dW has the wrong size")
    if ws is None:
        ws = _workspace(load().dk_workspace_bytes(C.byref(lay), DK_OP_WGRAD, G, K), delta, stream)
    _check(load().dk_wgrad(C.byref(lay), _ptr(delta), _ptr(B), _ptr(gamma), _ptr(xbar), _ptr(dW),
                           G, K, float(scale), int(bool(accumulate)), _ptr(ws), ws.numel(),
                           _stream(stream)), "dk_wgrad")
    return dW


def dk_decode(ybar, Ainv, K, y=None, stream=None):
    """ybar[G*S, ...], Ainv[G,S,S] (device) -> y[G*K, ...] (device)."""
    torch = _torch()
    ybar, Ainv = _dev(ybar, "ybar"), _dev(Ainv, "Ainv")
    G = Ainv.shape[0]
    S = K + 2
    if Ainv.shape != (G, S, S) or ybar.shape[0] != G * S:
        raise ValueError("dk_decode: inconsistent shapes")
    m = ybar[0].numel()
    if y is None:
        y = torch.empty((G * K,) + tuple(ybar.shape[1:]), dtype=torch.float32, device=ybar.device)
    _dev(y, "y")
    if y.numel() != G * K * m:
        raise ValueError("dk_decode: y has the wrong size")
    _check(load().dk_decode(_ptr(ybar), _ptr(Ainv), _ptr(y), G, K, m, _stream(stream)), "dk_decode")
    return y


def dk_verify(ybar, nvec, K, tol=1e-3, verdict=None, resid=None, ws=None, stream=None):
    """ybar[G*S, ...], nvec[G,S] (device) -> (verdict[G] int32, resid[G] fp32) (device)."""
    torch = _torch()
    ybar, nvec = _dev(ybar, "ybar"), _dev(nvec, "nvec")
    G, S = nvec.shape
    if S != K + 2 or ybar.shape[0] != G * S:
        raise ValueError("dk_verify: inconsistent shapes")
    m = ybar[0].numel()
    if verdict is None:
        verdict = torch.empty(G, dtype=torch.int32, device=ybar.device)
    if resid is None:
        resid = torch.empty(G, dtype=torch.float32, device=ybar.device)
    if ws is None:
        ws = _workspace(load().dk_workspace_bytes(None, DK_OP_VERIFY, G, K), ybar, stream)
    _check(load().dk_verify(_ptr(ybar), _ptr(nvec), float(tol), _ptr(verdict), _ptr(resid), G, K, m,
                            _ptr(ws), ws.numel(), _stream(stream)), "dk_verify")
    return verdict, resid


def dk_decode_verify(ybar, Ainv, nvec, K, tol=1e-3, y=None, verdict=None, resid=None, ws=None,
                     stream=None):
    """dk_decode and dk_verify in one sweep: returns (y, verdict, resid)."""
    torch = _torch()
    ybar, Ainv, nvec = _dev(ybar, "ybar"), _dev(Ainv, "Ainv"), _dev(nvec, "nvec")
    G = Ainv.shape[0]
    S = K + 2
    if Ainv.shape != (G, S, S) or nvec.shape != (G, S) or ybar.shape[0] != G * S:
        raise ValueError("dk_decode_verify: inconsistent shapes")
    m = ybar[0].numel()
    if y is None:
        y = torch.empty((G * K,) + tuple(ybar.shape[1:]), dtype=torch.float32, device=ybar.device)
    _dev(y, "y")
    if y.numel() != G * K * m:
        raise ValueError("dk_decode_verify: y has the wrong size")
    if verdict is None:
        verdict = torch.empty(G, dtype=torch.int32, device=ybar.device)
    if resid is None:
        resid = torch.empty(G, dtype=torch.float32, device=ybar.device)
    if ws is None:
        ws = _workspace(load().dk_workspace_bytes(None, DK_OP_VERIFY, G, K), ybar, stream)
    _check(load().dk_decode_verify(_ptr(ybar), _ptr(Ainv), _ptr(nvec), float(tol), _ptr(y), _ptr(verdict),
                                   _ptr(resid), G, K, m, _ptr(ws), ws.numel(), _stream(stream)),
           "dk_decode_verify")
    return y, verdict, resid


def dk_conv_fwd_decode_verify(layer, W, xbar, Ainv, nvec, K, tol=1e-3, y=None, verdict=None, resid=None,
                              ws=None, stream=None):
    """dk_conv_fwd + dk_decode_verify as one call: returns (y, verdict, resid)."""
    torch = _torch()
    lay = DkLayer.of(layer)
    W, xbar, Ainv, nvec = _dev(W, "W"), _dev(xbar, "xbar"), _dev(Ainv, "Ainv"), _dev(nvec, "nvec")
    G = Ainv.shape[0]
    S = K + 2
    n, m = dk_layer_in_len(lay), dk_layer_out_len(lay)
    if n == 0:
        raise DkError(2, "dk_conv_fwd_decode_verify")
    if (Ainv.shape != (G, S, S) or nvec.shape != (G, S) or xbar.numel() != G * S * n
            or W.numel() != int(np.prod(_wshape(lay)))):
        raise ValueError("dk_conv_fwd_decode_verify: inconsistent shapes")
    if y is None:
        Ho = (lay.H + 2 * lay.pad - lay.kh) // lay.stride + 1
        Wo = (lay.W + 2 * lay.pad - lay.kw) // lay.stride + 1
        y = torch.empty((G * K, lay.Co, Ho, Wo), dtype=torch.float32, device=W.device)
    _dev(y, "y")
    if y.numel() != G * K * m:
        raise ValueError("dk_conv_fwd_decode_verify: y has the wrong size")
    if verdict is None:
        verdict = torch.empty(G, dtype=torch.int32, device=W.device)
    if resid is None:
        resid = torch.empty(G, dtype=torch.float32, device=W.device)
    if ws is None:
        ws = _workspace(load().dk_conv_fwd_decode_verify_workspace_bytes(C.byref(lay), G, K), W, stream)
    _check(load().dk_conv_fwd_decode_verify(C.byref(lay), _ptr(W), _ptr(xbar), _ptr(Ainv), _ptr(nvec),
                                            float(tol), _ptr(y), _ptr(verdict), _ptr(resid), G, K, _ptr(ws),
                                            ws.numel(), _stream(stream)), "dk_conv_fwd_decode_verify")
    return y, verdict, resid


def dk_conv_fwd_decode_verify_workspace_bytes(layer, G, K) -> int:
    return int(load().dk_conv_fwd_decode_verify_workspace_bytes(C.byref(DkLayer.of(layer)), int(G), int(K)))


def dk_set_option(which, value):
    """DK_OPT_FUSE_FWD / DK_OPT_FUSE_WGRAD <- DK_FUSE_NEVER / DK_FUSE_ALWAYS / DK_FUSE_AUTO."""
    _check(load().dk_set_option(int(which), int(value)), "dk_set_option")


def dk_get_option(which) -> int:
    return int(load().dk_get_option(int(which)))


def dk_decode_verify_static(ybar, Ainv, nvec, K, y, verdict, resid=None, tol=1e-3, stream=None):
    """dk_decode_verify without a workspace and without any allocation: the
    caller passes every output (resid may be None)."""
    ybar, Ainv, nvec, y = _dev(ybar, "ybar"), _dev(Ainv, "Ainv"), _dev(nvec, "nvec"), _dev(y, "y")
    G = Ainv.shape[0]
    S = K + 2
    if Ainv.shape != (G, S, S) or nvec.shape != (G, S) or ybar.shape[0] != G * S:
        raise ValueError("dk_decode_verify_static: inconsistent shapes")
    m = ybar[0].numel()
    if y.numel() != G * K * m or verdict.numel() != G or (resid is not None and resid.numel() != G):
        raise ValueError("dk_decode_verify_static: an output has the wrong size")
    _check(load().dk_decode_verify_static(_ptr(ybar), _ptr(Ainv), _ptr(nvec), float(tol), _ptr(y),
                                          _ptr(verdict), _ptr(resid), G, K, m, _stream(stream)),
           "dk_decode_verify_static")
    return y, verdict, resid


def dk_static_scratch_bytes() -> int:
    return int(load().dk_static_scratch_bytes())


# ---- several colluding accelerators: M noise rows per group, S = K+M+1 ----

def dk_coeffs_m(A, gamma, K):
    """Host arrays A[G,S,S], gamma[G,S] (fp32), S = K+M+1 -> Ainv[G,S,S], nvec[G,S], B[G,S,K]."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    gamma = np.ascontiguousarray(gamma, dtype=np.float32)
    G, S, _ = A.shape
    M = S - K - 1
    Ainv = np.empty((G, S, S), dtype=np.float32)
    nvec = np.empty((G, S), dtype=np.float32)
    B = np.empty((G, S, K), dtype=np.float32)
    _check(load().dk_coeffs_m(A.ctypes.data, gamma.ctypes.data, G, K, M, Ainv.ctypes.data,
                              nvec.ctypes.data, B.ctypes.data), "dk_coeffs_m")
    return Ainv, nvec, B


def dk_encode_m(x, r, A, K, M, xbar=None, stream=None):
    """x[G*K, ...], r[G*M, ...], A[G,S,S] (device) -> xbar[G*S, ...] (device)."""
    torch = _torch()
    x, r, A = _dev(x, "x"), _dev(r, "r"), _dev(A, "A")
    G = A.shape[0]
    S = K + M + 1
    n = x[0].numel()
    if x.shape[0] != G * K or r.shape[0] != G * M or A.shape != (G, S, S) or r[0].numel() != n:
        raise ValueError("dk_encode_m: inconsistent shapes")
    if xbar is None:
        xbar = torch.empty((G * S,) + tuple(x.shape[1:]), dtype=torch.float32, device=x.device)
    _dev(xbar, "xbar")
    if xbar.numel() != G * S * n:
        raise ValueError("dk_encode_m: xbar has the wrong size")
    _check(load().dk_encode_m(_ptr(x), _ptr(r), _ptr(A), _ptr(xbar), G, K, M, n, _stream(stream)),
           "dk_encode_m")
    return xbar


def dk_decode_verify_m(ybar, Ainv, nvec, K, M, tol=1e-3, y=None, verdict=None, resid=None, ws=None,
                       stream=None):
    """Returns (y[G*K, ...], verdict[G], resid[G])."""
    torch = _torch()
    ybar, Ainv, nvec = _dev(ybar, "ybar"), _dev(Ainv, "Ainv"), _dev(nvec, "nvec")
    G = Ainv.shape[0]
    S = K + M + 1
    if Ainv.shape != (G, S, S) or nvec.shape != (G, S) or ybar.shape[0] != G * S:
        raise ValueError("dk_decode_verify_m: inconsistent shapes")
    m = ybar[0].numel()
    if y is None:
        y = torch.empty((G * K,) + tuple(ybar.shape[1:]), dtype=torch.float32, device=ybar.device)
    _dev(y, "y")
    if y.numel() != G * K * m:
        raise ValueError("dk_decode_verify_m: y has the wrong size")
    if verdict is None:
        verdict = torch.empty(G, dtype=torch.int32, device=ybar.device)
    if resid is None:
        resid = torch.empty(G, dtype=torch.float32, device=ybar.device)
    if ws is None:
        ws = _workspace(load().dk_workspace_bytes_m(None, DK_OP_VERIFY, G, K, M), ybar, stream)
    _check(load().dk_decode_verify_m(_ptr(ybar), _ptr(Ainv), _ptr(nvec), float(tol), _ptr(y), _ptr(verdict),
                                     _ptr(resid), G, K, M, m, _ptr(ws), ws.numel(), _stream(stream)),
           "dk_decode_verify_m")
    return y, verdict, resid


def dk_wgrad_m(layer, delta, B, gamma, xbar, K, M, dW=None, scale=1.0, accumulate=False, ws=None,
               stream=None):
    """delta[G*K, ...], B[G,S,K], gamma[G,S], xbar[G*S, ...] (device) -> dW (device)."""
    torch = _torch()
    lay = DkLayer.of(layer)
    delta, B, gamma, xbar = _dev(delta, "delta"), _dev(B, "B"), _dev(gamma, "gamma"), _dev(xbar, "xbar")
    G, S = gamma.shape
    n, m = dk_layer_in_len(lay), dk_layer_out_len(lay)
    if n == 0:
        raise DkError(2, "dk_wgrad_m")
    if (S != K + M + 1 or B.shape != (G, S, K) or delta.numel() != G * K * m
            or xbar.numel() != G * S * n):
        raise ValueError("dk_wgrad_m: inconsistent shapes")
    wshape = _wshape(lay)
    if dW is None:
        if accumulate:
            raise ValueError("dk_wgrad_m: accumulate needs an existing dW")
        dW = torch.empty(wshape, dtype=torch.float32, device=delta.device)
    _dev(dW, "dW")
    if dW.numel() != int(np.prod(wshape)):
        raise ValueError("dk_wgrad_m: dW has the wrong size")
    if ws is None:
        ws = _workspace(load().dk_workspace_bytes_m(C.byref(lay), DK_OP_WGRAD, G, K, M), delta, stream)
    _check(load().dk_wgrad_m(C.byref(lay), _ptr(delta), _ptr(B), _ptr(gamma), _ptr(xbar), _ptr(dW),
                             G, K, M, float(scale), int(bool(accumulate)), _ptr(ws), ws.numel(),
                             _stream(stream)), "dk_wgrad_m")
    return dW


def dk_dgrad(layer, W, delta, dx=None, ws=None, stream=None):
    """Un-encoded data gradient: W (layer's weight shape), delta[R, ...out] -> dx[R, ...in] (device)."""
    torch = _torch()
    lay = DkLayer.of(layer)
    W, delta = _dev(W, "W"), _dev(delta, "delta")
    R = delta.shape[0]
    n, m = dk_layer_in_len(lay), dk_layer_out_len(lay)
    if n == 0:
        raise DkError(2, "dk_dgrad")
    if delta[0].numel() != m or W.numel() != int(np.prod(_wshape(lay))):
        raise ValueError("dk_dgrad: inconsistent shapes")
    if dx is None:
        shape = (R, lay.N) if lay.kind == 0 else (R, lay.Ci, lay.H, lay.W)
        dx = torch.empty(shape, dtype=torch.float32, device=W.device)
    _dev(dx, "dx")
    if dx.numel() != R * n:
        raise ValueError("dk_dgrad: dx has the wrong size")
    if ws is None:
        ws = _workspace(load().dk_dgrad_workspace_bytes(C.byref(lay), R), W, stream)
    _check(load().dk_dgrad(C.byref(lay), _ptr(W), _ptr(delta), _ptr(dx), R, _ptr(ws), ws.numel(),
                           _stream(stream)), "dk_dgrad")
    return dx


# ---- noise drawn by the library's counter-based generator ----

def dk_noise_rng(G, M, feat, seed, noise_std, device="cuda", stream=None):
    """r[G*M, *feat] (device): the noise rows the seed stands for."""
    torch = _torch()
    feat = tuple(int(v) for v in np.atleast_1d(feat))
    r = torch.empty((G * M,) + feat, dtype=torch.float32, device=device)
    _check(load().dk_noise_rng(_ptr(r), G, M, int(np.prod(feat)), int(seed), float(noise_std),
                               _stream(stream)), "dk_noise_rng")
    return r


def dk_encode_rng(x, A, K, M, seed, noise_std, xbar=None, stream=None):
    """x[G*K, ...], A[G,S,S] (device), S = K+M+1 -> xbar[G*S, ...]; noise from the seed."""
    torch = _torch()
    x, A = _dev(x, "x"), _dev(A, "A")
    G = A.shape[0]
    S = K + M + 1
    n = x[0].numel()
    if x.shape[0] != G * K or A.shape != (G, S, S):
        raise ValueError("dk_encode_rng: inconsistent shapes")
    if xbar is None:
        xbar = torch.empty((G * S,) + tuple(x.shape[1:]), dtype=torch.float32, device=x.device)
    _dev(xbar, "xbar")
    if xbar.numel() != G * S * n:
        raise ValueError("dk_encode_rng: xbar has the wrong size")
    _check(load().dk_encode_rng(_ptr(x), _ptr(A), _ptr(xbar), G, K, M, n, int(seed), float(noise_std),
                                _stream(stream)), "dk_encode_rng")
    return xbar


def dk_profile_enable(on=True):
    """Start (clearing old records) or stop per-kernel event timing."""
    _check(load().dk_profile_enable(1 if on else 0), "dk_profile_enable")


def dk_probe_mfma_rate(random_operands, iterations=20000, stream=None):
    """Launches the fp32 matrix-instruction rate probe; returns the FLOP of the launch."""
    flop = C.c_double(0.0)
    _check(load().dk_probe_mfma_rate(int(random_operands), int(iterations), C.byref(flop), _stream(stream)),
           "dk_probe_mfma_rate")
    return flop.value


def dk_profile_read():
    """{kernel label: (average launch ms, launches)} of the recorded launches."""
    lib = load()
    n = lib.dk_profile_read(-1, None, 0, None, None)
    out = {}
    for i in range(n):
        name = C.create_string_buffer(128)
        ms, cnt = C.c_double(0.0), C.c_int(0)
        lib.dk_profile_read(i, name, 128, C.byref(ms), C.byref(cnt))
        out[name.value.decode()] = (ms.value, cnt.value)
    return out
