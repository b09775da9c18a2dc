"""ctypes binding of the finite-field entry points (include/darknight_field.h).

Argument marshalling only.  Field elements travel as 4-byte integer tensors:
torch.int32 on the device (every element is below 2^25, so the bit pattern
equals the uint32 the C ABI names) and numpy uint32 on the host.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .binding import (DkError, DkLayer, _check, _dev, _ptr, _stream, _torch, _workspace, dk_layer_in_len,
                      dk_layer_out_len, load)

DKF_P = (1 << 25) - 39
DKF_L = 8


def _fe(t, name):
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype not in (torch.int32, torch.uint32) or not t.is_contiguous():
        raise TypeError("%s must be a contiguous 4-byte integer tensor" % name)
    return t


def _new_fe(shape, like):
    torch = _torch()
    return torch.empty(shape, dtype=torch.int32, device=like.device)


def _scales(t, count, name):
    """A float32 device tensor of `count` normalisation factors, or None."""
    if t is None:
        return None
    t = _dev(t, name)
    if t.numel() != count:
        raise ValueError("%s must hold %d factors" % (name, count))
    return t


def dkf_norm_scales(x, limit, rows=None, scale=None, stream=None):
    """One normalisation factor per row of x (device): 1/max|row| when that
    maximum exceeds `limit`, else 1.  rows defaults to x.shape[0]; rows=1 treats
    the whole tensor (a weight tensor) as one vector."""
    torch = _torch()
    x = _dev(x, "x")
    rows = int(x.shape[0] if rows is None else rows)
    if rows < 1 or x.numel() % rows:
        raise ValueError("dkf_norm_scales: rows does not divide the tensor")
    if scale is None:
        scale = torch.empty(rows, dtype=torch.float32, device=x.device)
    _scales(scale, rows, "scale")
    _check(load().dkf_norm_scales(_ptr(x), _ptr(scale), rows, x.numel() // rows, float(limit),
                                  _stream(stream)), "dkf_norm_scales")
    return scale


def dkf_coeffs(A, gamma):
    """Host arrays A[G,S,S], gamma[G,S] (uint32 field elements) ->
    host Ainv[G,S,S], nvec[G,S], B[G,S,K] (uint32)."""
    A = np.ascontiguousarray(A, dtype=np.uint32)
    gamma = np.ascontiguousarray(gamma, dtype=np.uint32)
    G, S, _ = A.shape
    K = S - 2
    Ainv = np.empty((G, S, S), dtype=np.uint32)
    nvec = np.empty((G, S), dtype=np.uint32)
    B = np.empty((G, S, K), dtype=np.uint32)
    _check(load().dkf_coeffs(A.ctypes.data, gamma.ctypes.data, G, K, Ainv.ctypes.data,
                             nvec.ctypes.data, B.ctypes.data), "dkf_coeffs")
    return Ainv, nvec, B


def dkf_quantize(x, l=DKF_L, xq=None, stream=None, scale=None):
    """scale (device, one factor per row; numel gives the number of rows)
    selects dkf_quantize_norm."""
    x = _dev(x, "x")
    if xq is None:
        xq = _new_fe(tuple(x.shape), x)
    _fe(xq, "xq")
    if xq.numel() != x.numel():
        raise ValueError("dkf_quantize: xq has the wrong size")
    if scale is not None:
        rows = _dev(scale, "scale").numel()
        if rows < 1 or x.numel() % rows:
            raise ValueError("dkf_quantize: the number of factors does not divide the tensor")
        _check(load().dkf_quantize_norm(_ptr(x), _ptr(scale), _ptr(xq), rows, x.numel() // rows, int(l),
                                        _stream(stream)), "dkf_quantize_norm")
        return xq
    _check(load().dkf_quantize(_ptr(x), _ptr(xq), x.numel(), int(l), _stream(stream)), "dkf_quantize")
    return xq


def dkf_dequantize(yq, l=DKF_L, y=None, stream=None):
    torch = _torch()
    yq = _fe(yq, "yq")
    if y is None:
        y = torch.empty(tuple(yq.shape), dtype=torch.float32, device=yq.device)
    _dev(y, "y")
    if y.numel() != yq.numel():
        raise ValueError("dkf_dequantize: y has the wrong size")
    _check(load().dkf_dequantize(_ptr(yq), _ptr(y), yq.numel(), int(l), _stream(stream)), "dkf_dequantize")
    return y


def dkf_encode(x, r, A, K, l=DKF_L, xbar=None, stream=None, xscale=None):
    """x[G*K, ...] float, r[G, ...], A[G,S,S] field elements (device) -> xbar[G*S, ...].
    xscale[G*K] (device) selects dkf_encode_norm."""
    x, r, A = _dev(x, "x"), _fe(r, "r"), _fe(A, "A")
    G, S = r.shape[0], K + 2
    n = x[0].numel()
    if x.shape[0] != G * K or tuple(A.shape) != (G, S, S) or r[0].numel() != n:
        raise ValueError("dkf_encode: inconsistent shapes")
    if xbar is None:
        xbar = _new_fe((G * S,) + tuple(x.shape[1:]), x)
    _fe(xbar, "xbar")
    if xbar.numel() != G * S * n:
        raise ValueError("dkf_encode: xbar has the wrong size")
    if xscale is not None:
        _scales(xscale, G * K, "xscale")
        _check(load().dkf_encode_norm(_ptr(x), _ptr(xscale), _ptr(r), _ptr(A), _ptr(xbar), G, K, n, int(l),
                                      _stream(stream)), "dkf_encode_norm")
        return xbar
    _check(load().dkf_encode(_ptr(x), _ptr(r), _ptr(A), _ptr(xbar), G, K, n, int(l), _stream(stream)),
           "dkf_encode")
    return xbar


def dkf_noise_rng(G, feat, seed, device="cuda", stream=None):
    """r[G, *feat] (device, field elements): the uniform noise the seed stands for."""
    torch = _torch()
    feat = tuple(int(v) for v in np.atleast_1d(feat))
    r = torch.empty((G,) + feat, dtype=torch.int32, device=device)
    _check(load().dkf_noise_rng(_ptr(r), G, int(np.prod(feat)), int(seed), _stream(stream)), "dkf_noise_rng")
    return r


def dkf_encode_rng(x, A, K, seed, l=DKF_L, xbar=None, stream=None, xscale=None):
    """x[G*K, ...] float, A[G,S,S] field elements (device) -> xbar[G*S, ...]; noise from the seed.
    xscale[G*K] (device) selects dkf_encode_rng_norm."""
    x, A = _dev(x, "x"), _fe(A, "A")
    G, S = A.shape[0], K + 2
    n = x[0].numel()
    if x.shape[0] != G * K or tuple(A.shape) != (G, S, S):
        raise ValueError("dkf_encode_rng: inconsistent shapes")
    if xbar is None:
        xbar = _new_fe((G * S,) + tuple(x.shape[1:]), x)
    _fe(xbar, "xbar")
    if xbar.numel() != G * S * n:
        raise ValueError("dkf_encode_rng: xbar has the wrong size")
    if xscale is not None:
        _scales(xscale, G * K, "xscale")
        _check(load().dkf_encode_rng_norm(_ptr(x), _ptr(xscale), _ptr(A), _ptr(xbar), G, K, n, int(l), int(seed),
                                          _stream(stream)), "dkf_encode_rng_norm")
        return xbar
    _check(load().dkf_encode_rng(_ptr(x), _ptr(A), _ptr(xbar), G, K, n, int(l), int(seed), _stream(stream)),
           "dkf_encode_rng")
    return xbar


def dkf_fwd_workspace_bytes(M, N, R) -> int:
    return int(load().dkf_fwd_workspace_bytes(int(M), int(N), int(R)))


def dkf_wgrad_workspace_bytes(layer, G, K) -> int:
    return int(load().dkf_wgrad_workspace_bytes(C.byref(DkLayer.of(layer)), int(G), int(K)))


def dkf_linear_fwd(Wq, xbar, ybar=None, ws=None, stream=None):
    """Wq[M,N], xbar[R,N] field elements (device) -> ybar[R,M]."""
    Wq, xbar = _fe(Wq, "Wq"), _fe(xbar, "xbar")
    M, N = Wq.shape
    R = xbar.shape[0]
    if xbar[0].numel() != N:
        raise ValueError("dkf_linear_fwd: inconsistent shapes")
    if ybar is None:
        ybar = _new_fe((R, M), Wq)
    _fe(ybar, "ybar")
    if ybar.numel() != R * M:
        raise ValueError("dkf_linear_fwd: ybar has the wrong size")
    if ws is None:
        ws = _workspace(dkf_fwd_workspace_bytes(M, N, R), Wq, stream)
    _check(load().dkf_linear_fwd(_ptr(Wq), _ptr(xbar), _ptr(ybar), M, N, R, _ptr(ws), ws.numel(),
                                 _stream(stream)), "dkf_linear_fwd")
    return ybar


def dkf_linear_fwd_w(W, xbar, l=DKF_L, ybar=None, ws=None, stream=None):
    """W[M,N] float, xbar[R,N] field elements (device) -> ybar[R,M]; the weights are quantised on the way."""
    W, xbar = _dev(W, "W"), _fe(xbar, "xbar")
    M, N = W.shape
    R = xbar.shape[0]
    if xbar[0].numel() != N:
        raise ValueError("dkf_linear_fwd_w: inconsistent shapes")
    if ybar is None:
        ybar = _new_fe((R, M), xbar)
    _fe(ybar, "ybar")
    if ybar.numel() != R * M:
        raise ValueError("dkf_linear_fwd_w: ybar has the wrong size")
    if ws is None:
        ws = _workspace(dkf_fwd_workspace_bytes(M, N, R), xbar, stream)
    _check(load().dkf_linear_fwd_w(_ptr(W), int(l), _ptr(xbar), _ptr(ybar), M, N, R, _ptr(ws), ws.numel(),
                                   _stream(stream)), "dkf_linear_fwd_w")
    return ybar


def dkf_conv_fwd_workspace_bytes(layer, R) -> int:
    return int(load().dkf_conv_fwd_workspace_bytes(C.byref(DkLayer.of(layer)), int(R)))


def dkf_conv_fwd(layer, Wq, xbar, ybar=None, ws=None, stream=None):
    """Wq[Co,Ci,kh,kw], xbar[R,Ci,H,W] field elements (device) -> ybar[R,Co,Ho,Wo]."""
    lay = DkLayer.of(layer)
    Wq, xbar = _fe(Wq, "Wq"), _fe(xbar, "xbar")
    R = xbar.shape[0]
    Ho = (lay.H + 2 * lay.pad - lay.kh) // lay.stride + 1
    Wo = (lay.W + 2 * lay.pad - lay.kw) // lay.stride + 1
    wcount = lay.Ci * lay.kh * lay.kw if lay.kind == 2 else lay.Co * lay.Ci * lay.kh * lay.kw
    if xbar[0].numel() != lay.Ci * lay.H * lay.W or Wq.numel() != wcount:
        raise ValueError("dkf_conv_fwd: inconsistent shapes")
    if ybar is None:
        ybar = _new_fe((R, lay.Co, Ho, Wo), Wq)
    _fe(ybar, "ybar")
    if ybar.numel() != R * lay.Co * Ho * Wo:
        raise ValueError("dkf_conv_fwd: ybar has the wrong size")
    if ws is None:
        ws = _workspace(dkf_conv_fwd_workspace_bytes(lay, R), Wq, stream)
    _check(load().dkf_conv_fwd(C.byref(lay), _ptr(Wq), _ptr(xbar), _ptr(ybar), R, _ptr(ws), ws.numel(),
                               _stream(stream)), "dkf_conv_fwd")
    return ybar


def dkf_decode_verify(ybar, Ainv, nvec, K, l=DKF_L, y=None, yq=None, verdict=None, want_yq=False,
                      stream=None, xscale=None, wscale=None):
    """Returns (y float, yq or None, verdict int32).  xscale[G*K] and wscale[1]
    (device, both or neither) select dkf_decode_verify_norm."""
    torch = _torch()
    ybar, Ainv, nvec = _fe(ybar, "ybar"), _fe(Ainv, "Ainv"), _fe(nvec, "nvec")
    G, S = Ainv.shape[0], K + 2
    if tuple(Ainv.shape) != (G, S, S) or tuple(nvec.shape) != (G, S) or ybar.shape[0] != G * S:
        raise ValueError("dkf_decode_verify: inconsistent shapes")
    m = ybar[0].numel()
    if y is None:
        y = torch.empty((G * K,) + tuple(ybar.shape[1:]), dtype=torch.float32, device=ybar.device)
    _dev(y, "y")
    if yq is None and want_yq:
        yq = _new_fe(tuple(y.shape), ybar)
    if yq is not None:
        _fe(yq, "yq")
    if y.numel() != G * K * m or (yq is not None and yq.numel() != G * K * m):
        raise ValueError("dkf_decode_verify: output has the wrong size")
    if verdict is None:
        verdict = torch.empty(G, dtype=torch.int32, device=ybar.device)
    if (xscale is None) != (wscale is None):
        raise ValueError("dkf_decode_verify: xscale and wscale come together")
    if xscale is not None:
        _scales(xscale, G * K, "xscale")
        _scales(wscale, 1, "wscale")
        _check(load().dkf_decode_verify_norm(_ptr(ybar), _ptr(Ainv), _ptr(nvec), _ptr(xscale), _ptr(wscale),
                                             _ptr(y), _ptr(yq), _ptr(verdict), G, K, m, int(l),
                                             _stream(stream)), "dkf_decode_verify_norm")
        return y, yq, verdict
    _check(load().dkf_decode_verify(_ptr(ybar), _ptr(Ainv), _ptr(nvec), _ptr(y), _ptr(yq), _ptr(verdict),
                                    G, K, m, int(l), _stream(stream)), "dkf_decode_verify")
    return y, yq, verdict


def dkf_wgrad(layer, delta, B, gamma, xbar, K, l=DKF_L, dW=None, dwq=None, want_dwq=False, scale=1.0,
              accumulate=False, ws=None, stream=None, xscale=None):
    """delta[G*K, ...] float, B[G,S,K], gamma[G,S], xbar[G*S, ...] (device) -> (dW float, dwq or None).
    xscale[G*K] (device, the factors the encodings were made with) selects dkf_wgrad_norm."""
    torch = _torch()
    lay = DkLayer.of(layer)
    delta, B, gamma, xbar = _dev(delta, "delta"), _fe(B, "B"), _fe(gamma, "gamma"), _fe(xbar, "xbar")
    G, S = gamma.shape
    n, m = dk_layer_in_len(lay), dk_layer_out_len(lay)
    if n == 0:
        raise DkError(2, "dkf_wgrad")
    if (S != K + 2 or tuple(B.shape) != (G, S, K) or delta.numel() != G * K * m
            or xbar.numel() != G * S * n):
        raise ValueError("dkf_wgrad: inconsistent shapes")
    wshape = ((lay.M, lay.N) if lay.kind == 0 else (lay.Ci, lay.kh, lay.kw) if lay.kind == 2
              else (lay.Co, lay.Ci, lay.kh, lay.kw))
    wcount = int(np.prod(wshape))
    if dW is None:
        if accumulate:
            raise ValueError("dkf_wgrad: accumulate needs an existing dW")
        dW = torch.empty(wshape, dtype=torch.float32, device=delta.device)
    _dev(dW, "dW")
    if dwq is None and want_dwq:
        dwq = _new_fe(wshape, delta)
    if dwq is not None:
        _fe(dwq, "dwq")
    if dW.numel() != wcount or (dwq is not None and dwq.numel() != wcount):
        raise ValueError("dkf_wgrad: output has the wrong size")
    if ws is None:
        ws = _workspace(dkf_wgrad_workspace_bytes(lay, G, K), delta, stream)
    if xscale is not None:
        _scales(xscale, G * K, "xscale")
        _check(load().dkf_wgrad_norm(C.byref(lay), _ptr(delta), _ptr(xscale), _ptr(B), _ptr(gamma), _ptr(xbar),
                                     _ptr(dW), _ptr(dwq), G, K, int(l), float(scale), int(bool(accumulate)),
                                     _ptr(ws), ws.numel(), _stream(stream)), "dkf_wgrad_norm")
        return dW, dwq
    _check(load().dkf_wgrad(C.byref(lay), _ptr(delta), _ptr(B), _ptr(gamma), _ptr(xbar), _ptr(dW),
                            _ptr(dwq), G, K, int(l), float(scale), int(bool(accumulate)), _ptr(ws),
                            ws.numel(), _stream(stream)), "dkf_wgrad")
    return dW, dwq


def dkf_add_bias(yq, bias, per, l=DKF_L, y=None, want_y=True, stream=None):
    """yq[rows, ...] field elements (device, updated in place) += Field(Round(bias 2^{2l}))[e // per];
    returns (yq, y) with y the de-quantised sums (None if want_y is False)."""
    torch = _torch()
    yq, bias = _fe(yq, "yq"), _dev(bias, "bias")
    rows = yq.shape[0]
    m = yq[0].numel()
    if bias.numel() * per != m:
        raise ValueError("dkf_add_bias: bias does not fit the rows")
    if y is None and want_y:
        y = torch.empty(tuple(yq.shape), dtype=torch.float32, device=yq.device)
    if y is not None:
        _dev(y, "y")
        if y.numel() != yq.numel():
            raise ValueError("dkf_add_bias: y has the wrong size")
    _check(load().dkf_add_bias(_ptr(yq), _ptr(y), _ptr(bias), rows, m, int(per), int(l), _stream(stream)),
           "dkf_add_bias")
    return yq, y


def dkf_probe_mfma_rate(random_operands, iterations=20000, stream=None):
    """Launches the int8 matrix-instruction rate probe; returns the int8 operations of the launch."""
    ops = C.c_double(0.0)
    _check(load().dkf_probe_mfma_rate(int(random_operands), int(iterations), C.byref(ops), _stream(stream)),
           "dkf_probe_mfma_rate")
    return ops.value


# ---- several colluding accelerators: M noise rows per group, S = K+M+1 ----

def dkf_coeffs_m(A, gamma, K):
    """Host arrays A[G,S,S], gamma[G,S] (uint32), S = K+M+1 -> Ainv[G,S,S], nvec[G,S], B[G,S,K]."""
    A = np.ascontiguousarray(A, dtype=np.uint32)
    gamma = np.ascontiguousarray(gamma, dtype=np.uint32)
    G, S, _ = A.shape
    M = S - K - 1
    Ainv = np.empty((G, S, S), dtype=np.uint32)
    nvec = np.empty((G, S), dtype=np.uint32)
    B = np.empty((G, S, K), dtype=np.uint32)
    _check(load().dkf_coeffs_m(A.ctypes.data, gamma.ctypes.data, G, K, M, Ainv.ctypes.data,
                               nvec.ctypes.data, B.ctypes.data), "dkf_coeffs_m")
    return Ainv, nvec, B


def dkf_encode_m(x, r, A, K, M, l=DKF_L, xbar=None, stream=None):
    """x[G*K, ...] float, r[G*M, ...], A[G,S,S] field elements (device) -> xbar[G*S, ...]."""
    x, r, A = _dev(x, "x"), _fe(r, "r"), _fe(A, "A")
    G, S = A.shape[0], K + M + 1
    n = x[0].numel()
    if x.shape[0] != G * K or r.shape[0] != G * M or tuple(A.shape) != (G, S, S) or r[0].numel() != n:
        raise ValueError("dkf_encode_m: inconsistent shapes")
    if xbar is None:
        xbar = _new_fe((G * S,) + tuple(x.shape[1:]), x)
    _fe(xbar, "xbar")
    if xbar.numel() != G * S * n:
        raise ValueError("dkf_encode_m: xbar has the wrong size")
    _check(load().dkf_encode_m(_ptr(x), _ptr(r), _ptr(A), _ptr(xbar), G, K, M, n, int(l), _stream(stream)),
           "dkf_encode_m")
    return xbar


def dkf_decode_verify_m(ybar, Ainv, nvec, K, M, l=DKF_L, y=None, yq=None, verdict=None, want_yq=False,
                        stream=None):
    """Returns (y float [G*K, ...], yq or None, verdict int32 [G])."""
    torch = _torch()
    ybar, Ainv, nvec = _fe(ybar, "ybar"), _fe(Ainv, "Ainv"), _fe(nvec, "nvec")
    G, S = Ainv.shape[0], K + M + 1
    if tuple(Ainv.shape) != (G, S, S) or tuple(nvec.shape) != (G, S) or ybar.shape[0] != G * S:
        raise ValueError("dkf_decode_verify_m: inconsistent shapes")
    m = ybar[0].numel()
    if y is None:
        y = torch.empty((G * K,) + tuple(ybar.shape[1:]), dtype=torch.float32, device=ybar.device)
    _dev(y, "y")
    if yq is None and want_yq:
        yq = _new_fe(tuple(y.shape), ybar)
    if yq is not None:
        _fe(yq, "yq")
    if y.numel() != G * K * m or (yq is not None and yq.numel() != G * K * m):
        raise ValueError("dkf_decode_verify_m: output has the wrong size")
    if verdict is None:
        verdict = torch.empty(G, dtype=torch.int32, device=ybar.device)
    _check(load().dkf_decode_verify_m(_ptr(ybar), _ptr(Ainv), _ptr(nvec), _ptr(y), _ptr(yq), _ptr(verdict),
                                      G, K, M, m, int(l), _stream(stream)), "dkf_decode_verify_m")
    return y, yq, verdict


def dkf_wgrad_workspace_bytes_m(layer, G, K, M) -> int:
    return int(load().dkf_wgrad_workspace_bytes_m(C.byref(DkLayer.of(layer)), int(G), int(K), int(M)))


def dkf_wgrad_m(layer, delta, B, gamma, xbar, K, M, l=DKF_L, dW=None, dwq=None, want_dwq=False, scale=1.0,
                accumulate=False, ws=None, stream=None):
    """delta[G*K, ...] float, B[G,S,K], gamma[G,S], xbar[G*S, ...] (device) -> (dW float, dwq or None)."""
    torch = _torch()
    lay = DkLayer.of(layer)
    delta, B, gamma, xbar = _dev(delta, "delta"), _fe(B, "B"), _fe(gamma, "gamma"), _fe(xbar, "xbar")
    G, S = gamma.shape
    n, m = dk_layer_in_len(lay), dk_layer_out_len(lay)
    if n == 0:
        raise DkError(2, "dkf_wgrad_m")
    if (S != K + M + 1 or tuple(B.shape) != (G, S, K) or delta.numel() != G * K * m
            or xbar.numel() != G * S * n):
        raise ValueError("dkf_wgrad_m: inconsistent shapes")
    wshape = (lay.M, lay.N) if lay.kind == 0 else (lay.Co, lay.Ci, lay.kh, lay.kw)
    wcount = int(np.prod(wshape))
    if dW is None:
        if accumulate:
            raise ValueError("dkf_wgrad_m: accumulate needs an existing dW")
        dW = torch.empty(wshape, dtype=torch.float32, device=delta.device)
    _dev(dW, "dW")
    if dwq is None and want_dwq:
        dwq = _new_fe(wshape, delta)
    if dwq is not None:
        _fe(dwq, "dwq")
    if dW.numel() != wcount or (dwq is not None and dwq.numel() != wcount):
        raise ValueError("dkf_wgrad_m: output has the wrong size")
    if ws is None:
        ws = _workspace(dkf_wgrad_workspace_bytes_m(lay, G, K, M), delta, stream)
    _check(load().dkf_wgrad_m(C.byref(lay), _ptr(delta), _ptr(B), _ptr(gamma), _ptr(xbar), _ptr(dW),
                              _ptr(dwq), G, K, M, int(l), float(scale), int(bool(accumulate)), _ptr(ws),
                              ws.numel(), _stream(stream)), "dkf_wgrad_m")
    return dW, dwq
