"""DarKnight finite-field ORACLE (Python side): test infrastructure, not product code.

The variant of the masked layer in which all values live in the prime field
F_p, p = 2^25 - 39, with l fractional bits of fixed point (section "Privacy
Guarantee": "Quantization", "Random Numbers", algorithm "The pseudo-code for
quantization").  The element-wise loops are in ``dk_field_oracle.c``; this
module marshals numpy arrays and derives the per-group coefficient matrices
with exact Python integers.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this module.  It imports nothing from the HIP library or its binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

P = (1 << 25) - 39          # section "Privacy Guarantee": the largest 25-bit prime
L_BITS = 8                  # fractional bits used for the paper's experiments

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dk_field_oracle.c")
_LIB = os.path.join(_HERE, "libdk_field_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                        "-o", _LIB, _SRC, "-lm"], check=True)
    return _LIB


def _L():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _u(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _l(v):
    return C.c_long(int(v))


def _fe(p):
    return C.c_uint32(int(p))


# ----------------------------------------------------------------------
# Coefficients, exact integer arithmetic
# ----------------------------------------------------------------------

def inv_mod_matrix(A, p=P):
    """Inverse of a square integer matrix over F_p by Gauss-Jordan elimination
    on Python integers; the scalar inverse is Fermat's a^(p-2).  Raises
    ValueError for a singular matrix."""
    n = len(A)
    M = [[int(A[i][j]) % p for j in range(n)] + [int(i == j) for j in range(n)] for i in range(n)]
    for c in range(n):
        piv = next((r for r in range(c, n) if M[r][c]), None)
        if piv is None:
            raise ValueError("matrix is singular over F_p")
        M[c], M[piv] = M[piv], M[c]
        inv = pow(M[c][c], p - 2, p)
        M[c] = [v * inv % p for v in M[c]]
        for r in range(n):
            if r != c and M[r][c]:
                f = M[r][c]
                M[r] = [(v - f * w) % p for v, w in zip(M[r], M[c])]
    return [row[n:] for row in M]


def coefficients(A, gamma, p=P):
    """A[G,S,S], gamma[G,S] (field elements; gamma non-zero) ->
    (Ainv[G,S,S], nvec[G,S], B[G,S,K]) as uint32.

    Same construction as in the real-valued path, over the field
    ("Random Numbers": A, B, Gamma are field elements and encoding and decoding
    are defined over F_p): Ainv = A^{-1}; its first K columns decode, its last
    column is the combination that must vanish (section "Computational
    Integrity"), and B[j][i] = Ainv[j][i] / gamma_j satisfies
    B^T Gamma A_ext^T = [I_K | 0] (Backward Propagation)."""
    A = np.asarray(A)
    gamma = np.asarray(gamma)
    G, S, _ = A.shape
    K = S - 2
    Ainv = np.zeros((G, S, S), dtype=np.uint32)
    nvec = np.zeros((G, S), dtype=np.uint32)
    B = np.zeros((G, S, K), dtype=np.uint32)
    for g in range(G):
        inv = inv_mod_matrix(A[g].tolist(), p)
        for j in range(S):
            gi = pow(int(gamma[g, j]), p - 2, p)
            if int(gamma[g, j]) % p == 0:
                raise ValueError("gamma must be non-zero")
            for i in range(S):
                Ainv[g, j, i] = inv[j][i]
            nvec[g, j] = inv[j][S - 1]
            for i in range(K):
                B[g, j, i] = inv[j][i] * gi % p
    return Ainv, nvec, B


# ----------------------------------------------------------------------
# Steps
# ----------------------------------------------------------------------

def quantize(x, l=L_BITS, p=P):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint32)
    _L().orf_quantize(_p(x), _p(out), _l(x.size), C.c_int(l), _fe(p))
    return out


def dequantize(yq, l=L_BITS, p=P):
    yq = _u(yq)
    out = np.empty(yq.shape, dtype=np.float32)
    _L().orf_dequantize(_p(yq), _p(out), _l(yq.size), C.c_int(l), _fe(p))
    return out


def encode(xq, r, A, p=P):
    xq, r, A = _u(xq), _u(r), _u(A)
    G, S, _ = A.shape
    K = S - 2
    feat = xq.shape[1:]
    n = int(np.prod(feat))
    assert xq.shape[0] == G * K and r.shape[0] == G
    out = np.empty((G * S,) + feat, dtype=np.uint32)
    _L().orf_encode(_p(xq), _p(r), _p(A), _p(out), _l(G), _l(K), _l(n), _fe(p))
    return out


def dense_fwd(Wq, X, p=P):
    Wq, X = _u(Wq), _u(X)
    M, N = Wq.shape
    R = X.shape[0]
    Y = np.empty((R, M), dtype=np.uint32)
    _L().orf_dense_fwd(_p(Wq), _p(X), _p(Y), _l(R), _l(M), _l(N), _fe(p))
    return Y


def dense_fwd_points(Wq, X, pts, p=P):
    Wq, X = _u(Wq), _u(X)
    pts = np.ascontiguousarray(pts, dtype=np.int64).reshape(-1, 2)
    out = np.empty(len(pts), dtype=np.uint32)
    _L().orf_dense_fwd_points(_p(Wq), _p(X), _l(Wq.shape[0]), _l(Wq.shape[1]), _p(pts),
                              _l(len(pts)), _p(out), _fe(p))
    return out


def decode(ybar, Ainv, ncols=None, p=P):
    ybar, Ainv = _u(ybar), _u(Ainv)
    G, S, _ = Ainv.shape
    K = S - 2
    ncols = K if ncols is None else ncols
    feat = ybar.shape[1:]
    m = int(np.prod(feat))
    out = np.empty((G * ncols,) + feat, dtype=np.uint32)
    _L().orf_decode(_p(ybar), _p(Ainv), _p(out), _l(G), _l(K), _l(m), _l(ncols), _fe(p))
    return out


def verify(ybar, nvec, p=P):
    ybar, nvec = _u(ybar), _u(nvec)
    G, S = nvec.shape
    m = int(np.prod(ybar.shape[1:]))
    verdict = np.zeros(G, dtype=np.int32)
    _L().orf_verify(_p(ybar), _p(nvec), _p(verdict), _l(G), _l(S - 2), _l(m), _fe(p))
    return verdict


def delta_mix(dq, B, gamma, p=P):
    dq, B, gamma = _u(dq), _u(B), _u(gamma)
    G, S, K = B.shape
    feat = dq.shape[1:]
    m = int(np.prod(feat))
    out = np.empty((G * S,) + feat, dtype=np.uint32)
    _L().orf_delta_mix(_p(dq), _p(B), _p(gamma), _p(out), _l(G), _l(K), _l(m), _fe(p))
    return out


def dense_wgrad(D, X, p=P):
    D, X = _u(D), _u(X)
    R, M = D.shape
    N = X.shape[1]
    out = np.empty((M, N), dtype=np.uint32)
    _L().orf_dense_wgrad(_p(D), _p(X), _p(out), _l(R), _l(M), _l(N), _fe(p))
    return out


def dense_wgrad_points(D, X, pts, p=P):
    D, X = _u(D), _u(X)
    pts = np.ascontiguousarray(pts, dtype=np.int64).reshape(-1, 2)
    out = np.empty(len(pts), dtype=np.uint32)
    _L().orf_dense_wgrad_points(_p(D), _p(X), _l(D.shape[0]), _l(D.shape[1]), _l(X.shape[1]),
                                _p(pts), _l(len(pts)), _p(out), _fe(p))
    return out


def noise_philox(G, feat, seed, p=P):
    """r[G, *feat] (uint32): the uniform field noise a seed stands for."""
    feat = tuple(int(v) for v in np.atleast_1d(feat))
    r = np.empty((G,) + feat, dtype=np.uint32)
    _L().orf_noise_philox(_p(r), _l(G), _l(int(np.prod(feat))), C.c_uint64(int(seed)), _fe(p))
    return r


def conv_out_hw(H, W, kh, kw, stride, pad):
    return (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1


def conv_fwd(Wq, X, stride=1, pad=0, p=P):
    Wq, X = _u(Wq), _u(X)
    Co, Ci, kh, kw = Wq.shape
    R, _, H, Wd = X.shape
    Ho, Wo = conv_out_hw(H, Wd, kh, kw, stride, pad)
    Y = np.empty((R, Co, Ho, Wo), dtype=np.uint32)
    _L().orf_conv_fwd(_p(Wq), _p(X), _p(Y), _l(R), _l(Ci), _l(H), _l(Wd), _l(Co), _l(kh), _l(kw),
                      _l(stride), _l(pad), _fe(p))
    return Y


def conv_fwd_points(Wq, X, pts, stride=1, pad=0, p=P):
    Wq, X = _u(Wq), _u(X)
    Co, Ci, kh, kw = Wq.shape
    _, _, H, Wd = X.shape
    pts = np.ascontiguousarray(pts, dtype=np.int64).reshape(-1, 4)
    out = np.empty(len(pts), dtype=np.uint32)
    _L().orf_conv_fwd_points(_p(Wq), _p(X), _l(Ci), _l(H), _l(Wd), _l(Co), _l(kh), _l(kw), _l(stride),
                             _l(pad), _p(pts), _l(len(pts)), _p(out), _fe(p))
    return out


def conv_wgrad(D, X, kh, kw, stride=1, pad=0, p=P):
    D, X = _u(D), _u(X)
    R, Co = D.shape[:2]
    _, Ci, H, Wd = X.shape
    out = np.empty((Co, Ci, kh, kw), dtype=np.uint32)
    _L().orf_conv_wgrad(_p(D), _p(X), _p(out), _l(R), _l(Ci), _l(H), _l(Wd), _l(Co), _l(kh), _l(kw),
                        _l(stride), _l(pad), _fe(p))
    return out


def conv_wgrad_points(D, X, kh, kw, pts, stride=1, pad=0, p=P):
    D, X = _u(D), _u(X)
    R, Co = D.shape[:2]
    _, Ci, H, Wd = X.shape
    pts = np.ascontiguousarray(pts, dtype=np.int64).reshape(-1, 4)
    out = np.empty(len(pts), dtype=np.uint32)
    _L().orf_conv_wgrad_points(_p(D), _p(X), _l(R), _l(Ci), _l(H), _l(Wd), _l(Co), _l(kh), _l(kw),
                               _l(stride), _l(pad), _p(pts), _l(len(pts)), _p(out), _fe(p))
    return out


def dwconv_fwd(Wq, X, stride=1, pad=0, p=P):
    """Depthwise cross-correlation over the field: Wq[C,kh,kw], X[R,C,H,W]."""
    Wq, X = _u(Wq), _u(X)
    Cc, kh, kw = Wq.shape
    R, _, H, Wd = X.shape
    Ho, Wo = conv_out_hw(H, Wd, kh, kw, stride, pad)
    Y = np.empty((R, Cc, Ho, Wo), dtype=np.uint32)
    _L().orf_dwconv_fwd(_p(Wq), _p(X), _p(Y), _l(R), _l(Cc), _l(H), _l(Wd), _l(kh), _l(kw), _l(stride),
                        _l(pad), _fe(p))
    return Y


def dwconv_wgrad(D, X, kh, kw, stride=1, pad=0, p=P):
    D, X = _u(D), _u(X)
    R, Cc, H, Wd = X.shape
    out = np.empty((Cc, kh, kw), dtype=np.uint32)
    _L().orf_dwconv_wgrad(_p(D), _p(X), _p(out), _l(R), _l(Cc), _l(H), _l(Wd), _l(kh), _l(kw), _l(stride),
                          _l(pad), _fe(p))
    return out


def add_bias(yq, bias, per, l=L_BITS, p=P):
    """Decoded field values plus the quantised bias b_q = Field(Round(b 2^{2l}))
    (quantisation algorithm); entry e of every row takes bias[e // per]
    (per = 1 for a dense layer, Ho*Wo for a convolution)."""
    out = _u(yq).copy()
    bias = np.ascontiguousarray(bias, dtype=np.float32)
    rows = out.shape[0]
    m = int(np.prod(out.shape[1:]))
    assert bias.size * per == m
    _L().orf_add_bias(_p(out), _p(bias), _l(rows), _l(m), _l(per), C.c_int(l), _fe(p))
    return out


def masked_dw_layer(W, X, r, delta, A, gamma, stride=1, pad=0, l=L_BITS, p=P):
    """masked_layer for a depthwise convolution W[C,kh,kw]: the same steps with
    the depthwise correlation as the linear operation."""
    Ainv, nvec, B = coefficients(A, gamma, p)
    Wq, Xq = quantize(W, l, p), quantize(X, l, p)
    Xbar = encode(Xq, r, A, p)
    Ybar = dwconv_fwd(Wq, Xbar, stride, pad, p)
    verdict = verify(Ybar, nvec, p)
    Yq = decode(Ybar, Ainv, None, p)
    Y = dequantize(Yq, l, p)
    Dq = quantize(delta, l, p)
    Dtilde = delta_mix(Dq, B, gamma, p)
    dWq = dwconv_wgrad(Dtilde, Xbar, W.shape[1], W.shape[2], stride, pad, p)
    dW = dequantize(dWq, l, p)
    return dict(Wq=Wq, Xq=Xq, Xbar=Xbar, Ybar=Ybar, verdict=verdict, Yq=Yq, Y=Y, Dq=Dq,
                Dtilde=Dtilde, dWq=dWq, dW=dW)


def masked_layer(W, X, r, delta, A, gamma, stride=1, pad=0, l=L_BITS, p=P):
    """masked_dense_layer for either kind of layer: W 2-D is the dense layer,
    W 4-D the NCHW convolution (same steps, the convolution as the linear
    operation and the correlation as the weight-gradient contraction)."""
    if np.ndim(W) == 2:
        return masked_dense_layer(W, X, r, delta, A, gamma, l, p)
    Ainv, nvec, B = coefficients(A, gamma, p)
    Wq, Xq = quantize(W, l, p), quantize(X, l, p)
    Xbar = encode(Xq, r, A, p)
    Ybar = conv_fwd(Wq, Xbar, stride, pad, p)
    verdict = verify(Ybar, nvec, p)
    Yq = decode(Ybar, Ainv, None, p)
    Y = dequantize(Yq, l, p)
    Dq = quantize(delta, l, p)
    Dtilde = delta_mix(Dq, B, gamma, p)
    dWq = conv_wgrad(Dtilde, Xbar, W.shape[2], W.shape[3], stride, pad, p)
    dW = dequantize(dWq, l, p)
    return dict(Wq=Wq, Xq=Xq, Xbar=Xbar, Ybar=Ybar, verdict=verdict, Yq=Yq, Y=Y, Dq=Dq,
                Dtilde=Dtilde, dWq=dWq, dW=dW)


def masked_dense_layer(W, X, r, delta, A, gamma, l=L_BITS, p=P):
    """The staged field path for a dense layer, in the order of the
    quantisation algorithm: quantise W and X, encode, multiply on encodings,
    verify, decode, de-quantise; then the masked weight gradient from the
    quantised output gradients.

    W[M,N], X[G*K,N], delta[G*K,M] are fp32; r[G,N], A[G,S,S], gamma[G,S] are
    field elements.  Returns dict(Wq, Xq, Xbar, Ybar, verdict, Yq, Y, Dq,
    Dtilde, dWq, dW)."""
    Ainv, nvec, B = coefficients(A, gamma, p)
    Wq, Xq = quantize(W, l, p), quantize(X, l, p)
    Xbar = encode(Xq, r, A, p)
    Ybar = dense_fwd(Wq, Xbar, p)
    verdict = verify(Ybar, nvec, p)
    Yq = decode(Ybar, Ainv, None, p)
    Y = dequantize(Yq, l, p)
    Dq = quantize(delta, l, p)
    Dtilde = delta_mix(Dq, B, gamma, p)
    dWq = dense_wgrad(Dtilde, Xbar, p)
    dW = dequantize(dWq, l, p)
    return dict(Wq=Wq, Xq=Xq, Xbar=Xbar, Ybar=Ybar, verdict=verdict, Yq=Yq, Y=Y, Dq=Dq,
                Dtilde=Dtilde, dWq=dWq, dW=dW)


# ----------------------------------------------------------------------
# Several colluding accelerators (section "Colluding GPUs" and the paragraph of
# "Privacy Guarantee" on it): M noise vectors per group, uniform over F_p,
# S = K + M + 1 encodings; rows of A are the K inputs (A_1), the M noise
# vectors (A_2) and the phantom zero source.
# ----------------------------------------------------------------------

def coefficients_m(A, gamma, K, p=P):
    """A[G,S,S], gamma[G,S], S = K+M+1 -> (Ainv[G,S,S], nvec[G,S], B[G,S,K]):
    the first K columns of A^{-1} decode, the last must vanish, and
    B[j][i] = Ainv[j][i] / gamma_j, so that B^T Gamma A = [I_K | 0] over the
    K+M real sources (the section's relation)."""
    A = np.asarray(A)
    gamma = np.asarray(gamma)
    G, S, _ = A.shape
    assert S >= K + 2
    Ainv = np.zeros((G, S, S), dtype=np.uint32)
    nvec = np.zeros((G, S), dtype=np.uint32)
    B = np.zeros((G, S, K), dtype=np.uint32)
    for g in range(G):
        inv = inv_mod_matrix(A[g].tolist(), p)
        for j in range(S):
            if int(gamma[g, j]) % p == 0:
                raise ValueError("gamma must be non-zero")
            gi = pow(int(gamma[g, j]), p - 2, p)
            for i in range(S):
                Ainv[g, j, i] = inv[j][i]
            nvec[g, j] = inv[j][S - 1]
            for i in range(K):
                B[g, j, i] = inv[j][i] * gi % p
    return Ainv, nvec, B


def encode_m(xq, r, A, K, p=P):
    xq, r, A = _u(xq), _u(r), _u(A)
    G, S, _ = A.shape
    M = S - K - 1
    feat = xq.shape[1:]
    n = int(np.prod(feat))
    assert xq.shape[0] == G * K and r.shape[0] == G * M and M >= 1
    out = np.empty((G * S,) + feat, dtype=np.uint32)
    _L().orf_encode_m(_p(xq), _p(r), _p(A), _p(out), _l(G), _l(K), _l(M), _l(n), _fe(p))
    return out


def decode_m(ybar, Ainv, ncols, p=P):
    ybar, Ainv = _u(ybar), _u(Ainv)
    G, S, _ = Ainv.shape
    feat = ybar.shape[1:]
    m = int(np.prod(feat))
    out = np.empty((G * ncols,) + feat, dtype=np.uint32)
    _L().orf_decode_s(_p(ybar), _p(Ainv), _p(out), _l(G), _l(S), _l(m), _l(ncols), _fe(p))
    return out


def verify_m(ybar, nvec, p=P):
    ybar, nvec = _u(ybar), _u(nvec)
    G, S = nvec.shape
    m = int(np.prod(ybar.shape[1:]))
    verdict = np.zeros(G, dtype=np.int32)
    _L().orf_verify_s(_p(ybar), _p(nvec), _p(verdict), _l(G), _l(S), _l(m), _fe(p))
    return verdict


def delta_mix_m(dq, B, gamma, p=P):
    dq, B, gamma = _u(dq), _u(B), _u(gamma)
    G, S, K = B.shape
    feat = dq.shape[1:]
    m = int(np.prod(feat))
    out = np.empty((G * S,) + feat, dtype=np.uint32)
    _L().orf_delta_mix_s(_p(dq), _p(B), _p(gamma), _p(out), _l(G), _l(K), _l(S), _l(m), _fe(p))
    return out


def masked_layer_m(W, X, r, delta, A, gamma, K, stride=1, pad=0, l=L_BITS, p=P):
    """masked_layer with M = S - K - 1 noise vectors per group (r[G*M, ...]):
    the same steps in the same order."""
    Ainv, nvec, B = coefficients_m(A, gamma, K, p)
    Wq, Xq = quantize(W, l, p), quantize(X, l, p)
    Xbar = encode_m(Xq, r, A, K, p)
    dense = np.ndim(W) == 2
    Ybar = dense_fwd(Wq, Xbar, p) if dense else conv_fwd(Wq, Xbar, stride, pad, p)
    verdict = verify_m(Ybar, nvec, p)
    Yq = decode_m(Ybar, Ainv, K, p)
    Y = dequantize(Yq, l, p)
    Dq = quantize(delta, l, p)
    Dtilde = delta_mix_m(Dq, B, gamma, p)
    dWq = (dense_wgrad(Dtilde, Xbar, p) if dense
           else conv_wgrad(Dtilde, Xbar, W.shape[2], W.shape[3], stride, pad, p))
    dW = dequantize(dWq, l, p)
    return dict(Wq=Wq, Xq=Xq, Xbar=Xbar, Ybar=Ybar, verdict=verdict, Yq=Yq, Y=Y, Dq=Dq,
                Dtilde=Dtilde, dWq=dWq, dW=dW)


# ----------------------------------------------------------------------
# Dynamic normalisation ("Quantization", the variant for networks without
# normalisation layers)
# ----------------------------------------------------------------------

def norm_scales(x, limit):
    """One factor per row of x (a row is one vector: one sample's features, or
    the whole weight tensor given as a single row).

    The paper divides a vector by its largest absolute entry when its values
    pass the limits.  Reading: the vector passes the limit when that largest
    entry m exceeds `limit`; its factor is then the fp32 value nearest to 1/m,
    otherwise 1.  NaN entries do not take part in the maximum, and an infinite
    maximum leaves the factor at 1 (the quantiser's clamp deals with it)."""
    x = np.asarray(x, dtype=np.float32)
    x = x.reshape(x.shape[0], -1)
    s = np.ones(x.shape[0], dtype=np.float32)
    for i in range(x.shape[0]):
        # fmax skips NaN operands
        m = float(np.fmax.reduce(np.abs(x[i]).astype(np.float64), initial=0.0))
        if m > float(np.float32(limit)) and m != np.inf:
            s[i] = np.float32(1.0 / m)
    return s


def quantize_scaled(x, scale, l=L_BITS, p=P):
    """Field(Round(x[i] * scale[i] * 2^l)), row i of x times its factor.  The
    product of two fp32 values and a power of two is exact in fp64, so Round
    sees the exact scaled value.  Clamp and NaN as in quantize()."""
    x = np.asarray(x, dtype=np.float32)
    scale = np.asarray(scale, dtype=np.float32).reshape(-1)
    rows = x.reshape(x.shape[0], -1).astype(np.float64)
    assert scale.shape[0] == rows.shape[0]
    v = np.floor(rows * scale.astype(np.float64)[:, None] * float(2 ** l) + 0.5)
    v = np.where(np.isnan(v), 0.0, v)
    v = np.clip(v, -2147483648.0, 2147483647.0).astype(np.int64)
    return np.mod(v, p).astype(np.uint32).reshape(x.shape)


def reciprocal(scale):
    """fp64 reciprocal of fp32 factors (one IEEE division each)."""
    return 1.0 / np.asarray(scale, dtype=np.float32).astype(np.float64)


def unscale(y, row_scale, wscale):
    """Undo the factors on de-quantised results: row i of y is multiplied by
    the fp64 reciprocal of (row_scale[i] * wscale) (that product is exact in
    fp64) and rounded to fp32."""
    y = np.asarray(y, dtype=np.float32)
    rs = np.asarray(row_scale, dtype=np.float32).astype(np.float64).reshape(-1)
    inv = 1.0 / (rs * float(np.float32(wscale)))
    out = y.reshape(y.shape[0], -1).astype(np.float64) * inv[:, None]
    return out.astype(np.float32).reshape(y.shape)


def quantize_unscaled_delta(delta, xscale, l=L_BITS, p=P):
    """Output gradients for the weight gradient when the stored encodings hold
    inputs times xscale: the sum over samples of delta_i (x) x_i equals the sum
    of (delta_i / s_i) (x) (s_i x_i), so row i is multiplied by the fp64
    reciprocal of s_i (product rounded to fp64 once), then Round and Field."""
    d = np.asarray(delta, dtype=np.float32)
    inv = reciprocal(xscale).reshape(-1)
    rows = d.reshape(d.shape[0], -1).astype(np.float64) * inv[:, None]
    v = np.floor(rows * float(2 ** l) + 0.5)
    v = np.where(np.isnan(v), 0.0, v)
    v = np.clip(v, -2147483648.0, 2147483647.0).astype(np.int64)
    return np.mod(v, p).astype(np.uint32).reshape(d.shape)


def masked_layer_normalized(W, X, r, delta, A, gamma, limit, stride=1, pad=0, l=L_BITS, p=P):
    """masked_layer with dynamic normalisation of the inputs (one factor per
    sample) and of the weights (one factor for the tensor).  The steps between
    quantisation and de-quantisation are those of masked_layer.  Y and dW come
    back in the units of the un-normalised layer: Y row i is divided by
    wscale * xscale[i]; the output gradients carry 1 / xscale[i] into the
    weight gradient, which therefore needs no factor afterwards."""
    W = np.asarray(W, dtype=np.float32)
    X = np.asarray(X, dtype=np.float32)
    Ainv, nvec, B = coefficients(A, gamma, p)
    xscale = norm_scales(X, limit)
    wscale = norm_scales(W.reshape(1, -1), limit)
    Wq = quantize_scaled(W.reshape(1, -1), wscale, l, p).reshape(W.shape)
    Xq = quantize_scaled(X, xscale, l, p)
    Xbar = encode(Xq, r, A, p)
    dense = W.ndim == 2
    Ybar = dense_fwd(Wq, Xbar, p) if dense else conv_fwd(Wq, Xbar, stride, pad, p)
    verdict = verify(Ybar, nvec, p)
    Yq = decode(Ybar, Ainv, None, p)
    Yn = dequantize(Yq, l, p)
    Y = unscale(Yn, xscale, wscale[0])
    Dq = quantize_unscaled_delta(delta, xscale, l, p)
    Dtilde = delta_mix(Dq, B, gamma, p)
    dWq = (dense_wgrad(Dtilde, Xbar, p) if dense
           else conv_wgrad(Dtilde, Xbar, W.shape[2], W.shape[3], stride, pad, p))
    dW = dequantize(dWq, l, p)
    return dict(xscale=xscale, wscale=wscale, Wq=Wq, Xq=Xq, Xbar=Xbar, Ybar=Ybar, verdict=verdict,
                Yq=Yq, Yn=Yn, Y=Y, Dq=Dq, Dtilde=Dtilde, dWq=dWq, dW=dW)
