"""DarKnight masked-layer ORACLE: test infrastructure, not product code.

A plain fp64 CPU implementation of everything the masked-layer hot path
computes, written from the paper (sections "Forward Pass", "Backward
Propagation", "Decoding Correctness Proof", "Computational Integrity").
The loops live in ``dk_oracle.c`` (naive C, fp64); this module only marshals
numpy arrays into it and derives the small per-group coefficient matrices
with numpy's fp64 linear algebra.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package.  It imports nothing from the HIP library or its binding.

Every array argument is converted to C-contiguous float64 first, so callers
may pass the very fp32 arrays the accelerator receives.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dk_oracle.c")
_LIB = os.path.join(_HERE, "libdk_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile dk_oracle.c into libdk_oracle.so with gcc (OpenMP, fp64)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    from . import field
    field.build(force)
    return _LIB


def _L():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ora_num_threads.restype = C.c_int
        _lib.ora_verify_two_subsets.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(_L().ora_num_threads())


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _l(v):
    return C.c_long(int(v))


def conv_out_hw(H, W, kh, kw, stride, pad):
    return (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1


# ----------------------------------------------------------------------
# Coefficients (the small matrices the trusted side draws and derives)
# ----------------------------------------------------------------------

def coefficients(A, gamma):
    """Derive decode / verify / backward coefficients from A and gamma.

    A[G,S,S] is the full square matrix whose first K+1 rows are the paper's
    (K+1)x(K+2) encoding matrix (Forward Pass Eq. "DarKnight Encoding" plus
    the extra integrity combination); its last row belongs to a phantom
    all-zero source.  With Ainv = A^{-1}:
      * Ainv[:, :K]  decodes the K outputs (Forward Pass, "DarKnight Decoding");
      * Ainv[:, K]   recovers <W, r>, which is dropped;
      * nvec = Ainv[:, K+1] is the combination of the K+2 results that must
        vanish (section "Computational Integrity");
      * B = Gamma^{-1} Ainv[:, :K] satisfies B^T Gamma A_ext^T = [I_K | 0]
        (Backward Propagation, matrix relation).
    Returns fp64 arrays (Ainv[G,S,S], nvec[G,S], B[G,S,K]).
    """
    A = _d(A)
    gamma = _d(gamma)
    G, S, _ = A.shape
    K = S - 2
    Ainv = np.linalg.inv(A)
    nvec = np.ascontiguousarray(Ainv[:, :, S - 1])
    B = np.ascontiguousarray(Ainv[:, :, :K] / gamma[:, :, None])
    return Ainv, nvec, B


# ----------------------------------------------------------------------
# Plain layer definitions
# ----------------------------------------------------------------------

def dense_fwd(W, X):
    W, X = _d(W), _d(X)
    M, N = W.shape
    R = X.shape[0]
    Y = np.empty((R, M))
    _L().ora_dense_fwd(_p(W), _p(X), _p(Y), _l(R), _l(M), _l(N))
    return Y


def conv_fwd(W, X, stride=1, pad=0):
    W, X = _d(W), _d(X)
    Co, Ci, kh, kw = W.shape
    R, _, H, Wd = X.shape
    Ho, Wo = conv_out_hw(H, Wd, kh, kw, stride, pad)
    Y = np.empty((R, Co, Ho, Wo))
    _L().ora_conv_fwd(_p(W), _p(X), _p(Y), _l(R), _l(Ci), _l(H), _l(Wd), _l(Co),
                      _l(kh), _l(kw), _l(stride), _l(pad))
    return Y


def dense_wgrad(D, X, scale=1.0):
    D, X = _d(D), _d(X)
    R, M = D.shape
    N = X.shape[1]
    dW = np.empty((M, N))
    _L().ora_dense_wgrad(_p(D), _p(X), _p(dW), _l(R), _l(M), _l(N), C.c_double(scale))
    return dW


def conv_wgrad(D, X, kh, kw, stride=1, pad=0, scale=1.0):
    D, X = _d(D), _d(X)
    R, Co = D.shape[:2]
    _, Ci, H, Wd = X.shape
    dW = np.empty((Co, Ci, kh, kw))
    _L().ora_conv_wgrad(_p(D), _p(X), _p(dW), _l(R), _l(Ci), _l(H), _l(Wd), _l(Co),
                        _l(kh), _l(kw), _l(stride), _l(pad), C.c_double(scale))
    return dW


# ---- the same definitions at sampled output coordinates (fp32 in, fp64 sum)

def _f(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _pts(pts, width):
    pts = np.ascontiguousarray(pts, dtype=np.int64).reshape(-1, width)
    return pts


def dense_fwd_points(W, X, pts):
    W, X, pts = _f(W), _f(X), _pts(pts, 2)
    out = np.empty(len(pts))
    _L().ora_dense_fwd_points(_p(W), _p(X), _l(W.shape[0]), _l(W.shape[1]),
                              _p(pts), _l(len(pts)), _p(out))
    return out


def dense_wgrad_points(D, X, pts, scale=1.0):
    D, X, pts = _f(D), _f(X), _pts(pts, 2)
    out = np.empty(len(pts))
    _L().ora_dense_wgrad_points(_p(D), _p(X), _l(D.shape[0]), _l(D.shape[1]),
                                _l(X.shape[1]), C.c_double(scale), _p(pts),
                                _l(len(pts)), _p(out))
    return out


def conv_fwd_points(W, X, pts, stride=1, pad=0):
    W, X, pts = _f(W), _f(X), _pts(pts, 4)
    Co, Ci, kh, kw = W.shape
    _, _, H, Wd = X.shape
    out = np.empty(len(pts))
    _L().ora_conv_fwd_points(_p(W), _p(X), _l(Ci), _l(H), _l(Wd), _l(Co), _l(kh),
                             _l(kw), _l(stride), _l(pad), _p(pts), _l(len(pts)), _p(out))
    return out


def conv_wgrad_points(D, X, kh, kw, pts, stride=1, pad=0, scale=1.0):
    D, X, pts = _f(D), _f(X), _pts(pts, 4)
    R, Co = D.shape[:2]
    _, Ci, H, Wd = X.shape
    out = np.empty(len(pts))
    _L().ora_conv_wgrad_points(_p(D), _p(X), _l(R), _l(Ci), _l(H), _l(Wd), _l(Co),
                               _l(kh), _l(kw), _l(stride), _l(pad), C.c_double(scale),
                               _p(pts), _l(len(pts)), _p(out))
    return out


# ----------------------------------------------------------------------
# The method's steps
# ----------------------------------------------------------------------

def encode(X, r, A):
    """X[G*K, ...], r[G, ...], A[G,S,S] -> Xbar[G*S, ...]."""
    X, r, A = _d(X), _d(r), _d(A)
    G, S, _ = A.shape
    K = S - 2
    feat = X.shape[1:]
    n = int(np.prod(feat))
    assert X.shape[0] == G * K and r.shape[0] == G
    Xbar = np.empty((G * S,) + feat)
    _L().ora_encode(_p(X), _p(r), _p(A), _p(Xbar), _l(G), _l(K), _l(n))
    return Xbar


def decode(Ybar, Ainv, ncols=None):
    """Ybar[G*S, ...], Ainv[G,S,S] -> Y[G*ncols, ...] (ncols defaults to K)."""
    Ybar, Ainv = _d(Ybar), _d(Ainv)
    G, S, _ = Ainv.shape
    K = S - 2
    ncols = K if ncols is None else ncols
    feat = Ybar.shape[1:]
    m = int(np.prod(feat))
    Y = np.empty((G * ncols,) + feat)
    _L().ora_decode(_p(Ybar), _p(Ainv), _p(Y), _l(G), _l(K), _l(m), _l(ncols))
    return Y


def verify(Ybar, nvec, tol):
    """Returns (verdict[G] int32, rho[G] fp64)."""
    Ybar, nvec = _d(Ybar), _d(nvec)
    G, S = nvec.shape
    m = int(np.prod(Ybar.shape[1:]))
    verdict = np.zeros(G, dtype=np.int32)
    rho = np.zeros(G)
    _L().ora_verify(_p(Ybar), _p(nvec), C.c_double(tol), _p(verdict), _p(rho),
                    _l(G), _l(S - 2), _l(m))
    return verdict, rho


def verify_two_subsets(Ybar, A, tol):
    """Literal redundant-decoding check; returns (verdict[G], maxdiff[G])."""
    Ybar, A = _d(Ybar), _d(A)
    G, S, _ = A.shape
    m = int(np.prod(Ybar.shape[1:]))
    verdict = np.zeros(G, dtype=np.int32)
    diff = np.zeros(G)
    rc = _L().ora_verify_two_subsets(_p(Ybar), _p(A), C.c_double(tol), _p(verdict),
                                     _p(diff), _l(G), _l(S - 2), _l(m))
    if rc:
        raise np.linalg.LinAlgError("singular encoding sub-block")
    return verdict, diff


def delta_mix(D, B, gamma):
    """D[G*K, ...], B[G,S,K], gamma[G,S] -> gamma_j * sum_i beta_ji delta_i, [G*S, ...]."""
    D, B, gamma = _d(D), _d(B), _d(gamma)
    G, S, K = B.shape
    feat = D.shape[1:]
    m = int(np.prod(feat))
    Dt = np.empty((G * S,) + feat)
    _L().ora_delta_mix(_p(D), _p(B), _p(gamma), _p(Dt), _l(G), _l(K), _l(m))
    return Dt


def masked_dense_wgrad(D, B, gamma, Xbar, scale=1.0):
    D, B, gamma, Xbar = _d(D), _d(B), _d(gamma), _d(Xbar)
    G, S, K = B.shape
    M, N = D.shape[1], Xbar.shape[1]
    dW = np.empty((M, N))
    _L().ora_masked_dense_wgrad(_p(D), _p(B), _p(gamma), _p(Xbar), _p(dW), _l(G),
                                _l(K), _l(M), _l(N), C.c_double(scale))
    return dW


def masked_conv_wgrad(D, B, gamma, Xbar, kh, kw, stride=1, pad=0, scale=1.0):
    D, B, gamma, Xbar = _d(D), _d(B), _d(gamma), _d(Xbar)
    G, S, K = B.shape
    Co = D.shape[1]
    _, Ci, H, Wd = Xbar.shape
    dW = np.empty((Co, Ci, kh, kw))
    _L().ora_masked_conv_wgrad(_p(D), _p(B), _p(gamma), _p(Xbar), _p(dW), _l(G), _l(K),
                               _l(Ci), _l(H), _l(Wd), _l(Co), _l(kh), _l(kw),
                               _l(stride), _l(pad), C.c_double(scale))
    return dW


def masked_layer(W, X, r, D, A, gamma, stride=1, pad=0, tol=1e-3, scale=1.0):
    """The whole staged path in the paper's order, fp64.

    encode -> linear op on encodings -> verify -> decode -> masked wgrad.
    W 2-D selects the dense layer, 4-D the convolution.
    Returns dict(Xbar, Ybar, verdict, rho, Y, dW).
    """
    Ainv, nvec, B = coefficients(A, gamma)
    Xbar = encode(X, r, A)
    conv = np.ndim(W) == 4
    Ybar = conv_fwd(W, Xbar, stride, pad) if conv else dense_fwd(W, Xbar)
    verdict, rho = verify(Ybar, nvec, tol)
    Y = decode(Ybar, Ainv)
    if conv:
        dW = masked_conv_wgrad(D, B, gamma, Xbar, W.shape[2], W.shape[3], stride, pad, scale)
    else:
        dW = masked_dense_wgrad(D, B, gamma, Xbar, scale)
    return dict(Xbar=Xbar, Ybar=Ybar, verdict=verdict, rho=rho, Y=Y, dW=dW)


# ----------------------------------------------------------------------
# Colluding accelerators: M noise vectors per group (section "Colluding GPUs")
# ----------------------------------------------------------------------

def coefficients_m(A, gamma, K):
    """A[G,S,S], gamma[G,S] with S = K+M+1 -> (Ainv[G,S,S], nvec[G,S], B[G,S,K]).

    Rows 0..K-1 of A are A_1, rows K..K+M-1 are A_2 (section "Colluding
    GPUs"), the last row is the phantom source of the integrity redundancy.
    B = Gamma^{-1} Ainv[:, :K] satisfies B^T Gamma A = [I_K | 0] over the K+M
    real sources (the section's matrix relation)."""
    A = _d(A)
    gamma = _d(gamma)
    S = A.shape[1]
    Ainv = np.linalg.inv(A)
    nvec = np.ascontiguousarray(Ainv[:, :, S - 1])
    B = np.ascontiguousarray(Ainv[:, :, :K] / gamma[:, :, None])
    return Ainv, nvec, B


def encode_m(X, Rn, A, K):
    """X[G*K, ...], Rn[G*M, ...], A[G,S,S] -> Xbar[G*S, ...]."""
    X, Rn, A = _d(X), _d(Rn), _d(A)
    G, S, _ = A.shape
    M = S - K - 1
    feat = X.shape[1:]
    n = int(np.prod(feat))
    assert M >= 1 and X.shape[0] == G * K and Rn.shape[0] == G * M
    Xbar = np.empty((G * S,) + feat)
    _L().ora_encode_m(_p(X), _p(Rn), _p(A), _p(Xbar), _l(G), _l(K), _l(M), _l(n))
    return Xbar


def decode_m(Ybar, Ainv, ncols):
    Ybar, Ainv = _d(Ybar), _d(Ainv)
    G, S, _ = Ainv.shape
    feat = Ybar.shape[1:]
    Y = np.empty((G * ncols,) + feat)
    _L().ora_decode_s(_p(Ybar), _p(Ainv), _p(Y), _l(G), _l(S), _l(int(np.prod(feat))), _l(ncols))
    return Y


def verify_m(Ybar, nvec, tol):
    Ybar, nvec = _d(Ybar), _d(nvec)
    G, S = nvec.shape
    verdict = np.zeros(G, dtype=np.int32)
    rho = np.zeros(G)
    _L().ora_verify_s(_p(Ybar), _p(nvec), C.c_double(tol), _p(verdict), _p(rho), _l(G), _l(S),
                      _l(int(np.prod(Ybar.shape[1:]))))
    return verdict, rho


def delta_mix_m(D, B, gamma):
    D, B, gamma = _d(D), _d(B), _d(gamma)
    G, S, K = B.shape
    feat = D.shape[1:]
    Dt = np.empty((G * S,) + feat)
    _L().ora_delta_mix_s(_p(D), _p(B), _p(gamma), _p(Dt), _l(G), _l(K), _l(S), _l(int(np.prod(feat))))
    return Dt


def masked_layer_m(W, X, Rn, D, A, gamma, K, stride=1, pad=0, tol=1e-3, scale=1.0):
    """The staged path with M = S-K-1 noise vectors per group, fp64:
    encode -> linear op on encodings -> verify -> decode -> mixed gradients ->
    the plain weight-gradient contraction of the mixed gradients with the
    encodings (the gamma-weighted sum of the Eq_j).
    Returns dict(Xbar, Ybar, verdict, rho, Y, Dt, dW)."""
    Ainv, nvec, B = coefficients_m(A, gamma, K)
    Xbar = encode_m(X, Rn, A, K)
    conv = np.ndim(W) == 4
    Ybar = conv_fwd(W, Xbar, stride, pad) if conv else dense_fwd(W, Xbar)
    verdict, rho = verify_m(Ybar, nvec, tol)
    Y = decode_m(Ybar, Ainv, K)
    Dt = delta_mix_m(D, B, gamma)
    if conv:
        dW = conv_wgrad(Dt, Xbar, W.shape[2], W.shape[3], stride, pad, scale)
    else:
        dW = dense_wgrad(Dt, Xbar, scale)
    return dict(Xbar=Xbar, Ybar=Ybar, verdict=verdict, rho=rho, Y=Y, Dt=Dt, dW=dW)


# ----------------------------------------------------------------------
# Noise from a counter-based generator
# ----------------------------------------------------------------------

def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) for v in key])
    out = (C.c_uint32 * 4)()
    _L().ora_philox4x32_10(c, k, out)
    return [int(v) for v in out]


def noise_philox(G, M, feat, seed, sigma):
    """r[G*M, *feat] (fp64): the noise rows a seed stands for."""
    feat = tuple(int(v) for v in np.atleast_1d(feat))
    n = int(np.prod(feat))
    r = np.empty((G * M,) + feat)
    _L().ora_noise_philox(_p(r), _l(G), _l(M), _l(n), C.c_uint64(int(seed)), C.c_double(sigma))
    return r


# ----------------------------------------------------------------------
# Depthwise convolution and data gradients
# ----------------------------------------------------------------------

def dwconv_fwd(W, X, stride=1, pad=0):
    """W[C,kh,kw], X[R,C,H,W] -> Y[R,C,Ho,Wo] (one filter per channel)."""
    W, X = _d(W), _d(X)
    Cc, kh, kw = W.shape
    R, _, H, Wd = X.shape
    Ho, Wo = conv_out_hw(H, Wd, kh, kw, stride, pad)
    Y = np.empty((R, Cc, Ho, Wo))
    _L().ora_dwconv_fwd(_p(W), _p(X), _p(Y), _l(R), _l(Cc), _l(H), _l(Wd), _l(kh), _l(kw), _l(stride), _l(pad))
    return Y


def dwconv_wgrad(D, X, kh, kw, stride=1, pad=0, scale=1.0):
    D, X = _d(D), _d(X)
    R, Cc, H, Wd = X.shape
    dW = np.empty((Cc, kh, kw))
    _L().ora_dwconv_wgrad(_p(D), _p(X), _p(dW), _l(R), _l(Cc), _l(H), _l(Wd), _l(kh), _l(kw), _l(stride),
                          _l(pad), C.c_double(scale))
    return dW


def dense_dgrad(D, W):
    D, W = _d(D), _d(W)
    M, N = W.shape
    dX = np.empty((D.shape[0], N))
    _L().ora_dense_dgrad(_p(D), _p(W), _p(dX), _l(D.shape[0]), _l(M), _l(N))
    return dX


def conv_dgrad(D, W, H, Wd, stride=1, pad=0):
    D, W = _d(D), _d(W)
    Co, Ci, kh, kw = W.shape
    R = D.shape[0]
    dX = np.empty((R, Ci, H, Wd))
    _L().ora_conv_dgrad(_p(D), _p(W), _p(dX), _l(R), _l(Ci), _l(H), _l(Wd), _l(Co), _l(kh), _l(kw),
                        _l(stride), _l(pad))
    return dX


def dwconv_dgrad(D, W, H, Wd, stride=1, pad=0):
    D, W = _d(D), _d(W)
    Cc, kh, kw = W.shape
    R = D.shape[0]
    dX = np.empty((R, Cc, H, Wd))
    _L().ora_dwconv_dgrad(_p(D), _p(W), _p(dX), _l(R), _l(Cc), _l(H), _l(Wd), _l(kh), _l(kw), _l(stride), _l(pad))
    return dX


def masked_dw_layer(W, X, r, D, A, gamma, stride=1, pad=0, tol=1e-3, scale=1.0):
    """masked_layer for a depthwise convolution W[C,kh,kw]: the same staged
    steps with the depthwise correlation as the bilinear operation."""
    Ainv, nvec, B = coefficients(A, gamma)
    Xbar = encode(X, r, A)
    Ybar = dwconv_fwd(W, Xbar, stride, pad)
    verdict, rho = verify(Ybar, nvec, tol)
    Y = decode(Ybar, Ainv)
    Dt = delta_mix(D, B, gamma)
    dW = dwconv_wgrad(Dt, Xbar, W.shape[1], W.shape[2], stride, pad, scale)
    return dict(Xbar=Xbar, Ybar=Ybar, verdict=verdict, rho=rho, Y=Y, dW=dW)
