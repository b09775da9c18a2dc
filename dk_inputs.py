"""Seeded synthetic inputs for the masked-layer workloads.

This module only draws random numbers: layer weights, private inputs, noise
vectors, output gradients, the random square matrices A (rejected until their
2-norm condition number is below a bound) and the random diagonal gamma.  It
holds none of the method's arithmetic (no encoding, decoding, inversion or
gradient mixing) and is the only thing the HIP path and the CPU oracle have
in common: both receive the same fp32 arrays.

Draw order for one layer (fixed, so a seed names a workload):
    W -> X (unless supplied) -> r -> delta -> for each group: A (with
    resampling) -> gamma signs -> gamma magnitudes.
"N(0, v)" in the workload descriptions is read as variance v.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np


@dataclass(frozen=True)
class Layer:
    """kind 'linear': y = W x, W[M, N].  kind 'conv': NCHW cross-correlation,
    W[Co, Ci, kh, kw], no bias.  kind 'dwconv': depthwise cross-correlation,
    one filter per channel, W[Ci, kh, kw], Co == Ci."""
    kind: str
    M: int = 0
    N: int = 0
    Ci: int = 0
    Co: int = 0
    H: int = 0
    W: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def in_shape(self):
        return (self.N,) if self.kind == "linear" else (self.Ci, self.H, self.W)

    @property
    def out_shape(self):
        return (self.M,) if self.kind == "linear" else (self.Co, self.Ho, self.Wo)

    @property
    def w_shape(self):
        if self.kind == "dwconv":
            return (self.Ci, self.kh, self.kw)
        return (self.M, self.N) if self.kind == "linear" else (self.Co, self.Ci, self.kh, self.kw)

    @property
    def fan_in(self):
        if self.kind == "dwconv":
            return self.kh * self.kw
        return self.N if self.kind == "linear" else self.Ci * self.kh * self.kw

    @property
    def macs_per_row(self):
        """Multiply-accumulates of the layer for one (encoded) input row."""
        if self.kind == "linear":
            return self.M * self.N
        if self.kind == "dwconv":
            return self.Ci * self.Ho * self.Wo * self.kh * self.kw
        return self.Co * self.Ho * self.Wo * self.Ci * self.kh * self.kw

    def asdict(self):
        return asdict(self)


def linear(M, N):
    return Layer("linear", M=M, N=N)


def conv(Ci, Co, H, W, k=3, stride=1, pad=None):
    return Layer("conv", Ci=Ci, Co=Co, H=H, W=W, kh=k, kw=k, stride=stride,
                 pad=(k // 2 if pad is None else pad))


def dwconv(C, H, W, k=3, stride=1, pad=None):
    return Layer("dwconv", Ci=C, Co=C, H=H, W=W, kh=k, kw=k, stride=stride,
                 pad=(k // 2 if pad is None else pad))


def _normal(rng, shape, std):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def sample_A(rng, S, cond_max=100.0):
    """One S x S matrix, entries U[-1,1], redrawn until cond_2 < cond_max
    (condition number of the fp64 draw, before rounding to fp32)."""
    while True:
        A = rng.uniform(-1.0, 1.0, size=(S, S))
        if np.linalg.cond(A, 2) < cond_max:
            return A.astype(np.float32)


def sample_coeff_draws(rng, G, K, cond_max=100.0):
    """A[G,S,S] fp32 and gamma[G,S] fp32 (sign * U[0.5,1.5]), S = K+2."""
    S = K + 2
    A = np.empty((G, S, S), dtype=np.float32)
    gamma = np.empty((G, S), dtype=np.float32)
    for g in range(G):
        A[g] = sample_A(rng, S, cond_max)
        sign = rng.integers(0, 2, size=S) * 2 - 1
        gamma[g] = (sign * rng.uniform(0.5, 1.5, size=S)).astype(np.float32)
    return A, gamma


def masked_layer_inputs(rng, layer: Layer, K: int, batch: int, *, w_std=None,
                        x=None, x_dist="normal", noise_std=10.0, delta_std=0.1,
                        cond_max=100.0):
    """All fp32 host arrays one masked layer needs.

    Returns dict(layer, K, G, W, X[batch,...], r[G,...], delta[batch,...],
    A[G,S,S], gamma[G,S]).  w_std None = He initialisation sqrt(2/fan_in).
    """
    if batch % K:
        raise ValueError("batch must be a multiple of K")
    G = batch // K
    if w_std is None:
        w_std = float(np.sqrt(2.0 / layer.fan_in))
    W = _normal(rng, layer.w_shape, w_std)
    if x is None:
        if x_dist == "normal":
            X = _normal(rng, (batch,) + layer.in_shape, 1.0)
        elif x_dist == "uniform":
            X = rng.random((batch,) + layer.in_shape, dtype=np.float32)
        elif x_dist == "relu_normal":
            X = np.maximum(_normal(rng, (batch,) + layer.in_shape, 1.0), 0)
        else:
            raise ValueError(x_dist)
    else:
        X = np.ascontiguousarray(x, dtype=np.float32).reshape((batch,) + layer.in_shape)
    r = _normal(rng, (G,) + layer.in_shape, noise_std)
    delta = _normal(rng, (batch,) + layer.out_shape, delta_std)
    A, gamma = sample_coeff_draws(rng, G, K, cond_max)
    return dict(layer=layer, K=K, G=G, W=W, X=X, r=r, delta=delta, A=A, gamma=gamma)


def collusion_layer_inputs(rng, layer: Layer, K: int, M: int, batch: int, *, w_std=None,
                           noise_std=10.0, delta_std=0.1, cond_max=100.0):
    """Host arrays for a masked layer that tolerates M colluding accelerators:
    as masked_layer_inputs, but M noise rows per group (r[G*M, ...]) and square
    matrices of size S = K+M+1 (A[G,S,S], gamma[G,S]); A is resampled until
    its 2-norm condition number is below cond_max."""
    if batch % K:
        raise ValueError("batch must be a multiple of K")
    G, S = batch // K, K + M + 1
    if w_std is None:
        w_std = float(np.sqrt(2.0 / layer.fan_in))
    W = _normal(rng, layer.w_shape, w_std)
    X = _normal(rng, (batch,) + layer.in_shape, 1.0)
    r = _normal(rng, (G * M,) + layer.in_shape, noise_std)
    delta = _normal(rng, (batch,) + layer.out_shape, delta_std)
    A = np.empty((G, S, S), dtype=np.float32)
    gamma = np.empty((G, S), dtype=np.float32)
    for g in range(G):
        A[g] = sample_A(rng, S, cond_max)
        sign = np.where(rng.random(S) < 0.5, -1.0, 1.0)
        gamma[g] = (sign * rng.uniform(0.5, 1.5, S)).astype(np.float32)
    return dict(layer=layer, K=K, M=M, G=G, W=W, X=X, r=r, delta=delta, A=A, gamma=gamma)


FIELD_P = (1 << 25) - 39     # the prime of the finite-field variant


def field_layer_inputs(rng, layer: Layer, K: int, batch: int, *, w_std=None,
                       delta_std=0.1, p=FIELD_P):
    """Host arrays for the finite-field variant of one masked layer: fp32 W, X
    and delta as in the real-valued workloads, and uniform draws from the
    field for the noise r[G,...] in [0,p), the matrices A[G,S,S] in [0,p) and
    the non-zero scalars gamma[G,S] in [1,p), all uint32.  A singular A has
    probability about 1/p per draw and is not screened here (no arithmetic in
    this module); the coefficient routines report it."""
    if batch % K:
        raise ValueError("batch must be a multiple of K")
    G, S = batch // K, K + 2
    if w_std is None:
        w_std = float(np.sqrt(2.0 / layer.fan_in))
    W = _normal(rng, layer.w_shape, w_std)
    X = _normal(rng, (batch,) + layer.in_shape, 1.0)
    r = rng.integers(0, p, size=(G,) + layer.in_shape, dtype=np.uint32)
    delta = _normal(rng, (batch,) + layer.out_shape, delta_std)
    A = rng.integers(0, p, size=(G, S, S), dtype=np.uint32)
    gamma = rng.integers(1, p, size=(G, S), dtype=np.uint32)
    return dict(layer=layer, K=K, G=G, W=W, X=X, r=r, delta=delta, A=A, gamma=gamma, p=p)


def field_collusion_layer_inputs(rng, layer: Layer, K: int, M: int, batch: int, *, w_std=None,
                                 delta_std=0.1, p=FIELD_P):
    """field_layer_inputs with M noise rows per group (r[G*M, ...]) and square
    matrices of size S = K+M+1 over the field."""
    if batch % K:
        raise ValueError("batch must be a multiple of K")
    G, S = batch // K, K + M + 1
    if w_std is None:
        w_std = float(np.sqrt(2.0 / layer.fan_in))
    W = _normal(rng, layer.w_shape, w_std)
    X = _normal(rng, (batch,) + layer.in_shape, 1.0)
    r = rng.integers(0, p, size=(G * M,) + layer.in_shape, dtype=np.uint32)
    delta = _normal(rng, (batch,) + layer.out_shape, delta_std)
    A = rng.integers(0, p, size=(G, S, S), dtype=np.uint32)
    gamma = rng.integers(1, p, size=(G, S), dtype=np.uint32)
    return dict(layer=layer, K=K, M=M, G=G, W=W, X=X, r=r, delta=delta, A=A, gamma=gamma, p=p)


def config5_field(seed=5, batch=1024, K=8, index=None):
    """The classifier shapes of config5 for the finite-field variant."""
    out = []
    for li, L in enumerate(config5_layers()):
        if index is not None and li != index:
            continue
        rng = np.random.default_rng([seed, li, 1])
        out.append(field_layer_inputs(rng, L, K=K, batch=batch))
    return out


def config2_field(seed=2, batch=256, hw=32, ch=64):
    """Conv 3x3 s1 p1, 64 -> 64 channels at 32x32, batch 256, K=4, finite-field variant."""
    rng = np.random.default_rng([seed, 0, 1])
    return field_layer_inputs(rng, conv(ch, ch, hw, hw, 3), K=4, batch=batch)


def config3_field(seed=3, batch=128, K=4, index=0):
    """One layer of the VGG-16 conv stack, finite-field variant."""
    rng = np.random.default_rng([seed, index, 1])
    return field_layer_inputs(rng, config3_layers()[index], K=K, batch=batch)


def config4_field(seed=4, batch=64, K=8, index=0):
    """One ResNet-50 conv shape, finite-field variant: (inputs, multiplicity)."""
    lay, count = resnet50_convs()[index]
    rng = np.random.default_rng([seed, index, 1])
    return field_layer_inputs(rng, lay, K=K, batch=batch), count


def config1_field(seed=0):
    """Dense 256 -> 512, K=2, one group, finite-field variant."""
    rng = np.random.default_rng([seed, 0, 1])
    return field_layer_inputs(rng, linear(512, 256), K=2, batch=2, w_std=1.0 / 16.0, delta_std=1.0)


# ----------------------------------------------------------------------
# The five workloads
# ----------------------------------------------------------------------

def config1(seed=0):
    """Single dense layer 256 -> 512, K=2, one group."""
    rng = np.random.default_rng(seed)
    return masked_layer_inputs(rng, linear(512, 256), K=2, batch=2, w_std=1.0 / 16.0,
                               noise_std=10.0, delta_std=1.0)


def config2(seed=2, batch=256, hw=32, ch=64):
    """Conv 3x3 s1 p1, 64 -> 64 channels at 32x32, batch 256, K=4."""
    rng = np.random.default_rng(seed)
    return masked_layer_inputs(rng, conv(ch, ch, hw, hw, 3), K=4, batch=batch,
                               noise_std=10.0, delta_std=0.1)


VGG16_CONVS = [(3, 64, 32), (64, 64, 32), (64, 128, 16), (128, 128, 16),
               (128, 256, 8), (256, 256, 8), (256, 256, 8),
               (256, 512, 4), (512, 512, 4), (512, 512, 4),
               (512, 512, 2), (512, 512, 2), (512, 512, 2)]


def config3_layers():
    """VGG-16 conv stack on 32x32 inputs: 13 conv 3x3 s1 p1."""
    return [conv(ci, co, hw, hw, 3) for ci, co, hw in VGG16_CONVS]


def config3(seed=3, batch=128, K=4, index=None):
    """Per-layer inputs for the VGG-16 conv stack.  Layer 0 sees images
    ~U[0,1]; deeper layers see max(0, N(0,1)) activations (each layer is an
    independent masked-layer problem: fresh A, r, gamma per layer and group)."""
    out = []
    for li, L in enumerate(config3_layers()):
        if index is not None and li != index:
            continue
        rng = np.random.default_rng([seed, li])   # one stream per layer
        out.append(masked_layer_inputs(rng, L, K=K, batch=batch,
                                       x_dist="uniform" if li == 0 else "relu_normal"))
    return out


def resnet50_convs(include_stem=False):
    """Distinct conv shapes of ResNet-50 bottlenecks at 224x224 input, with
    multiplicity: list of (Layer, count).  Stride 2 sits on the 3x3."""
    L = []
    if include_stem:
        L.append((conv(3, 64, 224, 224, 7, stride=2, pad=3), 1))
    hw, cin = 56, 64
    for stage, (mid, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)]):
        cout = mid * 4
        for b in range(blocks):
            st = 2 if (b == 0 and stage > 0) else 1
            L.append((conv(cin, mid, hw, hw, 1), 1))
            L.append((conv(mid, mid, hw, hw, 3, stride=st), 1))
            if b == 0:
                L.append((conv(cin, cout, hw, hw, 1, stride=st), 1))  # downsample
            hw //= st
            L.append((conv(mid, cout, hw, hw, 1), 1))
            cin = cout
    merged = {}
    for lay, c in L:
        merged[lay] = merged.get(lay, 0) + c
    return list(merged.items())


def config4(seed=4, batch=64, K=8, include_stem=False, index=None):
    """Generator over (inputs dict, multiplicity) for the ResNet-50 shapes
    (all of them, or only shape number `index`)."""
    for li, (lay, count) in enumerate(resnet50_convs(include_stem)):
        if index is not None and li != index:
            continue
        rng = np.random.default_rng([seed, li])   # one stream per layer
        d = masked_layer_inputs(rng, lay, K=K, batch=batch,
                                x_dist="uniform" if lay.Ci == 3 else "relu_normal")
        yield d, count


MOBILENETV2_DW = [(32, 112, 1, 1), (96, 112, 2, 1), (144, 56, 1, 1), (144, 56, 2, 1), (192, 28, 1, 2),
                  (192, 28, 2, 1), (384, 14, 1, 4), (576, 14, 1, 2), (576, 14, 2, 1), (960, 7, 1, 3)]


def mobilenetv2_dw(seed=6, batch=64, K=8, index=None):
    """The depthwise 3x3 layers of MobileNetV2 at 224x224 input (channels,
    input size, stride, multiplicity): list of (inputs dict, multiplicity)."""
    out = []
    for li, (c, hw, st, count) in enumerate(MOBILENETV2_DW):
        if index is not None and li != index:
            continue
        rng = np.random.default_rng([seed, li])
        out.append((masked_layer_inputs(rng, dwconv(c, hw, hw, 3, st), K=K, batch=batch,
                                        x_dist="relu_normal"), count))
    return out


def mobilenetv2_dw_field(seed=6, batch=64, K=8, index=0):
    """One depthwise 3x3 layer of MobileNetV2, finite-field variant: (inputs, multiplicity)."""
    c, hw, st, count = MOBILENETV2_DW[index]
    rng = np.random.default_rng([seed, index, 1])
    return field_layer_inputs(rng, dwconv(c, hw, hw, 3, st), K=K, batch=batch), count


def config5_layers():
    return [linear(4096, 25088), linear(4096, 4096), linear(1000, 4096)]


def config5(seed=5, batch=1024, K=8, index=None):
    """VGG classifier shape 25088 -> 4096 -> 4096 -> 1000, batch 1024, K=8."""
    out = []
    for li, L in enumerate(config5_layers()):
        if index is not None and li != index:
            continue
        rng = np.random.default_rng([seed, li])   # one stream per layer
        out.append(masked_layer_inputs(rng, L, K=K, batch=batch))
    return out
