"""Seeded synthetic inputs for the feature-whitening hot path.

This module only draws random numbers and shapes them like ResNet layer inputs
(activations, weight gradients).  It holds none of the method's arithmetic:
no covariance, no whitening, no transforms.  Both the CPU oracle's tests and
the GPU path's tests / benchmark take their inputs from here so that the two
sides see byte-identical data.

The shapes stand in for the CIFAR ResNet-110 and ImageNet ResNet-50/18 layers
the paper trained on (Sec. 6); only layer geometry is used, never dataset items.

Conventions
-----------
* A convolution layer input is an activation tensor, returned in NHWC order
  ``[B, H, W, Cin]`` (float32 numpy).  ``to_layout`` converts to NCHW.
* ``dtype == "bf16"`` means every value has already been rounded to the nearest
  bfloat16 (ties to even) and is exactly representable; ``bf16_bits`` gives the
  16-bit patterns for upload.
* A fully connected layer input is a plain row matrix ``[N_rows, M]``.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

LAYOUT_ROWS = 0
LAYOUT_NCHW = 1
LAYOUT_NHWC = 2
LAYOUT_NHWC_KKC = 3   # NHWC tensor, features ordered (ky, kx, c)


@dataclass
class ConvDesc:
    """Geometry of one layer input.  For LAYOUT_ROWS: B = N_rows, Cin = M, H=W=kh=kw=stride=1, pad=0."""
    B: int
    Cin: int
    H: int
    W: int
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def P(self) -> int:
        return self.Ho * self.Wo

    @property
    def M(self) -> int:
        return self.Cin * self.kh * self.kw

    @property
    def n_rows(self) -> int:
        return self.B * self.P

    def astuple(self):
        return (self.B, self.Cin, self.H, self.W, self.kh, self.kw, self.stride, self.pad)


@dataclass
class Layer:
    name: str
    desc: ConvDesc
    S: int
    dtype: str                     # "f32" or "bf16" (dtype of the activation)
    act: np.ndarray                # NHWC [B,H,W,Cin] float32, or rows [N_rows, M]
    G: np.ndarray                  # [S, M] float32 weight gradient
    is_rows: bool = False
    meta: dict = field(default_factory=dict)


# ----------------------------------------------------------------------------- bf16 helpers
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """16-bit patterns of values that are already exactly representable in bfloat16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value not representable in bf16"
    return (u >> np.uint32(16)).astype(np.uint16)


def to_layout(act_nhwc: np.ndarray, layout: int) -> np.ndarray:
    if layout in (LAYOUT_NHWC, LAYOUT_NHWC_KKC):
        return np.ascontiguousarray(act_nhwc)
    if layout == LAYOUT_NCHW:
        return np.ascontiguousarray(np.transpose(act_nhwc, (0, 3, 1, 2)))
    raise ValueError("layout")


# ----------------------------------------------------------------------------- random pieces
def _orthogonal(rng: np.random.Generator, n: int) -> np.ndarray:
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.sign(np.diag(r))


def _gaussian_grad(rng, S, M, var):
    return (rng.standard_normal((S, M)) * np.sqrt(var)).astype(np.float32)


def _correlated_halfnormal(rng, n_pix, mix: np.ndarray, relu: bool = False) -> np.ndarray:
    """Rows z = mix @ w with w ~ N(0, I), then |z| (half-normal) or max(z, 0)."""
    C = mix.shape[0]
    out = np.empty((n_pix, C), dtype=np.float32)
    step = 1 << 18
    mt = np.ascontiguousarray(mix.T)
    for lo in range(0, n_pix, step):
        hi = min(n_pix, lo + step)
        z = rng.standard_normal((hi - lo, mix.shape[1])) @ mt
        out[lo:hi] = np.maximum(z, 0.0) if relu else np.abs(z)
    return out


# ----------------------------------------------------------------------------- the five configurations
def config1(seed: int = 0) -> Layer:
    """Fully connected layer, M=64, S=32, B=128; X = Z A with singular values of A log-spaced 1..100."""
    rng = np.random.default_rng(seed)
    M, S, B = 64, 32, 128
    Z = rng.standard_normal((B, M))
    U = _orthogonal(rng, M)
    V = _orthogonal(rng, M)
    sv = np.logspace(0.0, 2.0, M)
    A = (U * sv) @ V.T
    X = (Z @ A).astype(np.float32)
    G = _gaussian_grad(rng, S, M, 1e-2)
    d = ConvDesc(B=B, Cin=M, H=1, W=1)
    return Layer("C1-fc64", d, S, "f32", X, G, is_rows=True)


def _toeplitz_mix(C: int, r: float) -> np.ndarray:
    idx = np.arange(C)
    cov = r ** np.abs(idx[:, None] - idx[None, :])
    return np.linalg.cholesky(cov)


def config2(seed: int = 1, B: int = 128, HW: int = 32, Cin: int = 64, S: int = 64) -> Layer:
    """CIFAR-ResNet 3x3 conv, Cin=64 (M=576), 32x32, pad 1; half-normal with Toeplitz(0.5) channel correlation."""
    rng = np.random.default_rng(seed)
    d = ConvDesc(B=B, Cin=Cin, H=HW, W=HW, kh=3, kw=3, stride=1, pad=1)
    act = _correlated_halfnormal(rng, B * HW * HW, _toeplitz_mix(Cin, 0.5)).reshape(B, HW, HW, Cin)
    G = _gaussian_grad(rng, S, d.M, 1e-3)
    return Layer("C2-cifar3x3", d, S, "f32", act, G)


def _powerlaw_layer(name, seed, B, HW, Cin, S) -> Layer:
    rng = np.random.default_rng(seed)
    d = ConvDesc(B=B, Cin=Cin, H=HW, W=HW, kh=3, kw=3, stride=1, pad=1)
    U = _orthogonal(rng, Cin)
    mix = U * (np.arange(1, Cin + 1, dtype=np.float64) ** -0.75)
    act = _correlated_halfnormal(rng, B * HW * HW, mix)
    act *= np.float32(1.0 / np.sqrt(np.mean(act.astype(np.float64) ** 2)))
    act = round_to_bf16(act).reshape(B, HW, HW, Cin)
    G = _gaussian_grad(rng, S, d.M, 1e-3)
    return Layer(name, d, S, "bf16", act, G)


def config3(seed: int = 2, B: int = 256) -> Layer:
    """ResNet-50 bottleneck 3x3, Cin=256 (M=2304), 14x14; bf16, channel eigenvalues ~ k^-1.5."""
    return _powerlaw_layer("C3-r50-14", seed, B, 14, 256, 256)


def config4(seed: int = 3, B: int = 256) -> Layer:
    """ResNet-50 last stage 3x3, Cin=512 (M=4608), 7x7; bf16, same spectrum."""
    return _powerlaw_layer("C4-r50-7", seed, B, 7, 512, 512)


# ResNet-18 at 224x224: (name, Cin, H, k, stride, pad, Cout)
RESNET18_LAYERS = [
    ("conv1", 3, 224, 7, 2, 3, 64),
    ("l1.0.c1", 64, 56, 3, 1, 1, 64), ("l1.0.c2", 64, 56, 3, 1, 1, 64),
    ("l1.1.c1", 64, 56, 3, 1, 1, 64), ("l1.1.c2", 64, 56, 3, 1, 1, 64),
    ("l2.0.c1", 64, 56, 3, 2, 1, 128), ("l2.0.ds", 64, 56, 1, 2, 0, 128),
    ("l2.0.c2", 128, 28, 3, 1, 1, 128), ("l2.1.c1", 128, 28, 3, 1, 1, 128), ("l2.1.c2", 128, 28, 3, 1, 1, 128),
    ("l3.0.c1", 128, 28, 3, 2, 1, 256), ("l3.0.ds", 128, 28, 1, 2, 0, 256),
    ("l3.0.c2", 256, 14, 3, 1, 1, 256), ("l3.1.c1", 256, 14, 3, 1, 1, 256), ("l3.1.c2", 256, 14, 3, 1, 1, 256),
    ("l4.0.c1", 256, 14, 3, 2, 1, 512), ("l4.0.ds", 256, 14, 1, 2, 0, 512),
    ("l4.0.c2", 512, 7, 3, 1, 1, 512), ("l4.1.c1", 512, 7, 3, 1, 1, 512), ("l4.1.c2", 512, 7, 3, 1, 1, 512),
    ("fc", 512, 1, 1, 1, 0, 1000),
]


def config5_layer(index: int, B: int = 256, scale: float = 1.0) -> Layer:
    """One layer of the ResNet-18 sweep; bf16 half-normal with a per-layer random channel correlation.

    ``scale`` < 1 shrinks the spatial size (for CPU-sized parity cases) while keeping Cin, k, stride.
    """
    name, Cin, H, k, stride, pad, Cout = RESNET18_LAYERS[index]
    rng = np.random.default_rng(100 + index)
    if scale != 1.0 and H > 1:
        H = max(k, int(round(H * scale)))
    A = rng.standard_normal((Cin, 2 * Cin))
    cov = A @ A.T
    dinv = 1.0 / np.sqrt(np.diag(cov))
    cov = cov * dinv[:, None] * dinv[None, :]
    mix = np.linalg.cholesky(cov)
    if name == "fc":
        d = ConvDesc(B=B, Cin=Cin, H=1, W=1)
        X = round_to_bf16(_correlated_halfnormal(rng, B, mix))
        G = _gaussian_grad(rng, Cout, Cin, 1e-3)
        return Layer("C5-" + name, d, Cout, "bf16", X, G, is_rows=True)
    d = ConvDesc(B=B, Cin=Cin, H=H, W=H, kh=k, kw=k, stride=stride, pad=pad)
    act = round_to_bf16(_correlated_halfnormal(rng, B * H * H, mix)).reshape(B, H, H, Cin)
    G = _gaussian_grad(rng, Cout, d.M, 1e-3)
    return Layer("C5-" + name, d, Cout, "bf16", act, G)


def small_conv(seed: int, B: int, Cin: int, H: int, W: int, k: int, stride: int, pad: int, S: int,
               dtype: str = "f32", relu: bool = False) -> Layer:
    """Small odd-shaped conv layer for parity tests (ragged tiles, strides, borders)."""
    rng = np.random.default_rng(seed)
    d = ConvDesc(B=B, Cin=Cin, H=H, W=W, kh=k, kw=k, stride=stride, pad=pad)
    mix = _toeplitz_mix(Cin, 0.6) if Cin > 1 else np.ones((1, 1))
    act = _correlated_halfnormal(rng, B * H * W, mix, relu=relu).reshape(B, H, W, Cin)
    if dtype == "bf16":
        act = round_to_bf16(act)
    G = _gaussian_grad(rng, S, d.M, 1e-3)
    return Layer(f"small-{seed}", d, S, dtype, act, G)


def small_rows(seed: int, n_rows: int, M: int, S: int, dtype: str = "f32", cond: float = 1e3) -> Layer:
    """Small fully connected layer input with a chosen population condition number."""
    rng = np.random.default_rng(seed)
    sv = np.logspace(0.0, 0.5 * np.log10(cond), M)
    A = (_orthogonal(rng, M) * sv) @ _orthogonal(rng, M).T
    X = (rng.standard_normal((n_rows, M)) @ A + rng.standard_normal(M)).astype(np.float32)
    if dtype == "bf16":
        X = round_to_bf16(X)
    G = _gaussian_grad(rng, S, M, 1e-2)
    return Layer(f"rows-{seed}", ConvDesc(B=n_rows, Cin=M, H=1, W=1), S, dtype, X, G, is_rows=True)


def spd_matrix(seed: int, M: int, spectrum: np.ndarray) -> np.ndarray:
    """Random symmetric positive definite matrix with the given eigenvalues (float64)."""
    rng = np.random.default_rng(seed)
    V = _orthogonal(rng, M)
    P = (V * np.asarray(spectrum, dtype=np.float64)) @ V.T
    return 0.5 * (P + P.T)
