"""Seeded synthetic workloads for the K-FAC hot path: layer shapes and input tensors.

This module holds no K-FAC arithmetic.  It only describes *shapes* (the ResNet-50 layer table the
paper's experiments run on, Sec. 5 "Experiments", and the three single-layer cases used by the
tests) and draws the random input tensors that both the float64 CPU oracle and the HIP library
are fed.  Everything is a plain numpy array in the logical (n, c, y, x) index order; how a tensor
is laid out in device memory is the binding's business.

Value distributions (stand-ins for ImageNet activations, which are not available here):
  * the input of the first convolution is plain N(0, 1) (it is the mean-subtracted image);
  * every other layer input is max(0, z), z ~ N(0, 1): about half the entries are exact zeros and
    the mean is 1/sqrt(2*pi), as after a ReLU;
  * output gradients are N(0, sigma^2 = 1e-2); weight gradients are N(0, sigma^2 = 1e-3).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List

import numpy as np

TENSOR_ACT, TENSOR_GOUT, TENSOR_GRADW = 0, 1, 2

SIGMA_GOUT = 0.1          # N(0, 1e-2): the second argument is the variance
SIGMA_GRADW = 1e-3 ** 0.5  # N(0, 1e-3)


@dataclass(frozen=True)
class LayerShape:
    """One conv / fc layer as the K-FAC factor builders see it (fc: H = W = kh = kw = 1)."""
    name: str
    N: int
    C_in: int
    H: int
    W: int
    C_out: int
    kh: int
    kw: int
    stride: int
    pad: int
    relu_input: bool = True
    has_bias: bool = True

    @property
    def H_out(self) -> int:
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def W_out(self) -> int:
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def R(self) -> int:
        """Number of unfolded rows: one per (image, output position)."""
        return self.N * self.H_out * self.W_out

    @property
    def d_A(self) -> int:
        return self.C_in * self.kh * self.kw + (1 if self.has_bias else 0)

    @property
    def d_G(self) -> int:
        return self.C_out

    def with_batch(self, N: int) -> "LayerShape":
        return replace(self, N=N)


def _bottleneck_stage(prefix: str, n_blocks: int, c_in: int, width: int, h_in: int, stride: int,
                      N: int) -> List[LayerShape]:
    """Bottleneck blocks of one ResNet stage, stride on the 3x3 convolution (the "v1.5" layout)."""
    layers = []
    c_out = 4 * width
    h = h_in
    for b in range(n_blocks):
        s = stride if b == 0 else 1
        cin_b = c_in if b == 0 else c_out
        h_b = h
        layers.append(LayerShape(f"{prefix}.{b}.conv1", N, cin_b, h_b, h_b, width, 1, 1, 1, 0))
        layers.append(LayerShape(f"{prefix}.{b}.conv2", N, width, h_b, h_b, width, 3, 3, s, 1))
        h_o = (h_b + 2 - 3) // s + 1
        layers.append(LayerShape(f"{prefix}.{b}.conv3", N, width, h_o, h_o, c_out, 1, 1, 1, 0))
        if b == 0:
            layers.append(LayerShape(f"{prefix}.{b}.downsample", N, cin_b, h_b, h_b, c_out, 1, 1, s, 0))
        h = h_o
    return layers


def resnet50_layers(N: int = 32) -> List[LayerShape]:
    """The 53 convolutions (incl. 4 projection shortcuts) and the fc layer of ResNet-50 at 224x224."""
    layers = [LayerShape("conv1", N, 3, 224, 224, 64, 7, 7, 2, 3, relu_input=False)]
    layers += _bottleneck_stage("layer1", 3, 64, 64, 56, 1, N)
    layers += _bottleneck_stage("layer2", 4, 256, 128, 56, 2, N)
    layers += _bottleneck_stage("layer3", 6, 512, 256, 28, 2, N)
    layers += _bottleneck_stage("layer4", 3, 1024, 512, 14, 2, N)
    layers.append(LayerShape("fc", N, 2048, 1, 1, 1000, 1, 1, 1, 0))
    return layers


def resnet50_bn_channels() -> List[int]:
    """Channel count of the batch-normalisation layer that follows each of the 53 convolutions."""
    return [l.C_out for l in resnet50_layers(1) if l.name != "fc"]


def config0() -> LayerShape:
    """Small single conv layer (fp32, NCHW): the case the oracle finishes in milliseconds."""
    return LayerShape("cfg0.conv3x3", 8, 16, 8, 8, 16, 3, 3, 1, 1)


def config1(N: int = 32) -> LayerShape:
    """ResNet-50 stage-5 3x3 convolution: d_A = 4609 from 1568 unfolded rows, d_G = 512."""
    return LayerShape("cfg1.stage5.conv3x3", N, 512, 7, 7, 512, 3, 3, 1, 1)


def config2(N: int = 32) -> LayerShape:
    """ResNet-50 first convolution: d_A = 148 from 401,408 unfolded rows, d_G = 64."""
    return LayerShape("cfg2.conv1", N, 3, 224, 224, 64, 7, 7, 2, 3, relu_input=False)


def _rng(seed: int, layer_idx: int, step: int, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng([seed, layer_idx, step, tensor_id])


def make_act(shape: LayerShape, seed: int = 0, layer_idx: int = 0, step: int = 0) -> np.ndarray:
    """Layer input, float32, logical index order (n, c, y, x)."""
    z = _rng(seed, layer_idx, step, TENSOR_ACT).standard_normal(
        (shape.N, shape.C_in, shape.H, shape.W), dtype=np.float32)
    if shape.relu_input:
        np.maximum(z, 0.0, out=z)
    return z


def make_gout(shape: LayerShape, seed: int = 0, layer_idx: int = 0, step: int = 0) -> np.ndarray:
    """Gradient of the loss w.r.t. the layer output, float32, index order (n, o, y, x)."""
    z = _rng(seed, layer_idx, step, TENSOR_GOUT).standard_normal(
        (shape.N, shape.C_out, shape.H_out, shape.W_out), dtype=np.float32)
    z *= np.float32(SIGMA_GOUT)
    return z


def make_gradw(shape: LayerShape, seed: int = 0, layer_idx: int = 0, step: int = 0) -> np.ndarray:
    """Weight gradient d_G x d_A (bias gradient in the last column), float32.

    The column order it is interpreted in is whichever order the factor A it is paired with uses.
    """
    z = _rng(seed, layer_idx, step, TENSOR_GRADW).standard_normal(
        (shape.d_G, shape.d_A), dtype=np.float32)
    z *= np.float32(SIGMA_GRADW)
    return z


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); returned as float32 holding bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that already are bf16-representable, as uint16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def random_spd(dim: int, seed: int, eig_lo: float = 1e-3, eig_hi: float = 10.0,
               n_zero: int = 0) -> np.ndarray:
    """A seeded symmetric positive semi-definite float32 test matrix with a prescribed spectrum.

    Eigenvalues are log-uniform in [eig_lo, eig_hi] (the first `n_zero` of them exactly 0, to mimic
    a rank-deficient factor) in a random orthonormal basis.
    """
    rng = np.random.default_rng([seed, dim, n_zero])
    Q, _ = np.linalg.qr(rng.standard_normal((dim, dim)))
    eig = np.exp(rng.uniform(np.log(eig_lo), np.log(eig_hi), size=dim))
    eig[:n_zero] = 0.0
    S = (Q * eig) @ Q.T
    S = 0.5 * (S + S.T)
    return S.astype(np.float32)
