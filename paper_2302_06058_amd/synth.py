"""Seeded synthetic inputs for the Bi-Mask hot path.

This module holds NO arithmetic of the method (no masks, scores, permutation
choice, compression or GEMM): only shapes, random draws and dtype conversion.
Both the CPU oracle's tests and the HIP path's tests / benchmark draw their
inputs from here, so the two sides always see identical bytes.

The layer shapes stand in for the networks the paper trains (Sec. 4.1:
ResNet-50 and DeiT-small on ImageNet); datasets and trained weights are not
used, only the GEMM shapes of the layers, with random values.

Host representation
  fp32 arrays : numpy float32
  bf16 arrays : numpy uint16 holding the bf16 bit pattern (round-to-nearest-even
                from float32); `bf16_to_f64` gives the exact real value.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------
# dtype conversion (exact, no method arithmetic)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest, ties to even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact real value of a stored array as float64."""
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def store(a32: np.ndarray, dtype: str) -> np.ndarray:
    """float32 draws -> the stored representation of `dtype`."""
    if dtype == BF16:
        return f32_to_bf16_bits(a32)
    return np.ascontiguousarray(a32, dtype=np.float32)


# --------------------------------------------------------------------------
# layer / config descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Layer:
    name: str
    I: int          # out features  (rows of W)
    J: int          # in features   (cols of W), already padded to a multiple of M
    T: int          # tokens = batch x spatial positions
    N: int = 2
    M: int = 4
    K: int = 100    # permutation candidates
    dtype: str = BF16
    seed: int = 0
    w_std: float = 1.0
    x_relu: bool = False
    x_std: float = 1.0
    dy_std: float = 1e-2
    j_real: Optional[int] = None   # un-padded J (ResNet stem: 147 -> 148)


@dataclass
class LayerData:
    layer: Layer
    W: np.ndarray          # I x J stored dtype
    X: Optional[np.ndarray]    # T x J
    dY: Optional[np.ndarray]   # T x I
    perms: np.ndarray      # K x I int32, each row a permutation of 0..I-1


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def gen_weights(layer: Layer) -> np.ndarray:
    rng = np.random.default_rng([layer.seed, 1])
    w = _normal(rng, (layer.I, layer.J), layer.w_std)
    if layer.j_real is not None and layer.j_real < layer.J:
        w[:, layer.j_real:] = 0.0          # zero padding columns
    return store(w, layer.dtype)


def gen_perms(layer: Layer, K: Optional[int] = None) -> np.ndarray:
    rng = np.random.default_rng([layer.seed, 2])
    K = layer.K if K is None else K
    out = np.empty((K, layer.I), dtype=np.int32)
    for c in range(K):
        out[c] = rng.permutation(layer.I).astype(np.int32)
    return out


def gen_activations(layer: Layer, T: Optional[int] = None) -> np.ndarray:
    rng = np.random.default_rng([layer.seed, 3])
    T = layer.T if T is None else T
    x = _normal(rng, (T, layer.J), layer.x_std)
    if layer.x_relu:
        np.maximum(x, 0.0, out=x)
    if layer.j_real is not None and layer.j_real < layer.J:
        x[:, layer.j_real:] = 0.0
    return store(x, layer.dtype)


def gen_out_grad(layer: Layer, T: Optional[int] = None) -> np.ndarray:
    rng = np.random.default_rng([layer.seed, 4])
    T = layer.T if T is None else T
    return store(_normal(rng, (T, layer.I), layer.dy_std), layer.dtype)


def gen_layer(layer: Layer, T: Optional[int] = None, K: Optional[int] = None,
              with_acts: bool = True) -> LayerData:
    """All arrays of one layer.  `T`/`K` may be reduced for bounded samples."""
    return LayerData(
        layer=layer,
        W=gen_weights(layer),
        X=gen_activations(layer, T) if with_acts else None,
        dY=gen_out_grad(layer, T) if with_acts else None,
        perms=gen_perms(layer, K),
    )


# --------------------------------------------------------------------------
# the five workload configurations
# --------------------------------------------------------------------------
def _pad(J: int, M: int) -> int:
    return (J + M - 1) // M * M


def config1() -> List[Layer]:
    return [Layer("c1.linear", 64, 128, 32, 2, 4, 4, F32, 1001, 1.0, False, 1.0, 1.0)]


def config2() -> List[Layer]:
    J = 2304
    return [Layer("c2.layer3.conv3x3", 256, J, 12544, 2, 4, 100, BF16, 1002,
                  float(np.sqrt(2.0 / J)), True, 1.0, 1e-2)]


def resnet50_gemm_shapes(batch: int = 64) -> List[Tuple[str, int, int, int]]:
    """(name, I, J, T) of every conv (as im2col GEMM) and the fc of a ResNet-50
    with 224x224 inputs, bottleneck blocks with the stride on the 3x3 conv."""
    out: List[Tuple[str, int, int, int]] = []
    out.append(("stem.conv7x7", 64, 3 * 7 * 7, batch * 112 * 112))
    inplanes, hw = 64, 56
    for li, (planes, blocks, stride) in enumerate(
            [(64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)], start=1):
        for b in range(blocks):
            s = stride if b == 0 else 1
            hw_in, hw_out = hw, hw // s
            p = f"layer{li}.{b}"
            out.append((p + ".conv1", planes, inplanes, batch * hw_in * hw_in))
            out.append((p + ".conv2", planes, planes * 9, batch * hw_out * hw_out))
            out.append((p + ".conv3", planes * 4, planes, batch * hw_out * hw_out))
            if b == 0:
                out.append((p + ".downsample", planes * 4, inplanes, batch * hw_out * hw_out))
            inplanes, hw = planes * 4, hw_out
    out.append(("fc", 1000, 2048, batch))
    return out


def config3(N: int = 2, M: int = 4) -> List[Layer]:
    layers = []
    for idx, (name, I, J, T) in enumerate(resnet50_gemm_shapes(64)):
        Jp = _pad(J, M)
        layers.append(Layer("c3." + name, I, Jp, T, N, M, 100, BF16, 1003 + idx,
                            float(np.sqrt(2.0 / J)), name != "stem.conv7x7", 1.0, 1e-2,
                            J if Jp != J else None))
    return layers


def config4() -> List[Layer]:
    layers = []
    T = 197 * 128
    shapes = [("qkv", 1152, 384), ("proj", 384, 384), ("fc1", 1536, 384), ("fc2", 384, 1536)]
    for (N, M) in [(2, 4), (1, 4), (4, 8)]:
        for si, (name, I, J) in enumerate(shapes):
            layers.append(Layer(f"c4.{name}.{N}of{M}", I, J, T, N, M, 100, BF16,
                                1004 + 10 * si, 0.02, False, 1.0, 1e-2))
    return layers


def config5() -> List[Layer]:
    return [
        Layer("c5.up", 11008, 4096, 8192, 2, 4, 100, BF16, 1005, 0.02, False, 1.0, 1e-2),
        Layer("c5.down", 4096, 11008, 8192, 2, 4, 100, BF16, 1006, 0.02, False, 1.0, 1e-2),
    ]


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def get_config(n: int) -> List[Layer]:
    return CONFIGS[n]()
