"""Seeded synthetic inputs and layer shapes for the SDGP backward-data path.

This module serves both the GPU library's callers and the CPU oracle's tests,
so it contains none of the method's arithmetic: only shapes, random tensors and
storage conversion.  Everything is generated on the host with numpy's PCG64 and
returned as numpy arrays; bfloat16 tensors are ``uint16`` bit patterns.

The tensors stand in for the CIFAR-10 / ImageNet gradients and trained weights
of the paper's evaluation (Sec. IV): output data gradients are Laplace
distributed with a fraction of exact zeros (Sec. III-C reports that almost a
quarter of a 16-bit gradient map is exactly zero), weights are He-normal.  The
zeros are independent Bernoulli draws, not spatially clustered as in Fig. 5.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F32, BF16 = 0, 1


# ----------------------------------------------------------------- storage

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even; inputs must be finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32, exact."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: int) -> np.ndarray:
    return f32_to_bf16_bits(x) if dtype == BF16 else np.ascontiguousarray(x, dtype=np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Stored tensor (uint16 bf16 bits or float32) -> float64 values."""
    return (bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


# --------------------------------------------------------------- generators

def normal(shape, std: float, seed: int, dtype: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return to_storage(x, dtype)


def laplace_with_zeros(shape, scale: float, zero_frac: float, seed: int, dtype: int) -> np.ndarray:
    """Laplace(0, scale) values with an independent fraction ``zero_frac`` set to +0."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == BF16 else np.float32)
    step = 1 << 24
    for lo in range(0, n, step):
        k = min(step, n - lo)
        mag = rng.standard_exponential(size=k, dtype=np.float32) * np.float32(scale)
        u = rng.random(size=k, dtype=np.float32)
        # one uniform decides both: [0, zero_frac) -> zero, the rest split evenly into signs
        x = np.where(u < zero_frac, np.float32(0.0),
                     np.where(u < zero_frac + (1.0 - zero_frac) / 2, -mag, mag)).astype(np.float32)
        out[lo:lo + k] = to_storage(x, dtype)
    return out.reshape(shape)


# ------------------------------------------------------------------- shapes

@dataclass(frozen=True)
class ConvLayer:
    """One convolution (or, with H = Wd = R = S = 1, linear) layer's backward-data problem."""
    name: str
    B: int
    H: int          # input height (the size of dD)
    Wd: int         # input width
    C_in: int
    C_out: int
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.Wd + 2 * self.pad - self.S) // self.stride + 1

    @property
    def dO_shape(self):
        return (self.B, self.P, self.Q, self.C_out)

    @property
    def W_shape(self):
        return (self.C_out, self.R, self.S, self.C_in)

    @property
    def dD_shape(self):
        return (self.B, self.H, self.Wd, self.C_in)

    @property
    def dense_flops(self) -> float:
        """Multiply-adds x2 of the unpruned backward-data product."""
        return 2.0 * self.B * self.P * self.Q * self.R * self.S * self.C_out * self.C_in

    def bytes_moved(self, elem: int = 2) -> float:
        """dO + W + dD, each touched once."""
        n = (self.B * self.P * self.Q * self.C_out + self.R * self.S * self.C_out * self.C_in
             + self.B * self.H * self.Wd * self.C_in)
        return float(n * elem)

    def with_batch(self, B: int) -> "ConvLayer":
        return ConvLayer(self.name, B, self.H, self.Wd, self.C_in, self.C_out, self.R, self.S,
                         self.stride, self.pad)


def resnet9_layers(B: int = 512):
    """3x3, stride 1, pad 1 layers of a 9-layer CIFAR ResNet (Sec. IV: ResNet-9 on CIFAR-10)."""
    spec = [(3, 64, 32), (64, 128, 32), (128, 128, 16), (128, 256, 16), (256, 512, 8), (512, 512, 4)]
    return [ConvLayer(f"r9_{ci}x{co}_{hw}", B, hw, hw, ci, co, 3, 3, 1, 1) for ci, co, hw in spec]


def resnet50_bottleneck_layers(B: int = 128):
    """The three convolutions of a ResNet-50 bottleneck at 56x56 and at 14x14 (Sec. IV: ResNet-50)."""
    out = []
    for hw, wide, narrow in ((56, 256, 64), (14, 1024, 256)):
        out.append(ConvLayer(f"r50_{hw}_1x1_{wide}x{narrow}", B, hw, hw, wide, narrow, 1, 1, 1, 0))
        out.append(ConvLayer(f"r50_{hw}_3x3_{narrow}x{narrow}", B, hw, hw, narrow, narrow, 3, 3, 1, 1))
        out.append(ConvLayer(f"r50_{hw}_1x1_{narrow}x{wide}", B, hw, hw, narrow, wide, 1, 1, 1, 0))
    return out


def resnet50_all_layers(B: int = 256):
    """All 53 convolutions of ResNet-50 at 224x224 plus the 2048->1000 classifier.

    Standard architecture (7x7/2 stem, max-pool, four stages of 3/4/6/3 bottleneck
    blocks, stride on the 3x3 of the first block of stages 2-4, 1x1 projection
    shortcuts).  The paper names the network only (Sec. IV).
    """
    layers = [ConvLayer("conv1_7x7s2", B, 224, 224, 3, 64, 7, 7, 2, 3)]
    hw, c_prev = 56, 64
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        for blk in range(blocks):
            st = 2 if (blk == 0 and stage > 1) else 1
            pre = f"l{stage}b{blk}"
            layers.append(ConvLayer(pre + "_1x1a", B, hw, hw, c_prev, width, 1, 1, 1, 0))
            layers.append(ConvLayer(pre + "_3x3", B, hw, hw, width, width, 3, 3, st, 1))
            hw_out = hw // st
            layers.append(ConvLayer(pre + "_1x1b", B, hw_out, hw_out, width, 4 * width, 1, 1, 1, 0))
            if blk == 0:
                layers.append(ConvLayer(pre + "_down", B, hw, hw, c_prev, 4 * width, 1, 1, st, 0))
            hw, c_prev = hw_out, 4 * width
    layers.append(ConvLayer("fc", B, 1, 1, 2048, 1000, 1, 1, 1, 0))
    return layers


def layer_inputs(layer: ConvLayer, scale: float, zero_frac: float, seed: int, dtype: int = BF16):
    """(dO, W) for one layer: Laplace gradients with zeros, He-normal weights."""
    dO = laplace_with_zeros(layer.dO_shape, scale, zero_frac, seed, dtype)
    W = normal(layer.W_shape, float(np.sqrt(2.0 / (layer.R * layer.S * layer.C_in))), seed + 500_000, dtype)
    return dO, W


def linear_config1(seed: int = 0):
    """Single linear layer: dO fp32 [256,128] ~ N(0,1), W fp32 [128,256] ~ N(0, 1/128)."""
    dO = normal((256, 128), 1.0, 1000 + seed, F32)
    W = normal((128, 256), float(np.sqrt(1.0 / 128.0)), 1500 + seed, F32)
    return dO, W


def resnet50_layer_stats(index: int):
    """Per-layer gradient scale 10^-U(3,5) and zero fraction U(0.2,0.5), drawn from PCG64(5000+index)."""
    rng = np.random.Generator(np.random.PCG64(5000 + index))
    u = rng.uniform(3.0, 5.0)
    z = rng.uniform(0.2, 0.5)
    return float(10.0 ** (-u)), float(z)
