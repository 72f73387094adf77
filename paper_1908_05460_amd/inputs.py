"""Seeded synthetic workloads: layer tables and input tensors.

Shared by the GPU tests, the oracle tests and the benchmark.  Holds none of the
method's arithmetic: only shapes and random inputs.

The paper trains a ResNet-20 and a VGG-19 on CIFAR-10 with batch size 128
(Section 3).  The tensors a weight-gradient kernel sees there are post-ReLU
activations and back-propagated output gradients; the stand-ins generated here
have the same shapes and the same gross structure:
  X  = max(z, 0),  z ~ N(0,1) i.i.d.   (about half exact zeros, half-normal otherwise)
  dY = 0.01 * z,   z ~ N(0,1) i.i.d.   (zero-mean, standard deviation 0.01)
in float32, optionally rounded once (round-to-nearest-even) to bfloat16 and
handed out as uint16 bit patterns.  Every tensor's stream is keyed by
(ROOT_SEED, config, batch, layer, tensor).
"""
from dataclasses import dataclass

import numpy as np

ROOT_SEED = 190805460
DY_STD = 0.01


@dataclass(frozen=True)
class Layer:
    name: str
    C: int
    K: int
    H: int
    W: int
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def flops(self, N):
        """Nominal FLOPs of the exact gradient (counts taps that fall on padding)."""
        return 2 * N * self.K * self.C * self.R * self.S * self.Ho * self.Wo

    def valid_flops(self, N):
        """FLOPs over taps that land inside X only."""
        def valid(H, Ho, R, st, pad):
            return sum(1 for h in range(Ho) for r in range(R) if 0 <= h * st + r - pad < H)
        vh = valid(self.H, self.Ho, self.R, self.stride, self.pad)
        vw = valid(self.W, self.Wo, self.S, self.stride, self.pad)
        return 2 * N * self.K * self.C * vh * vw


def smoke_stack():
    """Single 3x3 layer of the small configuration (N=16)."""
    return [Layer("c1", 16, 16, 32, 32)]


def resnet20_stack():
    """The 19 3x3 convolutions of a CIFAR ResNet-20 (first conv + 3 stages of 6)."""
    L = [Layer("r01", 3, 16, 32, 32)]
    L += [Layer(f"r{i:02d}", 16, 16, 32, 32) for i in range(2, 8)]
    L += [Layer("r08", 16, 32, 32, 32, stride=2)]
    L += [Layer(f"r{i:02d}", 32, 32, 16, 16) for i in range(9, 14)]
    L += [Layer("r14", 32, 64, 16, 16, stride=2)]
    L += [Layer(f"r{i:02d}", 64, 64, 8, 8) for i in range(15, 20)]
    return L


def vgg19_stack():
    """The 16 3x3 convolutions of a CIFAR VGG-19 (2x2 pooling between stages)."""
    spec = [(3, 64, 32), (64, 64, 32), (64, 128, 16), (128, 128, 16),
            (128, 256, 8), (256, 256, 8), (256, 256, 8), (256, 256, 8),
            (256, 512, 4), (512, 512, 4), (512, 512, 4), (512, 512, 4),
            (512, 512, 2), (512, 512, 2), (512, 512, 2), (512, 512, 2)]
    return [Layer(f"v{i + 1:02d}", c, k, hw, hw) for i, (c, k, hw) in enumerate(spec)]


# name -> (config id used in the seed, layer stack, batch size, element type)
WORKLOADS = {
    "single3x3_n16_fp32": (1, smoke_stack, 16, "fp32"),
    "resnet20_n128_fp32": (2, resnet20_stack, 128, "fp32"),
    "vgg19_n128_fp32": (3, vgg19_stack, 128, "fp32"),
    "vgg19_n512_bf16": (4, vgg19_stack, 512, "bf16"),
    "resnet20_schedule_sweep": (5, resnet20_stack, 128, "fp32"),
    "vgg19_schedule_sweep": (6, vgg19_stack, 128, "fp32"),      # the same sweep on the other stack the paper trains
}


def float32_to_bf16_bits(a):
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    bits = np.ascontiguousarray(a, np.float32).view(np.uint32)
    rounded = bits + (((bits >> 16) & 1) + np.uint32(0x7FFF))
    return (rounded >> 16).astype(np.uint16)


def bf16_bits_to_float32(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def _rng(config, batch, layer_index, tensor):
    return np.random.default_rng(np.random.SeedSequence([ROOT_SEED, config, batch, layer_index, tensor]))


def make_X(layer, N, config=0, batch=0, layer_index=0, dtype="fp32"):
    z = _rng(config, batch, layer_index, 0).standard_normal((N, layer.C, layer.H, layer.W), np.float32)
    np.maximum(z, 0, out=z)
    return float32_to_bf16_bits(z) if dtype == "bf16" else z


def make_dY(layer, N, config=0, batch=0, layer_index=0, dtype="fp32"):
    z = _rng(config, batch, layer_index, 1).standard_normal((N, layer.K, layer.Ho, layer.Wo), np.float32)
    z *= np.float32(DY_STD)
    return float32_to_bf16_bits(z) if dtype == "bf16" else z


def make_layer_inputs(layer, N, config=0, batch=0, layer_index=0, dtype="fp32"):
    """(X, dY) for one layer; float32 arrays, or uint16 bf16 bit patterns."""
    return (make_X(layer, N, config, batch, layer_index, dtype),
            make_dY(layer, N, config, batch, layer_index, dtype))
