"""Seeded synthetic inputs and the workload table.

This module serves both the GPU library's tests/benchmark and the CPU oracle's tests.  It holds
NONE of the method's arithmetic: it only draws random fp32 tensors (numpy) and lists layer
shapes.  It imports neither the GPU binding nor the oracle.

The paper measures single binary convolutions and Bi-Real Net 18 on ImageNet-sized inputs
(Sec. 2.2, Fig. 5; Sec. 2.3, Table 2).  Neither trained weights nor images are available here, so
tensors of the same shapes stand in for them: activations ~ N(0,1) fp32 (what a batch-normed
feature map looks like to the sign function), weights i.i.d. +-1.
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 190805858


@dataclass(frozen=True)
class ConvLayer:
    """One binary convolution: NHWC input H x W x Cin, weights [Cout, k, k, Cin]."""
    H: int
    W: int
    Cin: int
    Cout: int
    stride: int = 1
    k: int = 3
    pad: int = 1

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.k) // self.stride + 1

    @property
    def K(self):
        """True number of bits under one output (kh*kw*Cin, not padded to words)."""
        return self.k * self.k * self.Cin

    def ops(self, N):
        """Binary operations as the metric counts them: 2*K*Cout*Ho*Wo*N."""
        return 2 * self.K * self.Cout * self.Ho * self.Wo * N


# The sixteen binary 3x3 convolutions of a Bi-Real-Net-18 body at 224x224 input (the stem and
# max-pool bring 224 down to 56): four stages of 64/128/256/512 channels, four convolutions per
# stage, the first convolution of stages 2-4 has stride 2.
BIREAL18_BODY = (
    [ConvLayer(56, 56, 64, 64)] * 4
    + [ConvLayer(56, 56, 64, 128, stride=2)] + [ConvLayer(28, 28, 128, 128)] * 3
    + [ConvLayer(28, 28, 128, 256, stride=2)] + [ConvLayer(14, 14, 256, 256)] * 3
    + [ConvLayer(14, 14, 256, 512, stride=2)] + [ConvLayer(7, 7, 512, 512)] * 3
)

CFG1_LAYER = ConvLayer(14, 14, 64, 64)
CFG2_LAYERS = [ConvLayer(56, 56, 64, 64), ConvLayer(28, 28, 128, 128),
               ConvLayer(14, 14, 256, 256), ConvLayer(7, 7, 512, 512)]
CFG2_BATCHES = (1, 64)
# (N, H, W, C) of the bit-pack-only workload; the last three exercise tails (C % 64 != 0).
CFG3_SHAPES = [(1, 56, 56, 64), (64, 28, 28, 128), (256, 56, 56, 256),
               (64, 28, 28, 80), (64, 28, 28, 200), (1, 7, 7, 80)]
CFG4_LAYERS = [ConvLayer(56, 56, 64, 128, stride=2), ConvLayer(28, 28, 128, 256, stride=2),
               ConvLayer(14, 14, 256, 512, stride=2)]
CFG4_BATCH = 128
CFG4_P_PLUS = 0.3
CFG5_BATCH = 256


def seed_for(cfg, layer=0):
    return BASE_SEED + 1000 * cfg + layer


def activations(shape, seed):
    """fp32 ~ N(0,1)."""
    return np.random.default_rng(seed).standard_normal(shape, dtype=np.float32)


def weights(shape, seed, p_plus=0.5):
    """fp32 +-1.0, P(+1) = p_plus."""
    rng = np.random.default_rng(seed ^ 0x5EED)
    return np.where(rng.random(shape, dtype=np.float32) < p_plus, np.float32(1.0), np.float32(-1.0))


def inject_zeros(x, seed, frac=0.01):
    """Set `frac` of the elements to +0.0 and a disjoint `frac` to -0.0 (in place, returns x)."""
    rng = np.random.default_rng(seed ^ 0x2E80)
    u = rng.random(x.shape, dtype=np.float32)
    x[u < frac] = np.float32(0.0)
    x[(u >= frac) & (u < 2 * frac)] = np.float32(-0.0)
    return x


def special_values():
    """A row of fp32 edge values: +-0, +-inf, +-NaN, +-denormal, +-max, +-tiny normal."""
    bits = np.array([0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC00000,
                     0x7F800001, 0xFF800001, 0x00000001, 0x80000001, 0x007FFFFF, 0x807FFFFF,
                     0x7F7FFFFF, 0xFF7FFFFF, 0x00800000, 0x80800000], dtype=np.uint32)
    return bits.view(np.float32).copy()


def affine(C, seed):
    """Per-channel scale ~ U(0.5, 1.5) and shift ~ N(0, 0.25^2) for the full-network glue."""
    rng = np.random.default_rng(seed ^ 0xAFF1)
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    beta = (0.25 * rng.standard_normal(C)).astype(np.float32)
    return gamma, beta
