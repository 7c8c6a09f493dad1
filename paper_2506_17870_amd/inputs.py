"""Seeded synthetic inputs with the shapes and value distributions of the paper's
workloads (ImageNet CNN layers and ViT MLPs, Sec. 4.1): NumPy only, no method arithmetic.

These generators hand out random draws only: fp32 values (what a trained layer or the
previous layer would hand to the quantiser of Eq. 1) and uniform int8 codes.  Quantisation,
decomposition, packing, GEMM and dequantisation are not done here: the library quantises on
the device (nq_quantize), the tests quantise with the CPU oracle.  Both the HIP
tests/benchmark and the CPU oracle's tests are fed from this one module so that they see
identical bytes.
"""
from __future__ import annotations

import numpy as np


def float_weights(N: int, K: int, sigma: float, seed: int = 0) -> np.ndarray:
    """fp32 N(0, sigma) weights [N,K] (the values a trained layer would hand to the quantiser)."""
    rng = np.random.default_rng(seed)
    return rng.normal(0.0, sigma, size=(N, K)).astype(np.float32)


def he_sigma(fan_in: int) -> float:
    return float(np.sqrt(2.0 / fan_in))


def uniform_activations(shape, seed: int = 0) -> np.ndarray:
    """int8 codes uniform over [-128, 127]."""
    rng = np.random.default_rng(seed + 1000003)
    return rng.integers(-128, 128, size=shape, dtype=np.int64).astype(np.int8)


def relu_floats(shape, seed: int = 0) -> np.ndarray:
    """fp32 ReLU-clipped N(0,1) data (what a layer after a ReLU hands to the activation quantiser)."""
    rng = np.random.default_rng(seed + 2000003)
    return np.maximum(rng.normal(0.0, 1.0, size=shape), 0.0).astype(np.float32)


def gaussian_floats(shape, seed: int = 0) -> np.ndarray:
    """fp32 N(0,1) data (a normalised image batch, a token matrix)."""
    rng = np.random.default_rng(seed + 3000003)
    return rng.normal(0.0, 1.0, size=shape).astype(np.float32)


def small_floats(n: int, scale: float, seed: int = 0) -> np.ndarray:
    rng = np.random.default_rng(seed + 4000003)
    return rng.normal(0.0, scale, size=n).astype(np.float32)


# The benchmark configurations (shapes of ResNet / ViT layers; values as above).
LINEAR_SMALL = dict(M=64, K=512, N=512, sigma=0.02, n_bits=8, l_bits=2)
CONV_RESNET18 = dict(B=32, H=56, W=56, Cin=64, Cout=64, KH=3, KW=3, stride=1, pad=1, n_bits=8, l_bits=2)
BOTTLENECK_RESNET101 = [
    dict(B=64, H=14, W=14, Cin=1024, Cout=256, KH=1, KW=1, stride=1, pad=0),
    dict(B=64, H=14, W=14, Cin=256, Cout=256, KH=3, KW=3, stride=1, pad=1),
    dict(B=64, H=14, W=14, Cin=256, Cout=1024, KH=1, KW=1, stride=1, pad=0),
]
VIT_MLP = [dict(M=12608, K=768, N=3072, sigma=0.02, n_bits=8, l_bits=3),
           dict(M=12608, K=3072, N=768, sigma=0.02, n_bits=8, l_bits=3)]
