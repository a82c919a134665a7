"""Seeded synthetic inputs with the shapes and value distributions of the paper's layers.

This module holds NO arithmetic of the method (no quantisation, rounding, GEMM or update):
only numpy random draws.  It is the one piece of code that both the CPU oracle's tests and
the HIP library's tests / benchmark use, so that both sides see the same bytes.

The tensors stand in for activations, weights and back-propagated errors of the networks
the paper trains (ResNet-50 on ImageNet-1K, GNMT and Transformer on WMT16, Section 4);
those datasets and trained weights are not available, only layer shapes and plausible
value distributions are borrowed.  "N(0, s)" takes s as the standard deviation.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 190512334 * 10


def _rng(config: int, ordinal: int) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + 1000 * config + ordinal)


def normal(config, ordinal, shape, std=1.0):
    return (_rng(config, ordinal).standard_normal(shape, dtype=np.float32) * np.float32(std))


def relu_normal(config, ordinal, shape, std=1.0):
    """max(0, z), z ~ N(0, std): a post-ReLU activation, about half exact zeros."""
    return np.maximum(normal(config, ordinal, shape, std), np.float32(0))


def uniform(config, ordinal, shape, lo, hi):
    return _rng(config, ordinal).uniform(lo, hi, size=shape).astype(np.float32)


def xavier_uniform(config, ordinal, fan_in, fan_out):
    a = float(np.sqrt(6.0 / (fan_in + fan_out)))
    return uniform(config, ordinal, (fan_in, fan_out), -a, a)


def kaiming_normal(config, ordinal, fan_in, fan_out):
    return normal(config, ordinal, (fan_in, fan_out), float(np.sqrt(2.0 / fan_in)))


@dataclass
class Layer:
    """One GEMM layer X[M,K] . W[K,N] = Y[M,N] with its error dY[M,N] (all FP32, unscaled)."""
    name: str
    M: int
    N: int
    K: int
    X: np.ndarray
    W: np.ndarray
    dY: np.ndarray
    loss_scale: float
    extra: dict = field(default_factory=dict)


def config1(n: int = 256) -> Layer:
    """Single forward GEMM, M=N=K=n, A and B ~ N(0,1)."""
    return Layer("cfg1_square", n, n, n, normal(1, 0, (n, n)), normal(1, 1, (n, n)),
                 normal(1, 2, (n, n)), 1.0)


def config2(batch: int = 32, hw: int = 28, cin: int = 128, cout: int = 128) -> Layer:
    """ResNet-50-style 3x3 convolution taken as a GEMM on an explicitly lowered operand:
    M = batch*hw*hw, K = 9*cin, N = cout; Kaiming-normal weights, post-ReLU activations,
    errors N(0,1e-4) with loss scale 2**12."""
    M, K, N = batch * hw * hw, 9 * cin, cout
    return Layer("cfg2_resnet_conv3x3", M, N, K, relu_normal(2, 0, (M, K)),
                 kaiming_normal(2, 1, K, N), normal(2, 2, (M, N), 1e-4), 2.0 ** 12)


def config3(tokens: int = 4096, d_model: int = 512, d_ff: int = 2048):
    """Transformer-base FFN, two layers; errors N(0,1e-5) with the loss scale pinned at the
    dynamic scaler's floor 2**10."""
    l1 = Layer("cfg3_ffn1", tokens, d_ff, d_model, normal(3, 0, (tokens, d_model)),
               xavier_uniform(3, 1, d_model, d_ff), normal(3, 2, (tokens, d_ff), 1e-5), 2.0 ** 10)
    l2 = Layer("cfg3_ffn2", tokens, d_model, d_ff, relu_normal(3, 3, (tokens, d_ff)),
               xavier_uniform(3, 4, d_ff, d_model), normal(3, 5, (tokens, d_model), 1e-5),
               2.0 ** 10)
    return l1, l2


def config4(batch: int = 128, hidden: int = 1024, steps: int = 50) -> Layer:
    """GNMT-style LSTM gate GEMM: [x;h] (K = 2*hidden) -> 4 gates (N = 4*hidden), `steps`
    timesteps.  X holds the x_t halves for all steps ([steps, batch, hidden], U(-1,1)); the
    h halves are produced by the caller's cell stub.  extra['h0'] is the initial state,
    dY the gate errors for all steps ([steps*batch, N], N(0,1e-4), loss scale 2**12)."""
    K, N = 2 * hidden, 4 * hidden
    lay = Layer("cfg4_gnmt_lstm", batch, N, K, uniform(4, 0, (steps, batch, hidden), -1.0, 1.0),
                uniform(4, 1, (K, N), -0.1, 0.1), normal(4, 2, (steps * batch, N), 1e-4), 2.0 ** 12)
    lay.extra["h0"] = uniform(4, 3, (batch, hidden), -1.0, 1.0)
    lay.extra["steps"] = steps
    lay.extra["hidden"] = hidden
    return lay


def config5(tokens: int = 16384, d_in: int = 1024, d_out: int = 4096) -> Layer:
    """Transformer-big weight gradient + update: contraction over `tokens`; errors
    N(0,1e-5) with loss scale 2**14; master weights Xavier-uniform (stored as float16 by
    the caller); lr = 1e-3."""
    lay = Layer("cfg5_wgrad_update", tokens, d_out, d_in, normal(5, 0, (tokens, d_in)),
                xavier_uniform(5, 1, d_in, d_out), normal(5, 2, (tokens, d_out), 1e-5), 2.0 ** 14)
    lay.extra["lr"] = 1e-3
    lay.extra["seed"] = 0x1905_1233_4000_0005
    return lay


def random_f32_bit_patterns(seed: int, n: int) -> np.ndarray:
    """n FP32 values drawn uniformly over all 2**32 bit patterns (includes NaN, Inf,
    denormals) -- for conversion tests."""
    bits = np.random.default_rng(seed).integers(0, 2 ** 32, size=n, dtype=np.uint64)
    return bits.astype(np.uint32).view(np.float32)


def random_e5m2_codes(seed: int, shape, finite_only: bool = True) -> np.ndarray:
    """Uniform random E5M2 byte codes; with finite_only the Inf/NaN codes are excluded."""
    rng = np.random.default_rng(seed)
    c = rng.integers(0, 256, size=shape, dtype=np.uint16).astype(np.uint8)
    if finite_only:
        bad = (c & 0x7C) == 0x7C
        c[bad] = (c[bad] & 0x83) | 0x38  # exponent 14 instead of 31
    return c
