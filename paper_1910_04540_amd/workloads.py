"""Seeded synthetic inputs shaped like the training tensors the quantizers are applied to.

This module only draws numbers.  It holds none of the quantizers' arithmetic and serves both
the GPU tests/benchmark and the CPU oracle's tests, so that both sides see identical arrays.
Every generator uses ``numpy.random.Generator(PCG64(seed))`` and returns contiguous float32.

The paper evaluates on tensors from CIFAR10 training runs (Sec. 4, "Validation"); those are not
reproduced here.  The recipes below stand in for them: activations, gradients, weights and
matrices with the value structure (sparsity, dynamic range, outliers) that exercises rounding,
saturation and underflow.
"""
from __future__ import annotations

import numpy as np

# Full sizes of the five workloads.
N_SMALL = 1 << 20                     # 1: small tensor, N(0,1)
N_FIXED = 1 << 26                     # 2: 64 Mi elements, uniform body + wide outliers
BLOCK_SHAPE = (4096, 4096)            # 3: matrix with per-row magnitudes
ACT_SHAPE = (128, 256, 56, 56)        # 4: activation / gradient tensors
N_PARAMS = 25_600_000                 # 5: parameter count of a ResNet-50-sized model
N_PARAMS_RAGGED = 25_557_032          #    the same with a length that is no multiple of a chunk


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def normal_tensor(n: int = N_SMALL, seed: int = 1) -> np.ndarray:
    """Workload 1: x ~ N(0, 1)."""
    return _rng(seed).standard_normal(n, dtype=np.float32)


def uniform_with_outliers(n: int = N_FIXED, seed: int = 2) -> np.ndarray:
    """Workload 2: 90 % uniform on [-4, 4), 10 % N(0, variance 100) outliers."""
    g = _rng(seed)
    mask = g.random(n, dtype=np.float32) < np.float32(0.1)
    body = (g.random(n, dtype=np.float32) * np.float32(8.0) - np.float32(4.0)).astype(np.float32)
    wide = g.standard_normal(n, dtype=np.float32) * np.float32(10.0)
    return np.where(mask, wide, body).astype(np.float32)


def row_scaled_matrix(rows: int = BLOCK_SHAPE[0], cols: int = BLOCK_SHAPE[1], seed: int = 3) -> np.ndarray:
    """Workload 3: x[i, j] = a_i * N(0, 1) with a_i log-uniform over [1e-6, 1e3]."""
    g = _rng(seed)
    a = np.power(10.0, g.uniform(-6.0, 3.0, size=rows)).astype(np.float32)
    x = g.standard_normal((rows, cols), dtype=np.float32)
    return (x * a[:, None]).astype(np.float32)


def relu_activations(shape=ACT_SHAPE, seed: int = 4) -> np.ndarray:
    """Workload 4a: half exact zeros, the rest |N(0, 1)| (the output of a ReLU)."""
    g = _rng(seed)
    n = int(np.prod(shape))
    keep = g.random(n, dtype=np.float32) < np.float32(0.5)
    x = np.abs(g.standard_normal(n, dtype=np.float32))
    return np.where(keep, x, np.float32(0.0)).astype(np.float32).reshape(shape)


def lognormal_gradients(shape=ACT_SHAPE, seed: int = 5, overflow_fraction: float = 0.0) -> np.ndarray:
    """Workload 4b: sign * 10^z, z ~ N(-4, sd 2) clipped to [-10, 2].

    With ``overflow_fraction`` > 0 that share of the elements is multiplied by 1e4 so that a
    16-bit float's overflow path is reached as well (used by the parity tests only).
    """
    g = _rng(seed)
    n = int(np.prod(shape))
    z = np.clip(g.standard_normal(n, dtype=np.float32) * np.float32(2.0) - np.float32(4.0), -10.0, 2.0)
    mag = np.power(np.float32(10.0), z.astype(np.float32)).astype(np.float32)
    sign = np.where(g.random(n, dtype=np.float32) < np.float32(0.5), np.float32(-1.0), np.float32(1.0))
    x = (mag * sign).astype(np.float32)
    if overflow_fraction > 0.0:
        big = g.random(n, dtype=np.float32) < np.float32(overflow_fraction)
        x = np.where(big, x * np.float32(1e4), x).astype(np.float32)
    return x.reshape(shape)


def sgd_state(n: int = N_PARAMS, seeds=(6, 7, 8)):
    """Workload 5: (weights ~ N(0, sd 0.02), gradients ~ N(0, sd 1e-3), raw momentum ~ N(0, sd 1e-3))."""
    w = _rng(seeds[0]).standard_normal(n, dtype=np.float32) * np.float32(0.02)
    g = _rng(seeds[1]).standard_normal(n, dtype=np.float32) * np.float32(1e-3)
    m = _rng(seeds[2]).standard_normal(n, dtype=np.float32) * np.float32(1e-3)
    return w.astype(np.float32), g.astype(np.float32), m.astype(np.float32)


def resnet50_parameter_sizes() -> list:
    """Element counts of the parameter tensors of a ResNet-50 (bottleneck stages of 3, 4, 6 and 3
    blocks, widths 64 to 512 with expansion 4, batch-norm scale and shift after every convolution,
    a 1000-way classifier): 161 tensors, 25,557,032 parameters.  Used to shape the multi-tensor
    optimizer step like a real model: a few large tensors and many tiny ones."""
    sizes = [64 * 3 * 7 * 7, 64, 64]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(blocks):
            sizes += [planes * inplanes, planes, planes]                 # 1x1 reduce + norm
            sizes += [planes * planes * 9, planes, planes]               # 3x3 + norm
            sizes += [4 * planes * planes, 4 * planes, 4 * planes]       # 1x1 expand + norm
            if blk == 0:
                sizes += [4 * planes * inplanes, 4 * planes, 4 * planes]  # projection shortcut + norm
            inplanes = 4 * planes
    sizes += [1000 * 2048, 1000]
    return sizes


def all_exponents_probe(dropped_bits: int, seed: int = 11) -> np.ndarray:
    """Every (sign, exponent field, leading mantissa bits) combined with the low-bit patterns that
    decide a rounding (zero, one, just below/at/above half, all ones, a few random ones).

    ``dropped_bits`` = how many low mantissa bits a format with 23 - dropped_bits mantissa bits
    removes from a normal number.  Used to sweep a float format over the whole fp32 range without
    visiting all 2^32 encodings.
    """
    d = int(dropped_bits)
    assert 1 <= d <= 22
    g = _rng(seed)
    half = 1 << (d - 1)
    lows = {0, 1, half - 1, half, half + 1, (1 << d) - 1, (1 << d) - 2}
    lows |= {int(v) for v in g.integers(0, 1 << d, size=9)}
    lows = np.array(sorted(v for v in lows if 0 <= v < (1 << d)), dtype=np.uint32)
    high = np.arange(1 << (32 - d), dtype=np.uint64)          # sign, field, kept mantissa bits
    bits = ((high[:, None] << np.uint64(d)) | lows[None, :].astype(np.uint64)).astype(np.uint32)
    return bits.reshape(-1).view(np.float32)


def mixed_scales(n: int, seed: int = 12, lo_exp: int = -160, hi_exp: int = 130) -> np.ndarray:
    """fp32 values with exponents spread uniformly over [2^lo_exp, 2^hi_exp) (clipped to what
    fp32 holds, so the tails become denormals, zeros and Inf), random sign."""
    g = _rng(seed)
    e = g.uniform(lo_exp, hi_exp, size=n)
    with np.errstate(over="ignore", under="ignore"):
        x = (np.exp2(e) * (1.0 + g.random(n))).astype(np.float32)
    s = np.where(g.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    return (x * s).astype(np.float32)
