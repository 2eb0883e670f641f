"""Front-end over the C-ABI: number-format descriptors, a functional ``quantize`` and the
``Quantizer`` autograd module that quantizes activations on the way forward and errors on the way
back (arXiv 1910.04540, Sec. 3.1 "Front-end interface": the quantization of activation and error
is injected into each layer as a separate module).

Nothing is computed here: every call goes to ``libqsim`` through ``binding``.  The descriptors only
carry the arguments of the corresponding entry point.
"""
from __future__ import annotations

import itertools
import math
from dataclasses import dataclass
from typing import Optional, Union

import torch

from . import binding as Q

ROUNDING = {"nearest": Q.RN_EVEN, "nearest_even": Q.RN_EVEN, "nearest_away": Q.RN_AWAY,
            "nearest_zero": Q.RN_ZERO, "stochastic": Q.STOCHASTIC}


def _rounding(mode: Union[str, int]) -> int:
    if isinstance(mode, str):
        if mode not in ROUNDING:
            raise ValueError(f"rounding must be one of {sorted(ROUNDING)}")
        return ROUNDING[mode]
    return int(mode)


@dataclass(frozen=True)
class FloatingPoint:
    """Floating point with ``exp`` exponent and ``man`` mantissa bits (Sec. 3.1 "Number Formats")."""
    exp: int
    man: int
    saturate: bool = True
    subnormal: bool = False

    def flags(self) -> int:
        return (Q.SATURATE if self.saturate else 0) | (Q.SUBNORMAL if self.subnormal else 0)


@dataclass(frozen=True)
class FixedPoint:
    """Fixed point with word length ``wl`` and ``fl`` fractional bits."""
    wl: int
    fl: int
    clamp: bool = True
    symmetric: bool = False

    def flags(self) -> int:
        return (Q.SATURATE if self.clamp else 0) | (Q.SYMMETRIC if self.symmetric else 0)


@dataclass(frozen=True)
class BlockFloatingPoint:
    """Block floating point with word length ``wl``; one shared exponent per index of ``dim``
    (``dim=None``: the whole tensor is one block)."""
    wl: int
    dim: Optional[int] = None
    symmetric: bool = False

    def flags(self) -> int:
        return Q.SYMMETRIC if self.symmetric else 0

    def layout(self, shape) -> tuple:
        """(outer, nblocks, inner) of a contiguous tensor of this shape."""
        n = math.prod(shape)
        if self.dim is None or len(shape) == 0:
            return 1, 1, max(n, 1)
        d = self.dim % len(shape)
        return max(math.prod(shape[:d]), 1), shape[d], max(math.prod(shape[d + 1:]), 1)


Number = Union[FloatingPoint, FixedPoint, BlockFloatingPoint, None]


def quantize(x: torch.Tensor, number: Number, rounding: Union[str, int] = "nearest", seed: int = 0,
             stream_id: int = 0, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Map ``x`` (float32, on the GPU) onto the values of ``number``; ``None`` is the identity."""
    if number is None:
        return x if out is None else out.copy_(x)
    x = x.contiguous()
    mode = _rounding(rounding)
    if x.numel() == 0:
        return torch.empty_like(x) if out is None else out
    if isinstance(number, FloatingPoint):
        return Q.float_quantize(x, number.exp, number.man, mode, number.flags(), seed, stream_id, out=out)
    if isinstance(number, FixedPoint):
        return Q.fixed_quantize(x, number.wl, number.fl, mode, number.flags(), seed, stream_id, out=out)
    if isinstance(number, BlockFloatingPoint):
        outer, nblocks, inner = number.layout(tuple(x.shape))
        return Q.block_quantize(x, outer, nblocks, inner, number.wl, mode, number.flags(), seed, stream_id, out=out)
    raise TypeError("number must be FloatingPoint, FixedPoint, BlockFloatingPoint or None")


class _QuantizeBothWays(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, module, call):
        ctx.module, ctx.call = module, call
        if module.forward_number is None:
            return x.view_as(x)
        return quantize(x, module.forward_number, module.forward_rounding, module.seed, 2 * call)

    @staticmethod
    def backward(ctx, grad_out):
        m = ctx.module
        if m.backward_number is None:
            return grad_out, None, None
        return quantize(grad_out, m.backward_number, m.backward_rounding, m.seed, 2 * ctx.call + 1), None, None


class Quantizer(torch.nn.Module):
    """Quantizes the activation passing forward and the error passing backward, each with its own
    number format and rounding mode.

    Stochastic rounding draws from Philox streams ``2 * call`` (forward) and ``2 * call + 1``
    (backward) of ``seed``, where ``call`` counts this module's forward calls: a run is
    reproducible from the seed, and no two calls share random words.  Two modules with the same
    seed would round with the same words, so without a seed every module takes the next of a
    process-wide sequence (reproducible as long as the modules are created in the same order).
    """

    _next_seed = itertools.count(1 << 32)

    def __init__(self, forward_number: Number = None, backward_number: Number = None,
                 forward_rounding: Union[str, int] = "nearest", backward_rounding: Union[str, int] = "nearest",
                 seed: Optional[int] = None):
        super().__init__()
        self.forward_number, self.backward_number = forward_number, backward_number
        self.forward_rounding, self.backward_rounding = _rounding(forward_rounding), _rounding(backward_rounding)
        self.seed = int(seed) if seed is not None else next(Quantizer._next_seed)
        self.calls = 0

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        call = self.calls
        self.calls += 1
        return _QuantizeBothWays.apply(x, self, call)

    def extra_repr(self) -> str:
        return (f"forward={self.forward_number}, backward={self.backward_number}, "
                f"rounding=({self.forward_rounding}, {self.backward_rounding}), seed={self.seed}")
