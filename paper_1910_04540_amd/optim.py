"""Low-precision SGD over a model's parameters (arXiv 1910.04540, Sec. 3.1 "Front-end interface":
the optimizer wrapper that quantizes gradient, momentum and weight, each with its own format).

Nothing is computed here: one ``step()`` is one call of ``qsim_quant_sgd_step_table`` over all
parameters.  The wrapper only keeps the tensor list (and its device table) in step with the
tensors PyTorch hands it.
"""
from __future__ import annotations

from typing import Iterable, Optional, Union

import torch

from . import binding as Q
from .quantizer import BlockFloatingPoint, FixedPoint, FloatingPoint, _rounding

Number = Union[FloatingPoint, FixedPoint, BlockFloatingPoint, None]


def sgd_format(number: Number, rounding: Union[str, int] = "nearest", chunk: int = 256) -> Q.Format:
    """The ``qsim_format`` of a number descriptor inside the SGD step.  Block floating point shares
    one exponent per ``chunk`` consecutive elements of the flat tensor (a power of two, 4..1024);
    ``BlockFloatingPoint.dim`` has no meaning there and must be None."""
    mode = _rounding(rounding)
    if number is None:
        return Q.Format(Q.KIND_IDENTITY, 0, 0, 0, 0)
    if isinstance(number, FloatingPoint):
        return Q.Format(Q.KIND_FLOAT, number.exp, number.man, mode, number.flags())
    if isinstance(number, FixedPoint):
        return Q.Format(Q.KIND_FIXED, number.wl, number.fl, mode, number.flags())
    if isinstance(number, BlockFloatingPoint):
        if number.dim is not None:
            raise ValueError("inside the SGD step a block is a chunk of consecutive elements: use dim=None and `chunk`")
        return Q.Format(Q.KIND_BLOCK, number.wl, chunk, mode, number.flags())
    raise TypeError("number must be FloatingPoint, FixedPoint, BlockFloatingPoint or None")


class QuantSGD:
    """SGD with momentum whose gradient, momentum buffer and weight pass through a quantizer each.

    Per element, in fp32 (``include/qsim.h``, qsim_sgd_options):
        gq = Qg(grad);  d = gq + weight_decay * w;  v = Qm(momentum * v + (1 - dampening) * d)
        w  = w - lr * (nesterov ? d + momentum * v : v);  quantized copy = Qw(w)
    The momentum buffers start at zero, so the first step gives v = Qm((1 - dampening) * d)
    (``torch.optim.SGD`` takes v = d on its first step: the two differ when dampening != 0).

    ``weights``:
        "master"    parameters stay fp32 (the high-precision copy for accumulation, Sec. 1
                    footnote); ``quantized[i]`` holds Qw of parameter i after each step.
        "in_place"  the parameters themselves are kept in the weight format.
        "none"      no quantized copy is produced.

    Stochastic rounding: step s (counted from 0) of parameter t draws from Philox stream
    ``(s * len(params) + t) mod 2^32`` of ``seed``.
    """

    def __init__(self, params: Iterable[torch.Tensor], lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                 dampening: float = 0.0, nesterov: bool = False, grad_number: Number = None,
                 momentum_number: Number = None, weight_number: Number = None, grad_rounding="stochastic",
                 momentum_rounding="stochastic", weight_rounding="nearest", chunk: int = 256, weights: str = "master",
                 seed: int = 0):
        self.params = [p for p in params]
        if not self.params:
            raise ValueError("no parameters")
        if weights not in ("master", "in_place", "none"):
            raise ValueError('weights must be "master", "in_place" or "none"')
        for p in self.params:
            Q._device_f32(p.data, "parameter")
        self.lr, self.momentum = float(lr), float(momentum)
        self.options = Q.SgdOptions(float(weight_decay), float(dampening), 1 if nesterov else 0)
        self.fmt_grad = sgd_format(grad_number, grad_rounding, chunk)
        self.fmt_mom = sgd_format(momentum_number, momentum_rounding, chunk)
        self.fmt_weight = sgd_format(weight_number, weight_rounding, chunk)
        self.weights = weights
        self.seed = int(seed)
        self.steps = 0
        self.momentum_buffers = [torch.zeros_like(p.data) for p in self.params]
        self.quantized: Optional[list] = [torch.empty_like(p.data) for p in self.params] if weights == "master" else None
        self._list: Optional[Q.SgdTensorList] = None
        self._grad_ptrs: Optional[list] = None

    def zero_grad(self, set_to_none: bool = False) -> None:
        """Zeroing in place (the default here) keeps the gradient tensors, and with them the device
        table, from one step to the next."""
        for p in self.params:
            if p.grad is not None:
                if set_to_none:
                    p.grad = None
                else:
                    p.grad.detach_()
                    p.grad.zero_()

    def _tensor_list(self) -> Q.SgdTensorList:
        grads = []
        for p in self.params:
            if p.grad is None:
                raise RuntimeError("every parameter needs a gradient (run backward() first)")
            grads.append(p.grad.contiguous())
        ptrs = [g.data_ptr() for g in grads]
        if self._list is None or ptrs != self._grad_ptrs:      # PyTorch handed out new gradient tensors
            data = [p.data for p in self.params]
            w_q = self.quantized if self.weights == "master" else (data if self.weights == "in_place" else None)
            self._list = Q.SgdTensorList(data, grads, self.momentum_buffers, w_q)
            self._grad_ptrs = ptrs
        return self._list

    @torch.no_grad()
    def step(self) -> None:
        lst = self._tensor_list()
        stream = (self.steps * len(self.params)) & 0xFFFFFFFF
        lst.step(self.lr, self.momentum, self.fmt_grad, self.fmt_mom, self.fmt_weight, self.seed, stream, self.options)
        self.steps += 1
