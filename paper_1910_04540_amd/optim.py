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


class _Group:
    """The parameters that share one set of hyper-parameters: one device table, one launch per step."""

    def __init__(self, params, lr, momentum, weight_decay, dampening, nesterov, weights, first_stream):
        self.params = list(params)
        if not self.params:
            raise ValueError("a parameter group is empty")
        for p in self.params:
            Q._device_f32(p.data, "parameter")
        self.lr, self.momentum = float(lr), float(momentum)
        self.options = Q.SgdOptions(float(weight_decay), float(dampening), 1 if nesterov else 0)
        self.weights = weights
        self.first_stream = first_stream            # position of the group's first parameter among all parameters
        self.momentum_buffers = [torch.zeros_like(p.data) for p in self.params]
        self.quantized = [torch.empty_like(p.data) for p in self.params] if weights == "master" else None
        self._list: Optional[Q.SgdTensorList] = None
        self._ptrs: Optional[list] = None

    def tensor_list(self) -> Q.SgdTensorList:
        grads = []
        for p in self.params:
            if p.grad is None:
                raise RuntimeError("every parameter needs a gradient (run backward() first)")
            grads.append(p.grad.contiguous())
        # the list (and its device table) holds addresses: of the gradients, which PyTorch may hand out
        # anew, and of the parameters' storage, which `p.data = ...`, `model.float()` and the like replace
        ptrs = [g.data_ptr() for g in grads] + [p.data.data_ptr() for p in self.params]
        if self._list is None or ptrs != self._ptrs:
            data = [p.data for p in self.params]
            for d, m in zip(data, self.momentum_buffers):
                Q._device_f32(d, "parameter")
                if d.numel() != m.numel() or d.device != m.device:
                    raise RuntimeError("a parameter changed its size or device after the optimizer was built")
            w_q = self.quantized if self.weights == "master" else (data if self.weights == "in_place" else None)
            self._list = Q.SgdTensorList(data, grads, self.momentum_buffers, w_q)
            self._ptrs = ptrs
        return self._list


class QuantSGD:
    """SGD with momentum whose gradient, momentum buffer and weight pass through a quantizer each.

    Per element, in fp32 (``include/qsim.h``, qsim_sgd_options):
        gq = Qg(grad);  d = gq + weight_decay * w;  v = Qm(momentum * v + (1 - dampening) * d)
        w  = w - lr * (nesterov ? d + momentum * v : v);  quantized copy = Qw(w)
    The momentum buffers start at zero, so the first step gives v = Qm((1 - dampening) * d)
    (``torch.optim.SGD`` takes v = d on its first step: the two differ when dampening != 0).

    ``params``: an iterable of parameters, or of dicts ``{"params": [...], "lr": ..., "momentum": ...,
    "weight_decay": ..., "dampening": ..., "nesterov": ...}`` as ``torch.optim`` takes them (weights
    with decay and biases without, say); a missing key takes the value given to the constructor.
    Each group is one fused launch per step.

    ``weights``:
        "master"    parameters stay fp32 (the high-precision copy for accumulation, Sec. 1
                    footnote); ``quantized[i]`` holds Qw of parameter i after each step.
        "in_place"  the parameters themselves are kept in the weight format.
        "none"      no quantized copy is produced.

    Stochastic rounding: step s (counted from 0) of parameter t (counted over all groups in order)
    draws from Philox stream ``(s * number of parameters + t) mod 2^32`` of ``seed``.
    """

    def __init__(self, params: Iterable, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                 dampening: float = 0.0, nesterov: bool = False, grad_number: Number = None,
                 momentum_number: Number = None, weight_number: Number = None, grad_rounding="stochastic",
                 momentum_rounding="stochastic", weight_rounding="nearest", chunk: int = 256, weights: str = "master",
                 seed: int = 0):
        if weights not in ("master", "in_place", "none"):
            raise ValueError('weights must be "master", "in_place" or "none"')
        items = list(params)
        if not items:
            raise ValueError("no parameters")
        if not isinstance(items[0], dict):
            items = [{"params": items}]
        defaults = {"lr": lr, "momentum": momentum, "weight_decay": weight_decay, "dampening": dampening, "nesterov": nesterov}
        self.groups = []
        count = 0
        for item in items:
            unknown = set(item) - set(defaults) - {"params"}
            if unknown:
                raise ValueError(f"unknown keys in a parameter group: {sorted(unknown)}")
            cfg = {k: item.get(k, v) for k, v in defaults.items()}
            group = _Group(item["params"], cfg["lr"], cfg["momentum"], cfg["weight_decay"], cfg["dampening"], cfg["nesterov"],
                           weights, count)
            count += len(group.params)
            self.groups.append(group)
        self.fmt_grad = sgd_format(grad_number, grad_rounding, chunk)
        self.fmt_mom = sgd_format(momentum_number, momentum_rounding, chunk)
        self.fmt_weight = sgd_format(weight_number, weight_rounding, chunk)
        self.weights = weights
        self.seed = int(seed)
        self.steps = 0
        self.params = [p for g in self.groups for p in g.params]
        self.momentum_buffers = [m for g in self.groups for m in g.momentum_buffers]
        self.quantized: Optional[list] = [q for g in self.groups for q in g.quantized] if weights == "master" else None

    def zero_grad(self, set_to_none: bool = False) -> None:
        """Zeroing in place (the default here) keeps the gradient tensors, and with them the device
        tables, from one step to the next."""
        for p in self.params:
            if p.grad is not None:
                if set_to_none:
                    p.grad = None
                else:
                    p.grad.detach_()
                    p.grad.zero_()

    @torch.no_grad()
    def step(self) -> None:
        lists = [g.tensor_list() for g in self.groups]          # every gradient is checked before anything is updated
        base = self.steps * len(self.params)
        for g, lst in zip(self.groups, lists):
            lst.step(g.lr, g.momentum, self.fmt_grad, self.fmt_mom, self.fmt_weight, self.seed,
                     (base + g.first_stream) & 0xFFFFFFFF, g.options)
        self.steps += 1
