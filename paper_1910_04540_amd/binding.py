"""Thin Python binding of the libqsim C-ABI (include/qsim.h): argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the computation runs in
the library's kernels.  There is no fallback: if libqsim.so is not built, importing the entry
points raises.
"""
from __future__ import annotations

import ctypes
import functools
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libqsim.so")

RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC = 0, 1, 2, 3
SATURATE, SUBNORMAL, SYMMETRIC = 1, 2, 4
WORKSPACE_KEPT = 8             # block_quantize only: see qsim_block_quantize in include/qsim.h
KIND_IDENTITY, KIND_FLOAT, KIND_FIXED, KIND_BLOCK = 0, 1, 2, 3

# Every symbol include/qsim.h declares.
EXPORTS = ("qsim_float_quantize", "qsim_fixed_quantize", "qsim_block_quantize", "qsim_block_workspace_bytes",
           "qsim_set_barrier_wait_us", "qsim_quant_sgd_step", "qsim_quant_sgd_step_multi", "qsim_quant_sgd_step_ex",
           "qsim_quant_sgd_step_multi_ex", "qsim_sgd_table_bytes", "qsim_sgd_table_build", "qsim_quant_sgd_step_table",
           "qsim_float_quantize_at", "qsim_fixed_quantize_at", "qsim_block_quantize_at", "qsim_quant_sgd_step_at",
           "qsim_block_max", "qsim_block_quantize_with_max", "qsim_block_quantize_static", "qsim_status_string")
STATIC_SCRATCH_BYTES = 4 << 20   # QSIM_STATIC_SCRATCH_BYTES


class Format(ctypes.Structure):
    """qsim_format: kind, a, b, rounding, flags."""
    _fields_ = [("kind", ctypes.c_int), ("a", ctypes.c_int), ("b", ctypes.c_int),
                ("rounding", ctypes.c_int), ("flags", ctypes.c_uint32)]


class SgdOptions(ctypes.Structure):
    """qsim_sgd_options: weight_decay, dampening, nesterov."""
    _fields_ = [("weight_decay", ctypes.c_float), ("dampening", ctypes.c_float), ("nesterov", ctypes.c_int)]


class SgdTable(ctypes.Structure):
    """qsim_sgd_table: device, bytes, tiles, count, aligned."""
    _fields_ = [("device", ctypes.c_void_p), ("bytes", ctypes.c_size_t), ("tiles", ctypes.c_uint32),
                ("count", ctypes.c_int32), ("aligned", ctypes.c_int32)]


class QsimError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libqsim status {status}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load libqsim.so.  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1910_04540_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, u64, u32, ci, sz = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_size_t
    L.qsim_float_quantize.argtypes = [vp, vp, u64, ci, ci, ci, u32, u64, u32, vp]
    L.qsim_fixed_quantize.argtypes = [vp, vp, u64, ci, ci, ci, u32, u64, u32, vp]
    L.qsim_block_quantize.argtypes = [vp, vp, u64, u64, u64, u64, ci, ci, u32, u64, u32, vp, sz, vp]
    L.qsim_float_quantize_at.argtypes = [vp, vp, u64, u64, ci, ci, ci, u32, u64, u32, vp]
    L.qsim_fixed_quantize_at.argtypes = [vp, vp, u64, u64, ci, ci, ci, u32, u64, u32, vp]
    L.qsim_block_quantize_at.argtypes = [vp, vp, u64, u64, u64, u64, u64, ci, ci, u32, u64, u32, vp, sz, vp]
    L.qsim_block_max.argtypes = [vp, u64, u64, u64, u64, vp, vp, sz, vp]
    L.qsim_block_quantize_with_max.argtypes = [vp, vp, u64, u64, u64, u64, u64, ci, ci, u32, u64, u32, vp, vp]
    L.qsim_block_quantize_static.argtypes = [vp, vp, u64, u64, u64, u64, ci, ci, u32, u64, u32, vp]
    L.qsim_block_quantize_static.restype = ci
    L.qsim_block_workspace_bytes.argtypes = [u64, u64, u64, u64]
    L.qsim_block_workspace_bytes.restype = sz
    L.qsim_quant_sgd_step.argtypes = [vp, vp, vp, vp, u64, ctypes.c_float, ctypes.c_float,
                                      ctypes.POINTER(Format), ctypes.POINTER(Format), ctypes.POINTER(Format),
                                      u64, u32, vp]
    pp = ctypes.POINTER(ctypes.c_void_p)
    L.qsim_quant_sgd_step_multi.argtypes = [ci, pp, pp, pp, pp, ctypes.POINTER(u64), ctypes.c_float, ctypes.c_float,
                                            ctypes.POINTER(Format), ctypes.POINTER(Format), ctypes.POINTER(Format),
                                            u64, u32, vp]
    L.qsim_quant_sgd_step_multi.restype = ci
    po = ctypes.POINTER(SgdOptions)
    L.qsim_quant_sgd_step_ex.argtypes = [vp, vp, vp, vp, u64, ctypes.c_float, ctypes.c_float, po,
                                         ctypes.POINTER(Format), ctypes.POINTER(Format), ctypes.POINTER(Format),
                                         u64, u32, vp]
    L.qsim_quant_sgd_step_ex.restype = ci
    L.qsim_quant_sgd_step_at.argtypes = [vp, vp, vp, vp, u64, u64, ctypes.c_float, ctypes.c_float, po,
                                         ctypes.POINTER(Format), ctypes.POINTER(Format), ctypes.POINTER(Format),
                                         u64, u32, vp]
    L.qsim_quant_sgd_step_multi_ex.argtypes = [ci, pp, pp, pp, pp, ctypes.POINTER(u64), ctypes.c_float, ctypes.c_float, po,
                                               ctypes.POINTER(Format), ctypes.POINTER(Format), ctypes.POINTER(Format),
                                               u64, u32, vp]
    L.qsim_quant_sgd_step_multi_ex.restype = ci
    L.qsim_sgd_table_bytes.argtypes = [ci, ctypes.POINTER(u64)]
    L.qsim_sgd_table_bytes.restype = sz
    L.qsim_sgd_table_build.argtypes = [ci, pp, pp, pp, pp, ctypes.POINTER(u64), vp, sz, vp, ctypes.POINTER(SgdTable)]
    L.qsim_sgd_table_build.restype = ci
    L.qsim_quant_sgd_step_table.argtypes = [ctypes.POINTER(SgdTable), ctypes.c_float, ctypes.c_float, po,
                                            ctypes.POINTER(Format), ctypes.POINTER(Format), ctypes.POINTER(Format),
                                            u64, u32, vp]
    L.qsim_quant_sgd_step_table.restype = ci
    L.qsim_set_barrier_wait_us.argtypes = [u32]
    L.qsim_set_barrier_wait_us.restype = None
    L.qsim_status_string.argtypes = [ci]
    L.qsim_status_string.restype = ctypes.c_char_p
    for name in ("qsim_float_quantize", "qsim_fixed_quantize", "qsim_block_quantize", "qsim_quant_sgd_step",
                 "qsim_float_quantize_at", "qsim_fixed_quantize_at", "qsim_block_quantize_at", "qsim_quant_sgd_step_at",
                 "qsim_block_max", "qsim_block_quantize_with_max"):
        getattr(L, name).restype = ci
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().qsim_status_string(status).decode()


def _check(status: int) -> None:
    if status != 0:
        raise QsimError(status, status_string(status))


def _device_f32(t: torch.Tensor, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous float32 tensor on the GPU")
    return t


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream() -> int:
    """Handle of torch's current HIP stream on the current device (the raw getter is ten times
    cheaper than going through torch.cuda.current_stream(), which matters for small tensors)."""
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


def _out_like(x: torch.Tensor, out) -> torch.Tensor:
    if out is None:
        return torch.empty_like(x)
    _device_f32(out, "out")
    if out.numel() != x.numel():
        raise ValueError("out must have as many elements as the input")
    return out


def float_quantize(x, exp_bits, man_bits, rounding=RN_EVEN, flags=SATURATE, seed=0, stream_id=0, out=None, index0=0):
    """qsim_float_quantize on a device tensor; returns the output tensor (``out`` may be ``x``).
    ``index0``: position of ``x[0]`` in the whole tensor when ``x`` is a shard (qsim_float_quantize_at)."""
    _device_f32(x, "x")
    out = _out_like(x, out)
    if index0:
        _check(lib().qsim_float_quantize_at(x.data_ptr(), out.data_ptr(), x.numel(), index0, exp_bits, man_bits, rounding,
                                            flags, seed, stream_id, _stream()))
    else:
        _check(lib().qsim_float_quantize(x.data_ptr(), out.data_ptr(), x.numel(), exp_bits, man_bits, rounding, flags,
                                         seed, stream_id, _stream()))
    return out


def fixed_quantize(x, wl, fl, rounding=RN_EVEN, flags=SATURATE, seed=0, stream_id=0, out=None, index0=0):
    """qsim_fixed_quantize on a device tensor (``index0``: qsim_fixed_quantize_at)."""
    _device_f32(x, "x")
    out = _out_like(x, out)
    if index0:
        _check(lib().qsim_fixed_quantize_at(x.data_ptr(), out.data_ptr(), x.numel(), index0, wl, fl, rounding, flags, seed,
                                            stream_id, _stream()))
    else:
        _check(lib().qsim_fixed_quantize(x.data_ptr(), out.data_ptr(), x.numel(), wl, fl, rounding, flags, seed,
                                         stream_id, _stream()))
    return out


def set_barrier_wait_us(microseconds: int) -> None:
    """qsim_set_barrier_wait_us: bound of the single-pass block kernel's wait (0 = fall back at once)."""
    lib().qsim_set_barrier_wait_us(microseconds)


@functools.lru_cache(maxsize=4096)
def block_workspace_bytes(n, outer, nblocks, inner) -> int:
    """qsim_block_workspace_bytes: a function of the shape alone, so the answers are remembered
    (a training loop asks for the same few shapes every step)."""
    return int(lib().qsim_block_workspace_bytes(n, outer, nblocks, inner))


_scratch = {}                    # (device index, stream handle) -> uint8 tensor, reused by calls on that stream
_kept = {}                       # (device index, stream handle, n, outer, nblocks, inner) -> what _workspace returns: the
                                 # pointer, size and tensor of a zero-filled buffer and the flag, or zeros for a shape that needs none
_SCRATCH_KEEP = 64 << 20         # larger scratch is allocated per call and released with it
_KEPT_LIMIT = 4 << 20            # a shape whose scratch is larger shares the stream's scratch instead


def _workspace(x, outer, nblocks, inner, workspace, may_keep=False, stream=None):
    """Scratch for a block call: (pointer, bytes, the tensor that owns them, QSIM_WORKSPACE_KEPT or 0)."""
    n = x.numel()
    if workspace is None and may_keep:
        # the common case first: a shape seen before on this stream (a call on a small tensor is bound
        # by what the host does per call)
        capturing = torch.cuda.is_current_stream_capturing()
        key = (x.device.index, _stream() if stream is None else stream, n, outer, nblocks, inner)
        entry = _kept.get(key)
        if entry is not None and not capturing:
            return entry
    need = block_workspace_bytes(n, outer, nblocks, inner)
    if not need:
        if workspace is None and may_keep and not capturing:
            _kept[key] = (0, 0, None, 0)
        return 0, 0, None, 0
    kept = 0
    if workspace is None:
        if not may_keep:
            capturing = torch.cuda.is_current_stream_capturing()
        if may_keep and need <= _KEPT_LIMIT and not capturing:
            # one zero-filled buffer per stream and shape, written by nothing but these calls: the
            # library then keeps its counters in it from call to call and launches no clearing kernel
            workspace = torch.zeros(need, dtype=torch.uint8, device=x.device)
            entry = _kept[key] = (workspace.data_ptr(), need, workspace, WORKSPACE_KEPT)
            return entry
        if need > _SCRATCH_KEEP or capturing:
            # (memory allocated during a graph capture belongs to the graph: never shared with eager calls)
            workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
        else:
            # calls on one stream run one after the other, so they can share a scratch buffer
            key = (x.device.index, _stream() if stream is None else stream)
            workspace = _scratch.get(key)
            if workspace is None or workspace.numel() < need:
                workspace = torch.empty(max(need, 1 << 20), dtype=torch.uint8, device=x.device)
                _scratch[key] = workspace
    return workspace.data_ptr(), workspace.numel() * workspace.element_size(), workspace, kept


def block_quantize(x, outer, nblocks, inner, wl, rounding=RN_EVEN, flags=0, seed=0, stream_id=0, out=None,
                   workspace=None, index0=0):
    """qsim_block_quantize on a device tensor viewed as [outer, nblocks, inner].

    ``workspace``: a device tensor of at least ``block_workspace_bytes(...)`` bytes.  When omitted
    and needed, the binding keeps a zero-filled one per stream and shape and passes
    ``WORKSPACE_KEPT`` with it.  A caller who brings a workspace and has kept it as
    ``include/qsim.h`` asks (zero-filled once, then used for this shape only) may add
    ``WORKSPACE_KEPT`` to ``flags``.  ``index0``: position of ``x[0]`` in the whole tensor when
    ``x`` is a shard of whole blocks (qsim_block_quantize_at)."""
    _device_f32(x, "x")
    out = _out_like(x, out)
    stream = _stream()
    ws_ptr, ws_bytes, workspace, kept = _workspace(x, outer, nblocks, inner, workspace, may_keep=True, stream=stream)
    flags |= kept
    if index0:
        _check(lib().qsim_block_quantize_at(x.data_ptr(), out.data_ptr(), x.numel(), outer, nblocks, inner, index0, wl,
                                            rounding, flags, seed, stream_id, ws_ptr, ws_bytes, stream))
    else:
        _check(lib().qsim_block_quantize(x.data_ptr(), out.data_ptr(), x.numel(), outer, nblocks, inner, wl, rounding,
                                         flags, seed, stream_id, ws_ptr, ws_bytes, stream))
    return out


def block_quantize_static(x, outer, nblocks, inner, wl, rounding=RN_EVEN, flags=0, seed=0, stream_id=0, out=None):
    """qsim_block_quantize_static: the scratch is the library's own array on the GPU, nothing is
    allocated (pass ``out``, or the binding allocates the result).  Calls that are in flight on one
    GPU at the same time race."""
    _device_f32(x, "x")
    out = _out_like(x, out)
    _check(lib().qsim_block_quantize_static(x.data_ptr(), out.data_ptr(), x.numel(), outer, nblocks, inner, wl, rounding,
                                            flags, seed, stream_id, _stream()))
    return out


def kept_workspace(x, outer, nblocks, inner):
    """The zero-filled scratch the binding keeps for block_quantize calls of this shape on the
    current stream (None before the first such call, or when the shape needs none)."""
    entry = _kept.get((x.device.index, _stream(), x.numel(), outer, nblocks, inner))
    return None if entry is None else entry[2]


def workspace_timeouts(workspace) -> int:
    """Workgroups of single-pass block_quantize calls that stopped waiting for the others since
    ``workspace`` was last zeroed (its first 32-bit word; waits for the device)."""
    return int(workspace[:4].view(torch.int32).item()) if workspace is not None and workspace.numel() >= 4 else 0


def block_max(x, outer, nblocks, inner, out=None, workspace=None):
    """qsim_block_max: the largest magnitude of every block within ``x``, as int32 bit patterns of
    fp32 magnitudes (non-negative, so ``torch.maximum`` of two results is the maximum over both)."""
    _device_f32(x, "x")
    if out is None:
        out = torch.empty(nblocks, dtype=torch.int32, device=x.device)
    elif not out.is_cuda or out.dtype != torch.int32 or not out.is_contiguous() or out.numel() != nblocks:
        raise TypeError("out must be a contiguous int32 tensor of nblocks elements on the GPU")
    ws_ptr, ws_bytes, workspace, _ = _workspace(x, outer, nblocks, inner, workspace)
    _check(lib().qsim_block_max(x.data_ptr(), x.numel(), outer, nblocks, inner, out.data_ptr(), ws_ptr, ws_bytes, _stream()))
    return out


def block_quantize_with_max(x, outer, nblocks, inner, wl, maxima, rounding=RN_EVEN, flags=0, seed=0, stream_id=0,
                            out=None, index0=0):
    """qsim_block_quantize_with_max: ``maxima`` is an int32 device tensor of nblocks block maxima."""
    _device_f32(x, "x")
    out = _out_like(x, out)
    if not maxima.is_cuda or maxima.dtype != torch.int32 or not maxima.is_contiguous() or maxima.numel() != nblocks:
        raise TypeError("maxima must be a contiguous int32 tensor of nblocks elements on the GPU")
    _check(lib().qsim_block_quantize_with_max(x.data_ptr(), out.data_ptr(), x.numel(), outer, nblocks, inner, index0, wl,
                                              rounding, flags, seed, stream_id, maxima.data_ptr(), _stream()))
    return out


def quant_sgd_step(w_master, grad, mom, lr, momentum, fmt_grad: Format, fmt_mom: Format, fmt_weight: Format,
                   seed=0, stream_id=0, w_q=None, options: SgdOptions = None, index0=0):
    """qsim_quant_sgd_step_at: updates ``w_master`` and ``mom`` in place, fills ``w_q`` when given.
    ``index0``: position of the arrays' first element in the whole parameter tensor when they are a shard."""
    _device_f32(w_master, "w_master")
    _device_f32(grad, "grad")
    _device_f32(mom, "mom")
    n = w_master.numel()
    if grad.numel() != n or mom.numel() != n or (w_q is not None and _device_f32(w_q, "w_q").numel() != n):
        raise ValueError("all tensors of the step must have the same number of elements")
    _check(lib().qsim_quant_sgd_step_at(w_master.data_ptr(), w_q.data_ptr() if w_q is not None else None,
                                        grad.data_ptr(), mom.data_ptr(), n, index0, lr, momentum,
                                        ctypes.byref(options) if options is not None else None, ctypes.byref(fmt_grad),
                                        ctypes.byref(fmt_mom), ctypes.byref(fmt_weight), seed, stream_id, _stream()))
    return w_q


class SgdTensorList:
    """A fixed list of tensors (a model's parameters, gradients, momentum buffers and optional
    quantized copies), marshalled once: the pointer arrays of qsim_quant_sgd_step_multi, and the
    device table of qsim_sgd_table_build, so that a training loop pays for neither every step.

    ``step`` is one launch for the whole list (qsim_quant_sgd_step_table); ``step_batched`` passes
    the pointer arrays (qsim_quant_sgd_step_multi_ex, one launch per 64 tensors).  Both give the
    same result."""

    def __init__(self, w_master, grad, mom, w_q=None):
        k = len(w_master)
        if len(grad) != k or len(mom) != k or (w_q is not None and len(w_q) != k):
            raise ValueError("the tensor lists must have the same length")
        for t in range(k):
            _device_f32(w_master[t], "w_master")
            _device_f32(grad[t], "grad")
            _device_f32(mom[t], "mom")
            n = w_master[t].numel()
            if grad[t].numel() != n or mom[t].numel() != n or (w_q is not None and w_q[t] is not None
                                                                and _device_f32(w_q[t], "w_q").numel() != n):
                raise ValueError("all tensors of one parameter must have the same number of elements")
        self._keep = (list(w_master), list(grad), list(mom), None if w_q is None else list(w_q))   # keeps the memory alive
        ptrs = lambda ts: (ctypes.c_void_p * k)(*[None if x is None else x.data_ptr() for x in ts])
        self.count = k
        self.w_master, self.grad, self.mom = ptrs(w_master), ptrs(grad), ptrs(mom)
        self.w_q = ptrs(w_q) if w_q is not None else None
        self.sizes = (ctypes.c_uint64 * k)(*[x.numel() for x in w_master])
        self.table = None            # built by the first step()
        self._table_memory = None

    def _build_table(self) -> None:
        if torch.cuda.is_current_stream_capturing():
            # qsim_sgd_table_build copies the table to the device and waits for the copy
            raise RuntimeError("the device table of an SgdTensorList cannot be built during a stream capture: "
                               "call build_table() (or take one eager step) before capturing")
        k = self.count
        table = SgdTable()
        need = int(lib().qsim_sgd_table_bytes(k, self.sizes))
        if need:
            self._table_memory = torch.empty(need, dtype=torch.uint8, device=self._keep[0][0].device)
        _check(lib().qsim_sgd_table_build(k, self.w_master, self.w_q, self.grad, self.mom, self.sizes,
                                          self._table_memory.data_ptr() if need else None, need, _stream(),
                                          ctypes.byref(table)))
        self.table = table

    def build_table(self) -> None:
        """Builds the device table now (``step`` does it on its first call otherwise); needed before
        a stream capture, which can record ``step`` but not the building of the table."""
        if self.table is None:
            self._build_table()

    def step(self, lr, momentum, fmt_grad: Format, fmt_mom: Format, fmt_weight: Format, seed=0, stream_id=0,
             options: SgdOptions = None) -> None:
        if self.table is None:
            self._build_table()
        _check(lib().qsim_quant_sgd_step_table(ctypes.byref(self.table), lr, momentum,
                                               ctypes.byref(options) if options is not None else None,
                                               ctypes.byref(fmt_grad), ctypes.byref(fmt_mom), ctypes.byref(fmt_weight),
                                               seed, stream_id, _stream()))

    def step_batched(self, lr, momentum, fmt_grad: Format, fmt_mom: Format, fmt_weight: Format, seed=0, stream_id=0,
                     options: SgdOptions = None) -> None:
        _check(lib().qsim_quant_sgd_step_multi_ex(self.count, self.w_master, self.w_q, self.grad, self.mom, self.sizes, lr,
                                                  momentum, ctypes.byref(options) if options is not None else None,
                                                  ctypes.byref(fmt_grad), ctypes.byref(fmt_mom), ctypes.byref(fmt_weight),
                                                  seed, stream_id, _stream()))


def quant_sgd_step_multi(w_master, grad, mom, lr, momentum, fmt_grad: Format, fmt_mom: Format, fmt_weight: Format,
                         seed=0, stream_id=0, w_q=None, options: SgdOptions = None):
    """qsim_quant_sgd_step_multi(_ex) over lists of tensors (``w_q``: None, or a list whose entries may be None)."""
    SgdTensorList(w_master, grad, mom, w_q).step_batched(lr, momentum, fmt_grad, fmt_mom, fmt_weight, seed, stream_id, options)
