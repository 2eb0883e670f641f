"""ctypes front of the CPU oracle (``qsim_ref.c``).  TEST INFRASTRUCTURE ONLY.

Works on numpy float32 arrays in host memory.  Nothing here touches the GPU library, and the
GPU library never imports this module.  ``build()`` compiles the C file with gcc; the loader
compiles on demand when the shared object is missing or older than its sources.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qsim_ref.c")
_HDR = os.path.join(_HERE, "qsim_ref.h")
_LIB = os.path.join(_HERE, "libqsim_ref.so")

RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC = 0, 1, 2, 3
SATURATE, SUBNORMAL, SYMMETRIC = 1, 2, 4
KIND_IDENTITY, KIND_FLOAT, KIND_FIXED, KIND_BLOCK = 0, 1, 2, 3


def build() -> str:
    """Compile the oracle.  -ffp-contract=off: no fused multiply-add may be formed behind our back."""
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", "-ffp-contract=off",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


class Format(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("a", ctypes.c_int), ("b", ctypes.c_int),
                ("rounding", ctypes.c_int), ("flags", ctypes.c_uint32)]


class SgdOptions(ctypes.Structure):
    _fields_ = [("weight_decay", ctypes.c_float), ("dampening", ctypes.c_float), ("nesterov", ctypes.c_int)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if stale:
        build()
    L = ctypes.CDLL(_LIB)
    fp = ctypes.POINTER(ctypes.c_float)
    u64, u32, ci = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
    L.qsim_ref_philox4x32_10.argtypes = [ctypes.POINTER(u32), ctypes.POINTER(u32), ctypes.POINTER(u32)]
    L.qsim_ref_philox4x32_10.restype = None
    L.qsim_ref_random_word.argtypes = [u64, u32, u32, u64]
    L.qsim_ref_random_word.restype = u32
    L.qsim_ref_fixed_scalar.argtypes = [ctypes.c_float, ci, ci, ci, u32, u32]
    L.qsim_ref_fixed_scalar.restype = ctypes.c_float
    L.qsim_ref_float_scalar.argtypes = [ctypes.c_float, ci, ci, ci, u32, u32]
    L.qsim_ref_float_scalar.restype = ctypes.c_float
    L.qsim_ref_float_quantize_at.argtypes = [fp, fp, u64, u64, ci, ci, ci, u32, u64, u32]
    L.qsim_ref_float_quantize.argtypes = [fp, fp, u64, ci, ci, ci, u32, u64, u32]
    L.qsim_ref_fixed_quantize_at.argtypes = [fp, fp, u64, u64, ci, ci, ci, u32, u64, u32]
    L.qsim_ref_fixed_quantize.argtypes = [fp, fp, u64, ci, ci, ci, u32, u64, u32]
    L.qsim_ref_block_quantize.argtypes = [fp, fp, u64, u64, u64, u64, ci, ci, u32, u64, u32]
    L.qsim_ref_block_exponents.argtypes = [fp, u64, u64, u64, u64, ctypes.POINTER(ci)]
    L.qsim_ref_quant_sgd_step.argtypes = [fp, fp, fp, fp, u64, ctypes.c_float, ctypes.c_float,
                                          ctypes.POINTER(Format), ctypes.POINTER(Format),
                                          ctypes.POINTER(Format), u64, u32]
    L.qsim_ref_quant_sgd_step_ex.argtypes = [fp, fp, fp, fp, u64, ctypes.c_float, ctypes.c_float,
                                             ctypes.POINTER(SgdOptions), ctypes.POINTER(Format),
                                             ctypes.POINTER(Format), ctypes.POINTER(Format), u64, u32]
    for name in ("float_quantize_at", "float_quantize", "fixed_quantize_at", "fixed_quantize",
                 "block_quantize", "block_exponents", "quant_sgd_step", "quant_sgd_step_ex"):
        getattr(L, "qsim_ref_" + name).restype = ci
    _lib = L
    return L


class OracleError(RuntimeError):
    def __init__(self, status: int):
        super().__init__(f"oracle returned status {status}")
        self.status = status


def _check(status: int) -> None:
    if status != 0:
        raise OracleError(status)


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def philox4x32_10(ctr, key) -> np.ndarray:
    c = (ctypes.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (ctypes.c_uint32 * 4)()
    lib().qsim_ref_philox4x32_10(c, k, o)
    return np.array(list(o), dtype=np.uint32)


def random_word(seed: int, stream_id: int, role: int, index: int) -> int:
    return int(lib().qsim_ref_random_word(seed, stream_id, role, index))


def random_words(seed: int, stream_id: int, role: int, n: int, index0: int = 0) -> np.ndarray:
    return np.array([random_word(seed, stream_id, role, index0 + i) for i in range(n)], dtype=np.uint32)


def fixed_scalar(x, wl, fl, rounding=RN_EVEN, flags=SATURATE, r=0) -> np.float32:
    return np.float32(lib().qsim_ref_fixed_scalar(np.float32(x), wl, fl, rounding, flags, r))


def float_scalar(x, exp_bits, man_bits, rounding=RN_EVEN, flags=SATURATE, r=0) -> np.float32:
    return np.float32(lib().qsim_ref_float_scalar(np.float32(x), exp_bits, man_bits, rounding, flags, r))


def _threaded(fn_at, x: np.ndarray, threads: int, *args) -> np.ndarray:
    """Split a flat array over `threads` calls of an `_at` entry (ctypes releases the GIL)."""
    flat = _f32(x).reshape(-1)
    out = np.empty_like(flat)
    n = flat.size
    if n == 0:
        _check(fn_at(_ptr(flat), _ptr(out), 0, 0, *args))
        return out.reshape(np.shape(x))
    threads = max(1, min(threads, n))
    bounds = [n * t // threads for t in range(threads + 1)]

    def run(t):
        lo, hi = bounds[t], bounds[t + 1]
        return fn_at(_ptr(flat[lo:hi]), _ptr(out[lo:hi]), hi - lo, lo, *args)

    if threads == 1:
        _check(run(0))
    else:
        with ThreadPoolExecutor(threads) as pool:
            for status in pool.map(run, range(threads)):
                _check(status)
    return out.reshape(np.shape(x))


def float_quantize(x, exp_bits, man_bits, rounding=RN_EVEN, flags=SATURATE, seed=0, stream_id=0,
                   threads=1) -> np.ndarray:
    return _threaded(lib().qsim_ref_float_quantize_at, x, threads, exp_bits, man_bits, rounding,
                     flags, seed, stream_id)


def fixed_quantize(x, wl, fl, rounding=RN_EVEN, flags=SATURATE, seed=0, stream_id=0,
                   threads=1) -> np.ndarray:
    return _threaded(lib().qsim_ref_fixed_quantize_at, x, threads, wl, fl, rounding, flags, seed,
                     stream_id)


def _at(fn_at, x, index0, *args) -> np.ndarray:
    """One call of an `_at` entry: the array holds elements index0 .. of a larger tensor."""
    flat = _f32(x).reshape(-1)
    out = np.empty_like(flat)
    _check(fn_at(_ptr(flat), _ptr(out), flat.size, index0, *args))
    return out.reshape(np.shape(x))


def float_quantize_at(x, index0, exp_bits, man_bits, rounding=RN_EVEN, flags=SATURATE, seed=0,
                      stream_id=0) -> np.ndarray:
    return _at(lib().qsim_ref_float_quantize_at, x, index0, exp_bits, man_bits, rounding, flags, seed,
               stream_id)


def fixed_quantize_at(x, index0, wl, fl, rounding=RN_EVEN, flags=SATURATE, seed=0,
                      stream_id=0) -> np.ndarray:
    return _at(lib().qsim_ref_fixed_quantize_at, x, index0, wl, fl, rounding, flags, seed, stream_id)


def block_quantize(x, outer, nblocks, inner, wl, rounding=RN_EVEN, flags=0, seed=0,
                   stream_id=0) -> np.ndarray:
    flat = _f32(x).reshape(-1)
    out = np.empty_like(flat)
    _check(lib().qsim_ref_block_quantize(_ptr(flat), _ptr(out), flat.size, outer, nblocks, inner, wl,
                                         rounding, flags, seed, stream_id))
    return out.reshape(np.shape(x))


def block_exponents(x, outer, nblocks, inner) -> np.ndarray:
    flat = _f32(x).reshape(-1)
    e = (ctypes.c_int * int(nblocks))()
    _check(lib().qsim_ref_block_exponents(_ptr(flat), flat.size, outer, nblocks, inner, e))
    return np.array(list(e), dtype=np.int32)


def quant_sgd_step(w_master, grad, mom, lr, momentum, fmt_grad: Format, fmt_mom: Format,
                   fmt_weight: Format, seed=0, stream_id=0, want_wq=True, in_place_weights=False,
                   options: SgdOptions = None):
    """Returns (w_master', w_q or None, mom') as new arrays; the inputs are left untouched.
    ``in_place_weights``: pass w_master as w_q too (the returned w_q is then w_master').
    ``options``: weight decay, dampening, Nesterov momentum (None = plain step)."""
    w = _f32(w_master).reshape(-1).copy()
    g = _f32(grad).reshape(-1)
    m = _f32(mom).reshape(-1).copy()
    wq = w if in_place_weights else (np.empty_like(w) if want_wq else None)
    want_wq = want_wq or in_place_weights
    null = ctypes.POINTER(ctypes.c_float)()
    opt = ctypes.byref(options) if options is not None else None
    _check(lib().qsim_ref_quant_sgd_step_ex(_ptr(w), _ptr(wq) if want_wq else null, _ptr(g), _ptr(m),
                                            w.size, lr, momentum, opt, ctypes.byref(fmt_grad),
                                            ctypes.byref(fmt_mom), ctypes.byref(fmt_weight), seed,
                                            stream_id))
    return w, wq, m
