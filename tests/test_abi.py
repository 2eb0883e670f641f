"""The C-ABI library loads, exports every symbol include/qsim.h declares, and validates its
arguments before touching the GPU (so all of this runs on a host without one)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

B = pytest.importorskip("paper_1910_04540_amd.binding")


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "qsim.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qsim_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS), names
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    for s in range(0, 9):
        assert B.status_string(s) and B.status_string(s) != "unknown status"
    assert B.status_string(99) == "unknown status"


FAKE = 0x10000   # a non-null, 16-byte aligned address that is never dereferenced on the host


def test_elementwise_validation_without_gpu():
    L = B.lib()
    ok = (8, 6, 0, 1, 0, 0, None)
    assert L.qsim_fixed_quantize(FAKE, FAKE, 0, *ok) == 0                           # n == 0: no-op
    assert L.qsim_fixed_quantize(None, None, 0, *ok) == 0
    assert L.qsim_fixed_quantize(None, FAKE, 16, *ok) == 1
    assert L.qsim_fixed_quantize(FAKE, None, 16, *ok) == 1
    assert L.qsim_fixed_quantize(FAKE, FAKE, 16, 0, 6, 0, 1, 0, 0, None) == 2
    assert L.qsim_fixed_quantize(FAKE, FAKE, 16, 25, 6, 0, 1, 0, 0, None) == 2
    assert L.qsim_fixed_quantize(FAKE, FAKE, 16, 8, 150, 0, 1, 0, 0, None) == 2
    assert L.qsim_fixed_quantize(FAKE, FAKE, 16, 8, -121, 0, 1, 0, 0, None) == 2
    assert L.qsim_fixed_quantize(FAKE, FAKE, 16, 8, 6, 0, 8, 0, 0, None) == 2       # unknown flag
    assert L.qsim_fixed_quantize(FAKE, FAKE, 16, 8, 6, 4, 1, 0, 0, None) == 3
    assert L.qsim_fixed_quantize(FAKE, FAKE, 16, 0, 6, 4, 1, 0, 0, None) == 3       # rounding is checked first
    assert L.qsim_fixed_quantize(FAKE, FAKE + 32, 16, *ok) == 5                     # partial overlap
    assert L.qsim_fixed_quantize(FAKE, FAKE, (1 << 40) + 1, *ok) == 4
    assert L.qsim_float_quantize(FAKE, FAKE, 16, 1, 2, 0, 1, 0, 0, None) == 2
    assert L.qsim_float_quantize(FAKE, FAKE, 16, 9, 2, 0, 1, 0, 0, None) == 2
    assert L.qsim_float_quantize(FAKE, FAKE, 16, 5, 0, 0, 1, 0, 0, None) == 2
    assert L.qsim_float_quantize(FAKE, FAKE, 16, 5, 24, 0, 1, 0, 0, None) == 2
    assert L.qsim_float_quantize(FAKE, FAKE, 16, 5, 2, -1, 1, 0, 0, None) == 3
    assert L.qsim_float_quantize(None, FAKE, 16, 5, 2, 0, 1, 0, 0, None) == 1
    assert L.qsim_float_quantize(FAKE, FAKE + 4, 16, 5, 2, 0, 1, 0, 0, None) == 5


def test_block_validation_without_gpu():
    L = B.lib()

    def call(n, outer, nblocks, inner, wl=8, rounding=0, flags=0, ws=None, ws_bytes=0, a=FAKE, b=FAKE):
        return L.qsim_block_quantize(a, b, n, outer, nblocks, inner, wl, rounding, flags, 0, 0, ws, ws_bytes, None)

    assert call(0, 1, 1, 1) == 0
    assert call(6, 1, 1, 6, wl=1) == 2 and call(6, 1, 1, 6, wl=25) == 2
    assert call(6, 1, 1, 6, rounding=9) == 3
    assert call(6, 1, 1, 5) == 4 and call(6, 2, 3, 2) == 4 and call(6, 1, 0, 6) == 4 and call(6, 1, 3, 3) == 4
    assert call(6, 1, 1, 6, a=None) == 1
    assert call(64, 1, 1, 64, b=FAKE + 16) == 5
    # a block spread over several workgroups needs the scratch the size query asks for
    n = 1 << 24
    need = B.block_workspace_bytes(n, 1, 1, n)
    assert need > 0 and need % 4 == 0
    assert call(n, 1, 1, n) == 6
    assert call(n, 1, 1, n, ws=FAKE + (1 << 30), ws_bytes=need - 4) == 6
    assert call(n, 1, 1, n, ws=FAKE + (1 << 30) + 4, ws_bytes=need) == 6            # misaligned
    assert B.block_workspace_bytes(4096 * 4096, 1, 4096, 4096) == 0                 # one workgroup per row
    assert B.block_workspace_bytes(0, 1, 1, 1) == 0
    assert B.block_workspace_bytes(7, 2, 2, 2) == 0                                 # invalid shape: nothing to do
    # the flag that says the caller keeps the workspace belongs to block quantize alone
    assert call(0, 1, 1, 1, flags=B.WORKSPACE_KEPT) == 0 and call(6, 1, 1, 6, flags=16) == 2
    assert call(n, 1, 1, n, flags=B.WORKSPACE_KEPT) == 6                            # kept or not, it has to be there
    assert L.qsim_fixed_quantize(FAKE, FAKE, 8, 8, 6, 0, B.WORKSPACE_KEPT, 0, 0, None) == 2
    assert L.qsim_float_quantize(FAKE, FAKE, 8, 5, 2, 0, B.WORKSPACE_KEPT, 0, 0, None) == 2
    assert L.qsim_block_quantize_with_max(FAKE, FAKE, 8, 1, 1, 8, 0, 8, 0, B.WORKSPACE_KEPT, 0, 0, FAKE + (1 << 20), None) == 2


def test_sgd_validation_without_gpu():
    L = B.lib()
    ident = B.Format(0, 0, 0, 0, 0)

    def call(fg=ident, fm=ident, fw=ident, n=64, w=FAKE, q=FAKE + (1 << 20), g=FAKE + (2 << 20), m=FAKE + (3 << 20)):
        return L.qsim_quant_sgd_step(w, q, g, m, n, 0.1, 0.9, ctypes.byref(fg), ctypes.byref(fm), ctypes.byref(fw),
                                     0, 0, None)

    assert call(n=0) == 0
    for bad in [B.Format(4, 0, 0, 0, 0), B.Format(1, 9, 2, 0, 0), B.Format(2, 30, 2, 0, 0), B.Format(3, 8, 100, 0, 0),
                B.Format(3, 8, 2048, 0, 0), B.Format(3, 8, 2, 0, 0), B.Format(3, 1, 64, 0, 0), B.Format(2, 8, 6, 0, 16)]:
        assert call(fg=bad) == 2 and call(fm=bad) == 2 and call(fw=bad) == 2
    assert call(fm=B.Format(2, 8, 6, 7, 0)) == 3
    assert call(w=None) == 1 and call(g=None) == 1 and call(m=None) == 1
    assert call(g=FAKE) == 5 and call(m=FAKE + 8) == 5 and call(q=FAKE + (3 << 20)) == 5
    assert call(q=FAKE + 16) == 5                    # w_q may be w_master itself, but not a shifted copy of it
    assert L.qsim_quant_sgd_step(FAKE, None, FAKE + 4096, FAKE + 8192, 64, 0.1, 0.9, None, ctypes.byref(ident),
                                 ctypes.byref(ident), 0, 0, None) == 1


def test_sgd_multi_validation_without_gpu():
    L = B.lib()
    ident = B.Format(0, 0, 0, 0, 0)
    vp = ctypes.c_void_p

    def call(ws, gs, ms, ns, qs=None, fmt=ident, count=None):
        k = len(ns)
        arr = lambda xs: (vp * k)(*xs) if xs is not None else None
        return L.qsim_quant_sgd_step_multi(k if count is None else count, arr(ws), arr(qs), arr(gs), arr(ms),
                                           (ctypes.c_uint64 * k)(*ns), 0.1, 0.9, ctypes.byref(fmt), ctypes.byref(fmt),
                                           ctypes.byref(fmt), 0, 0, None)

    a, b, c = FAKE, FAKE + (1 << 20), FAKE + (2 << 20)
    assert call([a], [b], [c], [0]) == 0                          # only empty tensors: nothing to launch
    assert call([a, None], [b, None], [c, None], [0, 0]) == 0
    assert call([a], [b], [c], [16], count=0) == 0
    assert call([a], [b], [c], [16], count=-1) == 4
    assert call([a, None], [b, b], [c, c], [0, 16]) == 1          # the second tensor has no weights
    assert call([a, a], [b, a], [c, c], [0, 16]) == 5             # grad aliases the weights
    assert call([a], [b], [c], [16], fmt=B.Format(3, 8, 100, 0, 0)) == 2
    assert L.qsim_quant_sgd_step_multi(1, None, None, None, None, None, 0.1, 0.9, ctypes.byref(ident), ctypes.byref(ident),
                                       ctypes.byref(ident), 0, 0, None) == 1


def test_sgd_table_validation_without_gpu():
    L = B.lib()
    ident = B.Format(0, 0, 0, 0, 0)
    vp, u64 = ctypes.c_void_p, ctypes.c_uint64
    sizes = lambda ns: (u64 * len(ns))(*ns)

    # 48 bytes per non-empty tensor (rounded up to 16), 4 bytes per tile of 1024 elements (rounded up to 16)
    assert L.qsim_sgd_table_bytes(0, None) == 0
    assert L.qsim_sgd_table_bytes(2, sizes([0, 0])) == 0
    assert L.qsim_sgd_table_bytes(1, sizes([1])) == 48 + 16
    assert L.qsim_sgd_table_bytes(3, sizes([1024, 0, 1025])) == 96 + 16
    assert L.qsim_sgd_table_bytes(3, sizes([1024, 5, 1024 * 9 + 1])) == 144 + 48
    assert L.qsim_sgd_table_bytes(1, sizes([(1 << 38) + 1])) == 0
    assert L.qsim_sgd_table_bytes(17, sizes([1 << 38] * 17)) == 0           # 17 * 2^28 tiles do not fit 32 bits

    def build(ws, gs, ms, ns, qs=None, mem=FAKE + (8 << 20), mem_bytes=1 << 20, count=None, table=True):
        k = len(ns)
        arr = lambda xs: (vp * k)(*xs) if xs is not None else None
        t = B.SgdTable()
        st = L.qsim_sgd_table_build(k if count is None else count, arr(ws), arr(qs), arr(gs), arr(ms), sizes(ns), mem,
                                    mem_bytes, None, ctypes.byref(t) if table else None)
        return st, t

    a, b, c = FAKE, FAKE + (1 << 20), FAKE + (2 << 20)
    assert build([a], [b], [c], [16], table=False)[0] == 1
    assert build([a], [b], [c], [16], count=-1)[0] == 4
    st, t = build([a], [b], [c], [16], count=0)
    assert st == 0 and t.count == 0 and t.tiles == 0
    st, t = build([a, None], [b, None], [c, None], [0, 0])                  # only empty tensors
    assert st == 0 and t.count == 0
    assert build([a, None], [b, b], [c, c], [0, 16])[0] == 1
    assert build([a, a], [b, a], [c, c], [0, 16])[0] == 5
    assert build([a], [b], [c], [(1 << 38) + 1])[0] == 4
    assert build([a], [b], [c], [16], mem=None)[0] == 6
    assert build([a], [b], [c], [16], mem=FAKE + (8 << 20) + 4)[0] == 6     # misaligned table memory
    assert build([a], [b], [c], [16], mem_bytes=63)[0] == 6

    def step(t, fmt=ident):
        return L.qsim_quant_sgd_step_table(ctypes.byref(t) if t is not None else None, 0.1, 0.9, None, ctypes.byref(fmt),
                                           ctypes.byref(fmt), ctypes.byref(fmt), 0, 0, None)

    assert step(B.SgdTable()) == 0                                          # an empty list: nothing to launch
    assert step(None) == 1
    assert step(B.SgdTable(), fmt=B.Format(3, 8, 100, 0, 0)) == 2
    assert step(B.SgdTable(None, 0, 1, 1, 1)) == 1
    assert step(B.SgdTable(FAKE, 48, 1, 1, 1)) == 6                         # too small for one entry and one tile
    assert step(B.SgdTable(FAKE + 8, 64, 1, 1, 1)) == 6


def test_shard_validation_without_gpu():
    L = B.lib()
    ident = B.Format(0, 0, 0, 0, 0)
    assert L.qsim_fixed_quantize_at(FAKE, FAKE, 16, 6, 8, 6, 0, 1, 0, 0, None) == 4          # index0 not a multiple of 4
    assert L.qsim_float_quantize_at(FAKE, FAKE, 16, (1 << 62) + 4, 5, 2, 0, 1, 0, 0, None) == 4
    assert L.qsim_float_quantize_at(FAKE, FAKE, 0, 8, 5, 2, 0, 1, 0, 0, None) == 0
    assert L.qsim_fixed_quantize_at(FAKE, FAKE, 16, 8, 25, 6, 0, 1, 0, 0, None) == 2          # the format is checked first
    assert L.qsim_block_quantize_at(FAKE, FAKE, 64, 1, 4, 16, 2, 8, 0, 0, 0, 0, None, 0, None) == 4
    blk = B.Format(3, 8, 256, 0, 0)

    def sgd(index0, fw=blk):
        return L.qsim_quant_sgd_step_at(FAKE, None, FAKE + (1 << 20), FAKE + (2 << 20), 0, index0, 0.1, 0.9, None,
                                        ctypes.byref(ident), ctypes.byref(ident), ctypes.byref(fw), 0, 0, None)

    assert sgd(0) == 0 and sgd(512) == 0
    assert sgd(128) == 4                                       # a shard must hold whole chunks of 256
    assert sgd(128, fw=ident) == 0 and sgd(130, fw=ident) == 4
    mx = FAKE + (4 << 20)
    assert L.qsim_block_max(FAKE, 0, 1, 1, 1, mx, None, 0, None) == 4
    assert L.qsim_block_max(FAKE, 64, 1, 4, 15, mx, None, 0, None) == 4
    assert L.qsim_block_max(None, 64, 1, 4, 16, mx, None, 0, None) == 1
    assert L.qsim_block_max(FAKE, 64, 1, 4, 16, None, None, 0, None) == 1
    assert L.qsim_block_max(FAKE, 64, 1, 4, 16, FAKE + 64, None, 0, None) == 5              # maxima inside the input
    assert L.qsim_block_max(FAKE, 1 << 20, 1, 1, 1 << 20, mx, None, 0, None) == 6           # several slices need scratch
    assert L.qsim_block_quantize_with_max(FAKE, FAKE, 64, 1, 4, 16, 0, 8, 0, 0, 0, 0, None, None) == 1
    assert L.qsim_block_quantize_with_max(FAKE, FAKE, 64, 1, 4, 16, 2, 8, 0, 0, 0, 0, mx, None) == 4
    assert L.qsim_block_quantize_with_max(FAKE, FAKE, 64, 1, 4, 16, 0, 1, 0, 0, 0, 0, mx, None) == 2
    assert L.qsim_block_quantize_with_max(FAKE, FAKE, 64, 1, 4, 16, 0, 8, 0, 0, 0, 0, FAKE + 16, None) == 5
    assert L.qsim_block_quantize_with_max(FAKE, FAKE, 0, 1, 4, 16, 0, 8, 0, 0, 0, 0, None, None) == 0


def test_header_is_plain_c():
    """The boundary is a C-ABI: the header must compile as C99 (and as C++) on its own."""
    import shutil
    import subprocess

    header = os.path.join(ROOT, "include", "qsim.h")
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", header], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", header], check=True)
