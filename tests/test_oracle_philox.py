"""Pins for the oracle's Philox4x32-10: published known-answer vectors and an independent,
installed implementation (the Philox engine header that ships with PyTorch)."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import qsim_ref as R


def _kat_rows(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                rows.append([int(t, 16) for t in line.split()])
    return rows


def test_known_answer_vectors(golden_dir):
    rows = _kat_rows(golden_dir)
    assert len(rows) == 3
    for row in rows:
        got = R.philox4x32_10(row[0:4], row[4:6])
        assert [int(v) for v in got] == row[6:10]


def test_word_layout():
    """Element i takes word i mod 4 of the block with counter (i div 4, stream_id, role), key = seed."""
    seed, stream, role = 0x0123456789ABCDEF, 77, 2
    for index in (0, 1, 2, 3, 4, 7, 1023, (1 << 34) + 5, (1 << 40) + 2):
        j = index // 4
        blk = R.philox4x32_10([j & 0xFFFFFFFF, j >> 32, stream, role], [seed & 0xFFFFFFFF, seed >> 32])
        assert R.random_word(seed, stream, role, index) == int(blk[index % 4])


ATEN_SRC = r"""
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdio>
#include <cstdlib>
int main(int argc, char** argv) {
  for (int a = 1; a + 2 < argc; a += 3) {
    uint64_t seed = strtoull(argv[a], 0, 0), sub = strtoull(argv[a + 1], 0, 0), off = strtoull(argv[a + 2], 0, 0);
    at::Philox4_32 eng(seed, sub, off);
    for (int i = 0; i < 4; ++i) printf("%08x ", eng());
    printf("\n");
  }
  return 0;
}
"""


def test_against_aten_philox(tmp_path):
    """at::Philox4_32(seed, subsequence, offset) is Philox4x32-10 with key = seed and counter =
    (offset, subsequence): an implementation written by other people, compiled here from the header
    that ships with the installed PyTorch."""
    torch = pytest.importorskip("torch")
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    if not os.path.exists(os.path.join(inc, "ATen", "core", "PhiloxRNGEngine.h")) or not shutil.which("g++"):
        pytest.skip("ATen Philox header or g++ not available")
    src = tmp_path / "aten_philox.cpp"
    src.write_text(ATEN_SRC)
    exe = tmp_path / "aten_philox"
    subprocess.run(["g++", "-O1", "-std=c++17", f"-I{inc}", str(src), "-o", str(exe)], check=True)
    g = np.random.Generator(np.random.PCG64(99))
    cases = [(int(g.integers(0, 1 << 63)) * 2 + int(g.integers(0, 2)),
              int(g.integers(0, 1 << 63)) * 2 + int(g.integers(0, 2)),
              int(g.integers(0, 1 << 63)) * 2 + int(g.integers(0, 2))) for _ in range(64)]
    args = [str(exe)] + [hex(v) for c in cases for v in c]
    lines = subprocess.run(args, check=True, capture_output=True, text=True).stdout.strip().splitlines()
    assert len(lines) == len(cases)
    for (seed, sub, off), line in zip(cases, lines):
        want = [int(t, 16) for t in line.split()]
        got = R.philox4x32_10([off & 0xFFFFFFFF, off >> 32, sub & 0xFFFFFFFF, sub >> 32],
                              [seed & 0xFFFFFFFF, seed >> 32])
        assert [int(v) for v in got] == want


def test_words_look_uniform():
    w = R.random_words(1234, 0, 0, 1 << 14).astype(np.float64) / 2.0 ** 32
    assert abs(w.mean() - 0.5) < 0.01
    assert abs(w.var() - 1.0 / 12.0) < 0.005
    # neighbouring words (same and adjacent Philox blocks) are uncorrelated
    assert abs(np.corrcoef(w[:-1], w[1:])[0, 1]) < 0.03
    # each bit is set about half the time
    raw = R.random_words(5, 3, 1, 1 << 13)
    for b in range(32):
        frac = ((raw >> np.uint32(b)) & np.uint32(1)).mean()
        assert 0.46 < frac < 0.54
