"""Pins for the oracle's random numbers: published known answers, a big-int Python
statement of the same algorithm, an independent library implementation, and statistics."""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

import pyref

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(tok, 16) for tok in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_published_known_answers(oracle_lib):
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert oracle_lib.philox4x32_10(ctr, key) == want


def test_python_bigint_statement_matches_known_answers():
    for ctr, key, want in _kat_rows():
        assert pyref.philox4x32_10(ctr, key) == want


def test_oracle_matches_bigint_statement_on_random_inputs(oracle_lib):
    rng = np.random.default_rng(123)
    for _ in range(500):
        ctr = [int(v) for v in rng.integers(0, 2**32, size=4)]
        key = [int(v) for v in rng.integers(0, 2**32, size=2)]
        assert oracle_lib.philox4x32_10(ctr, key) == pyref.philox4x32_10(ctr, key)


def test_counter_and_key_layout_of_random_block(oracle_lib):
    # key = (seed lo, seed hi); counter = (env, agent, g lo, stream | g hi << 8)
    cases = [(0, 0, 0, 0, 0), (0x1122334455667788, 7, 9, 3, 1), (2, 1999, 999, 2**32 + 5, 0), (2**64 - 1, 2**31, 8191, 2**40, 1)]
    for seed, env, agent, g, stream in cases:
        want = pyref.philox4x32_10([env, agent, g & 0xFFFFFFFF, stream | ((g >> 32) << 8)], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle_lib.random_block(seed, env, agent, g, stream) == want
    # distinct coordinates give distinct blocks
    blocks = {tuple(oracle_lib.random_block(5, e, a, g, s)) for e in range(3) for a in range(3) for g in range(3) for s in range(2)}
    assert len(blocks) == 54


SHIM = r"""
#include <ATen/core/PhiloxRNGEngine.h>
extern "C" void aten_philox_block(unsigned long long seed, unsigned long long subsequence,
                                  unsigned long long offset, unsigned int* out) {
  at::Philox4_32 engine(seed, subsequence, offset);
  for (int i = 0; i < 4; ++i) out[i] = engine();
}
"""


@pytest.fixture(scope="module")
def aten_philox():
    torch = pytest.importorskip("torch")
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    if not os.path.exists(os.path.join(inc, "ATen", "core", "PhiloxRNGEngine.h")):
        pytest.skip("ATen Philox header not present")
    tmp = tempfile.mkdtemp(prefix="aten_philox_")
    src, lib = os.path.join(tmp, "shim.cpp"), os.path.join(tmp, "shim.so")
    with open(src, "w") as f:
        f.write(SHIM)
    r = subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-I", inc, "-o", lib, src],
                       capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("could not compile the ATen Philox shim: " + r.stderr[-300:])
    dll = ctypes.CDLL(lib)
    dll.aten_philox_block.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint32)]

    def block(seed, subsequence, offset):
        out = (ctypes.c_uint32 * 4)()
        dll.aten_philox_block(seed, subsequence, offset, out)
        return [int(v) for v in out]

    return block


def test_library_implementation_agrees(oracle_lib, aten_philox):
    """PyTorch's header-only CPU Philox4x32-10 engine: key = seed, counter = (offset, subsequence)."""
    rng = np.random.default_rng(7)
    for _ in range(200):
        seed, sub, off = (int(v) for v in rng.integers(0, 2**63, size=3))
        ctr = [off & 0xFFFFFFFF, off >> 32, sub & 0xFFFFFFFF, sub >> 32]
        key = [seed & 0xFFFFFFFF, seed >> 32]
        assert oracle_lib.philox4x32_10(ctr, key) == aten_philox(seed, sub, off)


def test_avalanche_and_uniformity(oracle_lib):
    rng = np.random.default_rng(11)
    flips = []
    for _ in range(300):
        ctr = [int(v) for v in rng.integers(0, 2**32, size=4)]
        key = [int(v) for v in rng.integers(0, 2**32, size=2)]
        base = oracle_lib.philox4x32_10(ctr, key)
        word, bit = int(rng.integers(0, 6)), int(rng.integers(0, 32))
        c2, k2 = list(ctr), list(key)
        if word < 4:
            c2[word] ^= 1 << bit
        else:
            k2[word - 4] ^= 1 << bit
        other = oracle_lib.philox4x32_10(c2, k2)
        flips.append(sum(bin(a ^ b).count("1") for a, b in zip(base, other)))
    assert 60 < np.mean(flips) < 68  # 128 output bits, about half flip
    # uniformity of the derived uniforms over sequential counters (chi-square, 64 bins)
    us = np.array([oracle_lib.uniform_from_word(oracle_lib.random_block(9, e, a, 3, 0)[0])
                   for e in range(40) for a in range(500)])
    assert us.min() >= 0.0 and us.max() < 1.0
    counts = np.histogram(us, bins=64, range=(0, 1))[0]
    chi2 = ((counts - len(us) / 64) ** 2 / (len(us) / 64)).sum()
    assert chi2 < 120  # 63 degrees of freedom; P(chi2 > 120) ~ 1e-5


def test_uniform_is_top_24_bits_exact(oracle_lib):
    assert oracle_lib.uniform_from_word(0) == 0.0
    assert oracle_lib.uniform_from_word(0xFF) == 0.0
    assert oracle_lib.uniform_from_word(0x100) == 2.0 ** -24
    assert oracle_lib.uniform_from_word(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert oracle_lib.uniform_from_word(0x80000000) == 0.5
