"""Pins of the oracle's variant functions (none of them is checked against itself).

Symmetric quantization (Section 2.1: z = 0 in Eq. 1, on signed codes; here the signed code is the stored code
minus 8 and there is no zero-point tensor): exact rationals on every weight, brute force with rationals on tiny
shapes, the closed form for a constant code, a BLAS GEMM on weights the test builds itself, agreement with the
general oracle fed an explicit zero-point tensor of eights (a different code path), and planted mistakes.
"""
import os
import subprocess
import sys
from fractions import Fraction

import numpy as np
import pytest

from oracle import w4a16_oracle as orc
from paper_2601_16536_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "w4a16_oracle.c")


def test_symmetric_dequant_every_code_and_scale_is_exact():
    """All 16 codes x every FP16 scale in [0.001, 0.02]: s (q - 8) as an exact rational."""
    lo, hi = np.float16(0.001).view(np.uint16), np.float16(0.02).view(np.uint16)
    bits = np.arange(lo, hi + 1, dtype=np.uint16)
    n = (len(bits) + 7) // 8 * 8
    s = np.resize(bits, n).view(np.float16)[None, :]
    for q in range(16):
        Wp = np.full((1, n), q * 0x11111111, np.uint32)  # K = 8, the same code in every nibble
        w = orc.dequant_symmetric(Wp, s, 8)
        for j in range(0, n, 37):
            assert Fraction(float(w[3, j])) == Fraction(float(s[0, j])) * (q - 8)
        assert np.array_equal(w, np.repeat(s.astype(np.float32) * np.float32(q - 8), 8, axis=0))


@pytest.mark.parametrize("M,K,N,group", [(2, 16, 8, 8), (3, 256, 16, 128), (1, 64, 8, 32)])
def test_symmetric_brute_force_rationals(M, K, N, group):
    X, Wp, s, _ = wl.make(M, K, N, index=700 + K, group=group)
    ref = orc.gemm_symmetric(X, Wp, s, group)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                qv = (int(Wp[k // 8, n]) >> (4 * (k % 8))) & 15
                acc += Fraction(float(X[m, k])) * Fraction(float(s[k // group, n])) * (qv - 8)
            want = float(acc)
            assert abs(ref[m, n] - want) <= 1e-13 * (1 + abs(want)), (m, n)


def test_symmetric_constant_code_gives_scaled_rowsum():
    rng = np.random.default_rng(71)
    M, K, N, group = 3, 512, 16, 128
    X = rng.standard_normal((M, K)).astype(np.float16)
    for c in (0, 3, 8, 15):
        s = np.full((K // group, N), np.float16(0.0123))
        ref = orc.gemm_symmetric(X, wl.pack_along_k(np.full((K, N), c, np.uint8)), s, group)
        want = float(np.float16(0.0123)) * (c - 8) * X.astype(np.float64).sum(axis=1)
        assert np.allclose(ref, np.repeat(want[:, None], N, axis=1), rtol=1e-12, atol=1e-13)
    assert not orc.gemm_symmetric(X, wl.pack_along_k(np.full((K, N), 8, np.uint8)), s, group).any()  # code 8 is weight 0


def test_symmetric_is_a_plain_gemm_on_signed_weights():
    rng = np.random.default_rng(72)
    M, K, N, group = 5, 1024, 40, 64
    signed = rng.integers(-8, 8, (K, N))
    s = rng.uniform(0.001, 0.02, (K // group, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    ref = orc.gemm_symmetric(X, wl.pack_along_k((signed + 8).astype(np.uint8)), s, group)
    want = X.astype(np.float64) @ (signed * np.repeat(s.astype(np.float64), group, axis=0))
    assert np.allclose(ref, want, rtol=1e-11, atol=1e-12)


def test_symmetric_equals_general_oracle_with_zero_point_eight():
    M, K, N, group = 4, 768, 24, 128
    X, Wp, s, _ = wl.make(M, K, N, index=73, group=group)
    Zp = wl.pack_along_n(np.full((K // group, N), 8, np.uint8))
    assert np.array_equal(orc.gemm_symmetric(X, Wp, s, group), orc.gemm(X, Wp, s, Zp, group))
    assert np.array_equal(orc.dequant_symmetric(Wp, s, group), orc.dequant(Wp, s, Zp, group))


MUTANTS = [
    ("offset of the signed code", "int signed_code = code_at(Wp, N, k, n) - 8;", "int signed_code = code_at(Wp, N, k, n) - 7;"),
    ("sign of the offset", "int signed_code = code_at(Wp, N, k, n) - 8;", "int signed_code = 8 - code_at(Wp, N, k, n);"),
    ("group of the scale", "int grp = k / group;", "int grp = k / 128;"),
    ("scale row", "scales[(size_t)grp * (size_t)N + (size_t)n]", "scales[(size_t)n]"),
    ("narrow sum", "double sum = 0.0;", "float sum = 0.0f;"),
]


def _run(lib):
    env = dict(os.environ, W4A16_ORACLE_LIB_OVERRIDE=lib)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-x", "-q", "-p", "no:cacheprovider",
                           "-k", "not planted and not unmodified"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True)


def _build(text, path):
    with open(path + ".c", "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", path, path + ".c", "-lm"])
    return path


def test_unmodified_source_passes_through_the_same_harness(tmp_path):
    r = _run(_build(open(SRC).read(), str(tmp_path / "clean.so")))
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site must be unique: %r" % old
    r = _run(_build(text.replace(old, new), str(tmp_path / "mutant.so")))
    assert r.returncode != 0, "the pins did not notice: %s" % name
