"""Pins of the oracle's variant functions (none of them is checked against itself).

Symmetric quantization (Section 2.1: z = 0 in Eq. 1, on signed codes; here the signed code is the stored code
minus 8 and there is no zero-point tensor): exact rationals on every weight, brute force with rationals on tiny
shapes, the closed form for a constant code, a BLAS GEMM on weights the test builds itself, agreement with the
general oracle fed an explicit zero-point tensor of eights (a different code path), and planted mistakes.

BF16 activations (the paper's A is a 16-bit float; bfloat16 is the upper half of a binary32): the decoding against
the bit cast and against a library's conversion on all 65536 patterns, the format's landmark values, brute force
with rationals, a BLAS GEMM, bit-equality with the FP16 oracle on inputs both formats hold, and the output rounding
against exact rationals, a library's cast and the case where rounding twice would differ.
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


def _bf16_values(bits):
    """bfloat16 patterns -> binary32 by the bit cast (the format's definition: the upper half of a binary32)."""
    return (np.asarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def test_bfloat_decoding_all_patterns():
    import torch
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    mine = np.array([orc.bfloat_to_float(int(b)) for b in allb], np.float32)
    cast = _bf16_values(allb)
    lib = torch.from_numpy(allb.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    fin = ~np.isnan(cast)
    assert np.array_equal(np.isnan(mine), np.isnan(cast)) and np.array_equal(np.isnan(lib), np.isnan(cast))
    assert np.array_equal(mine[fin].view(np.uint32), cast[fin].view(np.uint32))  # signed zeros included
    assert np.array_equal(lib[fin].view(np.uint32), cast[fin].view(np.uint32))
    # landmarks of the format (1 sign, 8 exponent, 7 fraction bits, bias 127)
    for bits, value in ((0x3F80, 1.0), (0x4049, 3.140625), (0xC2F7, -123.5), (0x0001, 2.0 ** -133), (0x0080, 2.0 ** -126),
                        (0x7F7F, (2 - 2.0 ** -7) * 2.0 ** 127), (0x3C00, 2.0 ** -7), (0xBF00, -0.5)):
        assert float(orc.bfloat_to_float(bits)) == value, hex(bits)
    assert np.isinf(orc.bfloat_to_float(0x7F80)) and orc.bfloat_to_float(0xFF80) < 0


@pytest.mark.parametrize("M,K,N,group", [(2, 16, 8, 8), (3, 256, 16, 128), (1, 64, 8, 32)])
def test_bf16_brute_force_rationals(M, K, N, group):
    _, Wp, s, Zp = wl.make(M, K, N, index=740 + K, group=group)
    Xb = wl.make_x_bf16(M, K, index=740 + K)
    ref = orc.gemm_bf16(Xb, Wp, s, Zp, group)
    xv = _bf16_values(Xb)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                qv = (int(Wp[k // 8, n]) >> (4 * (k % 8))) & 15
                zv = (int(Zp[k // group, n // 8]) >> (4 * (n % 8))) & 15
                acc += Fraction(float(xv[m, k])) * Fraction(float(s[k // group, n])) * (qv - zv)
            want = float(acc)
            assert abs(ref[m, n] - want) <= 1e-13 * (1 + abs(want)), (m, n)


def test_bf16_is_a_plain_gemm():
    rng = np.random.default_rng(75)
    M, K, N, group = 5, 1024, 40, 64
    q = rng.integers(0, 16, (K, N))
    z = rng.integers(0, 16, (K // group, N))
    s = rng.uniform(0.001, 0.02, (K // group, N)).astype(np.float16)
    Xb = wl.make_x_bf16(M, K, index=75, outliers=True)
    ref = orc.gemm_bf16(Xb, wl.pack_along_k(q.astype(np.uint8)), s, wl.pack_along_n(z.astype(np.uint8)), group)
    want = _bf16_values(Xb).astype(np.float64) @ ((q - np.repeat(z, group, axis=0)) * np.repeat(s.astype(np.float64), group, axis=0))
    assert np.allclose(ref, want, rtol=1e-11, atol=1e-12)


def test_bf16_equals_the_fp16_oracle_where_both_formats_hold_x():
    """Values with 8 significant bits and a modest exponent are both an FP16 and a bfloat16: the two oracles
    (different decoders) must then agree bit for bit."""
    M, K, N, group = 4, 768, 24, 128
    _, Wp, s, Zp = wl.make(M, K, N, index=76, group=group)
    Xb = wl.make_x_bf16(M, K, index=76)
    xv = _bf16_values(Xb)
    keep = (np.abs(xv) >= 2.0 ** -14) & (np.abs(xv) < 60000)
    Xb = np.where(keep, Xb, 0).astype(np.uint16)
    xh = _bf16_values(Xb).astype(np.float16)
    assert np.array_equal(xh.astype(np.float32), _bf16_values(Xb))
    assert np.array_equal(orc.gemm_bf16(Xb, Wp, s, Zp, group), orc.gemm(xh, Wp, s, Zp, group))


def test_bf16_output_rounding():
    import torch
    rng = np.random.default_rng(77)
    v32 = (rng.standard_normal(200000) * 10.0 ** rng.integers(-44, 39, 200000)).astype(np.float32)
    v32 = np.concatenate([v32, np.array([0.0, -0.0, np.inf, -np.inf, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 2.0 ** -133, 2.0 ** -134,
                                         1.5 * 2.0 ** -134, 2.0 ** -126, 3.3895313892515355e38, 3.39e38, 3.4e38], np.float32)])
    got = orc.to_bf16_bits(v32.astype(np.float64))
    lib = torch.from_numpy(v32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, lib)
    assert orc.to_bf16_bits(np.array([np.nan]))[0] & 0x7FFF > 0x7F80
    # ties go to the even significand; one rounding only: 1 + 2^-8 + 2^-40 is above the tie, although its
    # binary32 rounding sits exactly on it
    assert orc.to_bf16_bits(np.array([1 + 2.0 ** -8]))[0] == 0x3F80
    assert orc.to_bf16_bits(np.array([1 + 3 * 2.0 ** -8]))[0] == 0x3F82
    assert orc.to_bf16_bits(np.array([1 + 2.0 ** -8 + 2.0 ** -40]))[0] == 0x3F81
    # nearest, against exact rationals: no neighbouring pattern is closer
    v64 = rng.standard_normal(3000) * 10.0 ** rng.integers(-30, 30, 3000)
    bits = orc.to_bf16_bits(v64)
    for v, b in zip(v64, bits):
        mine = abs(Fraction(float(_bf16_values([b])[0])) - Fraction(v))
        for nb in (int(b) - 1, int(b) + 1):
            other = float(_bf16_values([nb & 0xFFFF])[0])
            if np.isfinite(other):
                assert mine <= abs(Fraction(other) - Fraction(v))


MUTANTS = [
    ("bias of the bfloat16 exponent", "(int)biased - 134);", "(int)biased - 133);"),
    ("bfloat16 subnormal spacing", "ldexpf((float)mant, -133);", "ldexpf((float)mant, -134);"),
    ("bfloat16 fraction width", "uint32_t mant = (uint32_t)b & 0x7Fu;", "uint32_t mant = (uint32_t)b & 0x3Fu;"),
    ("bfloat16 hidden bit", "(float)(128u + mant)", "(float)(mant)"),
    ("bf16 narrow sum", "double total = 0.0;", "float total = 0.0f;"),
    ("bf16 dropped last term", "for (int kk = 0; kk < K; ++kk) {", "for (int kk = 0; kk < K - 1; ++kk) {"),
    ("bf16 row stride of X", "Xb[(size_t)m * K + kk]", "Xb[(size_t)m * (K - 8) + kk]"),
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
