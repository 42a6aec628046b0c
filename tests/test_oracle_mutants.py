"""The pins must notice a plausible mistake anywhere in the oracle.

Each case plants one mistake in a copy of the oracle's C source (on the CPU,
in a temporary folder), builds it, and runs the pin suite against that build
in a child process: the suite has to fail.  The unmodified source has to pass
the same way, so a failure is the mutant's and not the harness's.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "w4a16_oracle.c")

MUTANTS = [
    ("sign of the zero point", "return s * (float)(q - z);", "return s * (float)(q + z);"),
    ("nibble order along k", "(word >> (4 * (k % 8)))", "(word >> (4 * (7 - k % 8)))"),
    ("nibble order along n", "(word >> (4 * (n % 8)))", "(word >> (4 * (7 - n % 8)))"),
    ("group index", "int g = k / group;", "int g = k / 128;"),
    ("scale ignores the group", "scales[(size_t)g * (size_t)N + (size_t)n]", "scales[(size_t)n]"),
    ("zero word index", "(size_t)g * (size_t)(N / 8) + (size_t)(n / 8)", "(size_t)g * (size_t)(N / 8) + (size_t)(n % (N / 8))"),
    ("dropped last term", "for (int k = 0; k < K; ++k) {\n        double x", "for (int k = 0; k < K - 1; ++k) {\n        double x"),
    ("narrow accumulator", "double acc = 0.0;", "float acc = 0.0f;"),
    ("rounded product", "acc += x * w;", "acc += (double)(float)(x * w);"),
    ("subnormal scale", "(1.0f / 16777216.0f)", "(1.0f / 8388608.0f)"),
    ("exponent bias", "(int)expo - 25)", "(int)expo - 24)"),
    ("packed row index", "Wp[(size_t)(k / 8) * (size_t)N + (size_t)n]", "Wp[(size_t)(k / 8) * (size_t)N + (size_t)(n ^ 1)]"),
]


def _run_pins(lib):
    env = dict(os.environ, W4A16_ORACLE_LIB_OVERRIDE=lib)
    return subprocess.run(
        [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
         "-p", "no:cacheprovider"],
        cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def _build(text, path):
    src = path + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", path, src, "-lm"])
    return path


def test_unmodified_source_passes_through_the_same_harness(tmp_path):
    lib = _build(open(SRC).read(), str(tmp_path / "clean.so"))
    r = _run_pins(lib)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site must be unique: %r" % old
    lib = _build(text.replace(old, new), str(tmp_path / "mutant.so"))
    r = _run_pins(lib)
    assert r.returncode != 0, "pins did not notice: " + name
    assert "failed" in r.stdout
