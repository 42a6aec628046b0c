"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU-side code: the oracle's C source, and the C-ABI
library's host code (argument checks, the Split-K planner, status strings, tuning knobs) with the device code
left unsanitized.  Each runs in a child process with the sanitizer runtime preloaded; any report fails."""
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _asan_runtime():
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    return out if os.path.sep in out and os.path.exists(out) else None


def _run(code, env_extra):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", **env_extra)
    return subprocess.run([sys.executable, "-c", textwrap.dedent(code)], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=600)


def test_oracle_under_asan_and_ubsan(tmp_path):
    rt = _asan_runtime()
    if not rt:
        pytest.skip("no libasan for gcc here")
    lib = str(tmp_path / "oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared", "-fPIC",
                           "-o", lib, os.path.join(ROOT, "oracle", "w4a16_oracle.c"), "-lm"])
    r = _run("""
        import numpy as np
        from oracle import w4a16_oracle as orc
        from paper_2601_16536_amd import workloads as wl
        for (M, K, N, g) in [(1, 128, 8, 128), (3, 1024, 72, 64), (5, 768, 1032, 128), (2, 256, 40, 32)]:
            X, Wp, s, Zp = wl.make(M, K, N, index=40 + M, group=g)
            ref = orc.gemm(X, Wp, s, Zp, g)
            cols = np.array([0, N - 1, N // 2], np.int32)
            assert np.array_equal(orc.gemm(X, Wp, s, Zp, g, cols=cols), ref[:, cols])
            assert orc.dequant(Wp, s, Zp, g).shape == (K, N)
            assert orc.unpack_codes(Wp).max() <= 15 and orc.unpack_zeros(Zp).max() <= 15
            assert np.array_equal(orc.gemm_symmetric(X, Wp, s, g), orc.gemm(X, Wp, s, wl.pack_along_n(np.full((K // g, N), 8, np.uint8)), g))
        assert orc.half_to_float(0x3C00) == 1.0
        print("oracle clean")
        """, {"LD_PRELOAD": rt, "W4A16_ORACLE_LIB_OVERRIDE": lib})
    assert r.returncode == 0 and "oracle clean" in r.stdout, r.stdout[-3000:]
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-3000:]


def test_library_host_code_under_asan_and_ubsan(tmp_path):
    """The planner and the argument checks need no GPU: they are called through the C ABI of a build whose host pass
    carries the sanitizers (every -fsanitize directly after -Xarch_host: the device pass stays as it is)."""
    rt = _asan_runtime()
    if not rt or not os.path.exists(HIPCC):
        pytest.skip("needs gcc's libasan and hipcc")
    from paper_2601_16536_amd import build
    lib = str(tmp_path / "libw4a16_san.so")
    cmd = [HIPCC, *build.FLAGS, "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared", "-shared-libsan", "-o", lib, *build.sources()]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if p.returncode:
        pytest.skip("hipcc cannot build the sanitized host pass here: " + p.stdout[-400:])
    clang_rt = subprocess.run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    preload = clang_rt if os.path.exists(clang_rt) else rt
    r = _run("""
        import ctypes, sys
        from paper_2601_16536_amd import binding
        binding.use_library(sys.argv[1] if len(sys.argv) > 1 else %r)
        L = binding.lib()
        import itertools
        for M, N, K, g in itertools.product((1, 2, 4, 5, 16, 17, 64, 200), (8, 64, 264, 4096, 8192), (128, 1024, 11008, 28672), (32, 64, 128)):
            if K %% g:
                continue
            for kernel in (-1, 0, 3, 4, 9):
                for split in (0, 1, 2, 7, K // g, K // g + 1):
                    try:
                        p = binding.query_plan(M, N, K, g, kernel, split)
                        assert p["split"] >= 1 and p["workgroups"] >= 1
                    except binding.W4A16Error as e:
                        assert e.status in (binding.ERR_UNSUPPORTED, binding.ERR_SHAPE, binding.ERR_GROUP)
            binding.workspace_bytes(M, N, K, g)
        for code in range(-1, 10):
            binding.status_string(code)
        for knob in ("stripe_waves", "tile_rows", "log", "bogus"):
            L.w4a16_tune(knob.encode(), 1); L.w4a16_tune(knob.encode(), 0)
        assert binding.raw_gemm(0, 16, 16, 16, 128, 1, 8, 128, 16, 0) == binding.ERR_NULL
        assert binding.raw_gemm(16, 16, 16, 16, 128, 1, 12, 128, 16, 0) == binding.ERR_SHAPE
        assert binding.raw_gemm_ws(16, 16, 16, 16, 128, 1, 8, 256, 16, 0, -1, 2, 128, 1 << 20) == binding.ERR_ALIGN
        assert L.w4a16_set_workspace(128, 1 << 20) == binding.ERR_ALIGN
        binding.shutdown()
        print("host code clean")
        """ % lib, {"LD_PRELOAD": preload})
    if "cannot open shared object" in r.stdout or "ASan runtime does not come first" in r.stdout:
        pytest.skip("sanitizer runtime cannot be preloaded here: " + r.stdout[-300:])
    assert r.returncode == 0 and "host code clean" in r.stdout, r.stdout[-3000:]
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-3000:]
