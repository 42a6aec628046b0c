"""Builds libw4a16.so (HIP, gfx950 only) in-tree, next to this file.

    python -m paper_2601_16536_amd.build

hipcc cross-compiles without a GPU.  Packed-FP32 instruction selection is
switched off for the device pass (ordinary float code must not be fused into
v_pk_*_f32 on the test machines); the host pass warns that it does not know
the feature, which is harmless.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libw4a16.so")
TIMELINE_LIB = os.path.join(HERE, "libw4a16_timeline.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


# Per-file additions.  The four-wave tile kernel reads its MFMA results back with vector instructions (Eq. 2's step per
# group): with the results in accumulation registers, the compiler's default under register pressure, every read costs
# a v_accvgpr_read first.
FILE_FLAGS = {"w4a16_tile_wide.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str, extra=(), objdir: str = OBJ) -> str:
    obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(os.path.basename(src), []), *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
    if out.strip():
        print(out)
    return obj


def build(verbose: bool = True, timeline: bool = False) -> str:
    """The library; timeline=True builds libw4a16_timeline.so instead, whose decode kernel records per-wave time
    stamps of its phases (bench.py --timeline reads them).  The product never loads that one by itself."""
    objdir = os.path.join(OBJ, "timeline") if timeline else OBJ
    lib = TIMELINE_LIB if timeline else LIB
    extra = ("-DW4A16_TIMELINE=1",) if timeline else ()
    os.makedirs(objdir, exist_ok=True)
    srcs = sources()
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda src: _compile(src, extra, objdir), srcs))
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, lib)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(timeline="--timeline" in sys.argv[1:])
    sys.exit(0)
