"""Seeded synthetic inputs for the W4A16 GEMM: shapes, value distributions and
storage layout only.  Holds none of the method's arithmetic (no dequantization,
no products, no sums), so the CPU oracle's tests and the GPU path's tests can
both draw their inputs here without sharing any computation.

Storage (Section 2.2 says only that 4-bit values travel packed in wider
integers such as INT32; the rest is this build's reading):
  Wp[K/8, N]   uint32, code of k = 8r+i in bits 4i..4i+3 of Wp[r, n]
  scales[G, N] float16, G = K/group
  Zp[G, N/8]   uint32, zero point of n = 8c+j in bits 4j..4j+3 of Zp[g, c]
  X[M, K]      float16 (A of Eq. 2)

Recipe: rng = numpy.random.default_rng([16536, config_index, stream]) with
stream 0 = X, 1 = codes, 2 = scales, 3 = zero points, 4 = outlier channels.
X ~ N(0,1) drawn in float64 then rounded to float16; codes and zero points
uniform on 0..15; scales uniform on [0.001, 0.02] rounded to float16.  The
outlier variant multiplies floor(K/100) distinct k-channels of X by 20.
The shapes stand for LLM decode projections (Section 4.1 derives its shapes
from published LLM layers); no dataset or trained weight is involved.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED = 16536
GROUP = 128


@dataclass(frozen=True)
class Config:
    name: str
    index: int
    K: int
    N: int
    Ms: tuple
    outliers: bool = False
    group: int = GROUP


CONFIGS = {
    "c1": Config("c1", 1, 4096, 1024, (1,)),
    "c2": Config("c2", 2, 11008, 4096, (1,)),
    "c3": Config("c3", 3, 14336, 4096, (1, 4, 16), outliers=True),
    "c4": Config("c4", 4, 28672, 8192, (1, 8)),
    "c5": Config("c5", 5, 8192, 8192, (32, 64, 128)),
}


# The (N, K) pairs of the paper's Split-K against data-parallel comparison (Section 4.1, Fig. 2, panels a to f;
# panel d prints K = 16348, read as 16384), with the batch sizes of a decode server.
FIG2_MS = (1, 2, 4, 8, 16, 32, 64)
FIG2 = {
    "f2a": Config("f2a", 21, 6144, 1536, FIG2_MS),
    "f2b": Config("f2b", 22, 8192, 2048, FIG2_MS),
    "f2c": Config("f2c", 23, 10240, 2048, FIG2_MS),
    "f2d": Config("f2d", 24, 16384, 4096, FIG2_MS),
    "f2e": Config("f2e", 25, 10240, 4608, FIG2_MS),
    "f2f": Config("f2f", 26, 18432, 7168, FIG2_MS),
}


# The opposite regime, K << N (up-projections of the same layers): Section 4.1 expects Split-K to gain only
# "when K >> N", so here it should not be chosen, and forcing it should lose.
WIDE = {
    "w1": Config("w1", 31, 4096, 11008, (1, 16)),
    "w2": Config("w2", 32, 4096, 14336, (1, 16)),
    "w3": Config("w3", 33, 8192, 28672, (1, 16)),
}


def config(name: str) -> Config:
    for table in (CONFIGS, FIG2, WIDE):
        if name in table:
            return table[name]
    raise KeyError(name)


def pack_along_k(q: np.ndarray) -> np.ndarray:
    """codes q[K, N] in 0..15 -> Wp[K/8, N] uint32 (layout only)."""
    q = np.asarray(q)
    K, N = q.shape
    if K % 8:
        raise ValueError("K must be a multiple of 8")
    if q.min(initial=0) < 0 or q.max(initial=0) > 15:
        raise ValueError("codes must lie in 0..15")
    q = q.astype(np.uint32).reshape(K // 8, 8, N)
    out = np.zeros((K // 8, N), np.uint32)
    for i in range(8):
        out |= q[:, i, :] << np.uint32(4 * i)
    return out


def pack_along_n(z: np.ndarray) -> np.ndarray:
    """zero points z[G, N] in 0..15 -> Zp[G, N/8] uint32 (layout only)."""
    z = np.asarray(z)
    G, N = z.shape
    if N % 8:
        raise ValueError("N must be a multiple of 8")
    if z.min(initial=0) < 0 or z.max(initial=0) > 15:
        raise ValueError("zero points must lie in 0..15")
    z = z.astype(np.uint32).reshape(G, N // 8, 8)
    out = np.zeros((G, N // 8), np.uint32)
    for j in range(8):
        out |= z[:, :, j] << np.uint32(4 * j)
    return out


def _rng(index: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([SEED, int(index), int(stream)])


def make_x(M: int, K: int, index: int, outliers: bool = False) -> np.ndarray:
    x = _rng(index, 0).standard_normal((M, K))
    if outliers:
        ch = _rng(index, 4).choice(K, size=K // 100, replace=False)
        x[:, ch] *= 20.0
    return x.astype(np.float16)


def make_x_bf16(M: int, K: int, index: int, outliers: bool = False) -> np.ndarray:
    """The same draw as make_x, stored as bfloat16 bit patterns (uint16): the binary32 value's upper half,
    the lower 16 bits dropped (a storage choice of this generator, no rounding rule involved)."""
    x = _rng(index, 0).standard_normal((M, K))
    if outliers:
        ch = _rng(index, 4).choice(K, size=K // 100, replace=False)
        x[:, ch] *= 20.0
    return (x.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def make_weights(K: int, N: int, index: int, group: int = GROUP):
    """Returns (Wp, scales, Zp) in the storage layout above."""
    if K % group or K % 8 or N % 8:
        raise ValueError("need K % group == 0, K % 8 == 0, N % 8 == 0")
    G = K // group
    q = _rng(index, 1).integers(0, 16, size=(K, N), dtype=np.uint8)
    Wp = pack_along_k(q)
    del q
    scales = _rng(index, 2).uniform(0.001, 0.02, size=(G, N)).astype(np.float16)
    z = _rng(index, 3).integers(0, 16, size=(G, N), dtype=np.uint8)
    return Wp, scales, pack_along_n(z)


def make(M: int, K: int, N: int, index: int, group: int = GROUP, outliers: bool = False):
    """One seeded problem instance: (X, Wp, scales, Zp)."""
    Wp, scales, Zp = make_weights(K, N, index, group)
    return make_x(M, K, index, outliers), Wp, scales, Zp


def make_config(name: str, M: int | None = None):
    """Inputs of a named configuration; X has max(Ms) rows unless M is given
    (then the leading M rows of that same draw)."""
    c = config(name)
    Mmax = max(c.Ms)
    X, Wp, scales, Zp = make(Mmax, c.K, c.N, c.index, c.group, c.outliers)
    if M is not None:
        if M > Mmax:
            raise ValueError("M beyond the configuration's largest batch")
        X = np.ascontiguousarray(X[:M])
    return X, Wp, scales, Zp


def algorithmic_bytes(M: int, K: int, N: int, group: int = GROUP) -> int:
    """Bytes one GEMM must move: packed W, fp16 scales, packed zero points, X, Y."""
    G = K // group
    return K * N // 2 + G * N * 2 + G * N // 2 + 2 * M * K + 2 * M * N
