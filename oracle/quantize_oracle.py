"""CPU oracle of the weight quantizer (TEST INFRASTRUCTURE, never the product path).

Section 2.1, Eq. 1 defines uniform affine quantization, x_q = round(x / s) + z, and
says nothing about how s and z are found.  This build's reading, per quantisation
group (``group`` consecutive k of one column n), in binary32 arithmetic throughout:

    lo = min(min_k w, 0), hi = max(max_k w, 0)      the range always holds 0, so z is a code
    s  = fp16((hi - lo) / 15), 1 if that is 0       scales cross the boundary as FP16
    z  = clamp(rint(-lo / s), 0, 15)
    q  = clamp(rint(w / s) + z, 0, 15)              Eq. 1; round = to nearest, ties to even

Plain numpy, one operation per line of the recipe; imports nothing from the GPU
package.  Outputs use the storage layout of the GEMM's inputs: codes packed eight
per uint32 along K (nibble i of word r = code of k = 8 r + i), zero points packed
eight per uint32 along N.
"""
from __future__ import annotations

import numpy as np


def quantize_codes(W, group: int):
    """(q[K, N] uint8, s[G, N] float16, z[G, N] uint8) of Eq. 1 for FP16 weights W[K, N]."""
    W = np.asarray(W)
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("W must be a float16 matrix [K, N]")
    K, N = W.shape
    if group < 1 or K % group:
        raise ValueError("K must be a multiple of group")
    G = K // group
    f32 = np.float32
    w = W.astype(f32).reshape(G, group, N)
    lo = np.minimum(w.min(axis=1), f32(0))
    hi = np.maximum(w.max(axis=1), f32(0))
    s32 = (hi - lo) / f32(15)
    assert s32.dtype == f32
    s16 = s32.astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(1), s16).astype(np.float16)
    s = s16.astype(f32)
    z = np.clip(np.rint((-lo) / s), f32(0), f32(15))
    q = np.clip(np.rint(w / s[:, None, :]) + z[:, None, :], f32(0), f32(15))
    assert q.dtype == f32 and z.dtype == f32
    return q.reshape(K, N).astype(np.uint8), s16, z.astype(np.uint8)


def quantize(W, group: int):
    """As quantize_codes, in storage layout: (Wp[K/8, N] uint32, scales[G, N] float16, Zp[G, N/8] uint32)."""
    q, s16, z = quantize_codes(W, group)
    K, N = q.shape
    if K % 8 or N % 8:
        raise ValueError("K and N must be multiples of 8")
    Wp = np.zeros((K // 8, N), np.uint32)
    for i in range(8):
        Wp |= q[i::8, :].astype(np.uint32) << np.uint32(4 * i)
    Zp = np.zeros((z.shape[0], N // 8), np.uint32)
    for j in range(8):
        Zp |= z[:, j::8].astype(np.uint32) << np.uint32(4 * j)
    return Wp, s16, Zp
