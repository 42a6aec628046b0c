"""The entry point that allocates nothing (w4a16_gemm_noalloc) against w4a16_gemm_ex: same plan, same kernels,
so the outputs must agree bit for bit; each is also checked against the oracle at the usual bar.  Calls in a
row, each with a smaller input than the one before (the shared array keeps the earlier call's contents), then
a plan that needs more than the array holds."""
import sys

import numpy as np
import pytest

from oracle import w4a16_oracle as orc
from paper_2601_16536_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-2


def err_ratio(Y, ref):
    Y = np.asarray(Y, dtype=np.float64)
    return float(np.max(np.abs(Y - ref) / (TOL * (1.0 + np.abs(ref)))))


def test_noalloc_entry_point_matches_gemm():
    import torch
    from paper_2601_16536_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    # (M, K, N, kernel, split): an accumulator plan of the stripe family, FP32 partials for the second pass, then
    # smaller inputs of both kinds and a direct plan, so that stale contents of the array would show
    T = binding.KERNEL_TILE
    # the first two: 32 rows of X per workgroup (the four-wave TILE form), FP32 partials, then the accumulator
    cases = [(48, 512, 8192, T, 2), (40, 512, 8192, T, 2), (2, 8192, 4104, -1, 0), (130, 768, 2056, T, 3), (1, 4096, 1024, -1, 0), (33, 512, 264, T, 4), (8, 2048, 520, -1, 0),
             (3, 1024, 264, -1, 0), (5, 256, 72, T, 1)]
    p = lambda t: t.data_ptr()
    st = torch.cuda.current_stream().cuda_stream
    for (M, K, N, kernel, split) in cases:
        X, Wp, s, Zp = wl.make(M, K, N, index=7000 + M + K + N)
        ref = orc.gemm(X, Wp, s, Zp, wl.GROUP)
        dX, dW, dS, dZ = binding.to_device(X, Wp, s, Zp)
        plan = binding.query_plan(M, N, K, wl.GROUP, kernel, split)
        assert plan["workspace_bytes"] <= 4 << 20
        print("[case] noalloc", (M, K, N), plan, flush=True)
        sys.stdout.flush()
        Y0 = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        Y1 = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        for rep in range(2):
            Y1.fill_(float("nan"))
            rc = binding.raw_gemm_noalloc(p(dX), p(dW), p(dS), p(dZ), wl.GROUP, M, N, K, p(Y1), st, kernel, split)
            assert rc == binding.OK, binding.status_string(rc)
            torch.cuda.synchronize()
            assert err_ratio(Y1.cpu().numpy(), ref) <= 1.0
        assert binding.raw_gemm_ex(p(dX), p(dW), p(dS), p(dZ), wl.GROUP, M, N, K, p(Y0), st, kernel, split) == binding.OK
        torch.cuda.synchronize()
        assert err_ratio(Y0.cpu().numpy(), ref) <= 1.0
        assert torch.equal(Y0, Y1), (M, K, N)
    # beyond the array: S * M * N * 4 bytes of FP32 partials > 4 MiB
    M, K, N, kernel, split = 130, 768, 2056, T, 6
    plan = binding.query_plan(M, N, K, wl.GROUP, kernel, split)
    assert plan["workspace_bytes"] > 4 << 20, plan
    X, Wp, s, Zp = wl.make(M, K, N, index=7999)
    dX, dW, dS, dZ = binding.to_device(X, Wp, s, Zp)
    Y = torch.full((M, N), 3.0, dtype=torch.float16, device="cuda")
    rc = binding.raw_gemm_noalloc(p(dX), p(dW), p(dS), p(dZ), wl.GROUP, M, N, K, p(Y), st, kernel, split)
    assert rc == binding.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (Y == 3.0).all()  # nothing was launched
