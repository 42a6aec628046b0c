"""GPU parity of the variants the paper names without evaluating them, through the C ABI, against the oracle's
variant functions (tests/test_oracle_variants.py pins those)."""
import sys

import numpy as np
import pytest

from oracle import w4a16_oracle as orc
from paper_2601_16536_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-2


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2601_16536_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return torch, binding


def err_ratio(Y, ref):
    Y = np.asarray(Y, dtype=np.float64)
    return float(np.max(np.abs(Y - ref) / (TOL * (1.0 + np.abs(ref)))))


SYM_SHAPES = [(1, 256, 264, 128), (2, 2048, 520, 128), (4, 1024, 72, 64), (3, 384, 136, 32), (8, 2048, 512, 128), (16, 1024, 776, 128),
              (33, 512, 256, 128), (100, 1536, 264, 64), (1, 8192, 4104, 128), (4, 6144, 1032, 128)]


@pytest.mark.parametrize("M,K,N,group", SYM_SHAPES)
def test_symmetric_quantisation_without_a_zeros_tensor(gpu, M, K, N, group):
    """zeros = NULL at the boundary (Section 2.1, symmetric: z = 0 on signed codes = stored code - 8): every family,
    with and without a split, the accumulator and the second pass."""
    torch, binding = gpu
    X, Wp, s, _ = wl.make(M, K, N, index=8000 + M + K + N, group=group)
    ref = orc.gemm_symmetric(X, Wp, s, group)
    dX, dW, dS, _ = binding.to_device(X, Wp, s, wl.pack_along_n(np.zeros((K // group, N), np.uint8)))
    G = K // group
    kernels = [binding.KERNEL_AUTO, binding.KERNEL_TILE] + ([binding.KERNEL_WAVE_SPLIT] if M <= 4 else []) + (
        [binding.KERNEL_STRIPE] if M <= 16 else [])
    for kernel in kernels:
        for split, fin in ((0, 0), (1, 0), (min(3, G), 0), (min(3, G), 2)):
            if split == 1 and fin:
                continue
            say("symmetric", (M, K, N, group), kernel, split, fin)
            binding.tune("stripe_finish", fin)
            try:
                Y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
                binding.gemm_ex(dX, dW, dS, None, group, kernel=kernel, split=split, out=Y)
                torch.cuda.synchronize()
            finally:
                binding.tune("stripe_finish", 0)
            out = Y.cpu().numpy()
            assert not np.isnan(out).any()
            assert err_ratio(out, ref) <= 1.0, (M, K, N, group, kernel, split, fin)


def test_symmetric_matches_explicit_zero_points_of_eight_bit_for_bit(gpu):
    """The same kernels, the same arithmetic: NULL and a tensor of eights must give identical bits."""
    torch, binding = gpu
    for (M, K, N) in [(1, 4096, 1032), (8, 2048, 520), (40, 1024, 264)]:
        X, Wp, s, _ = wl.make(M, K, N, index=8100 + M)
        Z8 = wl.pack_along_n(np.full((K // wl.GROUP, N), 8, np.uint8))
        dX, dW, dS, dZ = binding.to_device(X, Wp, s, Z8)
        say("symmetric vs eights", (M, K, N))
        assert torch.equal(binding.gemm(dX, dW, dS, None, wl.GROUP), binding.gemm(dX, dW, dS, dZ, wl.GROUP))


def test_symmetric_dequant_entry_point_bit_exact(gpu):
    torch, binding = gpu
    for (K, N, group) in [(256, 264, 128), (1024, 72, 64), (2304, 1000, 128)]:
        _, Wp, s, Zp = wl.make(1, K, N, index=8200 + K + N, group=group)
        want = orc.dequant_symmetric(Wp, s, group).astype(np.float16)
        _, dW, dS, _ = binding.to_device(np.zeros((1, K), np.float16), Wp, s, Zp)
        say("symmetric dequant", K, N, group)
        W16 = torch.full((K, N), float("nan"), dtype=torch.float16, device="cuda")
        binding.dequant(dW, dS, None, group, out=W16)
        torch.cuda.synchronize()
        assert np.array_equal(W16.cpu().numpy().view(np.uint16), want.view(np.uint16))
