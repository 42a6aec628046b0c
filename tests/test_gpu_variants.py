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


# ---- BF16 activations (w4a16_gemm_bf16) ----

def _bf16_to_device(torch, Xb):
    return torch.from_numpy(Xb.view(np.int16)).to("cuda").view(torch.bfloat16)


def _bf16_values(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _bf16_out(torch, M, N):
    return torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")


def _bits(Y):
    import torch
    return Y.view(torch.int16).cpu().numpy().view(np.uint16)


BF16_SHAPES = [(1, 256, 264, 128), (1, 8192, 4104, 128), (2, 20480, 2048, 128), (4, 6144, 1032, 128), (3, 384, 136, 32), (4, 1024, 72, 64),
               (8, 2048, 512, 128), (16, 1024, 776, 128), (12, 1536, 264, 64), (33, 512, 256, 128), (100, 1536, 264, 64), (130, 1024, 520, 128)]


@pytest.mark.parametrize("M,K,N,group", BF16_SHAPES)
def test_bf16_activations(gpu, M, K, N, group):
    """X and Y in bfloat16 against the oracle's BF16 form: the scheduler's plan and forced plans of both families,
    with and without a split, the accumulator and the second pass, with and without a zeros tensor."""
    torch, binding = gpu
    _, Wp, s, Zp = wl.make(1, K, N, index=8300 + M + K + N, group=group)
    Xb = wl.make_x_bf16(M, K, index=8300 + M + K + N, outliers=True)
    ref = orc.gemm_bf16(Xb, Wp, s, Zp, group)
    ref_sym = orc.gemm_bf16(Xb, Wp, s, wl.pack_along_n(np.full((K // group, N), 8, np.uint8)), group)
    _, dW, dS, dZ = binding.to_device(np.zeros((1, 8), np.float16), Wp, s, Zp)
    dX = _bf16_to_device(torch, Xb)
    G = K // group
    kernels = [binding.KERNEL_AUTO, binding.KERNEL_TILE] + ([binding.KERNEL_STRIPE] if M <= 4 else [])
    for kernel in kernels:
        for split, fin in ((0, 0), (1, 0), (min(3, G), 0), (min(3, G), 2), (min(5, G), 1)):
            if split == 1 and fin:
                continue
            for zeros, want in ((dZ, ref), (None, ref_sym)):
                say("bf16", (M, K, N, group), kernel, split, fin, "symmetric" if zeros is None else "zeros")
                binding.tune("stripe_finish", fin)
                try:
                    Y = _bf16_out(torch, M, N)
                    binding.gemm_bf16(dX, dW, dS, zeros, group, kernel=kernel, split=split, out=Y)
                    torch.cuda.synchronize()
                finally:
                    binding.tune("stripe_finish", 0)
                out = _bf16_values(_bits(Y)).astype(np.float64)
                assert not np.isnan(out).any()
                assert err_ratio(out, want) <= 1.0, (M, K, N, group, kernel, split, fin)
                # and close to the one rounding the format asks for: half a unit in the last place (2^-9) plus the sums' own error
                assert np.all(np.abs(out - want) <= 2.0 ** -8 * np.abs(want) + 2e-3), (M, K, N, group, kernel, split, fin)


def test_bf16_exact_sums_round_like_the_oracle(gpu):
    """Small integers in X and a power of two as scale: every product and sum is exact in FP32, so the output must be
    the oracle's single rounding to bfloat16 bit for bit (ties to even included)."""
    torch, binding = gpu
    rng = np.random.default_rng(8400)
    for (M, K, N) in [(1, 4096, 1032), (3, 8192, 4096), (8, 2048, 520), (40, 1024, 264)]:
        group = 128
        xi = rng.integers(-4, 5, (M, K)).astype(np.float32)
        Xb = (xi.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
        assert np.array_equal(_bf16_values(Xb), xi)
        _, Wp, _, Zp = wl.make(1, K, N, index=8400 + M, group=group)
        s = np.full((K // group, N), np.float16(2.0 ** -6))
        ref = orc.gemm_bf16(Xb, Wp, s, Zp, group)
        _, dW, dS, dZ = binding.to_device(np.zeros((1, 8), np.float16), Wp, s, Zp)
        say("bf16 exact", (M, K, N))
        Y = _bf16_out(torch, M, N)
        binding.gemm_bf16(_bf16_to_device(torch, Xb), dW, dS, dZ, group, out=Y)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(Y), orc.to_bf16_bits(ref))


def test_bf16_headline_shape_every_output(gpu):
    """M = 1, K = 28672, N = 8192 in bfloat16: every output against the oracle, and repeated calls give the same bits."""
    torch, binding = gpu
    c = wl.config("c4")
    _, Wp, s, Zp = wl.make_config("c4", 1)
    Xb = wl.make_x_bf16(1, c.K, index=c.index)
    ref = orc.gemm_bf16(Xb, Wp, s, Zp, c.group)
    _, dW, dS, dZ = binding.to_device(np.zeros((1, 8), np.float16), Wp, s, Zp)
    dX = _bf16_to_device(torch, Xb)
    say("bf16 c4 M=1")
    first = None
    for _ in range(3):
        Y = _bf16_out(torch, 1, c.N)
        binding.gemm_bf16(dX, dW, dS, dZ, c.group, out=Y)
        torch.cuda.synchronize()
        bits = _bits(Y)
        assert err_ratio(_bf16_values(bits).astype(np.float64), ref) <= 1.0
        first = bits if first is None else first
        assert np.array_equal(bits, first)


def test_bf16_forced_plans_outside_its_families_are_refused(gpu):
    torch, binding = gpu
    _, Wp, s, Zp = wl.make(1, 256, 64, index=8500)
    _, dW, dS, dZ = binding.to_device(np.zeros((1, 8), np.float16), Wp, s, Zp)
    for M, kernel in ((2, binding.KERNEL_WAVE_SPLIT), (8, binding.KERNEL_STRIPE)):
        dX = torch.zeros((M, 256), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(binding.W4A16Error) as e:
            binding.gemm_bf16(dX, dW, dS, dZ, 128, kernel=kernel)
        assert e.value.status == binding.ERR_UNSUPPORTED
