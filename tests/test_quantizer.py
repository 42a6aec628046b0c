"""The offline quantizer (Section 2.1, Eq. 1): pins of its CPU oracle, then the HIP kernel against it.

The paper prints no numeric example of Eq. 1 and does not fix how s and z are chosen, so the oracle is
tied down by what the formula and its stated reading force: a grid of weights that is its own
quantization, Eq. 1 re-evaluated code by code with exact rationals, the half-step reconstruction bound,
the special groups (all zero, one sign only), and the storage constants of tests/golden.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import quantize_oracle as qo
from oracle import w4a16_oracle as orc


def _random_weights(K, N, seed, scale=0.05):
    rng = np.random.default_rng([16536, 77, seed])
    return (rng.standard_normal((K, N)) * scale).astype(np.float16)


def test_grid_of_weights_is_its_own_quantization(qo=qo):
    """w = s0 (q0 - z0) with s0 a power of two and the codes 0 and 15 present in every group: the range is
    15 s0 wide, so s = s0, z = z0 and q = q0 exactly.  A wrong sign, axis or zero-point formula moves them."""
    rng = np.random.default_rng(5)
    K, N, group = 256, 24, 64
    G = K // group
    q0 = rng.integers(0, 16, (K, N)).astype(np.int32)
    for g in range(G):  # both ends of the range in every (group, column)
        q0[g * group + rng.integers(0, group // 2, N), np.arange(N)] = 0
        q0[g * group + group // 2 + rng.integers(0, group // 2, N), np.arange(N)] = 15
    z0 = rng.integers(0, 16, (G, N)).astype(np.int32)
    s0 = (2.0 ** rng.integers(-9, -3, (G, N))).astype(np.float16)
    W = (s0.astype(np.float64).repeat(group, axis=0) * (q0 - z0.repeat(group, axis=0))).astype(np.float16)
    q, s, z = qo.quantize_codes(W, group)
    assert np.array_equal(s.view(np.uint16), s0.view(np.uint16))
    assert np.array_equal(z, z0)
    assert np.array_equal(q, q0)


def test_codes_are_eq1_evaluated_with_rationals(qo=qo):
    """Each code is clamp(round(x / s) + z) of Eq. 1 with x / s taken exactly (ties to even), given the
    oracle's own s and z; s and z are the stated functions of the group's range."""
    W = _random_weights(128, 16, seed=1)
    group = 32
    q, s, z = qo.quantize_codes(W, group)
    K, N = W.shape

    def rne(fr):
        fl = fr.numerator // fr.denominator
        rem = fr - fl
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
            fl += 1
        return fl

    for n in range(N):
        for g in range(K // group):
            col = [Fraction(float(W[g * group + k, n])) for k in range(group)]
            lo, hi = min(min(col), 0), max(max(col), 0)
            want_s = np.float32(float(hi - lo)) / np.float32(15)  # hi - lo is exact in binary32 here (FP16 inputs, close exponents)
            assert np.float16(want_s) == s[g, n]
            sf = Fraction(float(s[g, n]))
            assert z[g, n] == min(max(rne(-lo / sf), 0), 15)
            for k in range(group):
                assert q[g * group + k, n] == min(max(rne(col[k] / sf) + int(z[g, n]), 0), 15)


def test_reconstruction_within_half_a_step(qo=qo):
    """Dequant(quantize(w)) is within s / 2 of w (plus the little the FP16 rounding of s clips at the ends),
    through the GEMM oracle's own dequantization of the packed tensors."""
    W = _random_weights(512, 40, seed=2)
    group = 128
    Wp, s, Zp = qo.quantize(W, group)
    back = orc.dequant(Wp, s, Zp, group).astype(np.float64)
    step = s.astype(np.float64).repeat(group, axis=0)
    assert np.all(np.abs(back - W.astype(np.float64)) <= step * 0.51)
    # and the codes use the whole range: every group holds a 0 or a 15
    q = orc.unpack_codes(Wp).reshape(512 // group, group, 40)
    assert np.all((q.min(axis=1) == 0) | (q.max(axis=1) == 15))


def test_special_groups(qo=qo):
    group = 32
    W = np.zeros((96, 8), np.float16)
    W[32:64] = np.float16(0.25)    # one sign only: lo = 0, so z = 0 and the value is code 15
    W[64:96] = np.float16(-0.5)    # negative only: hi = 0, so z = 15 and the value is code 0
    q, s, z = qo.quantize_codes(W, group)
    assert np.all(q[:32] == 0) and np.all(z[0] == 0) and np.all(s[0] == 1)           # all-zero group: s = 1
    assert np.all(z[1] == 0) and np.all(q[32:64] == 15) and np.all(s[1] == np.float16(0.25 / 15))
    assert np.all(z[2] == 15) and np.all(q[64:96] == 0) and np.all(s[2] == np.float16(0.5 / 15))


def test_storage_layout_of_the_outputs(qo=qo):
    """Packed outputs unpack (with the GEMM oracle's unpackers, pinned by tests/golden) to the codes."""
    W = _random_weights(64, 24, seed=3)
    q, s, z = qo.quantize_codes(W, 32)
    Wp, s2, Zp = qo.quantize(W, 32)
    assert np.array_equal(orc.unpack_codes(Wp), q)
    assert np.array_equal(orc.unpack_zeros(Zp), z)
    assert np.array_equal(s.view(np.uint16), s2.view(np.uint16))
    # nibble i of word r is the code of k = 8 r + i
    assert int(Wp[0, 0]) == sum(int(q[i, 0]) << (4 * i) for i in range(8))
    assert int(Zp[0, 0]) == sum(int(z[0, j]) << (4 * j) for j in range(8))


PINS = (test_grid_of_weights_is_its_own_quantization, test_codes_are_eq1_evaluated_with_rationals,
        test_reconstruction_within_half_a_step, test_special_groups, test_storage_layout_of_the_outputs)

MUTATIONS = [  # (text in oracle/quantize_oracle.py, what a plausible mistake would put there)
    ("np.rint((-lo) / s)", "np.rint(lo / s)"),                    # sign of the zero point
    ("/ f32(15)", "/ f32(16)"),                                   # number of steps
    ("np.rint(w / s[:, None, :]) + z[:, None, :]", "np.rint(w / s[:, None, :])"),  # zero point dropped from Eq. 1
    ("np.rint(w / s[:, None, :])", "np.floor(w / s[:, None, :])"),                 # truncation for rounding
    ("np.minimum(w.min(axis=1), f32(0))", "w.min(axis=1)"),       # range without 0
    ("np.maximum(w.max(axis=1), f32(0))", "w.max(axis=1)"),
    ("w.min(axis=1)", "w.min(axis=2)[:, :, None].repeat(w.shape[2], axis=2).min(axis=1)"),  # group statistics over the wrong axis
    ("q[i::8, :]", "q[7 - i::8, :]"),                             # nibble order along K
    ("z[:, j::8]", "z[:, 7 - j::8]"),                             # nibble order along N
    ("(hi - lo)", "(hi + lo)"),
    ("np.where(s16 == 0, np.float16(1), s16)", "s16"),            # all-zero group left with s = 0
]


@pytest.mark.parametrize("old,new", MUTATIONS)
def test_pins_catch_planted_mistakes(old, new):
    """Each planted mistake in a copy of the oracle must fail at least one pin."""
    import types
    src = open(qo.__file__).read()
    assert src.count(old) >= 1, old
    mod = types.ModuleType("quantize_oracle_mutant")
    exec(compile(src.replace(old, new), "quantize_oracle_mutant", "exec"), mod.__dict__)
    caught = False
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin(mod)
        except Exception:
            caught = True
            break
    assert caught, "no pin noticed: %s -> %s" % (old, new)


# ----------------------------------------------------------------- the GPU ---

@pytest.fixture(scope="module")
def gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2601_16536_amd import binding
    binding.lib()
    return torch, binding


@pytest.mark.gpu
def test_hip_quantizer_bit_exact(gpu):
    """Codes, scales and zero points bit for bit the oracle's (both decide every code in binary32), on ragged
    shapes, several group sizes, and the special groups; then the round trip through w4a16_dequant."""
    torch, binding = gpu
    for (K, N, group, seed) in [(128, 8, 128, 1), (256, 264, 128, 2), (1024, 72, 64, 3), (384, 136, 32, 4), (2304, 1000, 128, 5),
                                (4096, 4104, 128, 6)]:
        W = _random_weights(K, N, seed=10 + seed, scale=0.02 * seed)
        W[:group, : N // 2] = 0                                  # all-zero groups
        W[group:2 * group, :8] = np.abs(W[group:2 * group, :8])  # one sign only
        want = qo.quantize(W, group)
        print("[case] quantize", K, N, group, flush=True)
        dW = torch.from_numpy(W).cuda()
        Wp, s, Zp = binding.quantize(dW, group)
        torch.cuda.synchronize()
        assert np.array_equal(Wp.cpu().numpy().view(np.uint32), want[0])
        assert np.array_equal(s.cpu().numpy().view(np.uint16), want[1].view(np.uint16))
        assert np.array_equal(Zp.cpu().numpy().view(np.uint32), want[2])
        back = binding.dequant(Wp, s, Zp, group)
        torch.cuda.synchronize()
        step = want[1].astype(np.float64).repeat(group, axis=0)
        assert np.all(np.abs(back.cpu().numpy().astype(np.float64) - W.astype(np.float64)) <= step * 0.52)
