"""GPU parity: the HIP library (through its C ABI) against the CPU oracle.

Bar (floating point): max |Y - ref| <= 1e-2 * (1 + |ref|) against the oracle's
unrounded binary64 result; bit-exact where the result is an exactly
representable integer.  Every case prints its name before touching the GPU so
that a fault names its case.
"""
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
    binding.lib()  # fails loudly when the HIP library is not built
    return torch, binding


def err_ratio(Y, ref):
    Y = np.asarray(Y, dtype=np.float64)
    return float(np.max(np.abs(Y - ref) / (TOL * (1.0 + np.abs(ref)))))


def run_gpu(gpu, X, Wp, s, Zp, group, kernel=-1, split=0, poison=True):
    torch, binding = gpu
    dX, dW, dS, dZ = binding.to_device(X, Wp, s, Zp)
    Y = torch.full((X.shape[0], Wp.shape[1]), float("nan"), dtype=torch.float16, device="cuda")
    binding.gemm_ex(dX, dW, dS, dZ, group, kernel=kernel, split=split, out=Y)
    torch.cuda.synchronize()
    out = Y.cpu().numpy()
    assert not np.isnan(out).any(), "output holds NaN (element not written?)"
    return out


SMALL = [
    # M, K, N, group
    (1, 128, 8, 128),
    (1, 256, 264, 128),
    (2, 512, 520, 128),
    (3, 1024, 72, 64),
    (4, 384, 136, 32),
    (5, 768, 1032, 128),
    (8, 2048, 512, 128),
    (11, 1280, 256, 256),
    (16, 2048, 776, 128),
    (17, 1024, 264, 128),
    (33, 512, 256, 128),
    (64, 2048, 520, 128),
    (100, 1536, 264, 64),
    (130, 768, 256, 128),
    (1, 4096, 4104, 128),
    (2, 8192, 40, 128),
    (4, 6144, 16416, 128),
    (3, 2304, 1000, 128),
]


@pytest.mark.parametrize("M,K,N,group", SMALL)
def test_small_shapes_every_split(gpu, M, K, N, group):
    _, binding = gpu
    X, Wp, s, Zp = wl.make(M, K, N, index=1000 + M + K + N, group=group)
    ref = orc.gemm(X, Wp, s, Zp, group)
    G = K // group
    kernels = [binding.KERNEL_AUTO, binding.KERNEL_TILE] + (
        [binding.KERNEL_WAVE_SPLIT] if M <= 4 else []) + ([binding.KERNEL_STRIPE] if M <= 16 else [])
    for kernel in kernels:
        for split in sorted({0, 1, 2, 3, G}):
            if split > G:
                continue
            say("small", M, K, N, group, "kernel", kernel, "split", split, binding.query_plan(M, N, K, group, kernel, split))
            Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=kernel, split=split)
            r = err_ratio(Y, ref)
            assert r <= 1.0, (M, K, N, group, kernel, split, r)


@pytest.mark.parametrize("form", ["scheduler", "eight waves at 32 and 64 rows"])
@pytest.mark.parametrize("rows_x", [16, 32, 64])
def test_tile_family_every_row_block(gpu, rows_x, form):
    """The TILE kernels for 16, 32 and 64 rows of X per workgroup (at 32 and 64 rows and group = 128: four waves per
    workgroup with q - z as the operand, and the eight-wave form with bare codes).  The scheduler takes the larger blocks only
    where N is large, so the library's tuning knobs force them here on small ragged shapes (rows past M, columns past N,
    fewer groups than waves, group sizes with and without the group-aligned loop)."""
    _, binding = gpu
    eight = form != "scheduler"
    if eight and rows_x == 16:
        pytest.skip("the four-wave form exists at 32 and 64 rows only")
    binding.tune("tile_rows", rows_x)
    binding.tune("tile_wide", 2 if eight else 0)
    binding.tune("tile_dyn", 2)  # not the ticket form, which 16 rows would take
    try:
        _tile_rows_cases(gpu, rows_x)
    finally:
        binding.tune("tile_rows", 0)
        binding.tune("tile_wide", 0)
        binding.tune("tile_dyn", 0)


def test_four_wave_form_exact_sums_and_one_hot_rows(gpu):
    """The four-wave TILE form multiplies X with q - z as exact FP16 integers and applies s per group in FP32.  With
    power-of-two scales and small integers in X every sum is exact: the result must be the oracle's, bit for bit; with
    one-hot rows of X the result is the FP16 rounding of the weight row itself."""
    torch, binding = gpu
    rng = np.random.default_rng(23)
    M, K, N, group = 70, 1024, 264, 128
    G = K // group
    _, Wp, _, Zp = wl.make(1, K, N, index=2300, group=group)
    s = (2.0 ** rng.integers(-8, -3, (G, N))).astype(np.float16)
    X = rng.integers(-3, 4, (M, K)).astype(np.float16)
    ref = orc.gemm(X, Wp, s, Zp, group)
    X1, Wp1, s1, Zp1 = wl.make(64, K, N, index=2301, group=group)
    X1[:] = 0
    ks = rng.choice(K, size=64, replace=False)
    X1[np.arange(64), ks] = 1
    try:
        for rows_x in (32, 64):
            binding.tune("tile_rows", rows_x)
            for split in (1, 3, 8):
                say("four waves exact", rows_x, split)
                assert binding.query_plan(M, N, K, group, binding.KERNEL_TILE, split)["waves_k"] == 4
                Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=binding.KERNEL_TILE, split=split)
                assert np.array_equal(Y, orc.to_fp16(ref)), (rows_x, split)
            say("four waves one-hot", rows_x)
            Y = run_gpu(gpu, X1, Wp1, s1, Zp1, group, kernel=binding.KERNEL_TILE, split=1)
            assert np.array_equal(Y, orc.dequant(Wp1, s1, Zp1, group)[ks].astype(np.float16)), rows_x
    finally:
        binding.tune("tile_rows", 0)


def test_tile_ticket_form_with_two_units_in_flight(gpu):
    """The M <= 16 TILE form hands its units out by ticket and sums them exactly: two units in flight per wave (knob
    tile_depth) and other wave counts must give the bits of the scheduler's form, on ragged shapes and group sizes."""
    _, binding = gpu
    for (M, K, N, group) in [(5, 1024, 136, 128), (16, 2048, 264, 128), (9, 768, 72, 64), (2, 1024, 520, 32), (13, 4096, 64, 256)]:
        X, Wp, s, Zp = wl.make(M, K, N, index=2400 + M + K + N, group=group)
        ref = orc.gemm(X, Wp, s, Zp, group)
        G = K // group
        for split in sorted({1, 2, 3, G}):
            if split > G or split > 63:
                continue
            say("ticket form", M, K, N, group, split)
            base = run_gpu(gpu, X, Wp, s, Zp, group, kernel=binding.KERNEL_TILE, split=split)
            assert err_ratio(base, ref) <= 1.0
            for depth, waves in [(2, 0), (2, 4), (1, 12), (2, 12)]:
                binding.tune("tile_depth", depth)
                binding.tune("tile_waves", waves)
                try:
                    Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=binding.KERNEL_TILE, split=split)
                finally:
                    binding.tune("tile_depth", 0)
                    binding.tune("tile_waves", 0)
                assert np.array_equal(Y, base), (M, K, N, group, split, depth, waves)


def _tile_rows_cases(gpu, rows_x):
    _, binding = gpu
    for (M, K, N, group) in [(33, 640, 72, 128), (130, 512, 136, 128), (200, 1024, 200, 128), (40, 256, 64, 128),
                             (64, 2048, 520, 128), (7, 128, 64, 128), (70, 768, 264, 64), (129, 1024, 72, 256)]:
        X, Wp, s, Zp = wl.make(M, K, N, index=2000 + M + K + N, group=group)
        ref = orc.gemm(X, Wp, s, Zp, group)
        G = K // group
        for split in sorted({0, 1, 2, 3, G}):
            if split > G:
                continue
            plan = binding.query_plan(M, N, K, group, binding.KERNEL_TILE, split)
            assert plan["tile_m"] == rows_x
            say("tile rows", rows_x, (M, K, N, group), "split", split, plan)
            Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=binding.KERNEL_TILE, split=split)
            r = err_ratio(Y, ref)
            assert r <= 1.0, (rows_x, M, K, N, group, split, r)


def test_seeded_random_shapes(gpu):
    """Forty-eight shapes drawn with a fixed seed (M 1..200, ragged N, K of 1..40 groups, group 32..256): the
    scheduler's plan and one forced (family, split) each, all outputs against the oracle."""
    _, binding = gpu
    rng = np.random.default_rng(20260116)
    for case in range(48):
        group = int(rng.choice([32, 64, 128, 128, 128, 256]))
        G = int(rng.integers(1, 41))
        K = G * group
        N = 8 * int(rng.integers(1, 160))
        M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 15, 16, 17, 31, 32, 33, 64, 65, 100, 128, 200]))
        X, Wp, s, Zp = wl.make(M, K, N, index=5000 + case, group=group)
        ref = orc.gemm(X, Wp, s, Zp, group)
        fams = [binding.KERNEL_TILE] + ([binding.KERNEL_STRIPE] if M <= 16 else []) + ([binding.KERNEL_WAVE_SPLIT] if M <= 4 else [])
        forced = (int(rng.choice(fams)), int(rng.integers(1, G + 1)))
        for kernel, split in ((binding.KERNEL_AUTO, 0), forced):
            say("random", case, (M, K, N, group), "kernel", kernel, "split", split)
            Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=kernel, split=split)
            r = err_ratio(Y, ref)
            assert r <= 1.0, (case, M, K, N, group, kernel, split, r)


def test_integer_case_bit_exact(gpu):
    """s = 1, z = 0, X in {-1,0,1}, K = 128: integers below 2048, exactly representable."""
    rng = np.random.default_rng(21)
    M, K, N, group = 9, 128, 264, 128
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    Xi = rng.integers(-1, 2, (M, K))
    X = Xi.astype(np.float16)
    Wp, Zp = wl.pack_along_k(q), wl.pack_along_n(np.zeros((1, N), np.uint8))
    s = np.ones((1, N), np.float16)
    ref = orc.gemm(X, Wp, s, Zp, group)
    assert np.array_equal(ref, (Xi @ q.astype(np.int64)).astype(np.float64))
    say("integer exact")
    Y = run_gpu(gpu, X, Wp, s, Zp, group)
    assert np.array_equal(Y.astype(np.float64), ref)
    for kernel in (0, 3):
        Y = run_gpu(gpu, X[:3], Wp, s, Zp, group, kernel=kernel)
        assert np.array_equal(Y.astype(np.float64), ref[:3])


def test_integer_case_bit_exact_with_zero_points_and_splits(gpu):
    """Integer scales, random zero points, several groups: still exact in fp32 and fp16."""
    rng = np.random.default_rng(22)
    M, K, N, group = 4, 512, 256, 128
    G = K // group
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    z = rng.integers(0, 16, (G, N), dtype=np.uint8)
    Xi = np.zeros((M, K), np.int64)
    for m in range(M):
        idx = rng.choice(K, size=24, replace=False)
        Xi[m, idx] = rng.integers(-2, 3, 24)
    X = Xi.astype(np.float16)
    s = rng.integers(1, 3, (G, N)).astype(np.float16)
    Wp, Zp = wl.pack_along_k(q), wl.pack_along_n(z)
    ref = orc.gemm(X, Wp, s, Zp, group)
    assert np.abs(ref).max() < 2048 and np.array_equal(ref, np.round(ref))
    for kernel in (0, 3, 4):
        for split in (1, 2, 4):
            say("integer exact zp", kernel, split)
            Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=kernel, split=split)
            assert np.array_equal(Y.astype(np.float64), ref)


def test_one_hot_rows_return_weight_rows(gpu):
    """X = e_k: Y row is the fp16 rounding of dequantized weight row k (indexing check)."""
    K, N, group = 256, 264, 128
    _, Wp, s, Zp = wl.make(1, K, N, index=1234, group=group)
    ks = [0, 1, 7, 8, 127, 128, 200, 255, 31, 32, 33, 64, 100, 129, 250, 5]
    X = np.zeros((len(ks), K), np.float16)
    for i, k in enumerate(ks):
        X[i, k] = 1.0
    w = orc.dequant(Wp, s, Zp, group)
    say("one hot")
    want = w[ks].astype(np.float16)  # exact fp32 weight, one rounding to fp16
    Y = run_gpu(gpu, X, Wp, s, Zp, group)
    assert np.array_equal(Y, want)
    for i in range(0, len(ks), 4):  # the M <= 4 kernels, four rows at a time
        for kernel, split in ((0, 0), (3, 1), (3, 2)):
            Y = run_gpu(gpu, X[i:i + 4], Wp, s, Zp, group, kernel=kernel, split=split)
            assert np.array_equal(Y, want[i:i + 4])


def test_closed_forms_on_gpu(gpu):
    """q = z everywhere gives zero (to fp32 accumulation noise: the kernel forms
    s 2^24 P - s z sum(x) from two separately rounded fp32 sums); a constant code
    gives s (c - z) rowsum(X)."""
    rng = np.random.default_rng(23)
    M, K, N, group = 3, 1024, 520, 128
    G = K // group
    z = rng.integers(0, 16, (G, N), dtype=np.uint8)
    s = rng.uniform(0.001, 0.02, (G, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    say("q == z")
    Y = run_gpu(gpu, X, wl.pack_along_k(np.repeat(z, group, axis=0)), s, wl.pack_along_n(z), group)
    assert np.abs(Y.astype(np.float64)).max() < 1e-3  # tolerance would allow 1e-2
    c, zv, sv = 11, 3, np.float16(0.0123)
    say("constant code")
    Y = run_gpu(gpu, X, wl.pack_along_k(np.full((K, N), c, np.uint8)), np.full((G, N), sv, np.float16),
                wl.pack_along_n(np.full((G, N), zv, np.uint8)), group)
    want = float(sv) * (c - zv) * X.astype(np.float64).sum(axis=1)
    assert err_ratio(Y, np.repeat(want[:, None], N, axis=1)) <= 1.0
    assert (Y == Y[:, :1]).all()  # every column went through the same arithmetic


def test_symmetric_int4_as_zero_point_eight(gpu):
    rng = np.random.default_rng(24)
    M, K, N, group = 2, 512, 256, 128
    signed = rng.integers(-8, 8, (K, N))
    s = rng.uniform(0.001, 0.02, (K // group, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    Wp = wl.pack_along_k((signed + 8).astype(np.uint8))
    Zp = wl.pack_along_n(np.full((K // group, N), 8, np.uint8))
    ref = orc.gemm(X, Wp, s, Zp, group)
    say("symmetric")
    assert err_ratio(run_gpu(gpu, X, Wp, s, Zp, group), ref) <= 1.0


def binding_kernels(gpu):
    _, binding = gpu
    return (binding.KERNEL_AUTO, binding.KERNEL_WAVE_SPLIT, binding.KERNEL_STRIPE, binding.KERNEL_TILE)


def test_deterministic_and_split_invariant(gpu):
    M, K, N, group = 4, 4096, 1024, 128
    X, Wp, s, Zp = wl.make(M, K, N, index=77, group=group)
    ref = orc.gemm(X, Wp, s, Zp, group)
    outs = {}
    for kernel in (binding_kernels(gpu)):
        for split in (0, 1, 4, 32):
            say("determinism kernel", kernel, "split", split)
            runs = [run_gpu(gpu, X, Wp, s, Zp, group, kernel=kernel, split=split) for _ in range(5)]
            for r in runs[1:]:
                assert np.array_equal(r.view(np.uint16), runs[0].view(np.uint16))
            outs[(kernel, split)] = runs[0]
            assert err_ratio(runs[0], ref) <= 1.0
    # different kernels and S re-associate the same sum: results agree far inside the tolerance
    base = outs[(-1, 0)].astype(np.float64)
    for key, out in outs.items():
        d = np.abs(out.astype(np.float64) - base)
        assert np.max(d / (1 + np.abs(ref))) < 2e-3, key


def test_non_default_stream_and_caller_workspace(gpu):
    torch, binding = gpu
    M, K, N, group = 2, 2048, 512, 128
    X, Wp, s, Zp = wl.make(M, K, N, index=78, group=group)
    ref = orc.gemm(X, Wp, s, Zp, group)
    dX, dW, dS, dZ = binding.to_device(X, Wp, s, Zp)
    plan = binding.query_plan(M, N, K, group, -1, 8)
    ws = torch.zeros(plan["workspace_bytes"] + 256, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + plan["workspace_bytes"]]
    ws[:] = 0xFF  # poison it (NaN bit patterns): the library must not rely on its contents
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    say("stream + caller workspace")
    with torch.cuda.stream(st):
        for _ in range(3):
            Y = binding.gemm_ws(dX, dW, dS, dZ, group, ws, split=8, stream=st)
    st.synchronize()
    assert err_ratio(Y.cpu().numpy(), ref) <= 1.0
    with pytest.raises(binding.W4A16Error) as e:
        binding.gemm_ws(dX, dW, dS, dZ, group, ws[:1024], split=8)
    assert e.value.status == binding.ERR_WORKSPACE


def test_hip_graph_replays_match_eager(gpu):
    """What bench.py times: GEMMs recorded into a HIP graph and replayed.  Every kind of finish is recorded
    (direct store, accumulator in the library's and in a caller's workspace - the latter with its clearing
    kernel -, FP32 partials with the second pass); the graph is replayed several times with eager work and
    synchronisations in between, and every replay must reproduce the eager results bit for bit."""
    torch, binding = gpu
    cases = [  # M, K, N, kernel, split
        (1, 4096, 1024, binding.KERNEL_STRIPE, 0),   # accumulator (library-owned)
        (8, 2048, 512, binding.KERNEL_TILE, 4),      # accumulator
        (3, 1024, 264, binding.KERNEL_TILE, 1),      # direct
        (130, 768, 2056, binding.KERNEL_TILE, 3),    # S M N > 640 K adds: FP32 partials + second pass
        (2, 2048, 520, binding.KERNEL_WAVE_SPLIT, 2),
    ]
    dev, eager, outs = [], [], []
    for (M, K, N, kernel, split) in cases:
        X, Wp, s, Zp = wl.make(M, K, N, index=4000 + M + K + N)
        d = binding.to_device(X, Wp, s, Zp)
        dev.append(d)
        ref = orc.gemm(X, Wp, s, Zp, 128)
        say("graph: eager", (M, K, N), kernel, split, binding.query_plan(M, N, K, 128, kernel, split))
        Y = binding.gemm_ex(*d, 128, kernel=kernel, split=split)  # also lets the library allocate what the plan needs
        torch.cuda.synchronize()
        assert err_ratio(Y.cpu().numpy(), ref) <= 1.0
        eager.append(Y.clone())
        outs.append(torch.empty_like(Y))
    # a caller's workspace for the second case, poisoned: its clearing kernel is part of the graph
    M, K, N, kernel, split = cases[1]
    plan = binding.query_plan(M, N, K, 128, kernel, split)
    assert plan["workspace_bytes"] == M * N * 8
    ws = torch.full((plan["workspace_bytes"],), 0xFF, dtype=torch.uint8, device="cuda")
    out_ws = torch.empty_like(eager[1])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    say("graph: capture")
    with torch.cuda.graph(g):
        for d, (M, K, N, kernel, split), Y in zip(dev, cases, outs):
            binding.gemm_ex(*d, 128, kernel=kernel, split=split, out=Y, stream=torch.cuda.current_stream())
        binding.gemm_ws(*dev[1], 128, ws, kernel=cases[1][3], split=cases[1][4], out=out_ws, stream=torch.cuda.current_stream())
    for rep in range(4):
        for Y in outs + [out_ws]:
            Y.fill_(float("nan"))
        ws.fill_(0xFF if rep % 2 else 0x5A)
        # eager work between the replays, on the same library state
        Ye = binding.gemm_ex(*dev[0], 128, kernel=cases[0][3], split=cases[0][4])
        torch.cuda.synchronize()
        assert torch.equal(Ye, eager[0])
        say("graph: replay", rep)
        g.replay()
        torch.cuda.synchronize()
        for Y, E in zip(outs, eager):
            assert torch.equal(Y, E), rep
        assert torch.equal(out_ws, eager[1]), rep


def test_stripe_accumulator_is_left_clean(gpu):
    """The STRIPE family adds the K slices of different workgroups into a 64-bit fixed-point accumulator
    (one atomic add each) that the last arriver clears: calls of different shapes and splits in a row, on the
    library's own accumulator and on a caller's (poisoned) one, must each be right."""
    torch, binding = gpu
    cases = [(1, 4096, 1024, 8), (4, 2048, 520, 3), (2, 4096, 264, 32), (1, 4096, 1024, 5), (3, 1024, 4104, 2)]
    data = {}
    for M, K, N, S in cases:
        if (M, K, N) not in data:
            X, Wp, s, Zp = wl.make(M, K, N, index=500 + M + K + N)
            data[(M, K, N)] = (binding.to_device(X, Wp, s, Zp), orc.gemm(X, Wp, s, Zp, wl.GROUP))
    for rep in range(3):
        for M, K, N, S in cases:
            (dX, dW, dS, dZ), ref = data[(M, K, N)]
            say("stripe clean", rep, M, K, N, S)
            Y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
            binding.gemm_ex(dX, dW, dS, dZ, wl.GROUP, kernel=binding.KERNEL_STRIPE, split=S, out=Y)
            torch.cuda.synchronize()
            assert err_ratio(Y.cpu().numpy(), ref) <= 1.0
    M, K, N, S = cases[0]
    (dX, dW, dS, dZ), ref = data[(M, K, N)]
    plan = binding.query_plan(M, N, K, wl.GROUP, binding.KERNEL_STRIPE, S)
    assert plan["workspace_bytes"] == M * N * 8
    ws = torch.full((plan["workspace_bytes"] + 256,), 0xFF, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + plan["workspace_bytes"]]
    for rep in range(2):
        Y = binding.gemm_ws(dX, dW, dS, dZ, wl.GROUP, ws, kernel=binding.KERNEL_STRIPE, split=S)
        torch.cuda.synchronize()
        assert err_ratio(Y.cpu().numpy(), ref) <= 1.0
        assert int(ws.view(torch.int64).abs().max().item()) == 0  # cleared by the last arrivers


def test_error_codes_leave_output_untouched(gpu):
    torch, binding = gpu
    M, K, N, group = 1, 256, 64, 128
    X, Wp, s, Zp = wl.make(M, K, N, index=79, group=group)
    dX, dW, dS, dZ = binding.to_device(X, Wp, s, Zp)
    Y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    p = lambda t: t.data_ptr()
    st = torch.cuda.current_stream().cuda_stream
    say("error codes")
    cases = [
        (binding.ERR_NULL, (0, p(dW), p(dS), p(dZ), group, M, N, K, p(Y), st)),
        (binding.ERR_NULL, (p(dX), p(dW), p(dS), p(dZ), group, M, N, K, 0, st)),
        (binding.ERR_SHAPE, (p(dX), p(dW), p(dS), p(dZ), group, 0, N, K, p(Y), st)),
        (binding.ERR_SHAPE, (p(dX), p(dW), p(dS), p(dZ), group, M, N + 4, K, p(Y), st)),
        (binding.ERR_SHAPE, (p(dX), p(dW), p(dS), p(dZ), group, M, N, K + 4, p(Y), st)),
        (binding.ERR_GROUP, (p(dX), p(dW), p(dS), p(dZ), 48, M, N, K, p(Y), st)),
        (binding.ERR_GROUP, (p(dX), p(dW), p(dS), p(dZ), 96, M, N, K, p(Y), st)),
        (binding.ERR_ALIGN, (p(dX) + 2, p(dW), p(dS), p(dZ), group, M, N, K, p(Y), st)),
        (binding.ERR_ALIGN, (p(dX), p(dW), p(dS), p(dZ), group, M, N, K, p(Y) + 8, st)),
    ]
    for want, args in cases:
        assert binding.raw_gemm(*args) == want
    assert binding.raw_gemm_ex(p(dX), p(dW), p(dS), p(dZ), group, M, N, K, p(Y), st, -1, 3) == binding.ERR_UNSUPPORTED
    assert binding.raw_gemm_ex(p(dX), p(dW), p(dS), p(dZ), group, M, N, K, p(Y), st, 9, 0) == binding.ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert (Y.cpu().numpy() == 7.0).all()
    assert binding.raw_gemm(p(dX), p(dW), p(dS), p(dZ), group, M, N, K, p(Y), st) == binding.OK
    torch.cuda.synchronize()
    assert err_ratio(Y.cpu().numpy(), orc.gemm(X, Wp, s, Zp, group)) <= 1.0


def test_reduce_entry_point(gpu):
    """Phase 3 alone: fixed-order fp32 sum, one RNE cast."""
    torch, binding = gpu
    rng = np.random.default_rng(25)
    S, M, N = 5, 3, 264
    P = rng.standard_normal((S, M, N)).astype(np.float32)
    acc = P[0].copy()
    for i in range(1, S):
        acc = (acc + P[i]).astype(np.float32)
    say("reduce")
    Y = binding.reduce(torch.from_numpy(P).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), acc.astype(np.float16))


def test_stream_probe_reads_and_keeps_nothing(gpu):
    """The measurement aid reads up to three arrays and must leave them and its sink as they were; argument errors come
    back as codes."""
    torch, binding = gpu
    X, Wp, s, Zp = wl.make(1, 2048, 264, index=2500)
    _, dW, dS, dZ = binding.to_device(X, Wp, s, Zp)
    before = (dW.clone(), dS.clone(), dZ.clone())
    sink = torch.full((4,), 12345, dtype=torch.int32, device="cuda")
    binding.stream_probe((dW, dS, dZ), sink)
    binding.stream_probe((dW,), sink)
    torch.cuda.synchronize()
    assert torch.equal(dW, before[0]) and torch.equal(dS, before[1]) and torch.equal(dZ, before[2])
    assert sink.tolist() == [12345] * 4
    L = binding.lib()
    assert L.w4a16_stream_probe(None, 0, None, 0, None, 0, sink.data_ptr(), None) == binding.ERR_NULL
    assert L.w4a16_stream_probe(dW.data_ptr(), 64, None, 0, None, 0, None, None) == binding.ERR_NULL
    assert L.w4a16_stream_probe(dW.data_ptr() + 4, 64, None, 0, None, 0, sink.data_ptr(), None) == binding.ERR_ALIGN


def test_dequant_entry_point_bit_exact(gpu):
    """Phase 1 alone: fp16(s (q - z)), one rounding of an exact FP32 product - bit for bit the oracle's
    dequantised weights rounded to FP16 (ragged N, several group sizes, every nibble and zero-point position)."""
    torch, binding = gpu
    for (K, N, group) in [(128, 8, 128), (256, 264, 128), (1024, 72, 64), (384, 136, 32), (2304, 1000, 128), (4096, 4104, 128)]:
        _, Wp, s, Zp = wl.make(1, K, N, index=3000 + K + N, group=group)
        want = orc.dequant(Wp, s, Zp, group).astype(np.float16)
        _, dW, dS, dZ = binding.to_device(np.zeros((1, K), np.float16), Wp, s, Zp)
        say("dequant", K, N, group)
        W16 = torch.full((K, N), float("nan"), dtype=torch.float16, device="cuda")
        binding.dequant(dW, dS, dZ, group, out=W16)
        torch.cuda.synchronize()
        got = W16.cpu().numpy()
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), (K, N, group)


# ------------------------------------------------------------ full configs ---

def _sample_cols(N, count, seed):
    rng = np.random.default_rng(seed)
    cols = set(rng.choice(N, size=count, replace=False).tolist())
    cols.update([0, 1, 7, 8, 255, 256, N - 257, N - 8, N - 1])  # tile edges
    return np.array(sorted(cols), dtype=np.int32)


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_baseline_configs_full_size(gpu, name):
    """Every configuration and every M it lists, in the plan the scheduler picks (the one bench.py times):
    every output against the oracle."""
    torch, binding = gpu
    cfg = wl.CONFIGS[name]
    Xall, Wp, s, Zp = wl.make_config(name)
    dW, dS, dZ = [t for t in binding.to_device(Xall, Wp, s, Zp)[1:]]
    for M in cfg.Ms:
        X = np.ascontiguousarray(Xall[:M])
        ref = orc.gemm(X, Wp, s, Zp, cfg.group)
        dX = torch.from_numpy(X).cuda()
        say(name, "M", M, binding.query_plan(M, cfg.N, cfg.K, cfg.group))
        Y = torch.full((M, cfg.N), float("nan"), dtype=torch.float16, device="cuda")
        binding.gemm(dX, dW, dS, dZ, cfg.group, out=Y)
        torch.cuda.synchronize()
        out = Y.cpu().numpy()
        assert not np.isnan(out).any()
        r = err_ratio(out, ref)
        print("   err/tol = %.4f" % r, flush=True)
        assert r <= 1.0, (name, M, r)
        # properties that hold for every output at any size
        assert np.isfinite(out).all()
        x = X.astype(np.float64)
        gs = x.reshape(M, cfg.K // cfg.group, cfg.group).sum(axis=2)
        es2 = (0.001 ** 2 + 0.001 * 0.02 + 0.02 ** 2) / 3
        pred = np.sqrt(es2 * (255.0 / 12.0) * ((x * x).sum(axis=1) + (gs * gs).sum(axis=1)))
        assert np.all(np.abs(out.astype(np.float64).std(axis=1) / pred - 1) < 0.1)
        # a forced different split re-associates the same sums: also against the oracle, every output
        S2 = 2 if binding.query_plan(M, cfg.N, cfg.K, cfg.group)["split"] != 2 else 4
        Y2 = binding.gemm_ex(dX, dW, dS, dZ, cfg.group, split=S2)
        torch.cuda.synchronize()
        assert err_ratio(Y2.cpu().numpy(), ref) <= 1.0, (name, M, "split", S2)


@pytest.mark.parametrize("name", sorted(wl.WIDE))
def test_wide_shapes_full_output(gpu, name):
    """K << N (up-projections): the regime in which Section 4.1 expects Split-K not to pay.  The scheduler's
    plan at M = 1 and M = 16, every output against the oracle."""
    torch, binding = gpu
    cfg = wl.WIDE[name]
    Xall, Wp, s, Zp = wl.make_config(name)
    dW, dS, dZ = [t for t in binding.to_device(Xall, Wp, s, Zp)[1:]]
    for M in (1, 16):
        X = np.ascontiguousarray(Xall[:M])
        ref = orc.gemm(X, Wp, s, Zp, cfg.group)
        dX = torch.from_numpy(X).cuda()
        say(name, "M", M, binding.query_plan(M, cfg.N, cfg.K, cfg.group))
        Y = torch.full((M, cfg.N), float("nan"), dtype=torch.float16, device="cuda")
        binding.gemm(dX, dW, dS, dZ, cfg.group, out=Y)
        torch.cuda.synchronize()
        r = err_ratio(Y.cpu().numpy(), ref)
        print("   err/tol = %.4f" % r, flush=True)
        assert r <= 1.0, (name, M, r)


# ------------------------------------------------- the method's own edge cases ---

def _families(binding, M):
    """(kernel, split) pairs that cover both families the scheduler uses and all three finishes."""
    fam = [(binding.KERNEL_TILE, 1), (binding.KERNEL_TILE, 4)]
    if M <= 16:
        fam += [(binding.KERNEL_STRIPE, 1), (binding.KERNEL_STRIPE, 4)]
    return fam


def test_tiny_and_subnormal_x(gpu):
    """The kernels divide half of the staged x by 16 in FP16 (the operand trick of the unpack): exact for
    |x| >= 2^-10, off by at most 2^-21 per element below.  X mixes normal values with values below 2^-10 and FP16
    subnormals; the result must stay within the bound that error model gives (far inside the tolerance), on both
    families, with and without a split, and through the second pass."""
    _, binding = gpu
    rng = np.random.default_rng(31)
    K, N, group = 2048, 520, 128
    _, Wp, s, Zp = wl.make(1, K, N, index=3100, group=group)
    for M in (1, 3, 9):
        mag = rng.choice([1.0, 2.0 ** -9, 2.0 ** -11, 2.0 ** -14, 2.0 ** -17, 2.0 ** -22], size=(M, K))
        X = (rng.standard_normal((M, K)) * mag).astype(np.float16)
        assert (np.abs(X[X != 0]) < 6.2e-5).any()  # FP16 subnormals are present
        ref = orc.gemm(X, Wp, s, Zp, group)
        bound = 2.0 ** -11 * np.abs(ref) + K * 2.0 ** -21 * 0.02 * 15 + 1e-4
        for kernel, split in _families(binding, M):
            say("tiny x", M, kernel, split)
            Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=kernel, split=split).astype(np.float64)
            assert err_ratio(Y, ref) <= 1.0
            assert np.all(np.abs(Y - ref) <= bound), (M, kernel, split, np.max(np.abs(Y - ref) / bound))
        binding.tune("stripe_finish", 2)
        try:
            Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=binding.KERNEL_TILE, split=4).astype(np.float64)
        finally:
            binding.tune("stripe_finish", 0)
        assert np.all(np.abs(Y - ref) <= bound)


def test_outputs_beyond_the_fp16_range(gpu):
    """Scales and X scaled up until outputs approach and pass 65504: the final cast (Section 3) gives +-inf
    where the oracle's value rounds to it, finite values within the tolerance elsewhere, whatever the finish.
    Columns whose exact value lies within one FP16 rounding step of the largest finite number may go either way."""
    _, binding = gpu
    rng = np.random.default_rng(32)
    K, N, group = 1024, 264, 128
    G = K // group
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    z = rng.integers(0, 16, (G, N), dtype=np.uint8)
    Wp, Zp = wl.pack_along_k(q), wl.pack_along_n(z)
    # column n has scale 2^(n mod 12): outputs from a few hundred up to a few hundred thousand
    s = np.repeat((2.0 ** (np.arange(N) % 12))[None, :], G, axis=0).astype(np.float16)
    for M in (1, 4, 7):
        X = (rng.standard_normal((M, K)) * 4).astype(np.float16)
        ref = orc.gemm(X, Wp, s, Zp, group)
        want = orc.to_fp16(ref)
        assert np.isinf(want).any() and np.isfinite(want).any()
        sure_inf = np.abs(ref) > 65536.0       # beyond the rounding boundary 65520 with margin
        sure_fin = np.abs(ref) < 65480.0
        finishes = [(k, sp, 0) for k, sp in _families(binding, M)] + [(binding.KERNEL_TILE, 4, 2)]
        for kernel, split, fin in finishes:
            say("overflow", M, kernel, split, fin)
            binding.tune("stripe_finish", fin)
            try:
                Y = run_gpu(gpu, X, Wp, s, Zp, group, kernel=kernel, split=split)
            finally:
                binding.tune("stripe_finish", 0)
            assert np.array_equal(np.isinf(Y)[sure_inf], np.ones(sure_inf.sum(), bool)), (M, kernel, split)
            assert np.array_equal(np.sign(Y[sure_inf]), np.sign(ref[sure_inf]))
            assert np.isfinite(Y[sure_fin]).all()
            assert err_ratio(Y[sure_fin], ref[sure_fin]) <= 1.0


def test_more_slices_than_the_accumulator_counts(gpu):
    """The accumulator counts arrivals in six bits: 63 slices still meet there, 64 and more go to the FP32
    workspace and the second pass."""
    _, binding = gpu
    M, G, N, group = 2, 300, 264, 32
    K = G * group
    X, Wp, s, Zp = wl.make(M, K, N, index=3300, group=group)
    ref = orc.gemm(X, Wp, s, Zp, group)
    for kernel in (binding.KERNEL_STRIPE, binding.KERNEL_TILE):
        for S, in_acc in ((60, True), (75, False), (G, False)):
            plan = binding.query_plan(M, N, K, group, kernel, S)
            assert plan["split"] == S and plan["workspace_bytes"] == (M * N * 8 if in_acc else S * M * N * 4), plan
            say("many slices", kernel, plan)
            assert err_ratio(run_gpu(gpu, X, Wp, s, Zp, group, kernel=kernel, split=S), ref) <= 1.0


def test_nan_in_x_gives_nan_whatever_the_finish(gpu):
    """The paper does not say what non-finite inputs give; here a NaN in X makes that row of Y NaN (as in the
    oracle) under every finish - direct store, accumulator (whose 64-bit integer sums cannot hold a NaN: a flag
    bit does) and second pass - and leaves the other rows alone."""
    _, binding = gpu
    rng = np.random.default_rng(33)
    K, N, group = 1024, 264, 128
    for M in (1, 4, 6):
        X, Wp, s, Zp = wl.make(M, K, N, index=3800 + M, group=group)
        X = X.copy()
        bad = M - 1
        X[bad, rng.integers(0, K)] = np.float16("nan")
        ref = orc.gemm(X, Wp, s, Zp, group)
        assert np.isnan(ref[bad]).all() and np.isfinite(np.delete(ref, bad, axis=0)).all()
        torch, _ = gpu
        for kernel, split in _families(binding, M):
            for fin in (0, 2):
                if split == 1 and fin:
                    continue
                say("nan", M, kernel, split, fin)
                binding.tune("stripe_finish", fin)
                try:
                    d = binding.to_device(X, Wp, s, Zp)
                    Y = binding.gemm_ex(*d, group, kernel=kernel, split=split)
                    torch.cuda.synchronize()
                finally:
                    binding.tune("stripe_finish", 0)
                Y = Y.cpu().numpy()
                assert np.isnan(Y[bad]).all(), (M, kernel, split, fin)
                if M > 1:
                    good = np.delete(np.arange(M), bad)
                    assert err_ratio(Y[good], ref[good]) <= 1.0


def test_per_channel_quantisation(gpu):
    """group = K: one scale and one zero point per output channel (the coarsest granularity Eq. 2 allows)."""
    _, binding = gpu
    for (M, K, N) in [(1, 1024, 264), (4, 2048, 520), (9, 512, 72), (40, 1024, 136)]:
        X, Wp, s, Zp = wl.make(M, K, N, index=3400 + M, group=K)
        assert s.shape == (1, N)
        ref = orc.gemm(X, Wp, s, Zp, K)
        for kernel in [binding.KERNEL_AUTO, binding.KERNEL_TILE] + ([binding.KERNEL_STRIPE] if M <= 16 else []):
            say("per channel", (M, K, N), kernel)
            assert err_ratio(run_gpu(gpu, X, Wp, s, Zp, K, kernel=kernel), ref) <= 1.0


# ------------------------------------------------------------- the boundary ---

def test_registered_workspace(gpu):
    """w4a16_set_workspace: the caller's split buffers replace the library's for every later call on the device."""
    torch, binding = gpu
    ws = torch.full((1 << 20,), 0xFF, dtype=torch.uint8, device="cuda")
    assert ws.data_ptr() % 256 == 0
    binding.set_workspace(ws)
    try:
        for (M, K, N, kernel, split) in [(1, 4096, 1024, binding.KERNEL_STRIPE, 0), (8, 2048, 520, binding.KERNEL_TILE, 4),
                                         (2, 2048, 520, binding.KERNEL_WAVE_SPLIT, 2), (3, 1024, 264, binding.KERNEL_TILE, 1)]:
            X, Wp, s, Zp = wl.make(M, K, N, index=3500 + M + K + N)
            ref = orc.gemm(X, Wp, s, Zp, wl.GROUP)
            say("registered workspace", (M, K, N), kernel, split)
            ws.fill_(0xFF)
            for _ in range(2):
                assert err_ratio(run_gpu(gpu, X, Wp, s, Zp, wl.GROUP, kernel=kernel, split=split), ref) <= 1.0
        # too small for this plan: 3 * 130 * 2056 * 4 bytes of partials
        X, Wp, s, Zp = wl.make(130, 768, 2056, index=3599)
        d = binding.to_device(X, Wp, s, Zp)
        with pytest.raises(binding.W4A16Error) as e:
            binding.gemm_ex(*d, wl.GROUP, kernel=binding.KERNEL_TILE, split=3)
        assert e.value.status == binding.ERR_WORKSPACE
    finally:
        binding.set_workspace(None)
    with pytest.raises(binding.W4A16Error) as e:
        binding.set_workspace(ws[8:])
    assert e.value.status == binding.ERR_ALIGN


def test_capture_never_allocates(gpu):
    """Under stream capture the library must not call hipMalloc: a plan whose split buffers it does not hold yet
    answers W4A16_ERR_WORKSPACE (and the capture stays usable), one that brings its buffers is recorded."""
    torch, binding = gpu
    binding.shutdown()  # the library holds no split buffers now
    M, K, N = 2, 2048, 520
    X, Wp, s, Zp = wl.make(M, K, N, index=3600)
    ref = orc.gemm(X, Wp, s, Zp, wl.GROUP)
    d = binding.to_device(X, Wp, s, Zp)
    plan = binding.query_plan(M, N, K, wl.GROUP, binding.KERNEL_TILE, 4)
    ws = torch.empty(plan["workspace_bytes"], dtype=torch.uint8, device="cuda")
    Y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()
    say("capture without buffers")
    g = torch.cuda.CUDAGraph()
    status = []
    with torch.cuda.graph(g):
        cs = torch.cuda.current_stream()
        for kernel, split in ((binding.KERNEL_TILE, 4), (binding.KERNEL_WAVE_SPLIT, 2)):  # accumulator; FP32 partials
            try:
                binding.gemm_ex(*d, wl.GROUP, kernel=kernel, split=split, out=Y, stream=cs)
                status.append(binding.OK)
            except binding.W4A16Error as e:
                status.append(e.status)
        binding.gemm_ws(*d, wl.GROUP, ws, kernel=binding.KERNEL_TILE, split=4, out=Y, stream=cs)
    assert status == [binding.ERR_WORKSPACE, binding.ERR_WORKSPACE]
    for _ in range(2):
        Y.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert err_ratio(Y.cpu().numpy(), ref) <= 1.0
    # outside a capture the same calls allocate and work
    assert err_ratio(binding.gemm_ex(*d, wl.GROUP, kernel=binding.KERNEL_TILE, split=4).cpu().numpy(), ref) <= 1.0


def test_plan_logging(gpu, capfd):
    """The "log" knob (W4A16_LOG=1 in the environment): one line per call on stderr, nothing otherwise."""
    _, binding = gpu
    X, Wp, s, Zp = wl.make(1, 256, 64, index=3700)
    run_gpu(gpu, X, Wp, s, Zp, wl.GROUP)
    assert "w4a16:" not in capfd.readouterr().err
    binding.tune("log", 1)
    try:
        run_gpu(gpu, X, Wp, s, Zp, wl.GROUP)
    finally:
        binding.tune("log", 0)
    err = capfd.readouterr().err
    assert "w4a16: gemm_ex M=1 N=64 K=256 group=128" in err and "S=" in err


@pytest.mark.parametrize("name", sorted(wl.FIG2))
def test_fig2_shapes_split_k_and_data_parallel(gpu, name):
    """The (N, K) pairs of the paper's Split-K against data-parallel comparison
    (Section 4.1, Fig. 2), as bench.py --fig2 times them: the scheduler's plan
    and the S = 1 plan of the TILE family, on all rows of sampled columns."""
    torch, binding = gpu
    cfg = wl.FIG2[name]
    Xall, Wp, s, Zp = wl.make_config(name)
    dW, dS, dZ = [t for t in binding.to_device(Xall, Wp, s, Zp)[1:]]
    for M in (1, 4, 16, 64):
        X = np.ascontiguousarray(Xall[:M])
        cols = _sample_cols(cfg.N, 96, seed=100 + M)
        ref = orc.gemm(X, Wp, s, Zp, cfg.group, cols=cols)
        dX = torch.from_numpy(X).cuda()
        for kernel, split in ((binding.KERNEL_AUTO, 0), (binding.KERNEL_TILE, 1)):
            say(name, "M", M, binding.query_plan(M, cfg.N, cfg.K, cfg.group, kernel, split))
            Y = torch.full((M, cfg.N), float("nan"), dtype=torch.float16, device="cuda")
            binding.gemm_ex(dX, dW, dS, dZ, cfg.group, kernel=kernel, split=split, out=Y)
            torch.cuda.synchronize()
            out = Y.cpu().numpy()
            assert np.isfinite(out).all()
            r = err_ratio(out[:, cols], ref)
            print("   err/tol = %.4f" % r, flush=True)
            assert r <= 1.0, (name, M, kernel, split, r)


# ------------------------------------------------------------- perf smoke ---

def test_headline_stays_under_its_time_ceiling(gpu):
    """M = 1, K = 28672, N = 8192 on cold weights, as bench.py times it (HIP-graph replays over rotating weight
    copies).  The build's target is 21.8 us (70 % of 8 TB/s); most boxes run it in 21.3 to 21.7 us, single ones were
    seen at 22.0 to 22.8 us and one ran everything 8 % slower, so the ceiling that must never be crossed is set at 26 us
    (on the fastest replay): a regression of the kernel or of the scheduler's plan fails loudly."""
    torch, binding = gpu
    import bench
    r, Y, _ = bench.time_gemm(torch, binding, wl, "c4", 1, 120, 24, replays=5)
    print("   c4 M=1: %.2f us per GEMM (fastest replay %.2f), %.1f %% of 8 TB/s" % (r["us_per_gemm"], r["us_per_gemm_min"], 100 * r["hbm_frac"]), flush=True)
    assert r["plan"]["kernel"] == binding.KERNEL_STRIPE and r["plan"]["workspace_bytes"] == 8192 * 8
    assert r["us_per_gemm_min"] < 26.0, r
