"""GPU parity: the HIP library against the CPU oracle, bit for bit, through the C ABI.

Every comparison is on the whole flat C buffer, leading-dimension padding
included, so a store outside the m x n matrix fails too.
"""
import os

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

VARIANTS = ["auto", "simple", "tile256", "tile128", "tile64", "tile64x256", "tile256x64",
            "dma256", "dma128", "dma64", "dma64x256", "dma256x64", "dma64x128", "dma128x64",
            "tile64x128", "tile128x64"]


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_11728_amd as M
    M.load_library()                       # raises if the HIP library is not built
    return M


class VariantEnv:
    """Pins the kernel variant (and optionally the split-k factor) for the calls inside."""

    def __init__(self, variant, splits=None):
        import paper_2506_11728_amd as M
        self.ctx = M.tuning(MIPGEMM_VARIANT=None if variant == "auto" else variant,
                            MIPGEMM_SPLITK=splits)

    def __enter__(self):
        self.ctx.__enter__()

    def __exit__(self, *a):
        self.ctx.__exit__(*a)


def gpu_gemm(M, case, A, B, C, variant="auto", splits=None):
    """Run the library on host buffers A, B, C (flat numpy); returns the flat C it produced."""
    import torch
    dA = torch.from_numpy(A.view(np.uint8)).cuda()
    dB = torch.from_numpy(B.view(np.uint8)).cuda()
    dC = torch.from_numpy(C).cuda()
    fn = getattr(M, "mipgemm_" + case.entry)
    with VariantEnv(variant, splits):
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
           dC, case.ldc, case.orderC, case.mode)
    torch.cuda.synchronize()
    return dC.cpu().numpy()


_expected = {}


def oracle_result(oracle, case, ops):
    if case.name not in _expected:
        C = ops.C.copy()
        oracle.gemm(case.a_unsigned, case.b_unsigned, case.m, case.n, case.k, ops.A, case.lda,
                    case.orderA, ops.B, case.ldb, case.orderB, C, case.ldc, case.orderC, case.mode)
        _expected[case.name] = C
    return _expected[case.name]


_ran = {}          # forced variant -> names of the kernels that served it, over the session


def kernel_that_runs(M, case, variant):
    """Name of the kernel the library takes for this case under this forced variant: a variant
    that cannot serve a case falls back (a direct-to-LDS variant on unaligned operands to the
    register-staged kernel of the same tile shape, the kernel for large problems and the
    skinny-m kernel to whatever the dispatcher picks), and a test that believes it covers a
    kernel has to know which one actually ran."""
    with VariantEnv(variant):
        name = M.mipgemm_variant_name_for_mode(case.m, case.n, case.k, case.lda, case.orderA, case.ldb,
                                               case.orderB, case.ldc, case.orderC, case.a_unsigned,
                                               case.b_unsigned, case.pad % 16 == 0, case.mode)
    if variant == "simple":
        assert name == "simple"
    elif variant.startswith("tile"):
        assert name == "mfma_" + variant
    elif variant == "dma128k128split":
        assert name == "mfma_dma128_k128_split" or not case.m * case.n * case.k
    elif variant == "dma256k128ragged":
        assert name == "mfma_dma256_k128_ragged" or not case.m * case.n * case.k
    elif variant.startswith("dma") and not variant.endswith("k128"):
        assert name in ("mfma_" + variant, "mfma_tile" + variant[3:])
    _ran.setdefault(variant, set()).add(name)
    return name


def check_case(M, oracle, case, variant, splits=None):
    if case.m and case.n and case.k:
        print("case", case.name, "variant", variant, "splits", splits, "kernel",
              kernel_that_runs(M, case, variant), flush=True)
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    got = gpu_gemm(M, case, ops.A, ops.B, ops.C, variant, splits)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        pytest.fail("%s [%s]: %d of %d words differ, first at %d: got %d want %d" % (
            case.name, variant, bad.size, got.size, bad[0], got[bad[0]], want[bad[0]]))


def _ops_count(c):
    return c.m * c.n * c.k


SMALL = [c for c in W.all_cases() if _ops_count(c) <= 2.5e9]
LARGE = [c for c in W.all_cases() if 2.5e9 < _ops_count(c) <= 7e10]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("case", SMALL, ids=lambda c: c.name)
def test_small_cases_every_variant(gpu, oracle, case, variant):
    check_case(gpu, oracle, case, variant)


@pytest.mark.parametrize("variant", ["dma256k128", "dma128k128"])
@pytest.mark.parametrize("case", SMALL, ids=lambda c: c.name)
def test_small_cases_deep_k_kernel(gpu, oracle, case, variant):
    """The kernel for large aligned problems in both its tile shapes, forced on every small case
    (those it cannot take fall back to whatever the dispatcher picks)."""
    check_case(gpu, oracle, case, variant)


@pytest.mark.parametrize("variant", ["auto", "tile256", "dma256", "dma256k128", "dma128k128"])
@pytest.mark.parametrize("case", LARGE, ids=lambda c: c.name)
def test_large_cases(gpu, oracle, case, variant):
    check_case(gpu, oracle, case, variant)


def test_every_forced_variant_ran_its_own_kernel_on_some_case():
    """After the two sweeps above: each direct-to-LDS and each staged variant was served by the
    kernel of its own name on at least one case (not only by its fall-back)."""
    assert _ran, "runs after test_small_cases_every_variant and test_large_cases"
    for variant in VARIANTS:
        if variant == "auto":
            continue
        own = "simple" if variant == "simple" else "mfma_" + variant
        assert own in _ran.get(variant, set()), (variant, _ran.get(variant))
    assert "mfma_dma256_k128" in _ran.get("dma256k128", set())
    assert "mfma_dma128_k128" in _ran.get("dma128k128", set())
    assert "mfma_dma256_k128" in _ran.get("auto", set())      # the 4096^3 cases as dispatched


SPLIT_CASES = [c for c in W.all_cases() if c.k >= 513 and _ops_count(c) <= 2.5e9]


@pytest.mark.parametrize("variant,splits", [("tile64", 3), ("tile64x256", 7), ("tile256x64", 2),
                                            ("tile128", 5), ("tile64", 1000), ("dma64", 3),
                                            ("dma64x256", 7), ("dma256x64", 2), ("dma128", 5), ("dma64x128", 3), ("tile128x64", 2),
                                            ("dma256", 2), ("dma64", 1000)])
@pytest.mark.parametrize("case", SPLIT_CASES, ids=lambda c: c.name)
def test_split_k_is_exact(gpu, oracle, case, variant, splits):
    """k cut into ranges added into C with integer atomics: same bits as one pass."""
    check_case(gpu, oracle, case, variant, splits)


@pytest.mark.parametrize("variant,splits", [("dma64", 2), ("dma64", 16), ("dma128", 4), ("dma64x256", 8),
                                            ("tile64", 5), ("tile128x64", 3), ("dma64", 64)])
def test_split_k_overwrite_on_garbage(gpu, oracle, variant, splits):
    """An overwriting call with split k must not depend on what C held: many tiles and ragged
    edges, C full of a different garbage before each of four calls in a row on the same
    buffers, padded ld (the padding keeps its sentinels)."""
    import torch
    case = W.Case("turns_%s_%d" % (variant, splits), 8, 3, 200, 328, 4096, pad=16, seed=41)
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dC = torch.from_numpy(ops.C).cuda()
    inside = np.zeros((case.m, case.ldc), dtype=bool)
    inside[:, :case.n] = True
    inside = torch.from_numpy(inside.reshape(-1)).cuda()
    with VariantEnv(variant, splits):
        for call in range(4):
            garbage = torch.full_like(dC, 0x01010101 * (call + 3))
            dC.copy_(torch.where(inside, garbage, torch.from_numpy(ops.C).cuda()))
            gpu.mipgemm_s8s8s32(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb,
                                case.orderB, dC, case.ldc, case.orderC, W.OVERWRITE)
            torch.cuda.synchronize()
            assert np.array_equal(dC.cpu().numpy(), want), "call %d" % call


@pytest.mark.parametrize("case", W.config3(), ids=lambda c: c.name)
def test_conv_cases_through_swapped_u8s8(gpu, oracle, case):
    """The same buffers through mipgemm_u8s8s32 with A and B swapped (C^T = B^T A^T)."""
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    sw = W.swapped(case)
    assert sw.entry == "u8s8s32"
    got = gpu_gemm(gpu, sw, ops.B, ops.A, ops.C)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------------------
# the headline size: every element against the oracle, closed form, Freivalds
# ---------------------------------------------------------------------------

def test_headline_8192_every_element_and_freivalds(gpu, oracle):
    """m = n = k = 8192, as dispatched (the kernel the benchmark times): all 2^26 elements of C
    against the oracle's (about 25 s of host time), then three exact integer identities."""
    case = W.headline_case()
    name = gpu.mipgemm_variant_name_for_mode(case.m, case.n, case.k, case.lda, case.orderA, case.ldb,
                                             case.orderB, case.ldc, case.orderC, False, False, True,
                                             case.mode)
    assert name == "mfma_dma256_k128"
    ops = W.materialize(case)
    got = gpu_gemm(gpu, case, ops.A, ops.B, ops.C)
    print("headline: oracle on all %d rows" % case.m, flush=True)
    want = oracle_result(oracle, case, ops)
    assert np.array_equal(got, want)
    got = got.reshape(case.m, case.ldc)
    rng = np.random.default_rng(99)
    # and through an exact integer identity that involves neither the oracle nor the GPU path: C x == A (B x)
    for _ in range(3):
        x = rng.integers(-2, 2, size=case.n, endpoint=True).astype(np.int64)
        lhs = got.astype(np.int64) @ x
        rhs = ops.A2d.astype(np.int64) @ (ops.B2d.astype(np.int64) @ x)
        assert np.array_equal(lhs, rhs)
    _expected.pop(case.name, None)   # 256 MB: not kept for the rest of the session


def test_headline_8192_extreme_values(gpu):
    case = next(c for c in W.config2() if c.name == "c2_8192_min")
    ops = W.materialize(case)
    got = gpu_gemm(gpu, case, ops.A, ops.B, ops.C)
    assert (got == 16384 * 8192).all()      # (-128) * (-128) * k = 2^27


# ---------------------------------------------------------------------------
# degenerate sizes, wraparound, error handling on the device
# ---------------------------------------------------------------------------

def test_wraparound_on_device(gpu, oracle):
    k = 131072 + 64 + 5
    case = W.Case("wrap", 9, 0, 40, 33, k, a_dist=("const", -128), b_dist=("const", -128))
    check_case(gpu, oracle, case, "auto")
    check_case(gpu, oracle, case, "tile128")
    # k a multiple of 128: the direct-to-LDS kernels, with and without split k
    case = W.Case("wrap_dma", 9, 1, 64, 48, 131072 + 128, a_dist=("const", -128),
                  b_dist=("const", -128))
    check_case(gpu, oracle, case, "dma64")
    check_case(gpu, oracle, case, "dma64", splits=1)
    case = W.Case("wrap_deepk", 9, 2, 256, 256, 131072 + 128, a_dist=("const", -128),
                  b_dist=("const", -128))
    check_case(gpu, oracle, case, "dma256k128")


def test_empty_problems(gpu):
    import torch
    C0 = np.arange(12, dtype=np.int32) + 5
    dA = torch.zeros(64, dtype=torch.uint8, device="cuda")
    dC = torch.from_numpy(C0).cuda()
    R, OVW, ACC = W.ROW_MAJOR, W.OVERWRITE, W.ACCUMULATE
    gpu.mipgemm_s8s8s32(0, 4, 5, dA, 5, R, dA, 4, R, dC, 4, R, OVW)
    gpu.mipgemm_s8s8s32(3, 0, 5, dA, 5, R, dA, 1, R, dC, 1, R, OVW)
    gpu.mipgemm_s8s8s32(3, 3, 0, dA, 1, R, dA, 3, R, dC, 4, R, ACC)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C0)
    gpu.mipgemm_s8s8s32(3, 3, 0, dA, 1, R, dA, 3, R, dC, 4, R, OVW)      # k == 0: C := 0
    torch.cuda.synchronize()
    want = C0.reshape(3, 4).copy()
    want[:, :3] = 0
    assert np.array_equal(dC.cpu().numpy().reshape(3, 4), want)
    # column-major C, k == 0
    dC = torch.from_numpy(C0).cuda()
    gpu.mipgemm_s8s8s32(3, 3, 0, dA, 1, R, dA, 3, R, dC, 4, W.COL_MAJOR, OVW)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy().reshape(3, 4), want)


def test_errors_touch_nothing(gpu):
    import torch
    C0 = np.full(16, 123, dtype=np.int32)
    dA = torch.zeros(64, dtype=torch.uint8, device="cuda")
    dC = torch.from_numpy(C0).cuda()
    R = W.ROW_MAJOR
    assert gpu.mipgemm_s8s8s32(4, 4, 4, dA, 3, R, dA, 4, R, dC, 4, R, 0, check=False) == -5
    assert gpu.mipgemm_s8s8s32(4, 4, 4, dA, 4, R, dA, 4, R, dC, 4, R, 7, check=False) == -13
    with pytest.raises(gpu.MipGemmError):
        gpu.mipgemm_u8s8s32(4, 4, 4, dA, 4, R, dA, 4, 3, dC, 4, R, 0)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C0)


def test_runs_on_a_side_stream(gpu, oracle):
    import torch
    case = W.config1()[0]
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    s = torch.cuda.Stream()
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dC = torch.from_numpy(ops.C).cuda()
    torch.cuda.synchronize()
    gpu.mipgemm_s8s8s32(case.m, case.n, case.k, dA, case.lda, 0, dB, case.ldb, 0, dC, case.ldc, 0,
                        case.mode, stream=s)
    s.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)


# ---------------------------------------------------------------------------
# seeded sweep over shapes, orders, leading dimensions, signedness and modes
# ---------------------------------------------------------------------------

def _sweep_cases():
    rng = np.random.default_rng(2024)
    cases = []
    for idx in range(160):
        aligned = idx % 2 == 0            # half the cases can take the direct-to-LDS kernels
        if aligned:
            k = int(rng.integers(1, 9)) * 64
            m = int(rng.integers(1, 420))
            n = int(rng.integers(1, 420))
            pad = int(rng.choice([0, 16, 32, 48]))
        else:
            k = int(rng.integers(1, 400))
            m = int(rng.integers(1, 300))
            n = int(rng.integers(1, 300))
            pad = int(rng.choice([0, 1, 3, 17]))
        oa, ob, oc = (int(x) for x in rng.integers(0, 2, size=3))
        if aligned:
            # leading dimensions become multiples of 16: round the contiguous extents up
            def up16(x):
                return (x + 15) // 16 * 16
            if oa == W.COL_MAJOR:
                m = up16(m)
            if ob == W.ROW_MAJOR:
                n = up16(n)
            if oa == W.ROW_MAJOR:
                pass                       # lda = k + pad, already a multiple of 16
            if ob == W.COL_MAJOR:
                pass                       # ldb = k + pad
        uns = int(rng.integers(0, 3))
        mode = int(rng.integers(0, 2))
        cases.append(W.Case(
            "sweep%03d_%dx%dx%d_%d%d%d_p%d_u%d_m%d" % (idx, m, n, k, oa, ob, oc, pad, uns, mode),
            8, idx, m, n, k, a_unsigned=uns == 1, b_unsigned=uns == 2,
            orderA=oa, orderB=ob, orderC=oc, pad=pad, mode=mode,
            a_dist=("uniform", 0, 255) if uns == 1 else ("uniform", -128, 127),
            b_dist=("uniform", 0, 255) if uns == 2 else ("uniform", -128, 127),
            c_dist=("uniform", -1000, 1000), seed=7))
    return cases


@pytest.mark.parametrize("case", _sweep_cases(), ids=lambda c: c.name)
def test_seeded_sweep(gpu, oracle, case):
    check_case(gpu, oracle, case, "auto")
    if case.k >= 128:
        check_case(gpu, oracle, case, "auto", splits=2)


def test_mfma_ceiling_probe(gpu):
    zero = gpu.mipgemm_mfma_ceiling(0, 2000)
    rand = gpu.mipgemm_mfma_ceiling(1, 2000)
    assert 500 < rand <= zero * 1.05 and zero < 5600      # TOPS, below the datasheet peak + margin
    with pytest.raises(gpu.MipGemmError):
        gpu.mipgemm_mfma_ceiling(2, 2000)
    # the clocked form: more patterns, and a shader clock between idle and the maximum
    for pattern in range(6):
        tops, mhz = gpu.mipgemm_mfma_ceiling_clocked(pattern, 3000)
        assert 500 < tops < 5600 and 300 < mhz < 2600, (pattern, tops, mhz)
        # the rate follows from the clock: 4 SIMDs x 2048 operations per clock and compute unit
        assert tops <= 256 * 4 * 2048 * mhz * 1e6 / 1e12 * 1.03
    with pytest.raises(gpu.MipGemmError):
        gpu.mipgemm_mfma_ceiling_clocked(6, 2000)


def test_clocked_entry_point_matches_the_plain_one(gpu, oracle):
    """mipgemm_s8s8s32_clocked: same bits as the oracle, counters filled for every tile."""
    import torch
    case = W.Case("clocked_512x768x1024", 8, 0, 512, 768, 1024, seed=31)
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dC = torch.from_numpy(ops.C).cuda()
    clocks = torch.zeros(2 * 8, dtype=torch.int64, device="cuda")     # 6 tiles, rounded up to 8
    gpu.mipgemm_s8s8s32_clocked(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb,
                                case.orderB, dC, case.ldc, case.orderC, case.mode, clocks, 16 * 8)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)
    c = clocks.cpu().numpy().reshape(8, 2)
    assert (c[:6] > 0).all() and (c[6:] == 0).all()
    mhz = c[:6, 0].sum() / c[:6, 1].sum() * 100.0
    assert 300 < mhz < 2600
    # too little room for the counters, a shape the kernel does not take: nothing is launched
    assert gpu.mipgemm_s8s8s32_clocked(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb,
                                       case.orderB, dC, case.ldc, case.orderC, case.mode, clocks, 15 * 8,
                                       check=False) == -16
    assert gpu.mipgemm_s8s8s32_clocked(100, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb,
                                       case.orderB, dC, case.ldc, case.orderC, case.mode, clocks, 16 * 8,
                                       check=False) == -1


def _deep_k_cases():
    out = []
    idx = 0
    for (m, n, k) in ((512, 768, 2048), (256, 256, 128), (768, 512, 384)):
        for uns in (0, 1, 2):
            for mode in (W.OVERWRITE, W.ACCUMULATE):
                for (oa, ob, oc) in ((0, 0, 0), (0, 1, 0), (1, 0, 1), (1, 1, 0)):
                    out.append(W.Case(
                        "deepk_%dx%dx%d_u%d_m%d_%d%d%d" % (m, n, k, uns, mode, oa, ob, oc), 8, idx,
                        m, n, k, a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob,
                        orderC=oc, pad=16 * (idx % 3), mode=mode,
                        a_dist=("uniform", 0, 255) if uns == 1 else ("uniform", -128, 127),
                        b_dist=("uniform", 0, 255) if uns == 2 else ("uniform", -128, 127),
                        c_dist=("uniform", -1000, 1000), seed=9))
                    idx += 1
    return out


@pytest.mark.parametrize("case", _deep_k_cases(), ids=lambda c: c.name)
def test_deep_k_kernel_unsigned_and_accumulate(gpu, oracle, case):
    """The 256 x 256, 128-deep kernel pinned on shapes it is eligible for."""
    name = gpu.mipgemm_variant_name
    with VariantEnv("dma256k128"):
        assert name(case.m, case.n, case.k, case.lda, case.orderA, case.ldb, case.orderB, case.ldc,
                    case.orderC, case.a_unsigned, case.b_unsigned, True) == "mfma_dma256_k128"
    check_case(gpu, oracle, case, "dma256k128")


def _k128_split_cases():
    out = []
    idx = 0
    shapes = ((208, 336, 640), (128, 128, 128), (400, 144, 1152), (96, 1568, 1024), (200, 330, 512))
    for (m, n, k) in shapes:
        for uns in (0, 1, 2):
            for mode in (W.OVERWRITE, W.ACCUMULATE):
                # extents that are no multiples of 16 need both operands k-contiguous
                orders = ((0, 1, 0), (0, 1, 1)) if m % 16 or n % 16 else ((0, 0, 0), (0, 1, 0), (1, 0, 1), (1, 1, 0))
                for (oa, ob, oc) in orders:
                    out.append((W.Case(
                        "k128split_%dx%dx%d_u%d_m%d_%d%d%d" % (m, n, k, uns, mode, oa, ob, oc), 8, idx,
                        m, n, k, a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob,
                        orderC=oc, pad=16 * (idx % 3), mode=mode,
                        a_dist=("uniform", 0, 255) if uns == 1 else ("uniform", -128, 127),
                        b_dist=("uniform", 0, 255) if uns == 2 else ("uniform", -128, 127),
                        c_dist=("uniform", -1000, 1000), seed=10), (1, 2, 3, 5, 1000)[idx % 5]))
                    idx += 1
    return out


@pytest.mark.parametrize("case,splits", _k128_split_cases(), ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_deep_k_kernel_general_form_with_k_ranges(gpu, oracle, case, splits):
    """The 128 x 128 form of the kernel with 128-deep blocks on ragged, unpadded operands, k in
    one to many ranges (1000: one block each) that meet in C through atomics; an overwriting
    call twice over different garbage."""
    import torch
    name = gpu.mipgemm_variant_name
    with VariantEnv("dma128k128split", splits):
        assert name(case.m, case.n, case.k, case.lda, case.orderA, case.ldb, case.orderB, case.ldc,
                    case.orderC, case.a_unsigned, case.b_unsigned, True) == "mfma_dma128_k128_split"
    check_case(gpu, oracle, case, "dma128k128split", splits)
    if case.mode == W.OVERWRITE:
        ops = W.materialize(case)
        want = oracle_result(oracle, case, ops)
        rows, cols = (case.n, case.m) if case.orderC else (case.m, case.n)
        inside = np.zeros((rows, case.ldc), dtype=bool)
        inside[:, :cols] = True
        C = np.where(inside.reshape(-1), np.int32(0x5a5a5a5a), ops.C[:rows * case.ldc])
        C = np.concatenate([C, ops.C[rows * case.ldc:]]).astype(np.int32)
        got = gpu_gemm(gpu, case, ops.A, ops.B, C, "dma128k128split", splits)
        assert np.array_equal(got, want)


def _k128_ragged_cases():
    out = []
    idx = 0
    for (m, n, k) in ((400, 528, 384), (256, 256, 128), (272, 1040, 256), (1008, 304, 640), (300, 530, 256)):
        for uns in (0, 1, 2):
            for mode in (W.OVERWRITE, W.ACCUMULATE):
                orders = ((0, 1, 0), (0, 1, 1)) if m % 16 or n % 16 else ((0, 0, 0), (0, 1, 0), (1, 0, 1), (1, 1, 0))
                for (oa, ob, oc) in orders:
                    out.append(W.Case(
                        "k128ragged_%dx%dx%d_u%d_m%d_%d%d%d" % (m, n, k, uns, mode, oa, ob, oc), 8, idx,
                        m, n, k, a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob,
                        orderC=oc, pad=16 * (idx % 3), mode=mode,
                        a_dist=("uniform", 0, 255) if uns == 1 else ("uniform", -128, 127),
                        b_dist=("uniform", 0, 255) if uns == 2 else ("uniform", -128, 127),
                        c_dist=("uniform", -1000, 1000), seed=11))
                    idx += 1
    return out


@pytest.mark.parametrize("case", _k128_ragged_cases(), ids=lambda c: c.name)
def test_deep_k_kernel_general_form_on_large_tiles(gpu, oracle, case):
    """The 256 x 256 form of the kernel with 128-deep blocks on ragged, unpadded operands: loads
    that would leave an operand are redirected inside it, the write-back stops at the edge."""
    name = gpu.mipgemm_variant_name
    with VariantEnv("dma256k128ragged"):
        assert name(case.m, case.n, case.k, case.lda, case.orderA, case.ldb, case.orderB, case.ldc,
                    case.orderC, case.a_unsigned, case.b_unsigned, True) == "mfma_dma256_k128_ragged"
    check_case(gpu, oracle, case, "dma256k128ragged")


@pytest.mark.parametrize("spec", [(272, 1008, 8192, 0, 0, W.OVERWRITE, 1), (256, 1024, 6144, 0, 1, W.ACCUMULATE, 0),
                                  (640, 400, 8320, 1, 0, W.OVERWRITE, 2), (384, 1536, 16384, 0, 0, W.ACCUMULATE, 0)],
                         ids=lambda s: "x".join(map(str, s)))
def test_deep_k_over_few_tiles_as_dispatched(gpu, oracle, spec):
    """A very long k over few tiles of C: the dispatcher itself takes the general 128 x 128 form
    with k ranges (the name is asserted), ragged edges and an unsigned operand included."""
    m, n, k, oa, ob, mode, uns = spec
    case = W.Case("deepfew_%dx%dx%d_%d%d_m%d_u%d" % (m, n, k, oa, ob, mode, uns), 8, 0, m, n, k,
                  a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob, pad=16, mode=mode,
                  a_dist=("uniform", 0, 255) if uns == 1 else ("uniform", -128, 127),
                  b_dist=("uniform", 0, 255) if uns == 2 else ("uniform", -128, 127),
                  c_dist=("uniform", -1000, 1000), seed=12)
    assert gpu.mipgemm_variant_name_for_mode(m, n, k, case.lda, oa, case.ldb, ob, case.ldc, 0, uns == 1,
                                             uns == 2, True, mode) == "mfma_dma128_k128_split"
    check_case(gpu, oracle, case, "auto")


@pytest.mark.parametrize("spec", [
    (3600, 3632, 2048, 0, 0, W.OVERWRITE, 0, "mfma_dma256_k128_ragged"),
    (3600, 3600, 2048, 0, 1, W.ACCUMULATE, 0, "mfma_dma256_k128_ragged"),
    (3600, 3600, 2176, 1, 0, W.OVERWRITE, 2, "mfma_dma256_k128_ragged"),
    (3600, 3600, 2048, 0, 0, W.ACCUMULATE, 1, "mfma_dma256_k128_ragged"),
    (3600, 3600, 1024, 0, 0, W.ACCUMULATE, 2, "mfma_dma128_k128_split"),
    (1000, 3072, 768, 0, 0, W.OVERWRITE, 1, "mfma_dma128_k128_split"),
    (1520, 1520, 2048, 0, 0, W.ACCUMULATE, 2, "mfma_dma128_k128_split")], ids=lambda s: "x".join(map(str, s)))
def test_aligned_ragged_shapes_as_dispatched(gpu, oracle, spec):
    """Aligned operands whose m or n is no multiple of the tile: the dispatcher itself takes the
    general forms of the kernel with 128-deep blocks (the name is asserted)."""
    m, n, k, oa, ob, mode, uns, want = spec
    case = W.Case("ragged_%dx%dx%d_%d%d_m%d_u%d" % (m, n, k, oa, ob, mode, uns), 8, 0, m, n, k,
                  a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob, pad=16, mode=mode,
                  a_dist=("uniform", 0, 255) if uns == 1 else ("uniform", -128, 127),
                  b_dist=("uniform", 0, 255) if uns == 2 else ("uniform", -128, 127),
                  c_dist=("uniform", -1000, 1000), seed=13)
    assert gpu.mipgemm_variant_name_for_mode(m, n, k, case.lda, oa, case.ldb, ob, case.ldc, 0, uns == 1,
                                             uns == 2, True, mode) == want
    check_case(gpu, oracle, case, "auto")


# ---------------------------------------------------------------------------
# the skinny-m kernel: one workgroup per 16-, 32- or 64-column slab of B
# ---------------------------------------------------------------------------

def _slab_cases():
    rng = np.random.default_rng(77)
    shapes = [(1, 4096, 4096), (16, 4096, 4096), (64, 4096, 4096), (1, 11008, 4096),
              (16, 4096, 11008), (64, 11008, 4096), (64, 3136, 576), (1, 16, 64), (64, 32, 64),
              (3, 48, 128), (17, 80, 192), (33, 176, 1088), (48, 32, 2048), (5, 4112, 320),
              (1, 64, 64), (9, 192, 4160), (40, 448, 704), (64, 128, 1024)]
    for _ in range(26):
        shapes.append((int(rng.integers(1, 65)), 16 * int(rng.integers(1, 40)),
                       64 * int(rng.integers(1, 24))))
    out = []
    for idx, (m, n, k) in enumerate(shapes):
        uns = idx % 3
        mode = (idx // 2) % 2
        ob = (idx // 3) % 2
        out.append(W.Case(
            "slab_%dx%dx%d_u%d_m%d_b%d" % (m, n, k, uns, mode, ob), 8, idx, m, n, k,
            a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=0, orderB=ob, orderC=0,
            pad=16 * (idx % 4), mode=mode,
            a_dist=("uniform", 0, 255) if uns == 1 else ("uniform", -128, 127),
            b_dist=("uniform", 0, 255) if uns == 2 else ("uniform", -128, 127),
            c_dist=("uniform", -1000, 1000), seed=21))
    return out


@pytest.mark.parametrize("variant", ["slab16", "slab32", "slab64", "auto"])
@pytest.mark.parametrize("case", _slab_cases(), ids=lambda c: c.name)
def test_skinny_m_slab_kernel(gpu, oracle, case, variant):
    """Forced through either slab width, and as the dispatcher routes it (an accumulating call
    with a long k goes to tiles with split k instead)."""
    width = {"slab16": 16, "slab32": 32, "slab64": 64}.get(variant, 0)
    if variant != "auto" and case.n % width == 0:
        with VariantEnv(variant):
            got = gpu.mipgemm_variant_name(case.m, case.n, case.k, case.lda, case.orderA, case.ldb,
                                           case.orderB, case.ldc, case.orderC, case.a_unsigned,
                                           case.b_unsigned, True)
        assert got == "mfma_" + variant
    check_case(gpu, oracle, case, variant)


def test_skinny_m_slab_kernel_wraps(gpu, oracle):
    """All(-128) x all(-128) over k = 2^17: every sum is 2^31, which wraps to -2^31."""
    m, n, k = 4, 32, 1 << 17
    A = np.full(m * k, -128, dtype=np.int8)
    B = np.full(k * n, -128, dtype=np.int8)
    case = W.Case("slab_wrap", 8, 0, m, n, k)
    for variant in ("slab16", "slab32"):
        got = gpu_gemm(gpu, case, A, B, np.full(m * n, 7, dtype=np.int32), variant)
        assert (got == -2 ** 31).all()
    case = W.Case("slab_wrap64", 8, 0, m, 64, k)
    got = gpu_gemm(gpu, case, A, np.full(k * 64, -128, dtype=np.int8), np.full(m * 64, 7, dtype=np.int32), "slab64")
    assert (got == -2 ** 31).all()


def test_calls_replay_from_a_hip_graph(gpu, oracle):
    """A captured call (here one that zero-fills C and then adds k ranges with atomics, and one
    single-kernel call) gives the oracle's result on every replay, with C overwritten by other
    work between the replays."""
    import torch
    for case in (W.Case("graph_splitk", 8, 0, 48, 256, 4096, seed=31),
                 W.Case("graph_slab", 8, 1, 8, 3072, 512, orderB=W.COL_MAJOR, seed=31)):
        ops = W.materialize(case)
        want = oracle_result(oracle, case, ops)
        dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
        dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
        dC = torch.from_numpy(ops.C).cuda()
        fn = getattr(gpu, "mipgemm_" + case.entry)

        def call():
            fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
               dC, case.ldc, case.orderC, case.mode)

        call()
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy(), want)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            call()
        for replay in range(4):
            dC.fill_(replay - 7)                     # eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(dC.cpu().numpy(), want), "replay %d of %s" % (replay, case.name)


# ---------------------------------------------------------------------------
# strided batches: every problem of the batch against the oracle on its own slices
# ---------------------------------------------------------------------------

def _batched_cases():
    # (m, n, k, orderA, orderB, orderC, pad, batch, share_a, mode)
    return [
        (256, 256, 64, 1, 0, 0, 0, 16, False, 0),      # K^T Q per head (M5 of the encoder block)
        (64, 256, 256, 0, 0, 0, 0, 16, False, 0),      # V E_1 per head (M7)
        (100, 37, 51, 0, 1, 0, 3, 3, False, 1),        # unaligned: the register-staged kernel
        (48, 80, 4096, 0, 0, 0, 0, 2, False, 0),       # few tiles, long k: split k inside a batch
        (130, 70, 128, 0, 0, 1, 16, 5, False, 1),      # column-major C: roles (and strides) swap
        (64, 64, 192, 0, 1, 0, 0, 7, True, 0),         # one A for every problem (stride 0)
        (1, 16, 64, 0, 1, 0, 0, 4, False, 0),
    ]


@pytest.mark.parametrize("signs", ["s8s8", "u8s8", "s8u8"])
@pytest.mark.parametrize("variant", ["auto", "simple", "tile64", "dma64", "dma128"])
@pytest.mark.parametrize("spec", _batched_cases(), ids=lambda s: "x".join(map(str, s)))
def test_batched_gemm(gpu, oracle, spec, variant, signs):
    import torch
    m, n, k, oa, ob, oc, pad, batch, share_a, mode = spec
    au, bu = signs[0] == "u", signs[2] == "u"
    print("batched", spec, variant, signs, flush=True)
    case = W.Case("batched", 8, 0, m, n, k, orderA=oa, orderB=ob, orderC=oc, pad=pad, mode=mode,
                  c_dist=("uniform", -1000, 1000), seed=51)
    sets = [W.materialize(W.Case("batched", 8, z, m, n, k, orderA=oa, orderB=ob, orderC=oc, pad=pad,
                                 mode=mode, c_dist=("uniform", -1000, 1000), seed=51))
            for z in range(batch)]
    gap = 48                                             # sentinel bytes / words between the slices
    sa = 0 if share_a else sets[0].A.size + gap
    sb, sc = sets[0].B.size + gap, sets[0].C.size + gap
    A = np.full(max(sa, sets[0].A.size) * (1 if share_a else batch), 0x5A, dtype=np.int8)
    B = np.full(sb * batch, 0x5A, dtype=np.int8)
    C = np.full(sc * batch, 0x5A5A5A5A, dtype=np.int32)
    want = C.copy()
    for z, o in enumerate(sets):
        a = sets[0].A if share_a else o.A
        if not share_a:
            A[z * sa:z * sa + a.size] = a
        elif z == 0:
            A[:a.size] = a
        B[z * sb:z * sb + o.B.size] = o.B
        C[z * sc:z * sc + o.C.size] = o.C
        w = o.C.copy()
        # the same bytes, read as unsigned where the entry point says so
        oracle.gemm(au, bu, m, n, k, a.view(np.uint8) if au else a, case.lda, oa,
                    o.B.view(np.uint8) if bu else o.B, case.ldb, ob, w, case.ldc, oc, mode)
        want[z * sc:z * sc + w.size] = w
    dA = torch.from_numpy(A.view(np.uint8)).cuda()
    dB = torch.from_numpy(B.view(np.uint8)).cuda()
    dC = torch.from_numpy(C).cuda()
    with VariantEnv(variant):
        getattr(gpu, "mipgemm_%ss32_batched" % signs)(m, n, k, dA, case.lda, oa, sa, dB, case.ldb, ob,
                                                      sb, dC, case.ldc, oc, sc, batch, mode)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)        # the gaps between the slices included


def test_batched_empty_sums(gpu):
    """k = 0 in a batch: overwrite zeroes every problem's m x n block and nothing else."""
    import torch
    m, n, batch, ldc, sc = 5, 7, 4, 9, 60
    C = np.full(sc * batch, 0x5A5A5A5A, dtype=np.int32)
    dC = torch.from_numpy(C.copy()).cuda()
    z = torch.zeros(64, dtype=torch.uint8, device="cuda")
    gpu.mipgemm_s8s8s32_batched(m, n, 0, z, 1, 0, 0, z, n, 0, 0, dC, ldc, 0, sc, batch, W.OVERWRITE)
    torch.cuda.synchronize()
    want = C.copy()
    for b in range(batch):
        for i in range(m):
            want[b * sc + i * ldc:b * sc + i * ldc + n] = 0
    assert np.array_equal(dC.cpu().numpy(), want)
    gpu.mipgemm_s8s8s32_batched(m, n, 0, z, 1, 0, 0, z, n, 0, 0, dC, ldc, 0, sc, batch, W.ACCUMULATE)
    gpu.mipgemm_s8s8s32_batched(0, n, 8, z, 8, 0, 0, z, n, 0, 0, dC, ldc, 0, sc, batch, W.OVERWRITE)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)


def test_calls_from_two_host_threads_on_two_streams(gpu, oracle):
    """The library keeps no state between calls: two host threads, each with a stream of its
    own, issue different problems (a split-k call with its zero fill, a skinny one, a square
    one) many times over at once; every result is the oracle's."""
    import threading
    import torch
    cases = [W.Case("mt_splitk", 8, 0, 48, 256, 4096, seed=41),
             W.Case("mt_slab", 8, 1, 8, 3072, 512, orderB=W.COL_MAJOR, seed=41),
             W.Case("mt_square", 8, 2, 512, 512, 512, a_unsigned=True, seed=41)]
    work = []
    for case in cases:
        ops = W.materialize(case)
        work.append((case, oracle_result(oracle, case, ops), ops))
    failures = []

    def worker(index):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()             # default priority
            with torch.cuda.stream(stream):
                bufs = [(torch.from_numpy(ops.A.view(np.uint8)).cuda(), torch.from_numpy(ops.B.view(np.uint8)).cuda(),
                         torch.from_numpy(ops.C).cuda()) for _, _, ops in work]
            stream.synchronize()
            for it in range(40):
                which = (it + index) % len(work)
                case, want, ops = work[which]
                dA, dB, dC = bufs[which]
                with torch.cuda.stream(stream):
                    dC.copy_(torch.from_numpy(ops.C), non_blocking=False)
                getattr(gpu, "mipgemm_" + case.entry)(
                    case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
                    dC, case.ldc, case.orderC, case.mode, stream=stream)
                stream.synchronize()
                if not np.array_equal(dC.cpu().numpy(), want):
                    failures.append((index, it, case.name))
        except Exception as e:                        # surfaced in the main thread below
            failures.append((index, "exception", repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads)
    assert failures == []


# ---------------------------------------------------------------------------
# the packed route: operands the direct-to-LDS kernels cannot stream, given a workspace
# ---------------------------------------------------------------------------

def _packed_bytes(m, n, k):
    kp = (k + 127) // 128 * 128 if k >= 1024 else (k + 63) // 64 * 64
    up = lambda x: (x + 255) // 256 * 256
    return (up(m) + up(n)) * kp


def _packed_cases():
    # (m, n, k, orderA, orderB, orderC, pad, a_unsigned, b_unsigned, mode)
    out = []
    for oa, ob, oc in ((0, 0, 0), (0, 1, 0), (1, 0, 0), (1, 1, 0), (0, 0, 1), (1, 0, 1)):
        out.append((1000, 999, 1001, oa, ob, oc, 0, False, False, oa ^ ob))
    out += [(1000, 999, 1001, 0, 0, 0, 3, True, False, 1), (1000, 999, 1001, 1, 1, 1, 5, False, True, 0),
            (1300, 1700, 257, 0, 0, 0, 0, False, False, 0),    # m not a multiple of the tile, short odd k
            (130, 4100, 1010, 1, 0, 0, 1, True, False, 0),
            (3000, 5000, 320, 0, 0, 0, 0, False, False, 1),    # k already fine, ldb = 5000 is not
            (515, 520, 2049, 0, 1, 0, 0, False, True, 0),      # long k: padded to a multiple of 128
            (2000, 3000, 1999, 0, 0, 0, 0, False, False, 0),
            # 14 x 14 ragged tiles of 256 x 256: the kernel with 128-deep k blocks on padded rows
            (3500, 3400, 1025, 1, 0, 0, 0, True, False, 1)]
    return out


@pytest.mark.parametrize("spec", _packed_cases(), ids=lambda s: "x".join(map(lambda v: str(int(v)), s)))
def test_packed_route_with_a_workspace(gpu, oracle, spec):
    import torch
    m, n, k, oa, ob, oc, pad, au, bu, mode = spec
    print("packed", spec, flush=True)
    case = W.Case("packed_" + "_".join(str(int(v)) for v in spec), 8, 0, m, n, k,
                  a_unsigned=au, b_unsigned=bu, orderA=oa, orderB=ob,
                  orderC=oc, pad=pad, mode=mode, c_dist=("uniform", -1000, 1000), seed=61)
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    name = gpu.mipgemm_variant_name_with_workspace(m, n, k, case.lda, oa, case.ldb, ob, case.ldc, oc,
                                                   au, bu, True)
    assert name.startswith("packed+mfma_"), name
    if (m, n, k) == (3500, 3400, 1025):
        assert name == "packed+mfma_dma256_k128"
    need = _packed_bytes(*((m, n, k) if oc == 0 else (n, m, k)))
    if pad == 0:
        assert gpu.mipgemm_workspace_size(m, n, k, oa, ob, oc) == need
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    fn = getattr(gpu, "mipgemm_" + case.entry)
    for given in (need, need - 1):                   # one byte short: the in-place kernels, same bits
        dC = torch.from_numpy(ops.C).cuda()
        ws = torch.full((need + 64,), 0x5A, dtype=torch.uint8, device="cuda")
        fn(m, n, k, dA, case.lda, oa, dB, case.ldb, ob, dC, case.ldc, oc, mode,
           workspace=ws, workspace_bytes=given)
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy(), want), "workspace_bytes %d" % given
        assert (ws[need:].cpu().numpy() == 0x5A).all()           # nothing written past the workspace
        if given < need:
            assert (ws.cpu().numpy() == 0x5A).all()              # and nothing at all when it is too small


def test_packed_route_for_unaligned_pointers_and_float_output(gpu, oracle):
    """Aligned sizes on pointers that are not: packed too.  And the dequantising entry point."""
    import torch
    m, n, k = 1024, 768, 1024
    case = W.Case("packed_ptr", 8, 1, m, n, k, seed=62)
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    assert gpu.mipgemm_variant_name_with_workspace(m, n, k, k, 0, n, 0, n, 0, False, False, False) \
        .startswith("packed+")
    assert gpu.mipgemm_workspace_size(m, n, k, 0, 0, 0) == 0     # by the sizes alone nothing to pack
    need = _packed_bytes(m, n, k)
    holdA = torch.zeros(ops.A.size + 16, dtype=torch.uint8, device="cuda")
    holdB = torch.zeros(ops.B.size + 16, dtype=torch.uint8, device="cuda")
    dA, dB = holdA[1:1 + ops.A.size], holdB[3:3 + ops.B.size]    # 1 and 3 bytes off
    dA.copy_(torch.from_numpy(ops.A.view(np.uint8)))
    dB.copy_(torch.from_numpy(ops.B.view(np.uint8)))
    dC = torch.from_numpy(ops.C).cuda()
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    gpu.mipgemm_s8s8s32(m, n, k, dA, k, 0, dB, n, 0, dC, n, 0, 0, workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)
    assert ws.cpu().numpy().any()                                 # the packed operands are there
    dF = torch.zeros(m * n, dtype=torch.float32, device="cuda")
    gpu.mipgemm_s8s8f32(m, n, k, dA, k, 0, dB, n, 0, dF, n, 0, 0, workspace=ws, workspace_bytes=need,
                        scale=0.25)
    torch.cuda.synchronize()
    assert np.array_equal(dF.cpu().numpy(), want.astype(np.float32) * np.float32(0.25))
    # a workspace that is itself off by a byte: the packed operands are then read in place
    ws1 = torch.zeros(need + 16, dtype=torch.uint8, device="cuda")
    dC.fill_(-5)
    gpu.mipgemm_s8s8s32(m, n, k, dA, k, 0, dB, n, 0, dC, n, 0, 0, workspace=ws1[1:], workspace_bytes=need)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)


@pytest.mark.parametrize("spec", [(65, 70, 100, 0, 0, 0, 0, False, False, 0), (7, 7, 3, 1, 0, 0, 17, True, False, 1),
                                  (1, 4097, 513, 0, 0, 0, 17, False, False, 0), (100, 37, 51, 1, 1, 1, 3, False, True, 1),
                                  (300, 200, 333, 0, 1, 0, 17, True, False, 1), (4095, 3, 2049, 0, 0, 1, 0, False, False, 0)],
                         ids=lambda s: "x".join(map(lambda v: str(int(v)), s)))
def test_packed_route_forced_on_small_and_skinny_shapes(gpu, oracle, spec):
    """MIPGEMM_PACK=always takes the packed route whatever the size: ragged everything."""
    import torch
    m, n, k, oa, ob, oc, pad, au, bu, mode = spec
    print("packed forced", spec, flush=True)
    case = W.Case("packedf_" + "_".join(str(int(v)) for v in spec), 8, 0, m, n, k,
                  a_unsigned=au, b_unsigned=bu, orderA=oa, orderB=ob, orderC=oc, pad=pad, mode=mode,
                  c_dist=("uniform", -1000, 1000), seed=63)
    ops = W.materialize(case)
    want = oracle_result(oracle, case, ops)
    need = _packed_bytes(m, n, k)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dC = torch.from_numpy(ops.C).cuda()
    ws = torch.full((need + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    with VariantEnv("auto"), gpu.tuning(MIPGEMM_PACK="always"):
        assert gpu.mipgemm_variant_name_with_workspace(m, n, k, case.lda, oa, case.ldb, ob, case.ldc,
                                                       oc, au, bu, True).startswith("packed")
        getattr(gpu, "mipgemm_" + case.entry)(m, n, k, dA, case.lda, oa, dB, case.ldb, ob, dC,
                                              case.ldc, oc, mode, workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)
    assert (ws[need:].cpu().numpy() == 0x5A).all()
    assert not (ws[:need].cpu().numpy() == 0x5A).all()           # the packed operands were written


def test_seeded_sweep_of_the_packed_route(gpu, oracle):
    """40 random small problems (any order, padded leading dimensions, either operand unsigned,
    both modes) forced through the packed route."""
    import torch
    rng = np.random.default_rng(2025)
    with gpu.tuning(MIPGEMM_PACK="always"):
        for it in range(40):
            m, n, k = int(rng.integers(1, 700)), int(rng.integers(1, 700)), int(rng.integers(1, 1500))
            oa, ob, oc = (int(x) for x in rng.integers(0, 2, size=3))
            au = bool(rng.integers(0, 2))
            bu = (not au) and bool(rng.integers(0, 2))
            pad, mode = int(rng.choice([0, 1, 3, 16, 17])), int(rng.integers(0, 2))
            case = W.Case("packsweep_%d" % it, 8, it, m, n, k, a_unsigned=au, b_unsigned=bu, orderA=oa,
                          orderB=ob, orderC=oc, pad=pad, mode=mode, c_dist=("uniform", -1000, 1000),
                          seed=64)
            print("packed sweep", (m, n, k, oa, ob, oc, pad, au, bu, mode), flush=True)
            ops = W.materialize(case)
            want = oracle_result(oracle, case, ops)
            need = _packed_bytes(m, n, k)
            ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
            dC = torch.from_numpy(ops.C).cuda()
            getattr(gpu, "mipgemm_" + case.entry)(
                m, n, k, torch.from_numpy(ops.A.view(np.uint8)).cuda(), case.lda, oa,
                torch.from_numpy(ops.B.view(np.uint8)).cuda(), case.ldb, ob, dC, case.ldc, oc, mode,
                workspace=ws, workspace_bytes=need)
            torch.cuda.synchronize()
            assert np.array_equal(dC.cpu().numpy(), want), (m, n, k, oa, ob, oc, pad, au, bu, mode)
