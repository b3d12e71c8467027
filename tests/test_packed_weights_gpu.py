"""GPU parity of the pre-packed weights: the packed object byte for byte against the oracle's,
and the GEMMs on it bit for bit against the GEMM oracle on the unpacked matrix."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_11728_amd as M
    M.load_library()
    return M


def _weights(k, n, order, pad, seed):
    """Flat int8 buffer holding a k x n matrix in the given order with padded ld (sentinels between)."""
    rng = np.random.default_rng([k, n, order, pad, seed])
    dense = rng.integers(-128, 128, size=(k, n), dtype=np.int8)
    ldb = max(1, (n if order == W.ROW_MAJOR else k)) + pad
    flat = np.full((max(1, k if order == W.ROW_MAJOR else n), ldb), 0x5A, dtype=np.uint8)
    if k and n:
        if order == W.ROW_MAJOR:
            flat[:k, :n] = dense.view(np.uint8)
        else:
            flat[:n, :k] = dense.T.view(np.uint8)
    return dense, flat.reshape(-1).view(np.int8), ldb


def _pack_on_gpu(M, k, n, flat, ldb, order, slack=64):
    import torch
    need = M.mipgemm_packed_weights_bytes(k, n)
    dP = torch.full((need + slack,), 0xC3, dtype=torch.uint8, device="cuda")
    dB = torch.from_numpy(flat.view(np.uint8)).cuda()
    M.mipgemm_pack_weights(k, n, dB, ldb, order, dP, need)
    torch.cuda.synchronize()
    return dP, need


@pytest.mark.parametrize("k,n,order,pad", [(2, 3, 0, 0), (64, 256, 1, 0), (100, 37, 0, 5), (1000, 300, 1, 17),
                                           (1024, 257, 0, 16), (1090, 513, 0, 3), (4096, 64, 1, 0),
                                           (1, 1, 0, 0), (200, 1, 1, 1), (0, 5, 0, 0), (7, 0, 1, 0)])
def test_pack_weights_matches_the_oracle(gpu, oracle, k, n, order, pad):
    dense, flat, ldb = _weights(k, n, order, pad, 1)
    dP, need = _pack_on_gpu(gpu, k, n, flat, ldb, order)
    want = oracle.pack_weights(k, n, flat, ldb, order)
    assert need == want.size == oracle.packed_weights_layout(k, n)[3]
    got = dP.cpu().numpy()
    assert np.array_equal(got[:need], want)
    assert (got[need:] == 0xC3).all()          # nothing written behind the object


def _check_gemm(M, oracle, m, n, k, a_unsigned, orderA, orderB, orderC, mode, pad, variant, splits=None,
                workspace=False, seed=0):
    import torch
    dense, flatB, ldb = _weights(k, n, orderB, pad, seed)
    case = W.Case("packed", 8, seed, m, n, k, a_unsigned=a_unsigned, orderA=orderA, orderB=orderB,
                  orderC=orderC, pad=pad, mode=mode,
                  a_dist=("uniform", 0, 255) if a_unsigned else ("uniform", -128, 127),
                  c_dist=("uniform", -1000, 1000), seed=seed)
    ops = W.materialize(case)
    want = ops.C.copy()
    oracle.gemm(a_unsigned, False, m, n, k, ops.A, case.lda, orderA, flatB, ldb, orderB, want, case.ldc,
                orderC, mode)
    dP, _ = _pack_on_gpu(M, k, n, flatB, ldb, orderB)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dC = torch.from_numpy(ops.C).cuda()
    kp = oracle.packed_weights_layout(k, n)[0]
    fn = M.mipgemm_u8s8s32_packed if a_unsigned else M.mipgemm_s8s8s32_packed
    ws = need = None
    if workspace:
        need = (-(-m // 256) * 256 + -(-n // 256) * 256) * (-(-k // 128) * 128) + 4096
        ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    with M.tuning(MIPGEMM_VARIANT=None if variant == "auto" else variant, MIPGEMM_SPLITK=splits,
                  MIPGEMM_PACK="always" if workspace else None):
        name = M.mipgemm_variant_name_for_mode(m, n, k, case.lda, orderA, kp, W.COL_MAJOR, case.ldc, orderC,
                                               a_unsigned, False, pad % 16 == 0, mode)
        print("packed gemm", (m, n, k), "u8" if a_unsigned else "s8", "orders", orderA, orderB, orderC,
              "mode", mode, "variant", variant, "kernel", name, flush=True)
        fn(m, n, k, dA, case.lda, orderA, dP, dC, case.ldc, orderC, mode,
           workspace=ws, workspace_bytes=need or 0)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        pytest.fail("%d of %d words differ, first at %d: got %d want %d" % (bad.size, got.size, bad[0],
                                                                          got[bad[0]], want[bad[0]]))
    return name


TILE_VARIANTS = ["auto", "dma256k128", "dma128k128", "dma256", "dma128", "dma64", "dma64x256", "dma256x64",
                 "dma64x128", "dma128x64", "tile64", "simple"]


@pytest.mark.parametrize("variant", TILE_VARIANTS)
@pytest.mark.parametrize("orderC", [W.ROW_MAJOR, W.COL_MAJOR])
def test_u8_gemm_on_packed_weights_every_kernel(gpu, oracle, variant, orderC):
    """Whole tiles, k a multiple of 128: every direct-to-LDS kernel takes the k-sums from the
    packed object (a column-major C swaps the operand roles: the sums then belong to the rows of
    the kernel's A); both orders of A, both modes."""
    name = None
    for orderA, mode in ((W.ROW_MAJOR, W.OVERWRITE), (W.COL_MAJOR, W.ACCUMULATE)):
        name = _check_gemm(gpu, oracle, 512, 768, 1024, True, orderA, W.ROW_MAJOR, orderC, mode, 0, variant,
                           seed=3)
    if variant.startswith("dma"):
        assert name == ("mfma_" + variant.replace("k128", "_k128"))


@pytest.mark.parametrize("variant", ["auto", "dma128", "dma64", "dma64x256", "dma128x64", "tile64"])
def test_u8_gemm_on_packed_weights_ragged_tiles(gpu, oracle, variant):
    """Ragged edges in both dimensions (columns past n read no k-sum), padded ld, weights that
    were stored column-major."""
    for orderC in (W.ROW_MAJOR, W.COL_MAJOR):
        _check_gemm(gpu, oracle, 200, 331, 512, True, W.ROW_MAJOR, W.COL_MAJOR, orderC, W.OVERWRITE, 16,
                    variant, seed=4)


def test_gemm_on_packed_weights_other_routes(gpu, oracle):
    """Kernels that ignore the supplied sums and compute their own, and the signed form: k not a
    multiple of 64 (register-staged kernel), a few rows (skinny-m kernel), split k (every range
    sums its own part), the packed route in front of the ragged form of the kernel for large
    problems."""
    _check_gemm(gpu, oracle, 100, 130, 200, True, W.ROW_MAJOR, W.ROW_MAJOR, W.ROW_MAJOR, W.ACCUMULATE, 3,
                "auto", seed=5)
    name = _check_gemm(gpu, oracle, 4, 4096, 1024, True, W.ROW_MAJOR, W.ROW_MAJOR, W.ROW_MAJOR, W.OVERWRITE,
                       0, "auto", seed=6)
    assert name.startswith("mfma_slab")
    _check_gemm(gpu, oracle, 64, 128, 4096, True, W.ROW_MAJOR, W.ROW_MAJOR, W.ROW_MAJOR, W.OVERWRITE, 0,
                "dma64", splits=4, seed=7)
    _check_gemm(gpu, oracle, 64, 128, 4096, True, W.ROW_MAJOR, W.ROW_MAJOR, W.COL_MAJOR, W.ACCUMULATE, 0,
                "dma64", splits=3, seed=7)
    for orderC in (W.ROW_MAJOR, W.COL_MAJOR):
        _check_gemm(gpu, oracle, 300, 520, 1024, True, W.ROW_MAJOR, W.ROW_MAJOR, orderC, W.OVERWRITE, 17,
                    "dma256k128", workspace=True, seed=8)
    for variant in ("auto", "dma128k128", "dma64"):
        _check_gemm(gpu, oracle, 256, 384, 768, False, W.ROW_MAJOR, W.ROW_MAJOR, W.ROW_MAJOR, W.ACCUMULATE, 0,
                    variant, seed=10)


def test_packed_weights_as_dispatched_on_a_large_product(gpu, oracle):
    """2048 x 2048 x 2048 and a conv-shaped product as the dispatcher runs them."""
    _check_gemm(gpu, oracle, 2048, 2048, 2048, True, W.ROW_MAJOR, W.ROW_MAJOR, W.ROW_MAJOR, W.OVERWRITE, 0,
                "auto", seed=11)
    _check_gemm(gpu, oracle, 6272, 256, 2304, True, W.ROW_MAJOR, W.ROW_MAJOR, W.ROW_MAJOR, W.OVERWRITE, 0,
                "auto", seed=12)


def test_packed_weights_error_paths_touch_nothing(gpu):
    import torch
    k, n, m = 128, 64, 32
    need = gpu.mipgemm_packed_weights_bytes(k, n)
    assert need == 128 * 256 + 4 * 64
    assert gpu.mipgemm_packed_weights_bytes(-1, 5) == 0
    dB = torch.zeros(k * n, dtype=torch.uint8, device="cuda")
    dP = torch.full((need + 16,), 7, dtype=torch.uint8, device="cuda")
    assert gpu.mipgemm_pack_weights(k, n, dB, n, W.ROW_MAJOR, dP, need - 1, check=False) == -7
    assert gpu.mipgemm_pack_weights(k, n, dB, n - 1, W.ROW_MAJOR, dP, need, check=False) == -4
    assert gpu.mipgemm_pack_weights(k, n, dB, n, 5, dP, need, check=False) == -5
    assert gpu.mipgemm_pack_weights(k, n, None, n, W.ROW_MAJOR, dP, need, check=False) == -3
    assert gpu.mipgemm_pack_weights(k, n, dB, n, W.ROW_MAJOR, dP[1:], need, check=False) == -6   # not 16-byte aligned
    torch.cuda.synchronize()
    assert (dP.cpu().numpy() == 7).all()
    dA = torch.zeros(m * k, dtype=torch.uint8, device="cuda")
    dC = torch.full((m * n,), 9, dtype=torch.int32, device="cuda")
    R, OVW = W.ROW_MAJOR, W.OVERWRITE
    assert gpu.mipgemm_u8s8s32_packed(m, n, k, dA, k, R, None, dC, n, R, OVW, check=False) == -7
    assert gpu.mipgemm_u8s8s32_packed(m, n, k, dA, k - 1, R, dP, dC, n, R, OVW, check=False) == -5
    assert gpu.mipgemm_u8s8s32_packed(m, n, k, dA, k, R, dP, None, n, R, OVW, check=False) == -8
    assert gpu.mipgemm_u8s8s32_packed(m, n, k, dA, k, R, dP, dC, n - 1, R, OVW, check=False) == -9
    assert gpu.mipgemm_u8s8s32_packed(m, n, k, dA, k, R, dP, dC, n, 7, OVW, check=False) == -10
    assert gpu.mipgemm_s8s8s32_packed(m, n, k, dA, k, R, dP, dC, n, R, 3, check=False) == -11
    torch.cuda.synchronize()
    assert (dC.cpu().numpy() == 9).all()


def test_packed_weights_seeded_sweep(gpu, oracle):
    """Forty random products as dispatched: sizes from a few rows to several tiles, ragged or
    whole, both signednesses of A, every order of A, B and C, both modes, aligned and padded ld."""
    rng = np.random.default_rng(20260)
    for i in range(40):
        m = int(rng.choice([1, 3, 16, 40, 64, 100, 128, 200, 256, 333, 512]))
        n = int(rng.choice([16, 48, 64, 100, 128, 256, 300, 384, 512, 1000]))
        k = int(rng.choice([64, 128, 192, 256, 320, 512, 1024, 1088, 2048, 77, 500]))
        pad = int(rng.choice([0, 0, 16, 5]))
        _check_gemm(gpu, oracle, m, n, k, bool(rng.integers(0, 2)), int(rng.integers(0, 2)),
                    int(rng.integers(0, 2)), int(rng.integers(0, 2)), int(rng.integers(0, 2)), pad, "auto",
                    seed=100 + i)


def test_packed_weights_replay_from_a_hip_graph(gpu, oracle):
    """A captured u8 x s8 call on packed weights gives the oracle's result on every replay."""
    import torch
    m, n, k = 256, 384, 1024
    dense, flatB, ldb = _weights(k, n, W.ROW_MAJOR, 0, 21)
    case = W.Case("packed_graph", 8, 21, m, n, k, a_unsigned=True, a_dist=("uniform", 0, 255), seed=21)
    ops = W.materialize(case)
    want = ops.C.copy()
    oracle.gemm(True, False, m, n, k, ops.A, case.lda, 0, flatB, ldb, 0, want, case.ldc, 0, W.OVERWRITE)
    dP, _ = _pack_on_gpu(gpu, k, n, flatB, ldb, W.ROW_MAJOR)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dC = torch.from_numpy(ops.C).cuda()

    def call():
        gpu.mipgemm_u8s8s32_packed(m, n, k, dA, case.lda, 0, dP, dC, case.ldc, 0, W.OVERWRITE)

    call()
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for replay in range(3):
        dC.fill_(replay + 11)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy(), want), "replay %d" % replay
