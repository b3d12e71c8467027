"""GPU parity of the product with 16-bit operands (byte planes on the 8-bit kernels) against
the int16 oracle, bit for bit, through the C ABI."""
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


def _flat(X, order, pad, fill):
    """X (r x c) as a flat buffer in the given order with padded ld; returns (buffer, ld)."""
    r, c = X.shape
    ld = max(1, (c if order == W.ROW_MAJOR else r)) + pad
    buf = np.full((max(1, r if order == W.ROW_MAJOR else c), ld), fill, dtype=X.dtype)
    if r and c:
        if order == W.ROW_MAJOR:
            buf[:r, :c] = X
        else:
            buf[:c, :r] = X.T
    return buf.reshape(-1), ld


def _operands(m, n, k, dist, seed):
    rng = np.random.default_rng([m, n, k, seed])
    if dist == "uniform":
        A = rng.integers(-32768, 32768, size=(m, k), dtype=np.int16)
        B = rng.integers(-32768, 32768, size=(k, n), dtype=np.int16)
    elif dist == "normal":          # what 16-bit quantized tensors look like
        A = np.clip(np.rint(rng.standard_normal((m, k)) * 3000), -32768, 32767).astype(np.int16)
        B = np.clip(np.rint(rng.standard_normal((k, n)) * 3000), -32768, 32767).astype(np.int16)
    elif dist == "min":
        A = np.full((m, k), -32768, dtype=np.int16)
        B = np.full((k, n), -32768, dtype=np.int16)
    else:                           # the byte boundaries: low byte 0x7f/0x80/0xff/0x00, high byte extremes
        vals = np.array([-32768, -32641, -32640, -129, -128, -1, 0, 1, 127, 128, 255, 256, 32639, 32640, 32767],
                        dtype=np.int16)
        A = rng.choice(vals, size=(m, k))
        B = rng.choice(vals, size=(k, n))
    return A, B


def _check(M, oracle, m, n, k, oa, ob, oc, mode, pad, dist="uniform", seed=0, variant=None, misalign=0):
    import torch
    A2, B2 = _operands(m, n, k, dist, seed)
    A, lda = _flat(A2, oa, pad, 0x5A5A)
    B, ldb = _flat(B2, ob, pad, 0x5A5A)
    rng = np.random.default_rng([seed, 7])
    ldc = max(1, (n if oc == W.ROW_MAJOR else m)) + pad
    C0 = rng.integers(-1000, 1000, size=max(1, m if oc == W.ROW_MAJOR else n) * ldc, dtype=np.int32)
    want = C0.copy()
    oracle.gemm_s16(m, n, k, A, lda, oa, B, ldb, ob, want, ldc, oc, mode)
    dA = torch.from_numpy(A.view(np.uint8)).cuda()
    dB = torch.from_numpy(B.view(np.uint8)).cuda()
    dC = torch.from_numpy(C0).cuda()
    need = M.mipgemm_workspace_size_s16(m, n, k)
    ws = torch.full((need + 64 + misalign,), 0x33, dtype=torch.uint8, device="cuda")
    with M.tuning(MIPGEMM_VARIANT=variant):
        M.mipgemm_s16s16s32(m, n, k, dA, lda, oa, dB, ldb, ob, dC, ldc, oc, mode,
                            workspace=ws[misalign:] if misalign else ws, workspace_bytes=need)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    if need:
        assert (ws[misalign + need:].cpu().numpy() == 0x33).all()      # nothing written past the workspace
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        pytest.fail("(%d, %d, %d) orders %d%d%d mode %d %s: %d of %d words differ, first at %d: got %d want %d" % (
            m, n, k, oa, ob, oc, mode, dist, bad.size, got.size, bad[0], got[bad[0]], want[bad[0]]))


@pytest.mark.parametrize("orders", [(0, 0, 0), (0, 1, 0), (1, 0, 0), (1, 1, 0), (0, 0, 1), (1, 0, 1), (0, 1, 1), (1, 1, 1)])
@pytest.mark.parametrize("mode", [0, 1])
def test_s16_every_order_and_mode(gpu, oracle, orders, mode):
    oa, ob, oc = orders
    for (m, n, k, pad) in ((37, 50, 70, 3), (128, 192, 256, 0), (200, 65, 1030, 17)):
        for dist in ("uniform", "edges"):
            _check(gpu, oracle, m, n, k, oa, ob, oc, mode, pad, dist, seed=1)


@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 64, 64), (7, 7, 3), (64, 1, 4096), (3, 4096, 512), (256, 256, 1024),
                                   (512, 384, 2048), (1000, 999, 1001), (130, 70, 63), (16, 2048, 128)],
                         ids=lambda s: "x".join(map(str, s)))
def test_s16_shapes(gpu, oracle, shape):
    m, n, k = shape
    _check(gpu, oracle, m, n, k, 0, 0, 0, W.OVERWRITE, 0, "uniform", seed=2)
    _check(gpu, oracle, m, n, k, 0, 1, 0, W.ACCUMULATE, 8, "normal", seed=3)


def test_s16_wraps_and_extremes(gpu, oracle):
    """All -32768: every product is 2^30, the sums wrap from k = 2 on; and the largest positive
    products next to them."""
    for k in (1, 2, 3, 4, 64, 100, 4097):
        _check(gpu, oracle, 5, 9, k, 0, 0, 0, W.OVERWRITE, 0, "min", seed=4)
    _check(gpu, oracle, 70, 130, 520, 0, 0, 0, W.ACCUMULATE, 0, "min", seed=5)


def test_s16_under_forced_kernels_and_a_misaligned_workspace(gpu, oracle):
    for variant in ("dma128k128", "dma64", "tile64", "dma64x256", "simple"):
        _check(gpu, oracle, 256, 384, 1024, 0, 0, 0, W.OVERWRITE, 0, "uniform", seed=6, variant=variant)
    _check(gpu, oracle, 100, 90, 200, 0, 0, 0, W.OVERWRITE, 0, "uniform", seed=7, misalign=3)


def test_s16_a_large_product_as_dispatched(gpu, oracle):
    _check(gpu, oracle, 1024, 1536, 2048, 0, 0, 0, W.OVERWRITE, 0, "normal", seed=8)


def test_s16_empty_problems_and_error_paths(gpu):
    import torch
    R, OVW, ACC = W.ROW_MAJOR, W.OVERWRITE, W.ACCUMULATE
    assert gpu.mipgemm_workspace_size_s16(0, 5, 5) == 0 and gpu.mipgemm_workspace_size_s16(-1, 5, 5) == 0
    dA = torch.zeros(256, dtype=torch.int16, device="cuda")
    C0 = np.arange(12, dtype=np.int32) + 5
    dC = torch.from_numpy(C0).cuda()
    gpu.mipgemm_s16s16s32(0, 4, 5, dA, 5, R, dA, 4, R, dC, 4, R, OVW)
    gpu.mipgemm_s16s16s32(3, 0, 5, dA, 5, R, dA, 1, R, dC, 1, R, OVW)
    gpu.mipgemm_s16s16s32(3, 3, 0, dA, 1, R, dA, 3, R, dC, 4, R, ACC)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C0)
    gpu.mipgemm_s16s16s32(3, 3, 0, dA, 1, R, dA, 3, R, dC, 4, R, OVW)        # k == 0: C := 0
    torch.cuda.synchronize()
    want = C0.reshape(3, 4).copy()
    want[:, :3] = 0
    assert np.array_equal(dC.cpu().numpy().reshape(3, 4), want)
    dC = torch.from_numpy(C0).cuda()
    need = gpu.mipgemm_workspace_size_s16(3, 4, 5)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    call = lambda *a, **kw: gpu.mipgemm_s16s16s32(*a, check=False, **kw)
    assert call(3, 4, 5, dA, 5, R, dA, 4, R, dC, 4, R, OVW) == -14                         # no workspace
    assert call(3, 4, 5, dA, 5, R, dA, 4, R, dC, 4, R, OVW, workspace=ws, workspace_bytes=need - 300) == -15
    assert call(3, 4, 5, dA, 4, R, dA, 4, R, dC, 4, R, OVW, workspace=ws, workspace_bytes=need) == -5
    assert call(3, 4, 5, dA, 5, R, dA, 3, R, dC, 4, R, OVW, workspace=ws, workspace_bytes=need) == -8
    assert call(3, 4, 5, dA, 5, R, dA, 4, R, dC, 3, R, OVW, workspace=ws, workspace_bytes=need) == -11
    assert call(3, 4, 5, dA, 5, R, dA, 4, R, dC, 4, R, 2, workspace=ws, workspace_bytes=need) == -13
    assert call(3, 4, 5, None, 5, R, dA, 4, R, dC, 4, R, OVW, workspace=ws, workspace_bytes=need) == -4
    assert call(-1, 4, 5, dA, 5, R, dA, 4, R, dC, 4, R, OVW, workspace=ws, workspace_bytes=need) == -1
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C0)
