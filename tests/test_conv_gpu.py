"""GPU parity of the steps around the GEMM against the CPU oracle, through the C ABI: the
convolution lowering (paper Section 7.2) -- the augmented matrix byte for byte, the
convolution bit for bit on the gathering ("implicit") path and on the written-out path --
and the pre-packing of a weight matrix (Section 4.1) byte for byte."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_11728_amd as M
    M.load_library()
    return M


class Env:
    """Tuning values of the library (kernel variant, k ranges, convolution route) for the calls inside."""

    def __init__(self, **kv):
        import paper_2506_11728_amd as M
        self.ctx = M.tuning(**kv)

    def __enter__(self):
        self.ctx.__enter__()

    def __exit__(self, *a):
        self.ctx.__exit__(*a)


def tensors(shape, seed):
    b, hi, wi, ci, co, hf, wf, s, p = shape
    rng = np.random.default_rng([seed] + list(shape))
    I = rng.integers(0, 256, size=(b, hi, wi, ci), dtype=np.uint8)
    F = np.clip(np.rint(rng.standard_normal((co, hf, wf, ci)) * 32), -128, 127).astype(np.int8)
    return I, F


# (b, hi, wi, ci, co, hf, wf, stride, pad): the ResNet-50-shaped layers of the conv workload at
# small batch, plus strides, paddings, non-square images and filters, ragged tile edges
CONV_SHAPES = [
    (1, 56, 56, 64, 64, 3, 3, 1, 1), (2, 28, 28, 128, 128, 3, 3, 1, 1),
    (3, 14, 14, 256, 256, 3, 3, 1, 1), (4, 7, 7, 512, 512, 3, 3, 1, 1),
    (2, 7, 7, 512, 2048, 1, 1, 1, 0), (2, 28, 28, 128, 128, 3, 3, 2, 1),
    (1, 17, 23, 64, 96, 3, 5, 2, 2), (2, 9, 13, 192, 40, 5, 3, 1, 0),
    (1, 30, 30, 64, 256, 3, 3, 3, 1), (5, 12, 12, 64, 64, 2, 2, 2, 0),
    (1, 8, 8, 128, 300, 3, 3, 1, 2)]


def run_conv(M, shape, I, F, O0, mode, **env):
    import torch
    b, hi, wi, ci, co, hf, wf, s, p = shape
    dI, dF = torch.from_numpy(I).cuda(), torch.from_numpy(F.view(np.uint8)).cuda()
    dO = torch.from_numpy(O0.copy()).cuda()
    with Env(**env):
        need = M.mipgemm_conv_workspace_size(*shape)
        ws = torch.full((need + 64,), 0x5A, dtype=torch.uint8, device="cuda") if need else None
        M.mipgemm_conv_s8u8s32(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, mode,
                               workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    if ws is not None:
        assert (ws[need:].cpu().numpy() == 0x5A).all()      # nothing written past the workspace
    return dO.cpu().numpy()


@pytest.mark.parametrize("path", ["implicit", "im2col"])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_matches_the_direct_convolution(gpu, oracle, shape, mode, path):
    print("conv", shape, "mode", mode, "path", path, flush=True)
    I, F = tensors(shape, 1)
    name = None
    with Env(MIPGEMM_CONV=None if path == "implicit" else "im2col"):
        name = gpu.mipgemm_conv_variant_name(*shape)
    assert name.startswith("implicit:" if path == "implicit" else "im2col+"), name
    ho = oracle.conv_out_extent(shape[1], shape[5], shape[7], shape[8])
    wo = oracle.conv_out_extent(shape[2], shape[6], shape[7], shape[8])
    rng = np.random.default_rng(3)
    O0 = rng.integers(-1000, 1000, size=(shape[0], ho, wo, shape[4]), dtype=np.int32)
    want = oracle.conv_direct(I, F, shape[7], shape[8], O=O0.copy() if mode else None, mode=mode)
    got = run_conv(gpu, shape, I, F, O0, mode, MIPGEMM_CONV=None if path == "implicit" else "im2col")
    assert np.array_equal(got, want)


@pytest.mark.parametrize("variant,splits", [("dma256", None), ("dma128", None), ("dma64", 3),
                                            ("dma64x256", None), ("dma256x64", 2), ("dma128", 5),
                                            ("dma128x64", None), ("dma64x128", 2)])
@pytest.mark.parametrize("shape", [(2, 28, 28, 128, 128, 3, 3, 1, 1), (1, 17, 23, 64, 96, 3, 5, 2, 2),
                                   (4, 7, 7, 512, 512, 3, 3, 1, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_implicit_conv_under_every_tile_shape_and_split_k(gpu, oracle, shape, variant, splits):
    print("conv", shape, variant, splits, flush=True)
    I, F = tensors(shape, 2)
    want = oracle.conv_direct(I, F, shape[7], shape[8])
    with Env(MIPGEMM_VARIANT=variant, MIPGEMM_SPLITK=splits):
        assert gpu.mipgemm_conv_variant_name(*shape) == "implicit:mfma_" + variant
    got = run_conv(gpu, shape, I, F, np.full(want.shape, 77, dtype=np.int32), 0,
                   MIPGEMM_VARIANT=variant, MIPGEMM_SPLITK=splits)
    assert np.array_equal(got, want)


# channel counts without 16-byte runs (and a few with, pinned to the same kernel): the
# row-segment kernel.  Several tiles per output row with a ragged last one, filter rows
# shorter and longer than a fragment's 16 bytes, filters past one workgroup's 64, windows
# that lie entirely in the padding, k from 4 to 245.
ROWS_SHAPES = [
    (2, 64, 48, 3, 64, 7, 7, 2, 3), (2, 20, 300, 3, 10, 3, 3, 1, 1), (1, 9, 9, 1, 65, 5, 5, 1, 2),
    (3, 12, 40, 5, 130, 3, 4, 3, 0), (1, 16, 16, 17, 7, 2, 2, 2, 1), (2, 10, 10, 4, 33, 1, 1, 1, 0),
    (1, 30, 260, 2, 64, 7, 1, 1, 3), (1, 5, 5, 3, 8, 3, 3, 1, 4), (1, 20, 20, 16, 40, 3, 3, 1, 1),
    (2, 12, 12, 64, 64, 1, 1, 1, 0), (1, 40, 131, 5, 3, 7, 7, 1, 0)]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", ROWS_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_through_the_row_segment_kernel(gpu, oracle, shape, mode):
    print("conv rows", shape, "mode", mode, flush=True)
    I, F = tensors(shape, 4)
    with Env(MIPGEMM_CONV="rows"):
        assert gpu.mipgemm_conv_variant_name(*shape) == "implicit:rows"
        assert gpu.mipgemm_conv_workspace_size(*shape) == 0
    ho = oracle.conv_out_extent(shape[1], shape[5], shape[7], shape[8])
    wo = oracle.conv_out_extent(shape[2], shape[6], shape[7], shape[8])
    rng = np.random.default_rng(9)
    O0 = rng.integers(-1000, 1000, size=(shape[0], ho, wo, shape[4]), dtype=np.int32)
    want = oracle.conv_direct(I, F, shape[7], shape[8], O=O0.copy() if mode else None, mode=mode)
    got = run_conv(gpu, shape, I, F, O0, mode, MIPGEMM_CONV="rows")
    assert np.array_equal(got, want)


def test_conv_first_layer_of_the_network(gpu, oracle):
    """224 x 224 x 3 images, 64 filters of 7 x 7, stride 2, padding 3: both routes that serve it."""
    import workloads as W
    hi, ci, co, hf, s, p = W.CONV_FIRST_LAYER
    shape = (2, hi, hi, ci, co, hf, hf, s, p)
    assert gpu.mipgemm_conv_variant_name(*shape) == "implicit:rows"
    I, F = tensors(shape, 4)
    want = oracle.conv_direct(I, F, s, p)
    got = run_conv(gpu, shape, I, F, np.zeros(want.shape, dtype=np.int32), 0)
    assert np.array_equal(got, want)
    with Env(MIPGEMM_CONV="im2col"):
        assert gpu.mipgemm_conv_variant_name(*shape).startswith("im2col+")
    got = run_conv(gpu, shape, I, F, np.zeros(want.shape, dtype=np.int32), 0, MIPGEMM_CONV="im2col")
    assert np.array_equal(got, want)


def test_conv_batch_32_layer_in_full(gpu, oracle):
    """The (64, 100352, 576) GEMM of the conv workload, as the convolution it stands for."""
    shape = (32, 56, 56, 64, 64, 3, 3, 1, 1)
    assert gpu.mipgemm_conv_variant_name(*shape) == "implicit:mfma_dma256x64"
    I, F = tensors(shape, 5)
    want = oracle.conv_direct(I, F, 1, 1)
    got = run_conv(gpu, shape, I, F, np.zeros(want.shape, dtype=np.int32), 0)
    assert np.array_equal(got, want)


def _network_layers():
    import workloads as W
    return [(name, geo) for (name, geo, count) in W.resnet50_conv_layers()]


@pytest.mark.parametrize("name,geo", _network_layers(), ids=lambda x: x if isinstance(x, str) else None)
def test_every_distinct_layer_of_the_network(gpu, oracle, name, geo):
    """The 23 distinct convolutions of the ResNet-50-type network, one image, bit for bit."""
    import workloads as W
    hi, ci, co, hf, stride, pad = geo
    shape = (1, hi, hi, ci, co, hf, hf, stride, pad)
    print("layer", name, shape, flush=True)
    image, filt = W.conv_tensors(1, geo)
    want = oracle.conv_direct(image, filt, stride, pad)
    got = run_conv(gpu, shape, image, filt, np.full(want.shape, -3, dtype=np.int32), 0)
    assert np.array_equal(got, want)


IM2COL_SHAPES = [(2, 9, 8, 16, 3, 3, 1, 1), (1, 14, 14, 64, 3, 3, 2, 1), (3, 7, 7, 48, 1, 1, 1, 0),
                 (1, 12, 10, 3, 7, 7, 2, 3), (2, 6, 5, 5, 2, 3, 1, 1), (1, 20, 20, 32, 5, 5, 3, 2),
                 (1, 40, 40, 512, 3, 3, 1, 1)]


@pytest.mark.parametrize("extra", [0, 16, 5])
@pytest.mark.parametrize("shape", IM2COL_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_im2col_matches_the_oracle(gpu, oracle, shape, extra):
    import torch
    print("im2col", shape, extra, flush=True)
    b, hi, wi, ci, hf, wf, s, p = shape
    rng = np.random.default_rng(list(shape))
    I = rng.integers(1, 256, size=(b, hi, wi, ci), dtype=np.uint8)
    ldm = hf * wf * ci + extra
    want = oracle.im2col_u8(I, hf, wf, s, p, ldm=ldm, fill=0x5A)
    dM = torch.full(want.shape, 0x5A, dtype=torch.uint8, device="cuda")
    gpu.mipgemm_im2col_u8(b, hi, wi, ci, hf, wf, s, p, torch.from_numpy(I).cuda(), dM, ldm)
    torch.cuda.synchronize()
    assert np.array_equal(dM.cpu().numpy(), want)            # row tails keep their sentinel


def test_conv_errors_and_empty(gpu):
    import torch
    shape = (1, 8, 8, 3, 4, 3, 3, 1, 1)
    with Env(MIPGEMM_CONV="im2col"):
        _conv_errors_and_empty(gpu, shape)


def _conv_errors_and_empty(gpu, shape):
    import torch
    need = gpu.mipgemm_conv_workspace_size(*shape)
    assert need == (256 + 256) * 64                          # positions and filters in tiles of 256, k 27 -> 64
    dI = torch.zeros(8 * 8 * 3, dtype=torch.uint8, device="cuda")
    dF = torch.zeros(4 * 27, dtype=torch.uint8, device="cuda")
    dO = torch.full((64 * 4,), 9, dtype=torch.int32, device="cuda")
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    b, hi, wi, ci, co, hf, wf, s, p = shape
    call = gpu.mipgemm_conv_s8u8s32
    assert call(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, 0, check=False) == -14
    assert call(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, 0, ws, need - 1, check=False) == -15
    assert call(b, hi, wi, ci, co, 11, wf, s, p, dF, dI, dO, 0, ws, need, check=False) == -6
    assert call(b, hi, wi, ci, co, hf, wf, 0, p, dF, dI, dO, 0, ws, need, check=False) == -8
    assert call(b, hi, wi, ci, co, hf, wf, s, -1, dF, dI, dO, 0, ws, need, check=False) == -9
    assert call(b, hi, wi, ci, co, hf, wf, s, p, None, dI, dO, 0, ws, need, check=False) == -10
    assert call(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, 5, ws, need, check=False) == -13
    assert call(0, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, 0, check=False) == 0
    torch.cuda.synchronize()
    assert (dO.cpu().numpy() == 9).all()                     # none of these touched O
    assert gpu.mipgemm_im2col_u8(1, 8, 8, 3, 3, 3, 1, 1, dI, ws, 26, check=False) == -11


@pytest.mark.parametrize("path", ["implicit", "im2col"])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape,scale", [((2, 28, 28, 128, 128, 3, 3, 1, 1), 0.0123),
                                         ((1, 17, 23, 64, 96, 3, 5, 2, 2), 2.0 ** -9),
                                         ((4, 7, 7, 512, 512, 3, 3, 1, 1), -3.3e-5),
                                         ((2, 12, 12, 3, 8, 5, 5, 1, 2), 0.5)],
                         ids=lambda x: "x".join(map(str, x)) if isinstance(x, tuple) else None)
def test_dequantised_conv(gpu, oracle, shape, scale, mode, path):
    """Float output = scale * integer sum (+ old O): within the two roundings the header states of
    the exact value, and for overwrite bit-equal to the same two IEEE operations done in numpy."""
    import torch
    print("conv f32", shape, scale, mode, path, flush=True)
    b, hi, wi, ci, co, hf, wf, s, p = shape
    I, F = tensors(shape, 6)
    S = oracle.conv_direct(I, F, s, p).astype(np.float64)            # exact integers
    rng = np.random.default_rng(8)
    O0 = (rng.standard_normal(S.shape) * 50).astype(np.float32)
    sc = float(np.float32(scale))
    want = sc * S + (O0.astype(np.float64) if mode else 0.0)
    dO = torch.from_numpy(O0.copy()).cuda()
    env = {"MIPGEMM_CONV": None if path == "implicit" else "im2col"}
    with Env(**env):
        need = gpu.mipgemm_conv_workspace_size(*shape)
        ws = torch.zeros(max(need, 16), dtype=torch.uint8, device="cuda")
        gpu.mipgemm_conv_s8u8f32(b, hi, wi, ci, co, hf, wf, s, p,
                                 torch.from_numpy(F.view(np.uint8)).cuda(),
                                 torch.from_numpy(I).cuda(), dO, mode, workspace=ws,
                                 workspace_bytes=need, scale=scale)
    torch.cuda.synchronize()
    got = dO.cpu().numpy().astype(np.float64)
    bound = 2.0 ** -23 * (np.abs(want) + (np.abs(O0) if mode else 0.0))
    assert (np.abs(got - want) <= bound).all()
    if mode == 0:
        assert np.array_equal(got.astype(np.float32), S.astype(np.float32) * np.float32(scale))


def test_dequantised_conv_rejects_a_bad_scale(gpu):
    import torch
    z = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    o = torch.zeros(4096, dtype=torch.float32, device="cuda")
    rc = gpu.mipgemm_conv_s8u8f32(1, 4, 4, 64, 4, 3, 3, 1, 1, z, z, o, 0, scale=float("nan"),
                                  check=False)
    assert rc == -17
    assert gpu.mipgemm_conv_s8u8f32(1, 4, 4, 64, 4, 3, 3, 1, 1, z, z, o, 3, scale=float("inf"),
                                    check=False) == -13


# ---------------------------------------------------------------------------
# weight pre-packing
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("k,n,order,pad,ppad", [
    (64, 64, 0, 0, 0), (4096, 4096, 0, 0, 0), (513, 4097, 0, 17, 3), (130, 200, 0, 16, 16),
    (1, 9, 0, 0, 0), (200, 1, 0, 0, 5), (100, 37, 1, 5, 0), (4096, 1024, 1, 16, 32),
    (77, 129, 1, 0, 3), (11008, 256, 0, 0, 0)])
def test_pack_b_matches_the_oracle(gpu, oracle, k, n, order, pad, ppad):
    import torch
    print("pack", k, n, order, pad, ppad, flush=True)
    rng = np.random.default_rng([k, n, order, pad])
    ldb = (n if order == 0 else k) + pad
    flat = rng.integers(0, 256, size=(k if order == 0 else n) * ldb, dtype=np.uint8)
    ldp = k + ppad
    want = oracle.pack_b(k, n, flat, ldb, order, ldp=ldp, fill=0x5A)
    dP = torch.full((n * ldp,), 0x5A, dtype=torch.uint8, device="cuda")
    gpu.mipgemm_pack_b(k, n, torch.from_numpy(flat).cuda(), ldb, order, dP, ldp)
    torch.cuda.synchronize()
    assert np.array_equal(dP.cpu().numpy().reshape(n, ldp), want)   # column tails keep their sentinel


def test_packed_weights_give_the_same_gemm_through_the_skinny_kernel(gpu, oracle):
    import torch
    import workloads as W
    case = W.Case("packed_decode", 8, 0, 16, 4096, 1024, seed=41)           # row-major B
    ops = W.materialize(case)
    want = ops.C.copy()
    oracle.gemm(False, False, case.m, case.n, case.k, ops.A, case.lda, 0, ops.B, case.ldb, 0,
                want, case.ldc, 0, 0)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dP = torch.empty(case.n * case.k, dtype=torch.uint8, device="cuda")
    dC = torch.from_numpy(ops.C).cuda()
    gpu.mipgemm_pack_b(case.k, case.n, dB, case.ldb, 0, dP, case.k)
    assert gpu.mipgemm_variant_name(case.m, case.n, case.k, case.lda, 0, case.k, 1, case.ldc,
                                    0) == "mfma_slab16"
    gpu.mipgemm_s8s8s32(case.m, case.n, case.k, dA, case.lda, 0, dP, case.k, 1, dC, case.ldc, 0, 0)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)


def test_pack_b_errors(gpu):
    import torch
    z = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    f = gpu.mipgemm_pack_b
    assert f(-1, 4, z, 4, 0, z, 4, check=False) == -1
    assert f(4, -1, z, 4, 0, z, 4, check=False) == -2
    assert f(4, 4, None, 4, 0, z, 4, check=False) == -3
    assert f(4, 8, z, 7, 0, z, 4, check=False) == -4
    assert f(4, 8, z, 8, 2, z, 4, check=False) == -5
    assert f(4, 8, z, 8, 0, None, 4, check=False) == -6
    assert f(4, 8, z, 8, 0, z, 3, check=False) == -7
    assert f(0, 8, None, 8, 0, None, 1, check=False) == 0


@pytest.mark.parametrize("shape", [(2, 64, 48, 3, 64, 7, 7, 2, 3), (2, 28, 28, 128, 128, 3, 3, 1, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_convolution_replays_from_a_hip_graph(gpu, oracle, shape):
    """A captured convolution (row-segment kernel; tile kernel that gathers) gives the oracle's
    result on every replay, with O overwritten by other work between the replays."""
    import torch
    print("conv graph", shape, flush=True)
    b, hi, wi, ci, co, hf, wf, s, p = shape
    assert gpu.mipgemm_conv_workspace_size(*shape) == 0
    I, F = tensors(shape, 11)
    want = oracle.conv_direct(I, F, s, p)
    dI, dF = torch.from_numpy(I).cuda(), torch.from_numpy(F.view(np.uint8)).cuda()
    dO = torch.zeros(want.shape, dtype=torch.int32, device="cuda")

    def call():
        gpu.mipgemm_conv_s8u8s32(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, 0)

    call()
    torch.cuda.synchronize()
    assert np.array_equal(dO.cpu().numpy(), want)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for replay in range(4):
        dO.fill_(replay - 7)                         # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(dO.cpu().numpy(), want), "replay %d" % replay


# neither gathering kernel serves these (channels not a multiple of 64, k too long for the
# row-segment kernel): the written-out route, whose matrix and filters are padded to whole
# k blocks so that the direct-to-LDS kernels multiply them
WRITTEN_OUT_SHAPES = [(2, 14, 14, 96, 40, 3, 3, 1, 1), (1, 10, 10, 160, 70, 3, 3, 2, 1),
                      (2, 9, 9, 48, 33, 5, 5, 1, 2), (1, 30, 30, 96, 300, 3, 3, 1, 0)]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", WRITTEN_OUT_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_on_the_written_out_route_by_default(gpu, oracle, shape, mode):
    print("conv written out", shape, mode, flush=True)
    name = gpu.mipgemm_conv_variant_name(*shape)
    assert name.startswith("im2col+mfma_dma") or name.startswith("im2col+mfma_slab"), name
    I, F = tensors(shape, 12)
    ho = oracle.conv_out_extent(shape[1], shape[5], shape[7], shape[8])
    wo = oracle.conv_out_extent(shape[2], shape[6], shape[7], shape[8])
    rng = np.random.default_rng(13)
    O0 = rng.integers(-1000, 1000, size=(shape[0], ho, wo, shape[4]), dtype=np.int32)
    want = oracle.conv_direct(I, F, shape[7], shape[8], O=O0.copy() if mode else None, mode=mode)
    got = run_conv(gpu, shape, I, F, O0, mode)
    assert np.array_equal(got, want)


def test_seeded_sweep_of_random_convolutions(gpu, oracle):
    """60 random geometries (1-48 channels, filters up to 7 x 7, strides 1-3, paddings 0-4, up to
    139 filters, both modes), each on the route the library picks and on the row-segment kernel
    where that can serve."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 60:
        ci = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 24, 32, 48]))
        hf, wf = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        s, p = int(rng.integers(1, 4)), int(rng.integers(0, 5))
        hi, wi = int(rng.integers(1, 40)), int(rng.integers(1, 300))
        if hi + 2 * p < hf or wi + 2 * p < wf:
            continue
        b, co = int(rng.integers(1, 4)), int(rng.integers(1, 140))
        shape = (b, hi, wi, ci, co, hf, wf, s, p)
        mode = int(rng.integers(0, 2))
        I = rng.integers(0, 256, size=(b, hi, wi, ci), dtype=np.uint8)
        F = rng.integers(-128, 128, size=(co, hf, wf, ci), dtype=np.int8)
        ho, wo = (hi + 2 * p - hf) // s + 1, (wi + 2 * p - wf) // s + 1
        O0 = rng.integers(-1000, 1000, size=(b, ho, wo, co), dtype=np.int32)
        want = oracle.conv_direct(I, F, s, p, O=O0.copy() if mode else None, mode=mode)
        for route in (None, "rows"):
            with Env(MIPGEMM_CONV=route):
                name = gpu.mipgemm_conv_variant_name(*shape)
            print("conv sweep", shape, mode, route, name, flush=True)
            got = run_conv(gpu, shape, I, F, O0, mode, MIPGEMM_CONV=route)
            assert np.array_equal(got, want), (shape, mode, route, name)
        done += 1


# ---------------------------------------------------------------------------
# the filters' k-sums supplied (mipgemm_conv_filter_sums, mipgemm_conv_*_with_sums)
# ---------------------------------------------------------------------------

def _filter_sums(M, oracle, F):
    """The sums on the device, checked against the oracle's column sums of the filter matrix
    (c_o columns of k = h_f w_f c_i signed bytes, k contiguous)."""
    import torch
    co, k = F.shape[0], int(np.prod(F.shape[1:]))
    dF = torch.from_numpy(F.view(np.uint8)).cuda()
    dS = torch.full((co + 4,), 0x55555555, dtype=torch.int32, device="cuda")
    M.mipgemm_conv_filter_sums(co, k, dF, dS)
    torch.cuda.synchronize()
    got = dS.cpu().numpy()
    want = oracle.column_sums(k, co, F.reshape(-1), k, oracle.COL_MAJOR)
    assert np.array_equal(got[:co], want) and (got[co:] == 0x55555555).all()
    return dS


def _run_conv_with_sums(M, shape, I, F, O0, mode, dS, **env):
    import torch
    b, hi, wi, ci, co, hf, wf, s, p = shape
    dI, dF = torch.from_numpy(I).cuda(), torch.from_numpy(F.view(np.uint8)).cuda()
    dO = torch.from_numpy(O0.copy()).cuda()
    with Env(**env):
        need = M.mipgemm_conv_workspace_size(*shape)
        ws = torch.full((need + 64,), 0x5A, dtype=torch.uint8, device="cuda") if need else None
        M.mipgemm_conv_s8u8s32_with_sums(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, mode, dS,
                                         workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    return dO.cpu().numpy()


@pytest.mark.parametrize("path", ["implicit", "im2col"])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_with_filter_sums(gpu, oracle, shape, mode, path):
    print("conv with sums", shape, "mode", mode, "path", path, flush=True)
    I, F = tensors(shape, 1)
    dS = _filter_sums(gpu, oracle, F)
    ho = oracle.conv_out_extent(shape[1], shape[5], shape[7], shape[8])
    wo = oracle.conv_out_extent(shape[2], shape[6], shape[7], shape[8])
    rng = np.random.default_rng(3)
    O0 = rng.integers(-1000, 1000, size=(shape[0], ho, wo, shape[4]), dtype=np.int32)
    want = oracle.conv_direct(I, F, shape[7], shape[8], O=O0.copy() if mode else None, mode=mode)
    got = _run_conv_with_sums(gpu, shape, I, F, O0, mode, dS,
                              MIPGEMM_CONV=None if path == "implicit" else "im2col")
    assert np.array_equal(got, want)


@pytest.mark.parametrize("variant,splits", [("dma256", None), ("dma128", None), ("dma64", None), ("dma64", 3),
                                            ("dma64x256", None), ("dma256x64", None), ("dma128x64", None),
                                            ("dma64x128", None)])
def test_conv_with_filter_sums_under_every_tile_shape(gpu, oracle, variant, splits):
    """The gathering tile kernel in its form that takes the sums (and, with split k, the form
    that ignores them), ragged tiles in both dimensions."""
    shape = (1, 17, 23, 64, 96, 3, 5, 2, 2)
    I, F = tensors(shape, 2)
    dS = _filter_sums(gpu, oracle, F)
    want = oracle.conv_direct(I, F, shape[7], shape[8])
    with Env(MIPGEMM_VARIANT=variant, MIPGEMM_SPLITK=splits):
        assert gpu.mipgemm_conv_variant_name(*shape) == "implicit:mfma_" + variant
    got = _run_conv_with_sums(gpu, shape, I, F, np.full(want.shape, 77, dtype=np.int32), 0, dS,
                              MIPGEMM_VARIANT=variant, MIPGEMM_SPLITK=splits)
    assert np.array_equal(got, want)


def test_conv_with_filter_sums_odd_channels_and_float_output(gpu, oracle):
    """Routes that compute their own sums (row-segment kernel), filters whose k is not a multiple
    of 16 (byte-wise sums), and the float-output form."""
    import torch
    for shape in ((2, 20, 300, 3, 10, 3, 3, 1, 1), (1, 12, 12, 24, 70, 3, 3, 1, 1)):
        I, F = tensors(shape, 5)
        dS = _filter_sums(gpu, oracle, F)
        want = oracle.conv_direct(I, F, shape[7], shape[8])
        got = _run_conv_with_sums(gpu, shape, I, F, np.zeros(want.shape, dtype=np.int32), 0, dS)
        assert np.array_equal(got, want)
    shape = (2, 14, 14, 64, 96, 3, 3, 1, 1)
    b, hi, wi, ci, co, hf, wf, s, p = shape
    I, F = tensors(shape, 6)
    dS = _filter_sums(gpu, oracle, F)
    scale = np.float32(0.0123)
    S = oracle.conv_direct(I, F, s, p)
    want = (S.astype(np.float32) * scale).astype(np.float32)       # int -> float32, one float32 multiply
    dO = torch.zeros(S.size, dtype=torch.float32, device="cuda")
    gpu.mipgemm_conv_s8u8f32_with_sums(b, hi, wi, ci, co, hf, wf, s, p, torch.from_numpy(F.view(np.uint8)).cuda(),
                                       torch.from_numpy(I).cuda(), dO, 0, dS, scale=float(scale))
    torch.cuda.synchronize()
    assert np.array_equal(dO.cpu().numpy(), want.reshape(-1))
    # a null pointer for the sums is argument 17
    dI = torch.from_numpy(I).cuda()
    dF = torch.from_numpy(F.view(np.uint8)).cuda()
    dOi = torch.full((S.size,), 5, dtype=torch.int32, device="cuda")
    assert gpu.mipgemm_conv_s8u8s32_with_sums(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dOi, 0, None,
                                              check=False) == -17
    torch.cuda.synchronize()
    assert (dOi.cpu().numpy() == 5).all()


# ---------------------------------------------------------------------------
# int8 output requantised for the next layer (mipgemm_conv_s8u8s8)
# ---------------------------------------------------------------------------

def _conv_requant_oracle(oracle, shape, I, F, scale):
    """clip(rint(scale * conv)) through two pinned oracle functions: the augmented matrix, then
    the requantising GEMM oracle on it (O is the column-major c_o x (b h_o w_o) result)."""
    b, hi, wi, ci, co, hf, wf, s, p = shape
    Mx = oracle.im2col_u8(I, hf, wf, s, p)                 # rows = output positions, k contiguous
    rows, k = Mx.shape
    Q = np.zeros(rows * co, dtype=np.int8)
    oracle.gemm_requant(False, True, co, rows, k, F.reshape(-1), k, oracle.ROW_MAJOR,
                        Mx.reshape(-1), k, oracle.COL_MAJOR, scale, Q, co, oracle.COL_MAJOR)
    return Q


@pytest.mark.parametrize("env", [{}, {"MIPGEMM_CONV": "im2col"}], ids=["as_dispatched", "written_out"])
@pytest.mark.parametrize("shape", CONV_SHAPES + ROWS_SHAPES[:6], ids=lambda s: "x".join(map(str, s)))
def test_conv_with_int8_output(gpu, oracle, shape, env):
    import torch
    print("conv s8 out", shape, env, flush=True)
    b, hi, wi, ci, co, hf, wf, s, p = shape
    I, F = tensors(shape, 7)
    S = oracle.conv_direct(I, F, s, p)
    scale = np.float32(100.0 / max(1.0, float(np.percentile(np.abs(S), 90))))   # about a tenth saturates
    want = _conv_requant_oracle(oracle, shape, I, F, scale)
    assert (want == 127).any() or (want == -128).any() or S.size < 50
    dI, dF = torch.from_numpy(I).cuda(), torch.from_numpy(F.view(np.uint8)).cuda()
    for with_sums in (False, True):
        dS = _filter_sums(gpu, oracle, F) if with_sums else None
        dO = torch.full((S.size + 32,), 0x11, dtype=torch.int8, device="cuda")
        with Env(**env):
            need = max(gpu.mipgemm_conv_workspace_size(*shape), gpu.mipgemm_conv_workspace_size_unaligned(*shape))
            ws = torch.zeros(need, dtype=torch.uint8, device="cuda") if need else None
            gpu.mipgemm_conv_s8u8s8(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, 0, dS, workspace=ws,
                                    workspace_bytes=need, scale=float(scale))
        torch.cuda.synchronize()
        got = dO.cpu().numpy()
        assert np.array_equal(got[:S.size], want), "with_sums=%s" % with_sums
        assert (got[S.size:] == 0x11).all()
    # accumulate mode is rejected, nothing touched
    dO = torch.full((S.size,), 0x11, dtype=torch.int8, device="cuda")
    assert gpu.mipgemm_conv_s8u8s8(b, hi, wi, ci, co, hf, wf, s, p, dF, dI, dO, 1, None, scale=1.0,
                                   check=False) == -13
    torch.cuda.synchronize()
    assert (dO.cpu().numpy() == 0x11).all()
