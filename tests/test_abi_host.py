"""Host-side checks of the C-ABI library: it loads, exports what include/mipgemm.h declares,
validates arguments before touching the GPU, and picks kernel variants as documented."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def M():
    import paper_2506_11728_amd as M
    if not os.path.exists(M.library_path()):
        from paper_2506_11728_amd.build import build_library
        build_library()
    M.load_library()
    return M


def test_header_symbols_are_exported(M):
    header = open(os.path.join(ROOT, "include", "mipgemm.h")).read()
    declared = set(re.findall(r"\b(mipgemm_[a-z0-9_]+)\s*\(", header))
    assert declared == set(M.exported_symbols())
    lib = M.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def test_header_constants_match_binding(M):
    header = open(os.path.join(ROOT, "include", "mipgemm.h")).read()
    consts = dict(re.findall(r"#define\s+MIPGEMM_(\w+)\s+(\d+)\b", header))
    assert int(consts["ROW_MAJOR"]) == M.ROW_MAJOR and int(consts["COL_MAJOR"]) == M.COL_MAJOR
    assert int(consts["OVERWRITE"]) == M.OVERWRITE and int(consts["ACCUMULATE"]) == M.ACCUMULATE


def call(M, name="mipgemm_s8s8s32", m=4, n=5, k=6, A=4096, lda=6, oa=0, B=4096, ldb=5, ob=0,
         C=4096, ldc=5, oc=0, mode=0, ws=None, wsb=0):
    # stream=0 keeps torch out of it; every call below must fail validation, so nothing launches
    return getattr(M, name)(m, n, k, A, lda, oa, B, ldb, ob, C, ldc, oc, mode, ws, wsb, 0,
                            check=False)


@pytest.mark.parametrize("entry", ["mipgemm_s8s8s32", "mipgemm_u8s8s32", "mipgemm_s8u8s32"])
def test_argument_validation_codes(M, entry):
    assert call(M, entry, m=-1) == -1
    assert call(M, entry, n=-1) == -2
    assert call(M, entry, k=-1) == -3
    assert call(M, entry, m=2**31) == -1
    assert call(M, entry, A=0) == -4
    assert call(M, entry, lda=5) == -5               # row-major A needs lda >= k
    assert call(M, entry, oa=1, lda=3) == -5         # column-major A needs lda >= m
    assert call(M, entry, oa=2) == -6
    assert call(M, entry, B=0) == -7
    assert call(M, entry, ldb=4) == -8
    assert call(M, entry, ob=1, ldb=5) == -8         # column-major B needs ldb >= k
    assert call(M, entry, ob=-1) == -9
    assert call(M, entry, C=0) == -10
    assert call(M, entry, ldc=4) == -11
    assert call(M, entry, oc=1, ldc=3) == -11        # column-major C needs ldc >= m
    assert call(M, entry, oc=5) == -12
    assert call(M, entry, mode=2) == -13
    assert call(M, entry, lda=0, k=0) == -5          # leading dimensions are at least 1


@pytest.mark.parametrize("entry", ["mipgemm_s8s8f32", "mipgemm_u8s8f32", "mipgemm_s8u8f32"])
def test_dequant_entry_points_share_the_numbering(M, entry):
    def callf(scale=0.5, **kw):
        args = dict(m=4, n=5, k=6, A=4096, lda=6, oa=0, B=4096, ldb=5, ob=0, C=4096, ldc=5, oc=0,
                    mode=0)
        args.update(kw)
        return getattr(M, entry)(args["m"], args["n"], args["k"], args["A"], args["lda"],
                                 args["oa"], args["B"], args["ldb"], args["ob"], args["C"],
                                 args["ldc"], args["oc"], args["mode"], None, 0, 0, scale=scale,
                                 check=False)
    assert callf(m=-1) == -1
    assert callf(lda=5) == -5
    assert callf(C=0) == -10
    assert callf(ldc=4) == -11
    assert callf(mode=3) == -13
    assert callf(scale=float("inf"), m=0) == -17
    assert callf(scale=float("nan"), lda=5) == -5
    assert "17" in M.mipgemm_strerror(-17)


def test_first_bad_argument_wins(M):
    assert call(M, m=-1, n=-1, mode=9) == -1
    assert call(M, lda=1, ldb=1, ldc=1) == -5


def test_empty_problems_need_no_pointers(M):
    assert call(M, m=0, A=0, C=0) == 0
    assert call(M, n=0, B=0, C=0, ldb=1, ldc=1) == 0
    assert call(M, k=0, A=0, B=0, lda=1, mode=1) == 0     # accumulate of an empty sum: no-op


def test_strerror_and_workspace(M):
    assert M.mipgemm_strerror(0) == "success"
    for code in range(-17, 0):
        assert str(-code) in M.mipgemm_strerror(code)
    assert "unknown" in M.mipgemm_strerror(-99)
    assert M.mipgemm_workspace_size(8192, 8192, 8192, 0, 0, 0) == 0
    # odd sizes that are worth packing: rows in whole tiles of 256, k padded to 64 (128 from 1024 on)
    assert M.mipgemm_workspace_size(1000, 999, 1001, 0, 0, 0) == (1024 + 1024) * 1024
    assert M.mipgemm_workspace_size(1000, 999, 1001, 1, 1, 1) == (1024 + 1024) * 1024
    assert M.mipgemm_workspace_size(300, 200, 333, 0, 0, 0) == (512 + 256) * 384
    assert M.mipgemm_workspace_size(4096, 4096, 4100, 0, 0, 0) == (4096 + 4096) * 4224
    assert M.mipgemm_workspace_size(64, 1000, 1001, 0, 0, 0) == 0          # skinny: packing does not pay
    assert M.mipgemm_workspace_size(3000, 5000, 65, 0, 0, 0) == 0          # short k: neither
    assert M.mipgemm_workspace_size(2**31 - 1, 2**31 - 1, 2**31 - 1, 0, 0, 0) == 0   # nothing overflows
    assert M.mipgemm_workspace_size(-1, 5, 5, 0, 0, 0) == 0 and M.mipgemm_workspace_size(5, 5, 5, 0, 3, 0) == 0


def test_variant_choice(M):
    name = M.mipgemm_variant_name
    assert name(8192, 8192, 8192, 8192, 0, 8192, 0, 8192, 0) == "mfma_dma256_k128"
    assert name(4096, 4096, 4096, 4096, 0, 4096, 0, 4096, 0) == "mfma_dma256_k128"
    assert name(4096, 4096, 1024, 1024, 0, 4096, 0, 4096, 0) == "mfma_dma256_k128"
    assert name(4096, 4096, 1088, 1088, 0, 4096, 0, 4096, 0) == "mfma_dma256"        # k % 128 != 0
    assert name(4352, 4352, 4096, 4096, 0, 4352, 0, 4352, 0) == "mfma_dma128_k128"      # 289 tiles of 256 x 256: a second round for 33
    assert name(4608, 4608, 4096, 4096, 0, 4608, 0, 4608, 0) == "mfma_dma256_k128"
    # unaligned operands cannot use the direct-to-LDS kernels
    assert name(8192, 8192, 8192, 8192, 0, 8192, 0, 8192, 0, aligned16=False) == "mfma_tile128x64"
    # a ragged row edge can, with the general form of the deep-k kernel; an unsigned operand can
    assert name(8191, 8192, 8192, 8192, 0, 8192, 0, 8192, 0) == "mfma_dma256_k128_ragged"
    assert name(8192, 8192, 8256, 8256, 0, 8192, 0, 8192, 0) == "mfma_dma256"        # k % 128 != 0
    assert name(8192, 8192, 8192, 8192, 0, 8192, 0, 8192, 0, a_unsigned=True) == "mfma_dma256_k128"
    # a row-major B with n not a multiple of 16 cannot
    assert name(8192, 8191, 8192, 8192, 0, 8192, 0, 8192, 0) == "mfma_tile128x64"
    # short in one dimension: a tile that is short there too
    assert name(16, 4096, 4096, 4096, 0, 4096, 0, 4096, 0) == "mfma_dma64"
    assert name(64, 100352, 576, 576, 0, 100352, 0, 100352, 0) == "mfma_dma64x256"
    # a few rows against a k-contiguous B, or a short k with few tiles: one workgroup per slab of B
    assert name(16, 4096, 4096, 4096, 0, 4096, 1, 4096, 0) == "mfma_slab16"
    assert name(1, 11008, 4096, 4096, 0, 4096, 1, 11008, 0) == "mfma_slab16"
    assert name(64, 4096, 4096, 4096, 0, 4096, 1, 4096, 0) == "mfma_dma64"
    assert name(64, 3136, 576, 576, 0, 3136, 0, 3136, 0, b_unsigned=True) == "mfma_slab16"
    assert name(16, 4096, 4096, 4096, 0, 4096, 1, 4096, 0, aligned16=False) == "mfma_tile64"
    assert name(64, 100352, 576, 576, 0, 100352, 0, 100352, 0, aligned16=False) == "mfma_tile64x256"
    assert name(4095, 3, 2049, 2049, 0, 3, 0, 3, 0) == "mfma_tile64"
    assert name(100000, 3, 2049, 2049, 0, 3, 0, 3, 0) == "mfma_tile256x64"
    # column-major C swaps the operand roles
    assert name(64, 100352, 576, 576, 0, 100352, 0, 64, 1) == "mfma_dma256x64"
    # unsigned operands and ragged m / n edges stay on the direct-to-LDS kernels: with 128-deep
    # blocks from k = 768 on (k a multiple of 128), the 64-deep kernel below and otherwise
    assert name(1000, 3072, 768, 768, 0, 3072, 0, 3072, 0, a_unsigned=True) == "mfma_dma128_k128_split"
    assert name(1000, 3072, 512, 512, 0, 3072, 0, 3072, 0, a_unsigned=True) == "mfma_dma128"
    assert name(1000, 3072, 832, 832, 0, 3072, 0, 3072, 0, a_unsigned=True) == "mfma_dma128"
    # an accumulating call with an unsigned operand stays on the large tile
    assert M.mipgemm_variant_name_for_mode(4096, 4096, 2048, 2048, 0, 4096, 0, 4096, 0, True, False, True,
                                           1) == "mfma_dma256_k128"
    assert M.mipgemm_variant_name_for_mode(4000, 4000, 2048, 2048, 0, 4000, 0, 4000, 0, True, False, True,
                                           1) == "mfma_dma256_k128_ragged"
    # whole 128 x 128 tiles and 128-deep k blocks: the kernel for large problems on that tile shape
    assert name(1024, 3072, 768, 768, 0, 3072, 0, 3072, 0, a_unsigned=True) == "mfma_dma128_k128"
    assert name(2048, 2048, 2048, 2048, 0, 2048, 0, 2048, 0) == "mfma_dma128_k128"
    # three quarters of a round of 64 x 128 tiles, long side along the row-major B
    assert name(256, 6272, 2304, 2304, 0, 6272, 0, 6272, 0) == "mfma_dma64x128"
    assert name(6272, 256, 2304, 2304, 0, 256, 0, 256, 0) == "mfma_dma64x128"
    # a very long k over few tiles: the 128 x 128 tiles with 128-deep blocks, k in ranges (an
    # accumulating call, which needs no zero-fill launch, from a shorter k on)
    assert name(768, 768, 8192, 8192, 0, 768, 0, 768, 0) == "mfma_dma128_k128_split"
    assert name(512, 1568, 16384, 16384, 0, 1568, 0, 1568, 0, b_unsigned=True) == "mfma_dma128_k128_split"
    assert name(768, 768, 6144, 6144, 0, 768, 0, 768, 0) == "mfma_dma64"
    assert M.mipgemm_variant_name_for_mode(768, 768, 6144, 6144, 0, 768, 0, 768, 0, False, False, True,
                                           1) == "mfma_dma128_k128_split"
    assert name(768, 776, 8192, 8192, 0, 776, 0, 776, 0) != "mfma_dma128_k128_split"   # n % 16 on a row-major B
    assert name(2048, 2048, 8192, 8192, 0, 2048, 0, 2048, 0) == "mfma_dma128_k128"     # enough tiles
    # k not a multiple of 64 does not
    assert name(1000, 3072, 770, 784, 0, 3072, 0, 3072, 0) == "mfma_tile128x64"
    assert name(4, 4, 0, 1, 0, 4, 0, 4, 0) == "fill_zero"
    assert name(0, 4, 4, 4, 0, 4, 0, 4, 0) == "none"
    assert name(4, 4, 4, 1, 0, 4, 0, 4, 0) == "invalid"
    assert name(256, 256, 256, 256, 0, 256, 0, 256, 0) == "mfma_dma64"


def test_binding_fails_loudly_without_library(M, monkeypatch):
    import paper_2506_11728_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libmipgemm.so")
    with pytest.raises(ImportError):
        b.load_library()


def test_conv_argument_validation_codes(M):
    """Every call below fails validation (or is empty), so nothing is launched: no GPU needed."""
    def conv(b=2, hi=8, wi=8, ci=64, co=16, hf=3, wf=3, stride=1, pad=1, F=4096, I=4096, O=4096,
             mode=0, ws=None, wsb=0):
        return M.mipgemm_conv_s8u8s32(b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, ws, wsb,
                                      0, check=False)
    assert conv(b=-1) == -1
    assert conv(hi=0) == -2
    assert conv(wi=0) == -3
    assert conv(ci=0) == -4
    assert conv(co=-1) == -5
    assert conv(hf=0) == -6
    assert conv(hf=11) == -6                         # 11 > 8 + 2 * 1: the filter does not fit
    assert conv(wf=11) == -7
    assert conv(stride=0) == -8
    assert conv(pad=-1) == -9
    assert conv(F=0) == -10
    assert conv(I=0) == -11
    assert conv(O=0) == -12
    assert conv(mode=2) == -13
    assert conv(ci=96) == -14                        # no kernel gathers these: the written-out route needs a workspace
    assert conv(ci=96, ws=4096, wsb=10) == -15
    assert conv(b=2**31) == -1
    assert conv(b=70000, hi=256, wi=256, ci=64) == -1    # the image tensor must stay below 2^31 bytes
    assert conv(b=1, hi=2**31 - 1, wi=1, ci=1, pad=2**31 - 1, hf=1, wf=1) == -9   # output extent beyond 2^31
    assert conv(b=0, I=0, O=0) == 0
    assert conv(co=0, F=0, O=0) == 0

    def im2col(b=2, hi=8, wi=8, ci=3, hf=3, wf=3, stride=1, pad=1, I=4096, Mat=4096, ldm=27):
        return M.mipgemm_im2col_u8(b, hi, wi, ci, hf, wf, stride, pad, I, Mat, ldm, 0, check=False)
    assert im2col(hf=0) == -5
    assert im2col(wf=12) == -6
    assert im2col(stride=0) == -7
    assert im2col(pad=-2) == -8
    assert im2col(I=0) == -9
    assert im2col(Mat=0) == -10
    assert im2col(ldm=26) == -11
    assert im2col(b=0, I=0, Mat=0) == 0


def test_conv_path_choice_and_workspace(M):
    name, ws = M.mipgemm_conv_variant_name, M.mipgemm_conv_workspace_size
    # channel counts that are multiples of 64 are gathered inside the GEMM kernel: no workspace
    assert name(32, 56, 56, 64, 64, 3, 3, 1, 1) == "implicit:mfma_dma256x64"
    assert ws(32, 56, 56, 64, 64, 3, 3, 1, 1) == 0
    assert name(32, 28, 28, 128, 128, 3, 3, 1, 1) == "implicit:mfma_dma128x64"
    assert name(1, 7, 7, 512, 2048, 1, 1, 1, 0).startswith("implicit:")
    # the 3-channel first layer is gathered too, from image row segments staged in LDS
    assert name(2, 64, 48, 3, 64, 7, 7, 2, 3) == "implicit:rows"
    assert ws(2, 64, 48, 3, 64, 7, 7, 2, 3) == 0
    # 96 channels: not a multiple of 64, k too long for the row-segment kernel: the augmented
    # matrix is written out, k padded to whole k blocks, and the filters re-pitched behind it
    assert name(2, 8, 8, 96, 16, 3, 3, 1, 1).startswith("im2col+")
    assert ws(2, 8, 8, 96, 16, 3, 3, 1, 1) == (256 + 256) * 896   # rows and filters in tiles of 256, k 864 -> 896
    assert name(0, 8, 8, 64, 16, 3, 3, 1, 1) == "none"
    assert name(2, 8, 8, 64, 16, 13, 3, 1, 1) == "invalid"
    assert ws(2, 8, 8, 64, 16, 13, 3, 1, 1) == 0


@pytest.mark.parametrize("entry", ["mipgemm_s8s8s32_batched", "mipgemm_u8s8s32_batched",
                                   "mipgemm_s8u8s32_batched"])
def test_batched_entry_point_validation(M, entry):
    def call_b(m=4, n=5, k=6, A=4096, lda=6, oa=0, sa=24, B=4096, ldb=5, ob=0, sb=30, C=4096, ldc=5,
               oc=0, sc=20, batch=3, mode=0):
        return getattr(M, entry)(m, n, k, A, lda, oa, sa, B, ldb, ob, sb, C, ldc, oc, sc,
                                 batch, mode, None, 0, 0, check=False)
    assert call_b(m=-1) == -1
    assert call_b(lda=5) == -5
    assert call_b(sa=-1) == -7
    assert call_b(B=0) == -8
    assert call_b(ob=3) == -10
    assert call_b(sb=-1) == -11
    assert call_b(C=0) == -12
    assert call_b(ldc=4) == -13
    assert call_b(oc=2) == -14
    assert call_b(sc=-5) == -15
    assert call_b(batch=-1) == -16
    assert call_b(batch=65536) == -16
    assert call_b(mode=7) == -17
    assert call_b(sa=-1, lda=5) == -5                 # the lowest-numbered bad argument wins
    assert call_b(batch=0) == 0                      # nothing to do, nothing launched
    for code in (-18, -19, -20):
        assert str(-code) in M.mipgemm_strerror(code)
