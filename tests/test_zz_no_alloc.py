"""The allocation-free GEMM entry point against the entry point it is a variant of.

mipgemm_s8s8s32_noalloc keeps the packed route's buffers in a static device array; its
results must be the bits mipgemm_s8s8s32 produces with a caller's workspace (and the
oracle's), call after call, whatever the previous call left in the array.
"""
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


def _run_both(M, oracle, case):
    import torch
    ops = W.materialize(case)
    want = ops.C.copy()
    oracle.gemm(case.a_unsigned, case.b_unsigned, case.m, case.n, case.k, ops.A, case.lda,
                case.orderA, ops.B, case.ldb, case.orderB, want, case.ldc, case.orderC, case.mode)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    need = M.mipgemm_workspace_size(case.m, case.n, case.k, case.orderA, case.orderB, case.orderC)
    assert 0 < need <= M.mipgemm_static_scratch_bytes()          # the packed route, and it fits
    assert M.mipgemm_variant_name_with_workspace(
        case.m, case.n, case.k, case.lda, case.orderA, case.ldb, case.orderB, case.ldc, case.orderC,
        False, False, True).startswith("packed+")
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    dC_ws = torch.from_numpy(ops.C).cuda()
    M.mipgemm_s8s8s32(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
                      dC_ws, case.ldc, case.orderC, case.mode, workspace=ws, workspace_bytes=need)
    dC = torch.from_numpy(ops.C).cuda()
    M.mipgemm_s8s8s32_noalloc(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb,
                              case.orderB, dC, case.ldc, case.orderC, case.mode)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    assert np.array_equal(got, dC_ws.cpu().numpy())              # bit for bit the existing entry point
    assert np.array_equal(got, want)                             # and the oracle, padding included


def test_two_calls_in_a_row_the_second_smaller(gpu, oracle):
    big = W.Case("noalloc_big", 8, 0, 1000, 999, 1001, orderB=W.COL_MAJOR, pad=17, mode=W.ACCUMULATE,
                 c_dist=("uniform", -1000, 1000), seed=71)
    small = W.Case("noalloc_small", 8, 1, 300, 200, 333, orderA=W.COL_MAJOR, pad=3, mode=W.OVERWRITE,
                   seed=71)
    _run_both(gpu, oracle, big)
    _run_both(gpu, oracle, small)      # finds the first call's packed operands in the array
    _run_both(gpu, oracle, big)        # and the other way round


def test_operands_that_need_no_buffer_run_in_place(gpu, oracle):
    import torch
    case = W.Case("noalloc_aligned", 8, 2, 256, 512, 1024, seed=71)
    ops = W.materialize(case)
    want = ops.C.copy()
    oracle.gemm(False, False, case.m, case.n, case.k, ops.A, case.lda, case.orderA, ops.B, case.ldb,
                case.orderB, want, case.ldc, case.orderC, case.mode)
    dC = torch.from_numpy(ops.C).cuda()
    gpu.mipgemm_s8s8s32_noalloc(case.m, case.n, case.k, torch.from_numpy(ops.A.view(np.uint8)).cuda(),
                                case.lda, case.orderA, torch.from_numpy(ops.B.view(np.uint8)).cuda(),
                                case.ldb, case.orderB, dC, case.ldc, case.orderC, case.mode)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)


def test_a_problem_beyond_the_static_buffer_is_rejected_and_touches_nothing(gpu):
    import torch
    m, n, k = 6001, 6001, 6001          # packed: (6144 + 6144) * 6016 bytes = 70.5 MiB > 64 MiB
    assert (6144 + 6144) * 6016 > gpu.mipgemm_static_scratch_bytes()
    dA = torch.zeros(m * k, dtype=torch.uint8, device="cuda")
    dB = torch.zeros(k * n, dtype=torch.uint8, device="cuda")
    dC = torch.full((m * n,), W.SENTINEL_WORD, dtype=torch.int32, device="cuda")
    rc = gpu.mipgemm_s8s8s32_noalloc(m, n, k, dA, k, W.ROW_MAJOR, dB, n, W.ROW_MAJOR, dC, n,
                                     W.ROW_MAJOR, W.OVERWRITE, check=False)
    torch.cuda.synchronize()
    assert rc == gpu.ERR_STATIC_SCRATCH
    assert "static" in gpu.mipgemm_strerror(rc)
    assert bool((dC == W.SENTINEL_WORD).all())
    # invalid arguments are reported as by mipgemm_s8s8s32
    assert gpu.mipgemm_s8s8s32_noalloc(-1, n, k, dA, k, 0, dB, n, 0, dC, n, 0, 0, check=False) == -1
    assert gpu.mipgemm_s8s8s32_noalloc(m, n, k, dA, k - 1, 0, dB, n, 0, dC, n, 0, 0, check=False) == -5
