"""GPU parity of the dequantised-output entry points (paper Section 7.3, C^r = s_A s_B C^q).

Floating point: compared with the fp64 oracle within the bound the arithmetic gives.  The
kernels convert the exact int32 sum to float (one rounding, relative 2^-24) and multiply by
the scale, or fuse multiply and add onto the old float (one more rounding, relative 2^-24 of
the result), so |got - want| <= 2^-23 * (|want| + |C0|).  Overwrite results are also compared
bit for bit with the same two float operations done by numpy.
"""
import os

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


def _cases():
    out = []
    idx = 0
    shapes = [(256, 256, 256), (300, 200, 333), (64, 3136, 576), (1024, 768, 768), (16, 4096, 1024),
              (40, 176, 640), (9, 64, 4096),
              (512, 768, 2048), (1000, 999, 1001), (7, 7, 3), (2048, 1568, 512), (768, 512, 384)]
    for (m, n, k) in shapes:
        for uns in (0, 1, 2):
            mode = (idx // 2) % 2
            oa, ob, oc = idx % 2, (idx // 3) % 2, (idx // 5) % 2
            pad = 0 if (m, n, k) not in ((1000, 999, 1001), (7, 7, 3), (300, 200, 333)) else 17
            out.append((W.Case(
                "deq_%dx%dx%d_u%d_m%d_%d%d%d" % (m, n, k, uns, mode, oa, ob, oc), 8, idx, m, n, k,
                a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob, orderC=oc, pad=pad,
                mode=mode,
                a_dist=("uniform", 0, 255) if uns == 1 else ("normal", 24.0),
                b_dist=("uniform", 0, 255) if uns == 2 else ("normal", 32.0),
                c_dist=("uniform", -1000, 1000), seed=13), [0.0123, 2.0 ** -8, -3.3e-5][idx % 3]))
            idx += 1
    return out


VARIANTS = ["auto", "simple", "tile64", "dma128", "dma256k128", "dma128k128", "dma128k128split", "dma256k128ragged",
            "slab16", "slab32"]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("case,scale", _cases(), ids=lambda x: x.name if hasattr(x, "name") else None)
def test_dequant_against_oracle(gpu, oracle, case, scale, variant):
    import torch
    print("case", case.name, "scale", scale, "variant", variant, flush=True)
    ops = W.materialize(case)
    rng = np.random.default_rng(case.index)
    C0 = (rng.standard_normal(ops.C.size) * 50).astype(np.float32)   # floats where the ints were
    pad_mask = W.padding_mask(case.m, case.n, case.orderC, case.ldc)
    want = oracle.gemm_dequant(case.a_unsigned, case.b_unsigned, case.m, case.n, case.k,
                               ops.A, case.lda, case.orderA, ops.B, case.ldb, case.orderB,
                               scale, C0, case.ldc, case.orderC, case.mode)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dC = torch.from_numpy(C0.copy()).cuda()
    fn = getattr(gpu, "mipgemm_" + case.entry.replace("s32", "f32"))
    with gpu.tuning(MIPGEMM_VARIANT=None if variant == "auto" else variant):
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
           dC, case.ldc, case.orderC, case.mode, scale=scale)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy()
    assert np.array_equal(raw[pad_mask], C0[pad_mask])               # padding untouched
    got = W.extract(raw, case.m, case.n, case.orderC, case.ldc).astype(np.float64)
    c0 = W.extract(C0, case.m, case.n, case.orderC, case.ldc).astype(np.float64)
    bound = 2.0 ** -23 * (np.abs(want) + (np.abs(c0) if case.mode == W.ACCUMULATE else 0.0))
    err = np.abs(got - want)
    assert (err <= bound).all(), "max excess %g at %s" % (
        (err - bound).max(), np.unravel_index(np.argmax(err - bound), err.shape))
    if case.mode == W.OVERWRITE:
        # the same two IEEE operations in numpy: float(S) then one float multiply
        S = np.rint(want / float(np.float32(scale)))                  # exact: want = scale * S
        emul = S.astype(np.float32) * np.float32(scale)
        assert np.array_equal(got.astype(np.float32), emul)


def test_dequant_scale_one_equals_integer_result(gpu):
    import torch
    case = W.config1()[0]
    ops = W.materialize(case)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dCi = torch.zeros(case.m * case.n, dtype=torch.int32, device="cuda")
    dCf = torch.zeros(case.m * case.n, dtype=torch.float32, device="cuda")
    gpu.mipgemm_s8s8s32(case.m, case.n, case.k, dA, case.lda, 0, dB, case.ldb, 0, dCi, case.n, 0, 0)
    gpu.mipgemm_s8s8f32(case.m, case.n, case.k, dA, case.lda, 0, dB, case.ldb, 0, dCf, case.n, 0, 0,
                        scale=1.0)
    torch.cuda.synchronize()
    assert np.array_equal(dCf.cpu().numpy(), dCi.cpu().numpy().astype(np.float32))


def test_dequant_rejects_bad_scale_and_empty_k(gpu):
    import torch
    dA = torch.zeros(64, dtype=torch.uint8, device="cuda")
    C0 = np.full(12, 7.5, dtype=np.float32)
    dC = torch.from_numpy(C0).cuda()
    R = W.ROW_MAJOR
    for bad in (float("nan"), float("inf")):
        assert gpu.mipgemm_s8s8f32(3, 3, 4, dA, 4, R, dA, 3, R, dC, 4, R, 0, scale=bad,
                                   check=False) == -17
    assert gpu.mipgemm_s8s8f32(3, 3, 4, dA, 3, R, dA, 3, R, dC, 4, R, 0, scale=float("nan"),
                               check=False) == -5                     # earlier argument first
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C0)
    gpu.mipgemm_s8s8f32(3, 3, 0, dA, 1, R, dA, 3, R, dC, 4, R, 0, scale=0.5)   # empty sum: zeros
    torch.cuda.synchronize()
    want = C0.reshape(3, 4).copy()
    want[:, :3] = 0.0
    assert np.array_equal(dC.cpu().numpy().reshape(3, 4), want)


# ---------------------------------------------------------------------------
# float output with k split over several workgroups per tile: the ranges meet in slots of
# int32 partial sums in the workspace, the last to arrive converts the complete sum
# ---------------------------------------------------------------------------

def _check_float(gpu, oracle, case, scale, variant, splits, with_workspace=True, replays=0):
    import torch
    ops = W.materialize(case)
    rng = np.random.default_rng(case.index)
    C0 = (rng.standard_normal(ops.C.size) * 50).astype(np.float32)
    pad_mask = W.padding_mask(case.m, case.n, case.orderC, case.ldc)
    want = oracle.gemm_dequant(case.a_unsigned, case.b_unsigned, case.m, case.n, case.k,
                               ops.A, case.lda, case.orderA, ops.B, case.ldb, case.orderB,
                               scale, C0, case.ldc, case.orderC, case.mode)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dC = torch.from_numpy(C0.copy()).cuda()
    need = max(gpu.mipgemm_workspace_size_f32(case.m, case.n, case.k, case.orderA, case.orderB,
                                              case.orderC), 64 << 20) if with_workspace else 0
    ws = torch.full((need + 64,), 0x5A, dtype=torch.uint8, device="cuda") if need else None
    fn = getattr(gpu, "mipgemm_" + case.entry.replace("s32", "f32"))

    def call():
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
           dC, case.ldc, case.orderC, case.mode, scale=scale, workspace=ws, workspace_bytes=need)

    def verify():
        torch.cuda.synchronize()
        raw = dC.cpu().numpy()
        assert np.array_equal(raw[pad_mask], C0[pad_mask])
        got = W.extract(raw, case.m, case.n, case.orderC, case.ldc).astype(np.float64)
        c0 = W.extract(C0, case.m, case.n, case.orderC, case.ldc).astype(np.float64)
        bound = 2.0 ** -23 * (np.abs(want) + (np.abs(c0) if case.mode == W.ACCUMULATE else 0.0))
        assert (np.abs(got - want) <= bound).all()
        if case.mode == W.OVERWRITE:       # bit for bit the two IEEE operations of an unsplit call
            S = np.rint(want / float(np.float32(scale)))
            assert np.array_equal(got.astype(np.float32), S.astype(np.float32) * np.float32(scale))
        if ws is not None:
            assert (ws[need:].cpu().numpy() == 0x5A).all()          # nothing behind the workspace

    with gpu.tuning(MIPGEMM_VARIANT=None if variant == "auto" else variant, MIPGEMM_SPLITK=splits):
        if replays == 0:
            call()
            verify()
        else:
            call()                                               # warm-up outside the capture
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            dC.copy_(torch.from_numpy(C0))
            with torch.cuda.graph(graph):
                call()
            for _ in range(replays):                             # same counters every replay
                dC.copy_(torch.from_numpy(C0))
                torch.cuda.synchronize()
                graph.replay()
                verify()


def _split_cases():
    out = []
    shapes = [(256, 256, 8192), (128, 1024, 4096), (64, 4096, 2048), (200, 136, 1024), (1, 4096, 1024),
              (512, 512, 4096), (33, 2000, 1536)]
    for idx, (m, n, k) in enumerate(shapes):
        uns, mode = idx % 3, (idx // 2) % 2
        oa, ob, oc = 0 if m % 16 else idx % 2, 0 if n % 16 else (idx // 2) % 2, (idx // 3) % 2
        out.append(W.Case("deqsplit_%dx%dx%d_u%d_m%d_%d%d%d" % (m, n, k, uns, mode, oa, ob, oc), 8, 100 + idx,
                          m, n, k, a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob,
                          orderC=oc, pad=16 * (idx % 2), mode=mode,
                          a_dist=("uniform", 0, 255) if uns == 1 else ("normal", 24.0),
                          b_dist=("uniform", 0, 255) if uns == 2 else ("normal", 32.0),
                          c_dist=("uniform", -1000, 1000), seed=17))
    return out


@pytest.mark.parametrize("variant,splits", [("dma64", 2), ("dma64", 5), ("dma64x128", 3), ("dma128x64", 4),
                                            ("dma128", 2), ("dma64x256", 7), ("dma256x64", 3),
                                            ("dma256", 2), ("dma64", 1000), ("auto", None)])
@pytest.mark.parametrize("case", _split_cases(), ids=lambda c: c.name)
def test_float_output_with_split_k_through_slots(gpu, oracle, case, variant, splits):
    _check_float(gpu, oracle, case, 0.0123, variant, splits)


def test_float_split_k_is_dispatched_with_a_workspace_and_not_without(gpu, oracle):
    """A long-k, few-tile float problem: with room for slots the dispatcher splits k (the
    workspace query says how much room), without it the call still gives the same result."""
    case = W.Case("deqsplit_auto", 8, 120, 256, 256, 8192, seed=17)
    assert gpu.mipgemm_workspace_size_f32(case.m, case.n, case.k, 0, 0, 0) > 0
    assert gpu.mipgemm_workspace_size(case.m, case.n, case.k, 0, 0, 0) == 0    # int32: atomics into C
    _check_float(gpu, oracle, case, 2.0 ** -9, "auto", None)
    _check_float(gpu, oracle, case, 2.0 ** -9, "auto", None, with_workspace=False)
    _check_float(gpu, oracle, case, 2.0 ** -9, "dma64", 4, with_workspace=False)  # no room: one range


def test_float_split_k_replays_from_a_hip_graph(gpu, oracle):
    case = W.Case("deqsplit_graph", 8, 121, 128, 1024, 4096, mode=W.ACCUMULATE, seed=17)
    _check_float(gpu, oracle, case, 0.004, "dma64", 6, replays=4)


def test_float_split_k_on_two_streams_at_once(gpu, oracle):
    """Two calls in flight at the same time take different ticket counters."""
    import torch
    case = W.Case("deqsplit_streams", 8, 122, 256, 512, 4096, seed=17)
    ops = W.materialize(case)
    want = oracle.gemm_dequant(False, False, case.m, case.n, case.k, ops.A, case.lda, 0, ops.B, case.ldb, 0,
                               0.01, None, case.ldc, 0, W.OVERWRITE)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    streams = [torch.cuda.Stream() for _ in range(2)]
    outs = [torch.zeros(case.m * case.n, dtype=torch.float32, device="cuda") for _ in range(2)]
    wss = [torch.empty(64 << 20, dtype=torch.uint8, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()
    with gpu.tuning(MIPGEMM_VARIANT="dma64", MIPGEMM_SPLITK=4):
        for rep in range(20):
            for s, o, w in zip(streams, outs, wss):
                gpu.mipgemm_s8s8f32(case.m, case.n, case.k, dA, case.lda, 0, dB, case.ldb, 0, o, case.ldc, 0,
                                    W.OVERWRITE, scale=0.01, workspace=w, workspace_bytes=w.numel(), stream=s)
    torch.cuda.synchronize()
    S = np.rint(want / float(np.float32(0.01)))
    for o in outs:
        assert np.array_equal(o.cpu().numpy().reshape(case.m, case.n), S.astype(np.float32) * np.float32(0.01))
