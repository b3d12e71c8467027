"""GPU parity of the requantised-output entry points (int8 C = clip(rint(scale * A B))).

Integer output: compared byte for byte with the oracle, leading-dimension padding
included.  Both sides take the rounding decision in float32 (paper silent; reading in
the oracle's header), so there is no tolerance.
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


def _run(gpu, oracle, case, scale, variant="auto", splits=None, workspace=False):
    import torch
    ops = W.materialize(case)
    # C as bytes: the int32 buffer of the case only gives the layout
    Q0 = np.full(ops.C.size, W.SENTINEL_BYTE, dtype=np.int8)
    want = Q0.copy()
    oracle.gemm_requant(case.a_unsigned, case.b_unsigned, case.m, case.n, case.k, ops.A, case.lda,
                        case.orderA, ops.B, case.ldb, case.orderB, scale, want, case.ldc, case.orderC)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dQ = torch.from_numpy(Q0.copy()).cuda()
    need = 0
    if workspace:
        need = max(gpu.mipgemm_workspace_size_f32(case.m, case.n, case.k, case.orderA, case.orderB,
                                                  case.orderC), 32 << 20)
    ws = torch.full((need + 64,), 0x5A, dtype=torch.uint8, device="cuda") if need else None
    fn = getattr(gpu, "mipgemm_" + case.entry.replace("s32", "s8"))
    with gpu.tuning(MIPGEMM_VARIANT=None if variant == "auto" else variant, MIPGEMM_SPLITK=splits):
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB, dQ, case.ldc,
           case.orderC, W.OVERWRITE, scale=scale, workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    got = dQ.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError("%s %s: %d bytes differ, first at %d: got %d want %d" % (
            case.name, variant, bad.size, bad[0], got[bad[0]], want[bad[0]]))
    if ws is not None:
        assert (ws[need:].cpu().numpy() == 0x5A).all()
    return want


def _cases():
    out = []
    shapes = [(256, 256, 256), (300, 200, 333), (64, 3136, 576), (1024, 768, 768), (16, 4096, 1024),
              (40, 176, 640), (512, 768, 2048), (1000, 999, 1001), (7, 7, 3), (2048, 1568, 512),
              (1, 4097, 513), (4095, 3, 2049), (768, 512, 384)]
    for idx, (m, n, k) in enumerate(shapes):
        for uns in (0, 1, 2):
            oa, ob, oc = idx % 2, (idx // 3) % 2, (idx // 2 + uns) % 2
            pad = 17 if (m * n * k) % 2 or m == 7 else 16 * (idx % 2)
            # scales that land the results inside the int8 range with many exact ties (powers of two)
            # and without; negative as well
            sigma = (24.0 if uns != 1 else 128.0) * (32.0 if uns != 2 else 128.0) * np.sqrt(k)
            scale = [2.0 ** -int(np.log2(sigma / 40)), 37.0 / sigma, -2.0 ** -int(np.log2(sigma / 25))][(idx + uns) % 3]
            out.append((W.Case("q8_%dx%dx%d_u%d_%d%d%d" % (m, n, k, uns, oa, ob, oc), 8, 200 + 3 * idx + uns,
                               m, n, k, a_unsigned=uns == 1, b_unsigned=uns == 2, orderA=oa, orderB=ob,
                               orderC=oc, pad=pad,
                               a_dist=("uniform", 0, 255) if uns == 1 else ("normal", 24.0),
                               b_dist=("uniform", 0, 255) if uns == 2 else ("normal", 32.0), seed=19),
                        float(scale)))
    return out


@pytest.mark.parametrize("variant", ["auto", "simple", "tile64", "tile128x64", "dma64", "dma128", "dma64x256",
                                     "dma256", "dma256k128", "dma128k128", "dma128k128split", "dma256k128ragged"])
@pytest.mark.parametrize("case,scale", _cases(), ids=lambda x: x.name if hasattr(x, "name") else None)
def test_requant_against_oracle(gpu, oracle, case, scale, variant):
    print("case", case.name, "scale", scale, "variant", variant, flush=True)
    want = _run(gpu, oracle, case, scale, variant)
    q = W.extract(want, case.m, case.n, case.orderC, case.ldc)
    if case.m * case.n >= 1000:            # the case exercises rounding, not only saturation or zeros
        assert 0.2 < np.mean((q > -128) & (q < 127) & (q != 0))


@pytest.mark.parametrize("variant,splits", [("dma64", 3), ("dma64x128", 2), ("dma128", 4), ("dma64x256", 5),
                                            ("auto", None)])
def test_requant_with_split_k_through_slots_and_packed_operands(gpu, oracle, variant, splits):
    for case, scale in _cases()[::4]:
        _run(gpu, oracle, case, scale, variant, splits, workspace=True)
    long_k = W.Case("q8_256x256x8192", 8, 260, 256, 256, 8192, a_dist=("normal", 24.0),
                    b_dist=("normal", 32.0), seed=19)
    _run(gpu, oracle, long_k, 2.0 ** -11, variant, splits, workspace=True)


def test_requant_hand_worked_values_on_the_device(gpu):
    """The ties, the saturation and the float32 decision of tests/golden/hand_worked_requant.txt."""
    import torch
    ones = torch.ones(3, dtype=torch.int8, device="cuda")
    B = np.array([[1, 1, 2, -1, -1, -2, 127, 127, -127, -128, -128],
                  [0, 1, 2, 0, -1, -2, 126, 127, -127, -128, -128],
                  [0, 1, 1, 0, -1, -1, 0, 1, -1, -1, -3]], dtype=np.int8)
    dB = torch.from_numpy(B.reshape(-1)).cuda()
    dQ = torch.zeros(11, dtype=torch.int8, device="cuda")
    gpu.mipgemm_s8s8s8(1, 11, 3, ones, 3, 0, dB, 11, 0, dQ, 11, 0, W.OVERWRITE, scale=0.5)
    torch.cuda.synchronize()
    assert dQ.cpu().tolist() == [0, 2, 2, 0, -2, -2, 126, 127, -128, -128, -128]
    a = np.full(1025, -128, dtype=np.int8)
    a[-1] = 1
    dA = torch.from_numpy(a).cuda()
    for scale, want in ((2.0 ** -25, 0), (3 * 2.0 ** -25, 2)):
        gpu.mipgemm_s8s8s8(1, 1, 1025, dA, 1025, 0, dA, 1, 0, dQ, 1, 0, W.OVERWRITE, scale=scale)
        torch.cuda.synchronize()
        assert int(dQ[0]) == want


def test_requant_errors_and_empty_sums(gpu):
    import torch
    dA = torch.zeros(64, dtype=torch.uint8, device="cuda")
    Q0 = np.full(12, 0x5A, dtype=np.int8)
    dQ = torch.from_numpy(Q0.copy()).cuda()
    R = W.ROW_MAJOR
    assert gpu.mipgemm_s8s8s8(3, 3, 4, dA, 4, R, dA, 3, R, dQ, 4, R, W.ACCUMULATE, scale=1.0, check=False) == -13
    for bad in (float("nan"), float("inf")):
        assert gpu.mipgemm_s8s8s8(3, 3, 4, dA, 4, R, dA, 3, R, dQ, 4, R, 0, scale=bad, check=False) == -17
    assert gpu.mipgemm_s8s8s8(3, 3, 4, dA, 3, R, dA, 3, R, dQ, 4, R, 0, scale=1.0, check=False) == -5
    torch.cuda.synchronize()
    assert np.array_equal(dQ.cpu().numpy(), Q0)
    gpu.mipgemm_s8s8s8(3, 3, 0, dA, 1, R, dA, 3, R, dQ, 4, R, 0, scale=0.5)      # empty sum: zeros
    torch.cuda.synchronize()
    want = Q0.reshape(3, 4).copy()
    want[:, :3] = 0
    assert np.array_equal(dQ.cpu().numpy().reshape(3, 4), want)
