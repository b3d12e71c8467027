"""Seeded randomized parity on the GPU: random shapes, storage orders, leading-dimension padding,
modes, entry points (int32, float and int8 outputs, packed weights, 16-bit operands), forced kernel
variants, split k and workspaces against the oracle; and random convolution geometries over all
routes, with and without supplied filter sums, with int32 and int8 outputs."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

VARIANTS = [None, None, None, "dma64", "dma128", "dma64x128", "dma128x64", "dma64x256", "dma256x64", "tile64",
            "tile128x64", "dma128k128", "dma256k128", "slab16", "slab32", "slab64", "dma256", "dma128k128split",
            "dma256k128ragged"]
ENTRIES = ["s8s8s32", "u8s8s32", "s8u8s32", "s8s8f32", "u8s8s8", "u8s8s32_packed", "s16"]


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_11728_amd as M
    M.load_library()
    return M


def _dims(rng):
    """Tiny and odd, skinny, whole 64-tiles, whole 128-tiles with 128-deep k, or anything up to 700."""
    kind = rng.integers(0, 5)
    if kind == 0:
        return int(rng.integers(1, 80)), int(rng.integers(1, 80)), int(rng.integers(1, 200))
    if kind == 1:
        return int(rng.integers(1, 20)), 16 * int(rng.integers(1, 80)), 64 * int(rng.integers(1, 40))
    if kind == 2:
        return 64 * int(rng.integers(1, 9)), 64 * int(rng.integers(1, 9)), 64 * int(rng.integers(1, 24))
    if kind == 3:
        return 128 * int(rng.integers(1, 5)), 128 * int(rng.integers(1, 5)), 128 * int(rng.integers(1, 17))
    return int(rng.integers(1, 700)), int(rng.integers(1, 700)), int(rng.integers(1, 1300))


def _flat16(X, order, pad):
    r, c = X.shape
    ld = (c if order == 0 else r) + pad
    buf = np.full(((r if order == 0 else c), ld), 0x5A5A, dtype=np.int16)
    if order == 0:
        buf[:, :c] = X
    else:
        buf[:, :r] = X.T
    return buf.reshape(-1), ld


def _one_s16(M, oracle, rng, m, n, k, oa, ob, oc, pad, mode, variant):
    import torch
    A, lda = _flat16(rng.integers(-32768, 32768, size=(m, k), dtype=np.int16), oa, pad)
    B, ldb = _flat16(rng.integers(-32768, 32768, size=(k, n), dtype=np.int16), ob, pad)
    ldc = (n if oc == 0 else m) + pad
    C0 = rng.integers(-1000, 1000, size=(m if oc == 0 else n) * ldc, dtype=np.int32)
    want = C0.copy()
    oracle.gemm_s16(m, n, k, A, lda, oa, B, ldb, ob, want, ldc, oc, mode)
    need = M.mipgemm_workspace_size_s16(m, n, k)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    dC = torch.from_numpy(C0).cuda()
    with M.tuning(MIPGEMM_VARIANT=variant):
        M.mipgemm_s16s16s32(m, n, k, torch.from_numpy(A).cuda(), lda, oa, torch.from_numpy(B).cuda(), ldb, ob,
                            dC, ldc, oc, mode, workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    return np.array_equal(dC.cpu().numpy(), want)


def _one_8bit(M, oracle, rng, seed, index, entry, m, n, k, oa, ob, oc, pad, mode, variant, splits, use_ws):
    import torch
    au, bu = entry.startswith("u8"), entry.startswith("s8u8")
    case = W.Case("random", 9, index, m, n, k, a_unsigned=au, b_unsigned=bu, orderA=oa, orderB=ob, orderC=oc,
                  pad=pad, mode=mode, a_dist=("uniform", 0, 255) if au else ("uniform", -128, 127),
                  b_dist=("uniform", 0, 255) if bu else ("uniform", -128, 127),
                  c_dist=("uniform", -1000, 1000), seed=seed)
    ops = W.materialize(case)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    need = M.mipgemm_workspace_size_f32(m, n, k, oa, ob, oc) + 4096 if use_ws else 0
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda") if need else None
    gemm_args = (m, n, k, ops.A, case.lda, oa, ops.B, case.ldb, ob)
    with M.tuning(MIPGEMM_VARIANT=variant, MIPGEMM_SPLITK=splits or None):
        if entry.endswith("s32"):
            want = ops.C.copy()
            oracle.gemm(au, bu, *gemm_args, want, case.ldc, oc, mode)
            dC = torch.from_numpy(ops.C).cuda()
            getattr(M, "mipgemm_" + entry)(m, n, k, dA, case.lda, oa, dB, case.ldb, ob, dC, case.ldc, oc, mode,
                                           workspace=ws, workspace_bytes=need)
            torch.cuda.synchronize()
            return np.array_equal(dC.cpu().numpy(), want)
        if entry.endswith("_packed"):
            want = ops.C.copy()
            oracle.gemm(au, False, *gemm_args, want, case.ldc, oc, mode)
            dP = torch.zeros(M.mipgemm_packed_weights_bytes(k, n), dtype=torch.uint8, device="cuda")
            M.mipgemm_pack_weights(k, n, dB, case.ldb, ob, dP)
            dC = torch.from_numpy(ops.C).cuda()
            M.mipgemm_u8s8s32_packed(m, n, k, dA, case.lda, oa, dP, dC, case.ldc, oc, mode,
                                     workspace=ws, workspace_bytes=need)
            torch.cuda.synchronize()
            return np.array_equal(dC.cpu().numpy(), want)
        inside = (np.arange(ops.C.size) % case.ldc) < (n if oc == 0 else m)   # not the ld padding
        if entry.endswith("f32"):
            scale = np.float32(0.0371)
            C0 = ops.C.astype(np.float32)
            S = np.zeros(ops.C.size, dtype=np.int32)
            oracle.gemm(au, bu, *gemm_args, S, case.ldc, oc, 0)
            dC = torch.from_numpy(C0.copy()).cuda()
            M.mipgemm_s8s8f32(m, n, k, dA, case.lda, oa, dB, case.ldb, ob, dC, case.ldc, oc, mode,
                              workspace=ws, workspace_bytes=need, scale=float(scale))
            torch.cuda.synchronize()
            got = dC.cpu().numpy()
            if not np.array_equal(got[~inside], C0[~inside]):
                return False
            if mode == 0:      # int -> float32, one float32 multiplication: the same two IEEE operations
                return np.array_equal(got[inside], (S.astype(np.float32) * scale)[inside])
            ref = C0.astype(np.float64) + np.float64(scale) * S.astype(np.float64)
            return bool(np.all(np.abs(got[inside] - ref[inside]) <=
                               2.0 ** -22 * (np.abs(ref[inside]) + np.abs(C0[inside]) + 1e-30)))
        # int8 output: overwrite only
        scale = np.float32(1.0 / (k * 60.0 + 1))
        Q0 = np.full(ops.C.size, 0x11, dtype=np.int8)
        want = Q0.copy()
        oracle.gemm_requant(au, bu, *gemm_args, scale, want, case.ldc, oc)
        dQ = torch.from_numpy(Q0.copy()).cuda()
        M.mipgemm_u8s8s8(m, n, k, dA, case.lda, oa, dB, case.ldb, ob, dQ, case.ldc, oc, 0,
                         workspace=ws, workspace_bytes=need, scale=float(scale))
        torch.cuda.synchronize()
        return np.array_equal(dQ.cpu().numpy(), want)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_gemm_calls(gpu, oracle, seed):
    rng = np.random.default_rng(seed)
    failures = []
    for index in range(400):
        m, n, k = _dims(rng)
        oa, ob, oc = (int(x) for x in rng.integers(0, 2, size=3))
        pad = int(rng.choice([0, 0, 16, 32, 1, 7]))
        mode = int(rng.integers(0, 2))
        entry = str(rng.choice(ENTRIES))
        variant = VARIANTS[int(rng.integers(0, len(VARIANTS)))]
        splits = int(rng.choice([0, 0, 0, 2, 3, 5]))
        use_ws = bool(rng.integers(0, 2))
        what = dict(m=m, n=n, k=k, orders=(oa, ob, oc), pad=pad, mode=mode, entry=entry, variant=variant,
                    splits=splits, workspace=use_ws)
        if entry == "s16":
            ok = _one_s16(gpu, oracle, rng, m, n, k, oa, ob, oc, pad, mode, variant)
        else:
            ok = _one_8bit(gpu, oracle, rng, seed, index, entry, m, n, k, oa, ob, oc, pad, mode, variant, splits,
                           use_ws)
        if not ok:
            failures.append(what)
    assert not failures, failures[:5]


def _one_conv(M, oracle, rng, shape, route, variant, mode, with_sums, int8_out):
    import torch
    b, hi, wi, ci, co, hf, wf, s, p = shape
    I = rng.integers(0, 256, size=(b, hi, wi, ci), dtype=np.uint8)
    F = rng.integers(-128, 128, size=(co, hf, wf, ci), dtype=np.int8)
    S = oracle.conv_direct(I, F, s, p)            # ValueError when the filter does not fit
    dI, dF = torch.from_numpy(I).cuda(), torch.from_numpy(F.view(np.uint8)).cuda()
    dS = None
    if with_sums:
        dS = torch.zeros(co, dtype=torch.int32, device="cuda")
        M.mipgemm_conv_filter_sums(co, hf * wf * ci, dF, dS)
    with M.tuning(MIPGEMM_CONV=route, MIPGEMM_VARIANT=variant):
        need = max(M.mipgemm_conv_workspace_size(*shape), M.mipgemm_conv_workspace_size_unaligned(*shape))
        ws = torch.zeros(need, dtype=torch.uint8, device="cuda") if need else None
        if int8_out:
            scale = np.float32(100.0 / max(1.0, float(np.abs(S).max()) * 0.7))
            Mx = oracle.im2col_u8(I, hf, wf, s, p)
            rows, k = Mx.shape
            want = np.zeros(rows * co, dtype=np.int8)
            oracle.gemm_requant(False, True, co, rows, k, F.reshape(-1), k, 0, Mx.reshape(-1), k, 1, scale,
                                want, co, 1)
            dO = torch.zeros(S.size, dtype=torch.int8, device="cuda")
            M.mipgemm_conv_s8u8s8(*shape, dF, dI, dO, 0, dS, workspace=ws, workspace_bytes=need,
                                  scale=float(scale))
        else:
            O0 = rng.integers(-1000, 1000, size=S.shape, dtype=np.int32)
            want = (S + O0 if mode else S).reshape(-1).astype(np.int32)
            dO = torch.from_numpy(O0.reshape(-1).copy()).cuda()
            if dS is not None:
                M.mipgemm_conv_s8u8s32_with_sums(*shape, dF, dI, dO, mode, dS, workspace=ws,
                                                 workspace_bytes=need)
            else:
                M.mipgemm_conv_s8u8s32(*shape, dF, dI, dO, mode, workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    return np.array_equal(dO.cpu().numpy(), want)


@pytest.mark.parametrize("seed", [1, 2])
def test_random_convolutions(gpu, oracle, seed):
    rng = np.random.default_rng(seed)
    failures = []
    count = 0
    while count < 400:
        b = int(rng.integers(1, 4))
        ci = int(rng.choice([1, 2, 3, 5, 16, 24, 48, 64, 128, 192]))
        hf, wf = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        s, p = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        hi = int(rng.integers(max(1, hf - 2 * p), 30))
        wi = int(rng.integers(max(1, wf - 2 * p), 40))
        co = int(rng.choice([1, 7, 16, 40, 64, 65, 130, 256]))
        shape = (b, hi, wi, ci, co, hf, wf, s, p)
        route = rng.choice([None, None, "im2col", "rows"])
        variant = rng.choice([None, None, "dma64", "dma128", "dma64x128", "dma256x64"])
        mode = int(rng.integers(0, 2))
        with_sums = bool(rng.integers(0, 2))
        int8_out = bool(rng.integers(0, 3) == 0)
        try:
            ok = _one_conv(gpu, oracle, rng, shape, route, variant, mode, with_sums, int8_out)
        except ValueError:
            continue
        count += 1
        if not ok:
            failures.append(dict(shape=shape, route=route, variant=variant, mode=mode, sums=with_sums,
                                 int8=int8_out))
    assert not failures, failures[:5]
