"""Pins for the CPU oracle: what the paper and the arithmetic fix, independent of the oracle's code.

Each test names the mistake it is meant to catch.  None of them touches the GPU.
"""
import os

import numpy as np
import pytest

import workloads as W
from workloads import ROW_MAJOR as R, COL_MAJOR as CM, OVERWRITE as OVW, ACCUMULATE as ACC

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ---------------------------------------------------------------------------
# helpers (layout only; the expected values come from separate code below)
# ---------------------------------------------------------------------------

def run(oracle, A2d, B2d, C2d=None, mode=OVW, oa=R, ob=R, oc=R, pad=0):
    """Call the oracle on logical matrices laid out as asked; return the logical C and the raw buffer."""
    m, k = A2d.shape
    k2, n = B2d.shape
    assert k == k2
    lda = (k if oa == R else m) + pad
    ldb = (n if ob == R else k) + pad
    ldc = (n if oc == R else m) + pad
    if C2d is None:
        C2d = np.full((m, n), 0x5A5A5A5A, dtype=np.int32)
    A = W.embed(A2d, oa, lda, A2d.dtype.type(W.SENTINEL_BYTE))
    B = W.embed(B2d, ob, ldb, B2d.dtype.type(W.SENTINEL_BYTE))
    C = W.embed(C2d.astype(np.int32), oc, ldc, np.int32(W.SENTINEL_WORD))
    oracle.gemm(A2d.dtype == np.uint8, B2d.dtype == np.uint8, m, n, k,
                A, lda, oa, B, ldb, ob, C, ldc, oc, mode)
    return W.extract(C, m, n, oc, ldc), C, W.padding_mask(m, n, oc, ldc)


def brute_force(A2d, B2d, C2d=None):
    """Per-element dot products in Python integers (unbounded), wrapped to int32 at the end.

    A different loop nest (j outermost, then i, then p, running downwards) and
    no numpy arithmetic: shares nothing with the oracle's C loops.
    """
    m, k = A2d.shape
    n = B2d.shape[1]
    a = [[int(x) for x in row] for row in A2d]
    b = [[int(x) for x in row] for row in B2d]
    out = np.zeros((m, n), dtype=np.int64)
    for j in range(n):
        for i in range(m):
            s = 0
            for p in range(k - 1, -1, -1):
                s += a[i][p] * b[p][j]
            if C2d is not None:
                s += int(C2d[i, j])
            s &= 0xFFFFFFFF
            out[i, j] = s - (1 << 32) if s >= (1 << 31) else s
    return out.astype(np.int32)


def rand(rng, shape, dtype):
    info = np.iinfo(dtype)
    return rng.integers(info.min, info.max, size=shape, endpoint=True).astype(dtype)


# ---------------------------------------------------------------------------
# P0  hand-worked example and closed forms stored as text
# ---------------------------------------------------------------------------

def _read_matrices(path):
    mats, cur = {}, None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0].isalpha() or tok[0][0].isalpha():
                cur = tok[0]
                mats[cur] = []
            else:
                mats[cur].append([int(t) for t in tok])
    return {k: np.array(v, dtype=np.int64) for k, v in mats.items()}


def test_hand_worked_example(oracle):
    g = _read_matrices(os.path.join(GOLDEN, "hand_worked_2x3x4.txt"))
    A, B, C0 = g["A"].astype(np.int8), g["B"].astype(np.int8), g["C0"].astype(np.int32)
    got, _, _ = run(oracle, A, B)
    assert np.array_equal(got, g["AB"])
    got, _, _ = run(oracle, A, B, C0, mode=ACC)
    assert np.array_equal(got, g["ACC"])
    got, _, _ = run(oracle, A.view(np.uint8), B)
    assert np.array_equal(got, g["AuB"])
    # B^T A^T = (AB)^T with the unsigned operand now second (catches a transposed operand)
    got, _, _ = run(oracle, np.ascontiguousarray(B.T), np.ascontiguousarray(A.view(np.uint8).T))
    assert np.array_equal(got, g["AuB"].T)


def test_closed_forms_constant_matrices(oracle):
    rows = []
    with open(os.path.join(GOLDEN, "closed_forms.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    assert len(rows) >= 12
    for at, bt, a, b, k, want in rows:
        a, b, k, want = int(a), int(b), int(k), int(want)
        A = np.full((3, k), a, dtype=np.uint8 if at == "u8" else np.int8)
        B = np.full((k, 2), b, dtype=np.uint8 if bt == "u8" else np.int8)
        got, _, _ = run(oracle, A, B)
        assert (got == want).all(), (at, bt, a, b, k, want, got[0, 0])


# ---------------------------------------------------------------------------
# P1  brute force on tiny shapes, incl. the instruction tiles the paper defines
# ---------------------------------------------------------------------------

TINY = [(1, 1, 1), (2, 8, 16), (4, 4, 8), (4, 16, 16), (16, 16, 64), (7, 7, 3), (3, 5, 2), (1, 9, 33)]


@pytest.mark.parametrize("m,n,k", TINY)
@pytest.mark.parametrize("types", ["s8s8", "u8s8", "s8u8"])
def test_brute_force_tiny(oracle, m, n, k, types):
    rng = np.random.default_rng(1000 + m * 131 + n * 17 + k)
    ta = np.uint8 if types == "u8s8" else np.int8
    tb = np.uint8 if types == "s8u8" else np.int8
    A, B = rand(rng, (m, k), ta), rand(rng, (k, n), tb)
    C0 = rng.integers(-1000, 1000, size=(m, n), endpoint=True).astype(np.int32)
    got, _, _ = run(oracle, A, B)
    assert np.array_equal(got, brute_force(A, B))
    got, _, _ = run(oracle, A, B, C0, mode=ACC)
    assert np.array_equal(got, brute_force(A, B, C0))


@pytest.mark.parametrize("types", ["s8s8", "u8s8", "s8u8"])
def test_exhaustive_byte_pairs(oracle, types):
    """Every (a, b) byte pair through a 1-deep product: catches any sign-extension slip.

    A is 256 x 1 holding every byte, B is 1 x 256 holding every byte, so
    C(i, j) must be value(i) * value(j).
    """
    ta = np.uint8 if types == "u8s8" else np.int8
    tb = np.uint8 if types == "s8u8" else np.int8
    a = np.arange(256, dtype=np.uint8).view(ta).reshape(256, 1)
    b = np.arange(256, dtype=np.uint8).view(tb).reshape(1, 256)
    got, _, _ = run(oracle, a, b)
    va = np.array([int(x) for x in a[:, 0]], dtype=np.int64)
    vb = np.array([int(x) for x in b[0, :]], dtype=np.int64)
    assert np.array_equal(got, np.multiply.outer(va, vb))
    assert got.min() == (-32640 if types != "s8s8" else -16256)
    assert got.max() == (32385 if types != "s8s8" else 16384)


# ---------------------------------------------------------------------------
# instruction-tile definitions printed in the paper, composed into a GEMM
# ---------------------------------------------------------------------------

def sdot_lane(v0, v1, v2, lane):
    """ARMv8.2 dot-product-by-lane as Section 5.2 defines it:
    r[i] = v0[i] + sum_{t<4} v1[4i+t] * v2[4*lane+t], i = 0..3."""
    r = [0] * 4
    for i in range(4):
        r[i] = int(v0[i]) + sum(int(v1[4 * i + t]) * int(v2[4 * lane + t]) for t in range(4))
    return r


def test_sdot_composition_matches_oracle(oracle):
    """A 4 x 16 x 16 GEMM assembled from the lane-dot instruction must equal the oracle.

    Row i of A_r (16 int8 along k) is one register; for each k-group g of four,
    the register of B holds four columns' k-group (4 columns x 4 k).  Output
    register (i, c4) holds C(i, 4*c4 .. 4*c4+3).
    """
    rng = np.random.default_rng(7)
    A = rand(rng, (4, 16), np.int8)
    B = rand(rng, (16, 16), np.int8)
    C0 = rng.integers(-1000, 1000, size=(4, 16), endpoint=True).astype(np.int32)
    C = [[int(x) for x in row] for row in C0]
    for g in range(4):                       # k-group: k = 4g .. 4g+3
        for c4 in range(4):                  # four output columns at a time
            v1 = [int(B[4 * g + t, 4 * c4 + jj]) for jj in range(4) for t in range(4)]
            for i in range(4):
                acc = C[i][4 * c4:4 * c4 + 4]
                C[i][4 * c4:4 * c4 + 4] = sdot_lane(acc, v1, list(A[i]), g)
    got, _, _ = run(oracle, A, B, C0, mode=ACC)
    assert np.array_equal(got, np.array(C))


def test_vmadot_tile_matches_oracle(oracle):
    """The 4 x 4 x 8 tile product of Section 6.1 (A_r row-major 4 x 8, B_r column-major 8 x 4,
    C_r += A_r B_r in INT32), evaluated from the register images."""
    rng = np.random.default_rng(8)
    reg_a = rand(rng, 32, np.int8)           # 4 rows x 8, row-major
    reg_b = rand(rng, 32, np.int8)           # 8 x 4 stored column by column
    c0 = rng.integers(-1000, 1000, size=(4, 4), endpoint=True).astype(np.int32)
    want = [[int(c0[i, j]) + sum(int(reg_a[8 * i + p]) * int(reg_b[8 * j + p]) for p in range(8))
             for j in range(4)] for i in range(4)]
    A = reg_a.reshape(4, 8)
    Bcm = reg_b.reshape(4, 8).T              # logical 8 x 4
    got, _, _ = run(oracle, A, np.ascontiguousarray(Bcm), c0, mode=ACC)
    assert np.array_equal(got, np.array(want))
    # the same bytes handed over as a column-major B, untouched
    C = c0.reshape(-1).copy()
    oracle.gemm_s8s8s32(4, 4, 8, reg_a, 8, R, reg_b, 8, CM, C, 4, R, ACC)
    assert np.array_equal(C.reshape(4, 4), np.array(want))


def test_amx_tile_matches_oracle(oracle):
    """The 16 x 16 x 64 tile product of Section 6.2: B held as 16 rows of 64 bytes where
    row r holds, for each column j, the four k values 4r .. 4r+3 next to each other."""
    rng = np.random.default_rng(9)
    A = rand(rng, (16, 64), np.int8)
    tile_b = rand(rng, (16, 64), np.int8)    # tile_b[r, 4*j + t] = B(4r + t, j)
    want = np.zeros((16, 16), dtype=np.int64)
    for i in range(16):
        for j in range(16):
            for r in range(16):
                for t in range(4):
                    want[i, j] += int(A[i, 4 * r + t]) * int(tile_b[r, 4 * j + t])
    B = np.zeros((64, 16), dtype=np.int8)
    for r in range(16):
        for j in range(16):
            for t in range(4):
                B[4 * r + t, j] = tile_b[r, 4 * j + t]
    got, _, _ = run(oracle, A, B)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------------------
# P3 / P4 / P5  identity, permutation, ones, ramp
# ---------------------------------------------------------------------------

def test_identity_and_permutation(oracle):
    rng = np.random.default_rng(3)
    k, n = 37, 23
    B = rand(rng, (k, n), np.int8)
    eye = np.eye(k, dtype=np.int8)
    got, _, _ = run(oracle, eye, B)
    assert np.array_equal(got, B.astype(np.int32))
    got, _, _ = run(oracle, eye.view(np.uint8), B)
    assert np.array_equal(got, B.astype(np.int32))
    perm = rng.permutation(k)
    P = np.zeros((k, k), dtype=np.int8)
    P[np.arange(k), perm] = 1                # row i of P picks row perm[i] of B
    got, _, _ = run(oracle, P, B)
    assert np.array_equal(got, B[perm].astype(np.int32))
    A = rand(rng, (19, k), np.uint8)
    got, _, _ = run(oracle, A, eye)
    assert np.array_equal(got, A.astype(np.int32))
    Bu = rand(rng, (k, n), np.uint8)
    got, _, _ = run(oracle, -eye, Bu)        # minus identity times unsigned B
    assert np.array_equal(got, -Bu.astype(np.int32))


def test_ones_give_row_and_column_sums(oracle):
    rng = np.random.default_rng(4)
    m, n, k = 9, 14, 301
    B = rand(rng, (k, n), np.int8)
    A = rand(rng, (m, k), np.uint8)
    got, _, _ = run(oracle, np.ones((m, k), dtype=np.int8), B)
    col = [sum(int(B[p, j]) for p in range(k)) for j in range(n)]
    assert np.array_equal(got, np.tile(np.array(col), (m, 1)))
    got, _, _ = run(oracle, A, np.ones((k, n), dtype=np.int8))
    row = [sum(int(A[i, p]) for p in range(k)) for i in range(m)]
    assert np.array_equal(got, np.tile(np.array(row)[:, None], (1, n)))


def test_ramp_closed_form(oracle):
    """a(i,p) = (p mod 256) - 128 against ones: each period of 256 sums to -128, so C = -k/2."""
    k = 1024
    A = np.tile(((np.arange(k) % 256) - 128).astype(np.int8), (5, 1))
    got, _, _ = run(oracle, A, np.ones((k, 6), dtype=np.int8))
    assert (got == -k // 2).all()
    # unsigned ramp 0..255: each period sums to 255*256/2 = 32640
    got, _, _ = run(oracle, np.tile((np.arange(k) % 256).astype(np.uint8), (5, 1)),
                    np.ones((k, 6), dtype=np.int8))
    assert (got == 32640 * (k // 256)).all()


# ---------------------------------------------------------------------------
# P6  linearity, modes, k-split
# ---------------------------------------------------------------------------

def test_modes_linearity_ksplit(oracle):
    rng = np.random.default_rng(5)
    m, n, k = 13, 11, 70
    A, B = rand(rng, (m, k), np.int8), rand(rng, (k, n), np.int8)
    C0 = rng.integers(-1000, 1000, size=(m, n), endpoint=True).astype(np.int32)
    ab, _, _ = run(oracle, A, B)
    acc1, _, _ = run(oracle, A, B, C0, mode=ACC)
    acc2, _, _ = run(oracle, A, B, acc1, mode=ACC)
    assert np.array_equal(acc1, C0 + ab)
    assert np.array_equal(acc2, C0 + 2 * ab)
    # overwrite never reads C: garbage in, same result out
    garbage = rng.integers(-2**31, 2**31 - 1, size=(m, n)).astype(np.int32)
    ovw, _, _ = run(oracle, A, B, garbage, mode=OVW)
    assert np.array_equal(ovw, ab)
    # k-split
    k1 = 29
    p1, _, _ = run(oracle, A[:, :k1].copy(), B[:k1].copy())
    p2, _, _ = run(oracle, A[:, k1:].copy(), B[k1:].copy())
    assert np.array_equal(p1 + p2, ab)
    # negating A (kept inside the int8 range) negates C
    A2 = np.clip(A, -127, 127).astype(np.int8)
    pos, _, _ = run(oracle, A2, B)
    neg, _, _ = run(oracle, (-A2).astype(np.int8), B)
    assert np.array_equal(neg, -pos)


def test_wraparound_modulo_2_32(oracle):
    """The accumulator wraps (reading of the paper's silence on overflow), it does not saturate."""
    k = 131072 + 5
    A = np.full((2, k), -128, dtype=np.int8)
    B = np.full((k, 3), -128, dtype=np.int8)
    got, _, _ = run(oracle, A, B)
    want = (16384 * k) % (1 << 32)
    want = want - (1 << 32) if want >= (1 << 31) else want
    assert (got == want).all()
    C0 = np.full((1, 1), 2**31 - 1, dtype=np.int32)
    got, _, _ = run(oracle, np.ones((1, 1), np.int8), np.ones((1, 1), np.int8), C0, mode=ACC)
    assert got[0, 0] == -2**31


# ---------------------------------------------------------------------------
# P7  layouts and leading dimensions
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("oa", [R, CM])
@pytest.mark.parametrize("ob", [R, CM])
@pytest.mark.parametrize("oc", [R, CM])
@pytest.mark.parametrize("pad", [0, 17])
def test_layouts_agree_and_padding_untouched(oracle, oa, ob, oc, pad):
    rng = np.random.default_rng(6)
    m, n, k = 10, 7, 13                     # all different: a transposed operand cannot pass
    A, B = rand(rng, (m, k), np.uint8), rand(rng, (k, n), np.int8)
    C0 = rng.integers(-1000, 1000, size=(m, n), endpoint=True).astype(np.int32)
    want = brute_force(A, B, C0)
    got, raw, mask = run(oracle, A, B, C0, mode=ACC, oa=oa, ob=ob, oc=oc, pad=pad)
    assert np.array_equal(got, want)
    assert (raw[mask] == W.SENTINEL_WORD).all()
    got, raw, mask = run(oracle, A, B, None, mode=OVW, oa=oa, ob=ob, oc=oc, pad=pad)
    assert np.array_equal(got, brute_force(A, B))
    assert (raw[mask] == W.SENTINEL_WORD).all()


def test_swap_identity_same_memory(oracle):
    """C^T = B^T A^T on the very same buffers (Section 3: column-major C by swapping A and B)."""
    case = W.Case("t", 9, 0, 12, 9, 31, b_unsigned=True, pad=5, mode=ACC,
                  b_dist=("uniform", 0, 255), c_dist=("uniform", -1000, 1000), seed=11)
    ops = W.materialize(case)
    C1 = ops.C.copy()
    oracle.gemm(case.a_unsigned, case.b_unsigned, case.m, case.n, case.k, ops.A, case.lda,
                case.orderA, ops.B, case.ldb, case.orderB, C1, case.ldc, case.orderC, case.mode)
    sw = W.swapped(case)
    assert (sw.lda, sw.ldb, sw.ldc) == (case.ldb, case.lda, case.ldc)
    C2 = ops.C.copy()
    oracle.gemm(sw.a_unsigned, sw.b_unsigned, sw.m, sw.n, sw.k, ops.B, sw.lda, sw.orderA,
                ops.A, sw.ldb, sw.orderB, C2, sw.ldc, sw.orderC, sw.mode)
    assert np.array_equal(C1, C2)
    assert np.array_equal(W.extract(C1, case.m, case.n, case.orderC, case.ldc),
                          brute_force(ops.A2d, ops.B2d, ops.C2d))


# ---------------------------------------------------------------------------
# P8  u8 <-> s8 identity
# ---------------------------------------------------------------------------

def test_u8_s8_identity(oracle):
    rng = np.random.default_rng(12)
    m, n, k = 21, 18, 95
    Au, B = rand(rng, (m, k), np.uint8), rand(rng, (k, n), np.int8)
    u, _, _ = run(oracle, Au, B)
    As = (Au.astype(np.int16) - 128).astype(np.int8)
    s, _, _ = run(oracle, As, B)
    colsum = B.astype(np.int64).sum(axis=0)
    assert np.array_equal(u, s + 128 * colsum[None, :])


# ---------------------------------------------------------------------------
# P9  numpy int64 matmul on the generated workloads
# ---------------------------------------------------------------------------

def _np_expected(ops, case):
    S = ops.A2d.astype(np.int64) @ ops.B2d.astype(np.int64)
    if case.mode == ACC:
        S = S + ops.C2d.astype(np.int64)
    return S.astype(np.int32)               # wraps modulo 2^32


def _small_enough(c):
    return c.m * c.n * c.k <= 3e8


CPU_CASES = [c for c in W.all_cases() if _small_enough(c)]


@pytest.mark.parametrize("case", CPU_CASES, ids=lambda c: c.name)
def test_workload_cases_against_numpy(oracle, case):
    assert W.magnitude_bound(case) < 2**31
    ops = W.materialize(case)
    C = ops.C.copy()
    oracle.gemm(case.a_unsigned, case.b_unsigned, case.m, case.n, case.k, ops.A, case.lda,
                case.orderA, ops.B, case.ldb, case.orderB, C, case.ldc, case.orderC, case.mode)
    got = W.extract(C, case.m, case.n, case.orderC, case.ldc)
    assert np.array_equal(got, _np_expected(ops, case))
    mask = W.padding_mask(case.m, case.n, case.orderC, case.ldc)
    assert (C[mask] == W.SENTINEL_WORD).all()


def test_every_case_is_overflow_free():
    for case in W.all_cases():
        assert W.magnitude_bound(case) < 2**31, case.name


# ---------------------------------------------------------------------------
# P10  integer Freivalds check on a mid-size product
# ---------------------------------------------------------------------------

def test_freivalds_midsize(oracle):
    rng = np.random.default_rng(13)
    m, n, k = 300, 280, 520
    A, B = rand(rng, (m, k), np.int8), rand(rng, (k, n), np.int8)
    got, _, _ = run(oracle, A, B)
    for _ in range(4):
        x = rng.integers(-3, 3, size=n, endpoint=True).astype(np.int64)
        assert np.array_equal(got.astype(np.int64) @ x, A.astype(np.int64) @ (B.astype(np.int64) @ x))


# ---------------------------------------------------------------------------
# degenerate sizes and argument checks
# ---------------------------------------------------------------------------

def test_degenerate_sizes(oracle):
    C = np.full(12, 77, dtype=np.int32)
    e8 = np.zeros(0, dtype=np.int8)
    # k == 0: overwrite zeroes the 3 x 3 matrix and leaves the padding, accumulate leaves all
    oracle.gemm_s8s8s32(3, 3, 0, e8, 1, R, e8, 3, R, C, 4, R, OVW)
    assert np.array_equal(C.reshape(3, 4), np.array([[0, 0, 0, 77]] * 3))
    C[:] = 77
    oracle.gemm_s8s8s32(3, 3, 0, e8, 1, R, e8, 3, R, C, 4, R, ACC)
    assert (C == 77).all()
    oracle.gemm_s8s8s32(0, 3, 5, e8, 5, R, np.zeros(15, np.int8), 3, R, C, 3, R, OVW)
    oracle.gemm_s8s8s32(3, 0, 5, np.zeros(15, np.int8), 5, R, e8, 1, R, C, 1, R, OVW)
    assert (C == 77).all()


def test_argument_checks(oracle):
    A, B, C = np.zeros(6, np.int8), np.zeros(6, np.int8), np.zeros(4, np.int32)
    with pytest.raises(ValueError):
        oracle.gemm_s8s8s32(2, 2, 3, A, 2, R, B, 2, R, C, 2, R, OVW)      # lda < k
    with pytest.raises(ValueError):
        oracle.gemm_s8s8s32(2, 2, 3, A, 3, R, B, 2, R, C, 1, R, OVW)      # ldc < n
    with pytest.raises(ValueError):
        oracle.gemm_s8s8s32(2, 2, 3, A, 3, 2, B, 2, R, C, 2, R, OVW)      # bad order
    with pytest.raises(TypeError):
        oracle.gemm_u8s8s32(2, 2, 3, A, 3, R, B, 2, R, C, 2, R, OVW)      # wrong dtype


# ---------------------------------------------------------------------------
# dequantised variant (paper Section 7.3: C^r = s_A s_B C^q)
# ---------------------------------------------------------------------------

def run_dequant(oracle, A2d, B2d, scale, C0=None, mode=OVW, oa=R, ob=R, oc=R, pad=0):
    m, k = A2d.shape
    n = B2d.shape[1]
    lda = (k if oa == R else m) + pad
    ldb = (n if ob == R else k) + pad
    ldc = (n if oc == R else m) + pad
    A = W.embed(A2d, oa, lda, A2d.dtype.type(W.SENTINEL_BYTE))
    B = W.embed(B2d, ob, ldb, B2d.dtype.type(W.SENTINEL_BYTE))
    C = None if C0 is None else W.embed(C0.astype(np.float32), oc, ldc, np.float32(-77.0))
    return oracle.gemm_dequant(A2d.dtype == np.uint8, B2d.dtype == np.uint8, m, n, k,
                               A, lda, oa, B, ldb, ob, scale, C, ldc, oc, mode)


def test_dequant_hand_worked_example(oracle):
    g = _read_matrices(os.path.join(GOLDEN, "hand_worked_2x3x4.txt"))
    A, B = g["A"].astype(np.int8), g["B"].astype(np.int8)
    got = run_dequant(oracle, A, B, 0.125)
    assert np.array_equal(got * 1000, g["DEQ_x1000"].astype(np.float64))
    # scale 1: the integer result itself, also for the unsigned reading of A
    assert np.array_equal(run_dequant(oracle, A, B, 1.0), g["AB"].astype(np.float64))
    assert np.array_equal(run_dequant(oracle, A.view(np.uint8), B, 1.0), g["AuB"].astype(np.float64))
    # accumulate: C0 + scale * S with exactly representable numbers
    C0 = np.array([[1.5, -2.25, 0.0], [1024.0, -0.5, 3.0]], dtype=np.float32)
    got = run_dequant(oracle, A, B, 0.5, C0, mode=ACC)
    assert np.array_equal(got, C0.astype(np.float64) + 0.5 * g["AB"])


@pytest.mark.parametrize("types", ["s8s8", "u8s8", "s8u8"])
def test_dequant_matches_integer_oracle_times_scale(oracle, types):
    rng = np.random.default_rng(31)
    m, n, k = 17, 13, 200
    ta = np.uint8 if types == "u8s8" else np.int8
    tb = np.uint8 if types == "s8u8" else np.int8
    A, B = rand(rng, (m, k), ta), rand(rng, (k, n), tb)
    S, _, _ = run(oracle, A, B)                       # integer oracle, pinned above
    for scale in (1.0, 2.0 ** -9, 0.1, 3.7e-4, -0.33):
        s32 = float(np.float32(scale))                # the entry points take a float
        got = run_dequant(oracle, A, B, scale, oa=CM, ob=CM, pad=3)
        want = np.array([[s32 * int(S[i, j]) for j in range(n)] for i in range(m)])
        assert np.array_equal(got, want)              # int32 * float is exact in double
    C0 = rng.standard_normal((m, n)).astype(np.float32)
    got = run_dequant(oracle, A, B, 0.25, C0, mode=ACC, oc=CM, pad=5)
    assert np.array_equal(got, C0.astype(np.float64) + 0.25 * S)


def test_dequant_closed_forms_and_wraparound(oracle):
    k = 4608
    A = np.full((3, k), 255, dtype=np.uint8)
    B = np.full((k, 2), -128, dtype=np.int8)
    got = run_dequant(oracle, A, B, 2.0 ** -10)
    assert (got == -150405120 / 1024).all()           # 255 * (-128) * 4608, closed_forms.txt
    # the scale applies to the wrapped int32 sum (reading of the paper's silence on overflow)
    k = 131072
    got = run_dequant(oracle, np.full((1, k), -128, np.int8), np.full((k, 1), -128, np.int8), 1.0)
    assert got[0, 0] == -2.0 ** 31


# ---------------------------------------------------------------------------
# requantised variant (paper Section 7.3 applied to the output: Q = clip(rint(scale * C^q)))
# ---------------------------------------------------------------------------

def run_requant(oracle, A2d, B2d, scale, oa=R, ob=R, oq=R, pad=0):
    m, k = A2d.shape
    n = B2d.shape[1]
    lda = (k if oa == R else m) + pad
    ldb = (n if ob == R else k) + pad
    ldq = (n if oq == R else m) + pad
    A = W.embed(A2d, oa, lda, A2d.dtype.type(W.SENTINEL_BYTE))
    B = W.embed(B2d, ob, ldb, B2d.dtype.type(W.SENTINEL_BYTE))
    Q = W.embed(np.full((m, n), 0x33, dtype=np.int8), oq, ldq, np.int8(W.SENTINEL_BYTE))
    oracle.gemm_requant(A2d.dtype == np.uint8, B2d.dtype == np.uint8, m, n, k, A, lda, oa, B, ldb, ob,
                        scale, Q, ldq, oq)
    mask = W.padding_mask(m, n, oq, ldq)
    assert (Q[mask] == np.int8(W.SENTINEL_BYTE)).all()          # padding untouched
    return W.extract(Q, m, n, oq, ldq)


def test_requant_hand_worked_values(oracle):
    """A dropped rounding, rounding half away from zero, a clip to +-127, or a decision taken in
    double instead of float32 each fail one of these."""
    g = _read_matrices(os.path.join(GOLDEN, "hand_worked_2x3x4.txt"))
    q = _read_matrices(os.path.join(GOLDEN, "hand_worked_requant.txt"))
    A, B = g["A"].astype(np.int8), g["B"].astype(np.int8)
    assert np.array_equal(run_requant(oracle, A, B, 2.0 ** -3), q["Q_EIGHTH"])
    assert np.array_equal(run_requant(oracle, A, B, 2.0 ** -5), q["Q_32ND"])
    # ties and saturation: the column sums are what the file says they are (checked here in
    # Python integers), and the oracle turns them into the hand-worked bytes
    ones, TB = np.ones((1, 3), dtype=np.int8), q["TIES_B"].astype(np.int8)
    assert [sum(int(TB[p, j]) for p in range(3)) for j in range(11)] == [int(x) for x in q["TIES_S"][0]]
    assert np.array_equal(run_requant(oracle, ones, TB, 0.5), q["TIES_Q"])
    # a sum above 2^24: its float32 image decides
    a = np.full((1, 1025), -128, dtype=np.int8)
    a[0, -1] = 1
    assert 1024 * 16384 + 1 == int(q["F32_S"][0, 0])
    assert run_requant(oracle, a, a.T.copy(), 2.0 ** -25)[0, 0] == q["F32_Q_SCALE_2POWMINUS25"][0, 0]
    assert run_requant(oracle, a, a.T.copy(), 3 * 2.0 ** -25)[0, 0] == q["F32_Q_SCALE_3x2POWMINUS25"][0, 0]


@pytest.mark.parametrize("types", ["s8s8", "u8s8", "s8u8"])
def test_requant_against_the_integer_and_the_fp64_functions(oracle, types):
    rng = np.random.default_rng(37)
    m, n, k = 19, 23, 96
    ta = np.uint8 if types == "u8s8" else np.int8
    tb = np.uint8 if types == "s8u8" else np.int8
    A, B = rand(rng, (m, k), ta), rand(rng, (k, n), tb)
    S, _, _ = run(oracle, A, B)                                  # integer oracle, pinned above
    # scale 1 on sums that fit: the sum itself; beyond, the nearer end of the range
    assert np.array_equal(run_requant(oracle, A, B, 1.0), np.clip(S, -128, 127))
    for scale in (2.0 ** -9, 1.0 / 3000, 7.3e-4, -2.0 ** -10, -1.9e-3):
        s32 = np.float32(scale)
        got = run_requant(oracle, A, B, scale, oa=CM, ob=CM, oq=CM, pad=3)
        # the same three IEEE float32 operations done by numpy on the integer oracle's sums
        want = np.clip(np.rint(S.astype(np.float32) * s32), -128, 127).astype(np.int8)
        assert np.array_equal(got, want)
        # and the fp64 dequantised oracle, wherever its value is not within 1e-4 of a tie
        D = run_dequant(oracle, A, B, scale)
        safe = np.abs(np.abs(D - np.floor(D)) - 0.5) > 1e-4
        assert safe.mean() > 0.99
        assert np.array_equal(got[safe], np.clip(np.rint(D), -128, 127).astype(np.int8)[safe])
        # odd symmetry of round-half-even, away from the asymmetric ends of the range
        neg = run_requant(oracle, A, B, -scale, oa=CM, ob=CM, oq=CM, pad=3)
        inner = (got > -128) & (got < 127) & (neg > -128) & (neg < 127)
        assert np.array_equal(neg[inner], -got[inner])


def test_requant_layouts_closed_forms_and_bad_scale(oracle):
    rng = np.random.default_rng(41)
    A, B = rand(rng, (5, 40), np.int8), rand(rng, (40, 7), np.uint8)
    ref = run_requant(oracle, A, B, 1e-3)
    for oa in (R, CM):
        for ob in (R, CM):
            for oq in (R, CM):
                assert np.array_equal(run_requant(oracle, A, B, 1e-3, oa, ob, oq, pad=17), ref)
    # all(-128) x all(-128), k = 8: S = 131072; times 2^-11 = 64; times 2^-10 = 128 -> 127
    A8, B8 = np.full((2, 8), -128, np.int8), np.full((8, 3), -128, np.int8)
    assert (run_requant(oracle, A8, B8, 2.0 ** -11) == 64).all()
    assert (run_requant(oracle, A8, B8, 2.0 ** -10) == 127).all()
    assert (run_requant(oracle, A8, B8, -2.0 ** -10) == -128).all()
    assert (run_requant(oracle, A8, B8, 0.0) == 0).all()
    # an empty sum is 0; empty matrices touch nothing
    assert (run_requant(oracle, np.zeros((2, 0), np.int8), np.zeros((0, 3), np.int8), 5.0) == 0).all()
    for bad in (float("nan"), float("inf")):
        with pytest.raises(ValueError):
            run_requant(oracle, A8, B8, bad)


# ---------------------------------------------------------------------------
# 16-bit operands (oracle_mip_gemm_s16)
# ---------------------------------------------------------------------------

def test_s16_hand_worked(oracle):
    # A = [[300, -2], [-32768, 7]], B = [[1000, -1], [5, 32767]]
    #   row 0: 300*1000 + (-2)*5 = 299990;      300*(-1) + (-2)*32767 = -65834
    #   row 1: -32768*1000 + 7*5 = -32767965;   -32768*(-1) + 7*32767 = 262137
    A = np.array([300, -2, -32768, 7], dtype=np.int16)
    B = np.array([1000, -1, 5, 32767], dtype=np.int16)
    C = np.full(4, 77, dtype=np.int32)
    oracle.gemm_s16(2, 2, 2, A, 2, 0, B, 2, 0, C, 2, 0, oracle.OVERWRITE)
    assert C.tolist() == [299990, -65834, -32767965, 262137]
    oracle.gemm_s16(2, 2, 2, A, 2, 0, B, 2, 0, C, 2, 0, oracle.ACCUMULATE)
    assert C.tolist() == [2 * 299990, 2 * -65834, 2 * -32767965, 2 * 262137]
    # the same matrices stored column-major, result column-major
    At = np.array([300, -32768, -2, 7], dtype=np.int16)
    Bt = np.array([1000, 5, -1, 32767], dtype=np.int16)
    Ct = np.zeros(4, dtype=np.int32)
    oracle.gemm_s16(2, 2, 2, At, 2, 1, Bt, 2, 1, Ct, 2, 1, oracle.OVERWRITE)
    assert Ct.tolist() == [299990, -32767965, -65834, 262137]


def test_s16_wraps_and_closed_forms(oracle):
    # (-32768)^2 = 2^30 per product: four of them are 2^32 = 0, three are 3 * 2^30 = -2^30 as int32
    for k, want in ((1, 1 << 30), (2, -(1 << 31)), (3, -(1 << 30)), (4, 0), (7, -(1 << 30))):
        A = np.full(k, -32768, dtype=np.int16)
        C = np.zeros(1, dtype=np.int32)
        oracle.gemm_s16(1, 1, k, A, k, 0, A, 1, 0, C, 1, 0, oracle.OVERWRITE)
        assert C[0] == want
    # all 32767: k * 32767^2 modulo 2^32
    k = 100
    A = np.full(3 * k, 32767, dtype=np.int16)
    B = np.full(k * 2, 32767, dtype=np.int16)
    C = np.zeros(6, dtype=np.int32)
    oracle.gemm_s16(3, 2, k, A, k, 0, B, 2, 0, C, 2, 0, oracle.OVERWRITE)
    want = (k * 32767 * 32767) % (1 << 32)
    want = want - (1 << 32) if want >= (1 << 31) else want
    assert (C == want).all()
    C0 = np.arange(6, dtype=np.int32)
    C = C0.copy()
    oracle.gemm_s16(3, 2, 0, A, 1, 0, B, 2, 0, C, 2, 0, oracle.ACCUMULATE)      # k = 0: nothing added
    assert np.array_equal(C, C0)


@pytest.mark.parametrize("m,n,k,oa,ob,oc,pad", [(5, 7, 9, 0, 0, 0, 0), (16, 3, 40, 1, 0, 1, 3), (1, 33, 65, 0, 1, 0, 5),
                                                (20, 20, 300, 1, 1, 1, 1)])
def test_s16_against_python_integers_numpy_and_the_byte_oracle(oracle, m, n, k, oa, ob, oc, pad):
    rng = np.random.default_rng([m, n, k, oa, ob, oc])
    Ad = rng.integers(-32768, 32768, size=(m, k), dtype=np.int16)
    Bd = rng.integers(-32768, 32768, size=(k, n), dtype=np.int16)
    Ad[0, 0], Bd[0, 0] = -32768, -32768

    def flat(X, order, pad):
        r, c = X.shape
        ld = (c if order == 0 else r) + pad
        buf = np.full(((r if order == 0 else c), ld), 0x5A5A, dtype=np.int16)
        if order == 0:
            buf[:, :c] = X
        else:
            buf[:, :r] = X.T
        return buf.reshape(-1), ld

    A, lda = flat(Ad, oa, pad)
    B, ldb = flat(Bd, ob, pad)
    ldc = (n if oc == 0 else m) + pad
    C0 = rng.integers(-1000, 1000, size=((m if oc == 0 else n), ldc), dtype=np.int32)
    C = C0.reshape(-1).copy()
    oracle.gemm_s16(m, n, k, A, lda, oa, B, ldb, ob, C, ldc, oc, oracle.ACCUMULATE)
    exact = Ad.astype(object) @ Bd.astype(object)                    # Python integers: no overflow anywhere
    got = C.reshape(C0.shape)
    got2d = got[:, :n] if oc == 0 else got[:, :m].T
    c02d = C0[:, :n] if oc == 0 else C0[:, :m].T
    for i in range(m):
        for j in range(n):
            want = (int(exact[i, j]) + int(c02d[i, j])) % (1 << 32)
            assert int(got2d[i, j]) % (1 << 32) == want
    pad_cols = got[:, (n if oc == 0 else m):]
    assert np.array_equal(pad_cols, C0[:, (n if oc == 0 else m):])    # padding untouched
    # operands that fit a byte: the same numbers through the 8-bit oracle
    A8 = rng.integers(-128, 128, size=(m, k), dtype=np.int8)
    B8 = rng.integers(-128, 128, size=(k, n), dtype=np.int8)
    C8 = np.zeros(m * n, dtype=np.int32)
    C16 = np.zeros(m * n, dtype=np.int32)
    oracle.gemm(False, False, m, n, k, A8.reshape(-1), k, 0, B8.reshape(-1), n, 0, C8, n, 0, oracle.OVERWRITE)
    oracle.gemm_s16(m, n, k, A8.astype(np.int16).reshape(-1), k, 0, B8.astype(np.int16).reshape(-1), n, 0,
                    C16, n, 0, oracle.OVERWRITE)
    assert np.array_equal(C8, C16)
    assert np.array_equal(C16.reshape(m, n), A8.astype(np.int64) @ B8.astype(np.int64))
