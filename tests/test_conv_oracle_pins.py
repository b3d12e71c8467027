"""Pins of the convolution-lowering and weight-packing oracle (oracle/mip_conv_oracle.c), CPU only.

Each test checks the oracle against something other than itself: hand-worked
values, brute force in Python integers, closed forms, the lowering identity
between its two independent functions and the GEMM oracle, a numpy
sliding-window product.  Paper Section 7.2 (CONV lowered by IM2COL to a GEMM of
dimensions (c_o, b h_o w_o, c_i h_f w_f)).
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_conv_3x3x2.txt")


def _golden():
    out, name, shape, vals = {}, None, None, []
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0][0].isalpha():
            if name:
                out[name] = np.array(vals, dtype=np.int64).reshape(shape)
            name, shape, vals = tok[0], tuple(int(t) for t in tok[1:]), []
        else:
            vals += [int(t) for t in tok]
    out[name] = np.array(vals, dtype=np.int64).reshape(shape)
    return out


def _rand(rng, b, hi, wi, ci, co, hf, wf):
    I = rng.integers(0, 256, size=(b, hi, wi, ci), dtype=np.uint8)
    F = rng.integers(-128, 128, size=(co, hf, wf, ci), dtype=np.int8)
    return I, F


def _brute(I, F, s, p):
    """Python integers, output-stationary dictionary walk over taps (a different loop nest)."""
    b, hi, wi, ci = I.shape
    co, hf, wf, _ = F.shape
    ho, wo = (hi + 2 * p - hf) // s + 1, (wi + 2 * p - wf) // s + 1
    O = {}
    for g in range(b):
        for iy in range(hi):
            for ix in range(wi):
                for y in range(hf):
                    for x in range(wf):
                        ty, tx = iy + p - y, ix + p - x          # s * oy, s * ox
                        if ty < 0 or tx < 0 or ty % s or tx % s:
                            continue
                        oy, ox = ty // s, tx // s
                        if oy >= ho or ox >= wo:
                            continue
                        for o in range(co):
                            acc = 0
                            for c in range(ci):
                                acc += int(F[o, y, x, c]) * int(I[g, iy, ix, c])
                            O[(g, oy, ox, o)] = O.get((g, oy, ox, o), 0) + acc
    out = np.zeros((b, ho, wo, co), dtype=np.int64)
    for key, v in O.items():
        out[key] = v
    return out


def test_hand_worked_example(oracle):
    gold = _golden()
    I = gold["I"].astype(np.uint8)[None]
    F = gold["F"].astype(np.int8)[None]
    assert np.array_equal(oracle.conv_direct(I, F, 1, 0)[0, :, :, 0], gold["O_s1_p0"])
    assert np.array_equal(oracle.conv_direct(I, F, 2, 1)[0, :, :, 0], gold["O_s2_p1"])
    M = oracle.im2col_u8(I, 2, 2, 1, 0)
    assert M.shape == (4, 8)
    assert np.array_equal(M[0], gold["M_s1_p0_row0"][0]) and np.array_equal(M[3], gold["M_s1_p0_row3"][0])
    M = oracle.im2col_u8(I, 2, 2, 2, 1)
    assert np.array_equal(M[0], gold["M_s2_p1_row0"][0]) and np.array_equal(M[2], gold["M_s2_p1_row2"][0])


@pytest.mark.parametrize("b,hi,wi,ci,co,hf,wf,s,p", [
    (1, 3, 3, 1, 1, 2, 2, 1, 0), (2, 5, 4, 3, 2, 3, 3, 1, 1), (1, 6, 7, 2, 3, 3, 2, 2, 1),
    (2, 4, 4, 4, 2, 1, 1, 1, 0), (1, 7, 5, 2, 2, 3, 3, 2, 0), (1, 5, 5, 1, 1, 5, 5, 1, 2),
    (1, 8, 3, 3, 2, 2, 3, 3, 1), (1, 2, 2, 5, 4, 3, 3, 1, 1)])
def test_brute_force_tiny(oracle, b, hi, wi, ci, co, hf, wf, s, p):
    I, F = _rand(np.random.default_rng([b, hi, wi, ci, co, hf, wf, s, p]), b, hi, wi, ci, co, hf, wf)
    assert np.array_equal(oracle.conv_direct(I, F, s, p), _brute(I, F, s, p))


def test_out_extent_formula(oracle):
    assert oracle.conv_out_extent(56, 3, 1, 1) == 56
    assert oracle.conv_out_extent(224, 7, 2, 3) == 112
    assert oracle.conv_out_extent(7, 1, 1, 0) == 7
    assert oracle.conv_out_extent(5, 3, 2, 0) == 2
    assert oracle.conv_out_extent(2, 3, 1, 0) == -1        # filter larger than the image


@pytest.mark.parametrize("shape", [(2, 9, 8, 16, 5, 3, 3, 1, 1), (1, 14, 14, 32, 8, 3, 3, 2, 1),
                                   (3, 7, 7, 64, 16, 1, 1, 1, 0), (1, 12, 10, 8, 4, 5, 3, 2, 2)])
def test_lowering_identity_against_the_gemm_oracle(oracle, shape):
    """CONV(F, I) equals the GEMM of F (c_o x k) with the augmented matrix (k x n): two
    routes through three independent functions."""
    b, hi, wi, ci, co, hf, wf, s, p = shape
    I, F = _rand(np.random.default_rng(list(shape)), b, hi, wi, ci, co, hf, wf)
    O = oracle.conv_direct(I, F, s, p)
    M = oracle.im2col_u8(I, hf, wf, s, p)
    n, k = M.shape
    assert n == O.shape[0] * O.shape[1] * O.shape[2] and k == ci * hf * wf
    C = np.zeros(n * co, dtype=np.int32)
    # A = F as c_o x k row-major; B = M as k x n column-major; C column-major with ldc = c_o,
    # which is the O tensor in its own memory order
    oracle.gemm(False, True, co, n, k, F.reshape(-1), k, oracle.ROW_MAJOR, M.reshape(-1), k,
                oracle.COL_MAJOR, C, co, oracle.COL_MAJOR, oracle.OVERWRITE)
    assert np.array_equal(C, O.reshape(-1))


def test_one_by_one_filter_is_a_plain_matrix_product(oracle):
    rng = np.random.default_rng(5)
    I, F = _rand(rng, 2, 6, 5, 24, 7, 1, 1)
    assert np.array_equal(oracle.im2col_u8(I, 1, 1, 1, 0), I.reshape(-1, 24))
    want = I.reshape(-1, 24).astype(np.int64) @ F.reshape(7, 24).astype(np.int64).T
    assert np.array_equal(oracle.conv_direct(I, F, 1, 0).reshape(-1, 7), want)


def test_delta_filter_copies_the_image(oracle):
    rng = np.random.default_rng(6)
    ci = 5
    I = rng.integers(0, 256, size=(2, 6, 7, ci), dtype=np.uint8)
    F = np.zeros((ci, 3, 3, ci), dtype=np.int8)
    for c in range(ci):
        F[c, 1, 1, c] = 1                                   # centre tap, channel c -> output c
    assert np.array_equal(oracle.conv_direct(I, F, 1, 1), I.astype(np.int32))
    F2 = np.zeros((1, 3, 3, ci), dtype=np.int8)
    F2[0, 0, 2, 3] = -1                                     # tap (0, 2): pixel (oy - 1, ox + 1), channel 3
    want = np.zeros((2, 6, 7, 1), dtype=np.int32)
    want[:, 1:, :-1, 0] = -I[:, :-1, 1:, 3].astype(np.int32)
    assert np.array_equal(oracle.conv_direct(I, F2, 1, 1), want)


def test_all_ones_counts_the_taps_inside_the_image(oracle):
    ci, hi, wi = 4, 6, 9
    I = np.ones((1, hi, wi, ci), dtype=np.uint8)
    F = np.ones((2, 3, 3, ci), dtype=np.int8)
    O = oracle.conv_direct(I, F, 1, 1)
    rows = np.array([2] + [3] * (hi - 2) + [2])
    cols = np.array([2] + [3] * (wi - 2) + [2])
    want = ci * rows[:, None] * cols[None, :]
    assert np.array_equal(O[0, :, :, 0], want) and np.array_equal(O[0, :, :, 1], want)
    # the augmented matrix holds a zero exactly where a tap falls outside
    M = oracle.im2col_u8(I, 3, 3, 1, 1)
    assert np.array_equal(M.sum(axis=1).reshape(hi, wi), want)
    assert int((M == 0).sum()) == M.size - int(want.sum())


def test_stride_subsamples_the_unit_stride_result(oracle):
    rng = np.random.default_rng(8)
    I, F = _rand(rng, 2, 11, 9, 6, 3, 3, 3)
    full = oracle.conv_direct(I, F, 1, 1)
    assert np.array_equal(oracle.conv_direct(I, F, 2, 1), full[:, ::2, ::2])
    assert np.array_equal(oracle.conv_direct(I, F, 3, 1), full[:, ::3, ::3])


@pytest.mark.parametrize("shape", [(2, 10, 12, 16, 6, 3, 3, 1, 1), (1, 15, 9, 8, 3, 5, 5, 2, 2),
                                   (2, 8, 8, 32, 4, 3, 3, 2, 0)])
def test_numpy_sliding_window_product(oracle, shape):
    b, hi, wi, ci, co, hf, wf, s, p = shape
    I, F = _rand(np.random.default_rng(list(shape)), b, hi, wi, ci, co, hf, wf)
    padded = np.pad(I.astype(np.int64), ((0, 0), (p, p), (p, p), (0, 0)))
    win = np.lib.stride_tricks.sliding_window_view(padded, (hf, wf), axis=(1, 2))[:, ::s, ::s]
    want = np.einsum("gabcyx,oyxc->gabo", win, F.astype(np.int64))
    assert np.array_equal(oracle.conv_direct(I, F, s, p), want)
    M = oracle.im2col_u8(I, hf, wf, s, p)
    assert np.array_equal(M.reshape(win.shape[0], win.shape[1], win.shape[2], hf, wf, ci),
                          win.transpose(0, 1, 2, 4, 5, 3))


def test_accumulate_wraparound_and_pitch(oracle):
    rng = np.random.default_rng(9)
    I, F = _rand(rng, 1, 5, 5, 3, 2, 3, 3)
    O0 = rng.integers(-1000, 1000, size=(1, 5, 5, 2), dtype=np.int32)
    got = oracle.conv_direct(I, F, 1, 1, O=O0.copy(), mode=oracle.ACCUMULATE)
    assert np.array_equal(got, O0 + oracle.conv_direct(I, F, 1, 1))
    # sums wrap modulo 2^32: 255 * (-128) * 65799 = -2147679360 = 2147287936 (mod 2^32)
    ci = 7311
    Ibig = np.full((1, 3, 3, ci), 255, dtype=np.uint8)
    Fbig = np.full((1, 3, 3, ci), -128, dtype=np.int8)
    assert oracle.conv_direct(Ibig, Fbig, 1, 0).reshape(-1)[0] == 2147287936
    # a row pitch larger than k leaves the tail of every row alone
    M = oracle.im2col_u8(I, 3, 3, 1, 1, ldm=27 + 5, fill=0x5A)
    assert (M[:, 27:] == 0x5A).all() and np.array_equal(M[:, :27], oracle.im2col_u8(I, 3, 3, 1, 1))


def test_rejects_a_filter_that_does_not_fit(oracle):
    I = np.zeros((1, 2, 2, 1), dtype=np.uint8)
    F = np.zeros((1, 3, 3, 1), dtype=np.int8)
    with pytest.raises(ValueError):
        oracle.conv_direct(I, F, 1, 0)
    with pytest.raises(ValueError):
        oracle.im2col_u8(I, 3, 3, 1, 0)


# ---------------------------------------------------------------------------
# weight pre-packing (oracle_pack_b): the same matrix with k contiguous
# ---------------------------------------------------------------------------

def test_pack_b_hand_worked(oracle):
    # B = [[1, 2, 3], [4, 5, 6]] (k = 2, n = 3): the columns (1,4), (2,5), (3,6) become rows
    Brow = np.array([1, 2, 3, 0x77, 4, 5, 6, 0x77], dtype=np.uint8)          # row-major, ldb = 4
    assert oracle.pack_b(2, 3, Brow, 4, oracle.ROW_MAJOR).tolist() == [[1, 4], [2, 5], [3, 6]]
    Bcol = np.array([1, 4, 0x77, 2, 5, 0x77, 3, 6, 0x77], dtype=np.uint8)    # column-major, ldb = 3
    assert oracle.pack_b(2, 3, Bcol, 3, oracle.COL_MAJOR).tolist() == [[1, 4], [2, 5], [3, 6]]
    P = oracle.pack_b(2, 3, Brow, 4, oracle.ROW_MAJOR, ldp=5, fill=0xEE)
    assert P.tolist() == [[1, 4, 0xEE, 0xEE, 0xEE], [2, 5, 0xEE, 0xEE, 0xEE], [3, 6, 0xEE, 0xEE, 0xEE]]


@pytest.mark.parametrize("k,n,order,pad", [(7, 5, 0, 0), (64, 64, 0, 3), (100, 37, 1, 5), (1, 9, 0, 0),
                                           (130, 200, 0, 17), (33, 1, 1, 0)])
def test_pack_b_is_the_numpy_transpose_and_leaves_the_product_unchanged(oracle, k, n, order, pad):
    rng = np.random.default_rng([k, n, order, pad])
    dense = rng.integers(-128, 128, size=(k, n), dtype=np.int8)
    ldb = (n if order == 0 else k) + pad
    flat = np.full(((k if order == 0 else n), ldb), 0x5A, dtype=np.uint8)
    if order == 0:
        flat[:, :n] = dense.view(np.uint8)
    else:
        flat[:, :k] = dense.T.view(np.uint8)
    P = oracle.pack_b(k, n, flat.reshape(-1), ldb, order, ldp=k + 2)
    assert np.array_equal(P[:, :k], dense.T.view(np.uint8)) and (P[:, k:] == 0x5A).all()
    # the GEMM on the packed matrix (column-major, ldb = ldp) equals the GEMM on the original
    m = 6
    A = rng.integers(-128, 128, size=m * k, dtype=np.int8)
    C1 = np.zeros(m * n, dtype=np.int32)
    C2 = np.zeros(m * n, dtype=np.int32)
    oracle.gemm(False, False, m, n, k, A, k, 0, flat.reshape(-1).view(np.int8), ldb, order, C1, n, 0, 0)
    oracle.gemm(False, False, m, n, k, A, k, 0, P.reshape(-1).view(np.int8), k + 2, 1, C2, n, 0, 0)
    assert np.array_equal(C1, C2)
    assert np.array_equal(C1.reshape(m, n), A.reshape(m, k).astype(np.int64) @ dense.astype(np.int64))


# ---------------------------------------------------------------------------
# k-sums of the weights and the packed-weights object (oracle_column_sums_s8, pack_weights)
# ---------------------------------------------------------------------------

def test_column_sums_hand_worked(oracle):
    # B = [[1, -2, 3], [-4, 5, -6], [7, -8, 127]] (k = 3, n = 3): columns sum to 4, -5, 124
    Brow = np.array([1, -2, 3, 99, -4, 5, -6, 99, 7, -8, 127, 99], dtype=np.int8)       # ldb = 4
    assert oracle.column_sums(3, 3, Brow, 4, oracle.ROW_MAJOR).tolist() == [4, -5, 124]
    Bcol = np.array([1, -4, 7, 2, -8, 2, 5 - 7, 0, -6 + 9, 127 - 3], dtype=np.int8)
    # column-major with ldb = 3 and nothing between the columns: (1,-4,7), (2,-8,2), (-2,0,3); the 10th byte is not read
    assert oracle.column_sums(3, 3, Bcol, 3, oracle.COL_MAJOR).tolist() == [4, -4, 1]
    assert oracle.column_sums(0, 2, np.zeros(0, dtype=np.int8), 2, oracle.ROW_MAJOR).tolist() == [0, 0]


@pytest.mark.parametrize("k,n,order,pad", [(7, 5, 0, 0), (64, 64, 1, 3), (300, 37, 0, 5), (1, 9, 1, 0),
                                           (1030, 20, 0, 17)])
def test_column_sums_are_a_row_of_ones_times_b(oracle, k, n, order, pad):
    """Pinned by the GEMM oracle (1^T B, a 1 x k matrix of ones as A), by numpy in 64 bits, and
    by the identity they exist for: with unsigned activations a,
    sum_p a b = sum_p (a - 128) b + 128 s, checked through three GEMM oracle calls."""
    rng = np.random.default_rng([k, n, order, pad, 5])
    dense = rng.integers(-128, 128, size=(k, n), dtype=np.int8)
    ldb = (n if order == 0 else k) + pad
    flat = np.full(((k if order == 0 else n), ldb), 0x5A, dtype=np.uint8)
    if order == 0:
        flat[:, :n] = dense.view(np.uint8)
    else:
        flat[:, :k] = dense.T.view(np.uint8)
    flat = flat.reshape(-1).view(np.int8)
    s = oracle.column_sums(k, n, flat, ldb, order)
    assert np.array_equal(s.astype(np.int64), dense.astype(np.int64).sum(axis=0))
    ones = np.ones(k, dtype=np.int8)
    C = np.zeros(n, dtype=np.int32)
    oracle.gemm(False, False, 1, n, k, ones, k, 0, flat, ldb, order, C, n, 0, 0)
    assert np.array_equal(C, s)
    m = 5
    Au = rng.integers(0, 256, size=m * k, dtype=np.uint8)
    As = (Au ^ 0x80).view(np.int8)                 # a - 128 as a signed byte
    Cu = np.zeros(m * n, dtype=np.int32)
    Cs = np.zeros(m * n, dtype=np.int32)
    oracle.gemm(True, False, m, n, k, Au, k, 0, flat, ldb, order, Cu, n, 0, 0)
    oracle.gemm(False, False, m, n, k, As, k, 0, flat, ldb, order, Cs, n, 0, 0)
    assert np.array_equal(Cu.reshape(m, n), Cs.reshape(m, n) + 128 * s[None, :])


def test_column_sums_wrap(oracle):
    # 2^24 + 5 entries of -128 in one column: -(2^31) - 640, which wraps to 2^31 - 640
    k = (1 << 24) + 5
    B = np.full(k, -128, dtype=np.int8)
    assert oracle.column_sums(k, 1, B, 1, oracle.ROW_MAJOR).tolist() == [(1 << 31) - 640]


def test_packed_weights_layout_and_contents(oracle):
    assert oracle.packed_weights_layout(1, 1) == (64, 256, 64 * 256, 64 * 256 + 4)
    assert oracle.packed_weights_layout(1000, 256) == (1024, 256, 1024 * 256, 1024 * 256 + 1024)
    assert oracle.packed_weights_layout(1024, 257) == (1024, 512, 1024 * 512, 1024 * 512 + 4 * 257)
    assert oracle.packed_weights_layout(1025, 300) == (1152, 512, 1152 * 512, 1152 * 512 + 1200)
    # B = [[1, 2, 3], [4, 5, -6]] row-major: columns (1,4), (2,5), (3,-6), each padded to 64 bytes,
    # 253 zero columns, then the sums 5, 7, -3
    B = np.array([1, 2, 3, 4, 5, -6], dtype=np.int8)
    P = oracle.pack_weights(2, 3, B, 3, oracle.ROW_MAJOR)
    kp, cols, at, total = oracle.packed_weights_layout(2, 3)
    assert P.size == total == 64 * 256 + 12
    body = P[:at].reshape(cols, kp).view(np.int8)
    assert body[0, :2].tolist() == [1, 4] and body[1, :2].tolist() == [2, 5] and body[2, :2].tolist() == [3, -6]
    assert not body[:, 2:].any() and not body[3:].any()
    assert P[at:].view(np.int32).tolist() == [5, 7, -3]
