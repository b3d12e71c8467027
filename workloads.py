"""Seeded synthetic inputs for the MIP GEMM: the one module both the GPU path's
tests/bench and the CPU oracle's tests draw their operands from.

It holds no arithmetic of the method: it only draws random bytes / words with
numpy's PCG64 and lays matrices out in flat buffers (row- or column-major, with
a leading dimension and sentinel-filled padding).

The shapes stand in for the workloads of the paper's Section 7.2: convolution
layers of a ResNet-50-type network lowered to GEMM with
(m, n, k) = (c_o, b*h_o*w_o, c_i*h_f*w_f), and the weight-times-activation
GEMMs of a transformer encoder block (Table "Dimensions of the GEMM operations
in the transformer encoder"), plus square sizes and odd shapes.  Trained
weights and datasets are not needed: the integer GEMM's result and run time
depend only on the operand types and shapes.

Value recipes:
  uniform(lo, hi)  integers, both ends included
  normal(sigma)    rint(N(0, sigma)) (round half to even), clipped to the type's range
  const(v)         every element v
Draw order inside one case: A, then B, then C.  One generator per case,
PCG64 seeded with [config seed, case index].
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Iterator, List, Tuple

import numpy as np

ROW_MAJOR, COL_MAJOR = 0, 1
OVERWRITE, ACCUMULATE = 0, 1

SENTINEL_BYTE = 0x5A
SENTINEL_WORD = 0x5A5A5A5A


@dataclass(frozen=True)
class Case:
    name: str
    config: int
    index: int                      # position inside its config (seeds the generator)
    m: int
    n: int
    k: int
    a_unsigned: bool = False
    b_unsigned: bool = False
    orderA: int = ROW_MAJOR
    orderB: int = ROW_MAJOR
    orderC: int = ROW_MAJOR
    pad: int = 0                    # ld = smallest legal ld + pad, for A, B and C
    mode: int = OVERWRITE
    a_dist: Tuple = ("uniform", -128, 127)
    b_dist: Tuple = ("uniform", -128, 127)
    c_dist: Tuple = ("sentinel",)   # what C holds before the call
    seed: int = 0

    @property
    def entry(self) -> str:
        return {(False, False): "s8s8s32", (True, False): "u8s8s32",
                (False, True): "s8u8s32"}[(self.a_unsigned, self.b_unsigned)]

    @property
    def lda(self) -> int:
        return (self.k if self.orderA == ROW_MAJOR else self.m) + self.pad

    @property
    def ldb(self) -> int:
        return (self.n if self.orderB == ROW_MAJOR else self.k) + self.pad

    @property
    def ldc(self) -> int:
        return (self.n if self.orderC == ROW_MAJOR else self.m) + self.pad

    @property
    def ops(self) -> int:
        """2*m*n*k, the paper's count of useful operations (Section 7.4)."""
        return 2 * self.m * self.n * self.k

    @property
    def algorithmic_bytes(self) -> int:
        """Each operand element read once, each C element written once (and read once when accumulating)."""
        c = 4 * self.m * self.n
        return self.m * self.k + self.k * self.n + c * (2 if self.mode == ACCUMULATE else 1)


@dataclass
class Operands:
    A: np.ndarray       # flat int8/uint8 buffer
    B: np.ndarray       # flat int8/uint8 buffer
    C: np.ndarray       # flat int32 buffer: contents before the call
    A2d: np.ndarray     # logical m x k view (a copy), same dtype
    B2d: np.ndarray     # logical k x n
    C2d: np.ndarray     # logical m x n contents before the call


def buffer_len(rows: int, cols: int, ld: int, order: int) -> int:
    """Elements in the flat buffer: every row (or column) owns a full ld."""
    return (rows if order == ROW_MAJOR else cols) * ld


def embed(X: np.ndarray, order: int, ld: int, sentinel) -> np.ndarray:
    """Lay the 2-D array X out in a flat buffer; padding elements hold ``sentinel``."""
    rows, cols = X.shape
    if order == ROW_MAJOR:
        buf = np.full((rows, ld), sentinel, dtype=X.dtype)
        buf[:, :cols] = X
    else:
        buf = np.full((cols, ld), sentinel, dtype=X.dtype)
        buf[:, :rows] = X.T
    return buf.reshape(-1)


def extract(buf: np.ndarray, rows: int, cols: int, order: int, ld: int) -> np.ndarray:
    """Logical rows x cols matrix held in the flat buffer (a copy)."""
    if order == ROW_MAJOR:
        return buf.reshape(rows, ld)[:, :cols].copy()
    return buf.reshape(cols, ld)[:, :rows].T.copy()


def padding_mask(rows: int, cols: int, order: int, ld: int) -> np.ndarray:
    """Boolean flat mask, True on leading-dimension padding."""
    if order == ROW_MAJOR:
        mask = np.ones((rows, ld), dtype=bool)
        mask[:, :cols] = False
    else:
        mask = np.ones((cols, ld), dtype=bool)
        mask[:, :rows] = False
    return mask.reshape(-1)


def _draw(rng: np.random.Generator, dist: Tuple, shape, dtype) -> np.ndarray:
    info = np.iinfo(dtype)
    kind = dist[0]
    if kind == "uniform":
        lo, hi = dist[1], dist[2]
        return rng.integers(lo, hi, size=shape, endpoint=True, dtype=np.int64).astype(dtype)
    if kind == "normal":
        x = np.rint(rng.normal(0.0, dist[1], size=shape))
        return np.clip(x, info.min, info.max).astype(dtype)
    if kind == "const":
        return np.full(shape, dist[1], dtype=dtype)
    if kind == "sentinel":
        return np.full(shape, np.array(SENTINEL_WORD, dtype=np.uint32).astype(dtype)
                       if dtype == np.int32 else SENTINEL_BYTE, dtype=dtype)
    raise ValueError("unknown distribution %r" % (dist,))


def materialize(case: Case) -> Operands:
    rng = np.random.Generator(np.random.PCG64([case.seed, case.index]))
    a_t = np.uint8 if case.a_unsigned else np.int8
    b_t = np.uint8 if case.b_unsigned else np.int8
    A2d = _draw(rng, case.a_dist, (case.m, case.k), a_t)
    B2d = _draw(rng, case.b_dist, (case.k, case.n), b_t)
    C2d = _draw(rng, case.c_dist, (case.m, case.n), np.int32)
    return Operands(
        A=embed(A2d, case.orderA, case.lda, a_t(SENTINEL_BYTE)),
        B=embed(B2d, case.orderB, case.ldb, b_t(SENTINEL_BYTE)),
        C=embed(C2d, case.orderC, case.ldc, np.int32(SENTINEL_WORD)),
        A2d=A2d, B2d=B2d, C2d=C2d)


def magnitude_bound(case: Case) -> int:
    """Largest |C| any element can reach: max|a| * max|b| * k + max|C0|.

    Every case below keeps this under 2^31, so wraparound versus saturation can
    never decide a comparison.
    """
    def amax(dist, unsigned):
        if dist[0] == "const":
            return abs(dist[1])
        if dist[0] == "uniform":
            return max(abs(dist[1]), abs(dist[2]))
        return 255 if unsigned else 128
    c0 = 1000 if case.c_dist[0] == "uniform" else 0
    if case.mode == ACCUMULATE and case.c_dist[0] == "sentinel":
        c0 = SENTINEL_WORD
    return amax(case.a_dist, case.a_unsigned) * amax(case.b_dist, case.b_unsigned) * case.k + c0


# ---------------------------------------------------------------------------
# The five configuration groups
# ---------------------------------------------------------------------------

SQUARE_SIZES = (1024, 2048, 4096, 8192)

# (c_o, h_o*w_o, c_i*h_f*w_f): convolution layers of a ResNet-50-type network
# lowered to GEMM (Section 7.2: (m, n, k) = (c_o, b*h_o*w_o, c_i*h_f*w_f)).
CONV_LAYERS = ((64, 3136, 576), (128, 784, 1152), (256, 196, 2304),
               (512, 49, 4608), (2048, 49, 512))
CONV_BATCHES = (1, 32)
# The convolutions those GEMMs stand for (hi = wi, ci, co, hf = wf, stride, pad): 3 x 3
# layers of the four stages and a 1 x 1 expansion, in the order of CONV_LAYERS.
CONV_GEOMETRY = ((56, 64, 64, 3, 1, 1), (28, 128, 128, 3, 1, 1), (14, 256, 256, 3, 1, 1),
                 (7, 512, 512, 3, 1, 1), (7, 512, 2048, 1, 1, 0))


# the 7 x 7, stride-2 first layer of such a network on 224 x 224 RGB images: 3 channels, so
# no 64-channel blocks to gather and a k (147) that no direct-to-LDS kernel takes
CONV_FIRST_LAYER = (224, 3, 64, 7, 2, 3)


def resnet50_conv_layers():
    """Every convolution of a ResNet-50 v1.5-type network on 224 x 224 images, the paper's first
    workload (Section 7.2: 49 convolutions in 16 bottleneck blocks plus the shortcut projections
    and the stem), as (name, geometry, how many times it occurs) with geometry = (hi, ci, co, hf,
    stride, pad); identical layers are merged as the paper merges them."""
    layers = [("stem", (224, 3, 64, 7, 2, 3))]
    size, cin = 56, 64                                   # after the stem's 3 x 3 / 2 pooling
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        for blk in range(blocks):
            stride = 2 if (blk == 0 and stage > 1) else 1   # v1.5: the 3 x 3 carries the stride
            tag = "s%db%d" % (stage, blk + 1)
            layers.append((tag + "_1x1a", (size, cin, width, 1, 1, 0)))
            layers.append((tag + "_3x3", (size, width, width, 3, stride, 1)))
            out = size // stride
            layers.append((tag + "_1x1b", (out, width, 4 * width, 1, 1, 0)))
            if blk == 0:
                layers.append((tag + "_proj", (size, cin, 4 * width, 1, stride, 0)))
            size, cin = out, 4 * width
    merged = {}
    for name, geo in layers:
        merged.setdefault(geo, [name, 0])[1] += 1
    return [(v[0], geo, v[1]) for geo, v in merged.items()]


def conv_tensors(b, geometry, seed=2):
    """Synthetic image tensor (uint8, b x hi x wi x ci) and filters (int8, co x hf x wf x ci)
    with the value distributions of the conv-as-GEMM workload."""
    hi, ci, co, hf, stride, pad = geometry
    rng = np.random.Generator(np.random.PCG64([seed, b, hi, ci, co, hf]))
    image = rng.integers(0, 256, size=(b, hi, hi, ci), dtype=np.uint8)
    filt = np.clip(np.rint(rng.standard_normal((co, hf, hf, ci)) * 32.0), -128, 127).astype(np.int8)
    return image, filt

# tokens x out-features x in-features, encoder linear layers with 1024 tokens
ENCODER_LAYERS = ((1024, 2304, 768), (1024, 768, 768), (1024, 3072, 768), (1024, 768, 3072))
DECODE_M = (1, 16, 64)
DECODE_NK = ((4096, 4096), (11008, 4096), (4096, 11008))

ODD_SHAPES = ((1000, 999, 1001), (1, 4097, 513), (4095, 3, 2049), (7, 7, 3), (3000, 5000, 64))
ODD_PAD = 17


def config1() -> List[Case]:
    return [Case("c1_256_acc", 1, 0, 256, 256, 256, mode=ACCUMULATE,
                 c_dist=("uniform", -1000, 1000), seed=0)]


def config2(sizes=SQUARE_SIZES) -> List[Case]:
    out, idx = [], 0
    for s in sizes:
        out.append(Case("c2_%d_rand" % s, 2, idx, s, s, s, seed=1)); idx += 1
        out.append(Case("c2_%d_min" % s, 2, idx, s, s, s, a_dist=("const", -128),
                        b_dist=("const", -128), seed=1)); idx += 1
    # "C initialised to 0" read literally: accumulate onto zeros gives the same C
    out.append(Case("c2_1024_zero_acc", 2, idx, 1024, 1024, 1024, mode=ACCUMULATE,
                    c_dist=("const", 0), seed=1))
    return out


def config3(batches=CONV_BATCHES) -> List[Case]:
    out, idx = [], 0
    for b in batches:
        for (co, hw, kk) in CONV_LAYERS:
            out.append(Case("c3_b%d_%dx%dx%d" % (b, co, hw * b, kk), 3, idx, co, hw * b, kk,
                            a_unsigned=False, b_unsigned=True,
                            a_dist=("normal", 32.0), b_dist=("uniform", 0, 255), seed=2))
            idx += 1
    return out


def config4() -> List[Case]:
    out, idx = [], 0
    for (m, n, k) in ENCODER_LAYERS:
        out.append(Case("c4_enc_%dx%dx%d" % (m, n, k), 4, idx, m, n, k,
                        a_dist=("normal", 24.0), b_dist=("normal", 24.0), seed=3)); idx += 1
    for (n, k) in DECODE_NK:
        for m in DECODE_M:
            out.append(Case("c4_dec_%dx%dx%d" % (m, n, k), 4, idx, m, n, k,
                            a_dist=("normal", 24.0), b_dist=("normal", 24.0), seed=3)); idx += 1
    # the same decode GEMMs with the weights stored n x k (k contiguous: column-major
    # B), the layout a linear layer's weight usually has
    for (n, k) in DECODE_NK:
        for m in DECODE_M:
            out.append(Case("c4_dec_%dx%dx%d_Bc" % (m, n, k), 4, idx, m, n, k, orderB=COL_MAJOR,
                            a_dist=("normal", 24.0), b_dist=("normal", 24.0), seed=3)); idx += 1
    return out


def config5() -> List[Case]:
    out, idx = [], 0
    for (m, n, k) in ODD_SHAPES:
        for a_unsigned in (False, True):
            for mode in (ACCUMULATE, OVERWRITE):
                for orderB in (ROW_MAJOR, COL_MAJOR):
                    out.append(Case(
                        "c5_%dx%dx%d_%s_%s_B%s" % (m, n, k, "u8s8" if a_unsigned else "s8s8",
                                                   "acc" if mode else "ovw", "cr"[1 - orderB]),
                        5, idx, m, n, k, a_unsigned=a_unsigned, orderB=orderB, pad=ODD_PAD,
                        mode=mode,
                        a_dist=("uniform", 0, 255) if a_unsigned else ("uniform", -128, 127),
                        c_dist=("uniform", -1000, 1000), seed=4))
                    idx += 1
    # every combination of storage orders for A, B and C on two of the shapes
    for (m, n, k) in ((7, 7, 3), (1000, 999, 1001)):
        for oa in (ROW_MAJOR, COL_MAJOR):
            for ob in (ROW_MAJOR, COL_MAJOR):
                for oc in (ROW_MAJOR, COL_MAJOR):
                    out.append(Case(
                        "c5_%dx%dx%d_orders_%d%d%d" % (m, n, k, oa, ob, oc), 5, idx, m, n, k,
                        orderA=oa, orderB=ob, orderC=oc, pad=ODD_PAD, mode=ACCUMULATE,
                        c_dist=("uniform", -1000, 1000), seed=4))
                    idx += 1
    return out


# One encoder block of a BERT-Large-type model as the paper tabulates it (Section 7.2, table
# "Dimensions of the GEMM operations in the transformer encoder"): d = 1024 embeddings,
# h = 16 heads, hidden dimension f = 4d, l tokens, b = 1; weights are A, activations B.
ENCODER_D, ENCODER_H = 1024, 16
ENCODER_TOKENS = (256, 512, 1024)


def encoder_block(l: int):
    """(case, how many times it runs per block) for the GEMMs of one encoder block on l tokens:
    M1-M3 the Q, K, V projections, M5 K^T Q and M7 V E_1 per head, M9 the output projection,
    F11 and F13 the feed-forward pair."""
    d, h, f = ENCODER_D, ENCODER_H, 4 * ENCODER_D
    dk = d // h
    dist = dict(a_dist=("normal", 24.0), b_dist=("normal", 24.0), seed=6)
    return [
        (Case("enc%d_M1-M3_%dx%dx%d" % (l, d, l, d), 6, 0, d, l, d, **dist), 3),
        # (K^i)^T is the d/h x l slice of K seen column-major: l x d/h with lda = l
        (Case("enc%d_M5_%dx%dx%d" % (l, l, l, dk), 6, 1, l, l, dk, orderA=COL_MAJOR, **dist), h),
        (Case("enc%d_M7_%dx%dx%d" % (l, dk, l, l), 6, 2, dk, l, l, **dist), h),
        (Case("enc%d_M9_%dx%dx%d" % (l, d, l, d), 6, 3, d, l, d, **dist), 1),
        (Case("enc%d_F11_%dx%dx%d" % (l, f, l, d), 6, 4, f, l, d, **dist), 1),
        (Case("enc%d_F13_%dx%dx%d" % (l, d, l, f), 6, 5, d, l, f, **dist), 1),
    ]


def config6() -> List[Case]:
    """The encoder-block GEMMs at the shortest sequence the paper uses (parity cases)."""
    return [case for (case, count) in encoder_block(ENCODER_TOKENS[0])]


def all_cases() -> Iterator[Case]:
    for group in (config1(), config2(), config3(), config4(), config5(), config6()):
        yield from group


def headline_case() -> Case:
    """m = n = k = 8192, s8 x s8 -> s32, row-major, overwrite: the size the metric is quoted on."""
    return next(c for c in config2() if c.name == "c2_8192_rand")


def swapped(case: Case) -> Case:
    """The same memory seen through C^T = B^T A^T (Section 3, last paragraph:
    a column-major C is handled by swapping the roles of A and B).

    A row-major X(r x c, ld) is the column-major X^T(c x r, ld), so the swapped
    problem reads the very same buffers with every order flipped.
    """
    return replace(case, name=case.name + "_swap", m=case.n, n=case.m,
                   a_unsigned=case.b_unsigned, b_unsigned=case.a_unsigned,
                   orderA=1 - case.orderB, orderB=1 - case.orderA, orderC=1 - case.orderC,
                   a_dist=case.b_dist, b_dist=case.a_dist)
