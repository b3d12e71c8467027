#!/usr/bin/env python3
"""Benchmark of the MIP GEMM hot path on one MI355X.

One step = one call of mipgemm_s8s8s32 on the headline workload (m = n = k =
8192, row-major int8 operands, int32 result, overwrite), operands resident in
HBM before the timed region.  Prints one JSON line: throughput in TOPS with
2*m*n*k operations per GEMM (the paper's count, Section 7.4), the roofline
fraction of the dominant kernel, and the CPU oracle timed on a bounded sample
of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

INT8_MFMA_PEAK_TOPS = 5033.2   # 256 CUs x 4 SIMDs x 2048 ops/clk x 2.4 GHz, dense int8
HBM_PEAK_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--size", type=int, default=8192, help="m = n = k of the square workload")
    ap.add_argument("--case", type=str, default=None, help="name of a workload case to run instead")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=8192,
                    help="rows of C the oracle computes (and the GPU result is compared on); "
                         "all 8192 take about 22 s on 16 host threads")
    ap.add_argument("--timeline", type=int, default=0,
                    help="time that many launches one by one, from a cold start, print them as one "
                         "JSON line and exit")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy and exit (scales the HBM byte counters)")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the register-resident MFMA rate probe")
    ap.add_argument("--conv-layer", type=str, default=None,
                    help="name of a layer of the convolution workload (see workloads.resnet50_conv_layers; "
                         "e.g. stem) to run as a convolution instead; --batch sets the batch")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--suite", action="store_true",
                    help="time every workload case once and print a table instead of the JSON line")
    return ap.parse_args()


def pick_case(args) -> W.Case:
    if args.case:
        for c in W.all_cases():
            if c.name == args.case:
                return c
        raise SystemExit("unknown case %r" % args.case)
    if args.size == 8192:
        return W.headline_case()
    return W.Case("square_%d" % args.size, 2, 0, args.size, args.size, args.size, seed=1)


def cpu_baseline(case: W.Case, ops: W.Operands, rows: int):
    """The oracle, as it stands, on the first `rows` rows of A (all of B): same k and n."""
    import oracle
    rows = min(rows, case.m)
    if case.orderA != W.ROW_MAJOR or case.orderC != W.ROW_MAJOR:
        rows = case.m
    C = np.zeros(rows * case.ldc, dtype=np.int32)
    t0 = time.perf_counter()
    oracle.gemm(case.a_unsigned, case.b_unsigned, rows, case.n, case.k, ops.A, case.lda,
                case.orderA, ops.B, case.ldb, case.orderB, C, case.ldc, case.orderC, W.OVERWRITE)
    dt = time.perf_counter() - t0
    return {
        "value": 2.0 * rows * case.n * case.k / dt / 1e12,
        "unit": "TOPS",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "first %d of %d rows of C (m=%d, n=%d, k=%d), %.2f s, plain C triple loop, "
                  "OpenMP over rows" % (rows, case.m, rows, case.n, case.k, dt),
    }, C


KERNEL_SOURCES = ("dma_common.h", "epilogue.h", "epilogue16.h", "lds_layout.h", "dma_k128.h", "kernel_dma_k128.hip")


def kernel_fingerprint() -> str:
    """Hash of the sources of the headline kernel: counters taken on other code do not count."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2506_11728_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def recorded_traffic(variant: str, case: W.Case):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None if the
    summary is missing, is for another kernel or workload, or predates a change of the kernel."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s_%dx%dx%d.txt" % (
        variant, case.m, case.n, case.k))
    if not os.path.exists(path):
        return None
    fields = {}
    with open(path) as f:
        for line in f:
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                fields[k.strip()] = v.strip()
    if fields.get("kernel_fingerprint") != kernel_fingerprint():
        return None
    try:
        return float(fields["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def copy_calibration():
    """A plain copy kernel of known size: 1 GiB read, 1 GiB written, five times."""
    import torch
    n = 1 << 30
    src = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "launches": 5}))


def time_case(M, case, steps, warmup, dequant=False, requant=False):
    """Average milliseconds per call, operands resident, events on the launch stream.

    dequant: time the float-output entry point (scale fused into the write-back) instead;
    requant: the int8-output entry point (the sum requantised for the next layer)."""
    import torch
    ops = W.materialize(case)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    stream = torch.cuda.current_stream()
    if requant:
        dC = torch.zeros(ops.C.size, dtype=torch.int8, device="cuda")      # ldc counts bytes here
        entry = getattr(M, "mipgemm_" + case.entry.replace("s32", "s8"))

        def fn(*a, **kw):
            return entry(*a, scale=0.00013, **kw)
    elif dequant:
        dC = torch.zeros(ops.C.size, dtype=torch.float32, device="cuda")
        entry = getattr(M, "mipgemm_" + case.entry.replace("s32", "f32"))

        def fn(*a, **kw):
            return entry(*a, scale=0.00731, **kw)
    else:
        dC = torch.from_numpy(ops.C).cuda()
        fn = getattr(M, "mipgemm_" + case.entry)
    for _ in range(warmup):
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
           dC, case.ldc, case.orderC, case.mode, stream=stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
           dC, case.ldc, case.orderC, case.mode, stream=stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / steps


def time_case_graph(M, case, calls=24, replays=6, footprint=0):
    """Microseconds per call as the GPU sees them: `calls` calls captured into one
    HIP graph and the graph replayed, so that the host's launch cost, which exceeds
    the run time of the small cases, stays out.  footprint > 0 rotates the calls over
    as many copies of the operands as it takes to exceed that many bytes, so that no
    call finds its operands in the 256 MB last-level cache ("cold")."""
    import torch
    ops = W.materialize(case)
    per_set = ops.A.size + ops.B.size + 4 * ops.C.size
    sets = 1 if footprint <= 0 else max(1, min(calls, -(-footprint // per_set)))
    hA, hB = torch.from_numpy(ops.A.view(np.uint8)), torch.from_numpy(ops.B.view(np.uint8))
    hC = torch.from_numpy(ops.C)
    bufs = [(hA.cuda(), hB.cuda(), hC.cuda()) for _ in range(sets)]
    fn = getattr(M, "mipgemm_" + case.entry)
    # the workspace the header recommends (operands that have to be packed first)
    need = M.mipgemm_workspace_size(case.m, case.n, case.k, case.orderA, case.orderB, case.orderC)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda") if need else None

    def call(i):
        dA, dB, dC = bufs[i % sets]
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
           dC, case.ldc, case.orderC, case.mode, workspace=ws, workspace_bytes=need)

    call(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(calls):
            call(i)
    graph.replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(replays):
        graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / (calls * replays) * 1e3


def run_suite(M, args):
    """One line per workload case: time per call warm (operands may sit in the
    last-level cache) and cold (operands rotated over more than 512 MB), TOPS,
    GB/s of algorithmic bytes, and the fraction of the roofline
    max(ops / int8 MFMA peak, bytes / HBM peak) reached by the cold time."""
    print("| case | entry | m | n | k | kernel | us warm | us cold | TOPS cold | GB/s warm | GB/s cold "
          "| bound | frac of roofline (cold) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    seen = set()
    for case in W.all_cases():
        key = (case.entry, case.m, case.n, case.k, case.orderA, case.orderB, case.orderC,
               case.pad, case.mode, case.a_dist[0])
        if key in seen:
            continue
        seen.add(key)
        big = case.ops > 2e11
        calls = 4 if big else 24
        warm = time_case_graph(M, case, calls=calls)
        cold = warm if big else time_case_graph(M, case, calls=calls, footprint=600 * 10 ** 6)
        t_mfma = case.ops / (INT8_MFMA_PEAK_TOPS * 1e12)
        t_hbm = case.algorithmic_bytes / (HBM_PEAK_GBS * 1e9)
        need = M.mipgemm_workspace_size(case.m, case.n, case.k, case.orderA, case.orderB, case.orderC)
        name_of = M.mipgemm_variant_name_with_workspace if need else M.mipgemm_variant_name
        variant = name_of(case.m, case.n, case.k, case.lda, case.orderA, case.ldb, case.orderB,
                          case.ldc, case.orderC, case.a_unsigned, case.b_unsigned, True)
        print("| %s | %s | %d | %d | %d | %s | %.1f | %.1f | %.1f | %.0f | %.0f | %s | %.3f |" % (
            case.name, case.entry, case.m, case.n, case.k, variant, warm, cold,
            case.ops / cold / 1e6, case.algorithmic_bytes / warm / 1e3,
            case.algorithmic_bytes / cold / 1e3,
            "mfma" if t_mfma >= t_hbm else "hbm", max(t_mfma, t_hbm) / (cold * 1e-6)), flush=True)
    print()
    print("Float output with the dequantising scale fused into the write-back (f32 entry points), and int8")
    print("output requantised for the next layer (s8 entry points, a quarter of the bytes of C); no split k")
    print("without a workspace there (float sums are not combined out of order); eager launches:")
    print()
    print("| case | entry | us (s32) | us (f32) | us (s8) |")
    print("|---|---|---|---|---|")
    for name in ("c2_8192_rand", "c2_4096_rand", "c3_b32_64x100352x576", "c3_b32_128x25088x1152",
                 "c3_b32_256x6272x2304", "c3_b32_2048x1568x512", "c4_enc_1024x3072x768", "c4_dec_16x4096x4096"):
        case = next(c for c in W.all_cases() if c.name == name)
        a = time_case(M, case, args.steps, args.warmup)
        b = time_case(M, case, args.steps, args.warmup, dequant=True)
        q = time_case(M, case, args.steps, args.warmup, requant=True)
        print("| %s | %s | %.1f | %.1f | %.1f |" % (name, case.entry.replace("s32", "f32"), a * 1e3, b * 1e3,
                                                    q * 1e3), flush=True)


def run_packed_table(M):
    """Large products on operands that cannot be streamed as they are stored (odd sizes:
    no 16-byte alignment, k not a multiple of 64): the kernels that read them in place
    against the packed route (Pack A / Pack B into the workspace, Section 4.1), HIP graph
    replay, warm."""
    import torch
    rng = np.random.default_rng(5)
    print()
    print("Unaligned operands, s8 x s8 -> s32, row-major C, us per call without and with the workspace:")
    print()
    print("| m | n | k | A | B | kernel in place | us | TOPS | with workspace | us | TOPS |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for (m, n, k) in ((1000, 999, 1001), (2000, 3000, 1999), (4095, 4097, 4099), (8191, 8193, 8195)):
        hA = torch.from_numpy(rng.integers(-128, 128, size=m * k, dtype=np.int8).view(np.uint8))
        hB = torch.from_numpy(rng.integers(-128, 128, size=k * n, dtype=np.int8).view(np.uint8))
        dA, dB = hA.cuda(), hB.cuda()
        dC = torch.zeros(m * n, dtype=torch.int32, device="cuda")
        for oa, ob in ((W.ROW_MAJOR, W.ROW_MAJOR), (W.ROW_MAJOR, W.COL_MAJOR), (W.COL_MAJOR, W.ROW_MAJOR)):
            lda = k if oa == W.ROW_MAJOR else m
            ldb = n if ob == W.ROW_MAJOR else k
            need = M.mipgemm_workspace_size(m, n, k, oa, ob, W.ROW_MAJOR)
            ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
            times = []
            for given in (0, need):
                def call():
                    M.mipgemm_s8s8s32(m, n, k, dA, lda, oa, dB, ldb, ob, dC, n, W.ROW_MAJOR, W.OVERWRITE,
                                      workspace=ws if given else None, workspace_bytes=given)
                call()
                torch.cuda.synchronize()
                calls = 4
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for _ in range(calls):
                        call()
                graph.replay()
                torch.cuda.synchronize()
                ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                ev0.record()
                for _ in range(3):
                    graph.replay()
                ev1.record()
                torch.cuda.synchronize()
                times.append(ev0.elapsed_time(ev1) / (calls * 3) * 1e3)
            names = (M.mipgemm_variant_name(m, n, k, lda, oa, ldb, ob, n, W.ROW_MAJOR),
                     M.mipgemm_variant_name_with_workspace(m, n, k, lda, oa, ldb, ob, n, W.ROW_MAJOR))
            ops = 2.0 * m * n * k
            print("| %d | %d | %d | %s | %s | %s | %.1f | %.0f | %s | %.1f | %.0f |" % (
                m, n, k, "row" if oa == W.ROW_MAJOR else "col", "row" if ob == W.ROW_MAJOR else "col",
                names[0], times[0], ops / times[0] / 1e6, names[1], times[1], ops / times[1] / 1e6),
                flush=True)


def run_deep_k_table(M):
    """A very long k over few tiles of C: the dispatcher's choice (128 x 128 tiles with 128-deep
    blocks, k in ranges) against the 64 x 64 and 64 x 128 tiles the general scheme would pick,
    unsplit and in the ranges it would give them when forced (HIP graph replay, warm / cold)."""
    print()
    print("Deep k over few tiles, s8 x s8 -> s32, row-major, us per call warm / cold:")
    print()
    print("| m | n | k | mode | as dispatched | us | 64x64 tiles | 64x128 tiles in 4 ranges |")
    print("|---|---|---|---|---|---|---|---|")
    for (m, n, k) in ((512, 512, 16384), (768, 768, 8192), (512, 1568, 8192), (1024, 1024, 8192),
                      (1024, 1024, 16384), (768, 2048, 16384), (768, 768, 6144), (512, 1568, 4608)):
        for mode in (W.OVERWRITE, W.ACCUMULATE):
            case = W.Case("deepk_%dx%dx%d_m%d" % (m, n, k, mode), 8, 0, m, n, k, mode=mode, seed=3)
            cells = []
            for variant, splits in ((None, None), ("dma64", None), ("dma64x128", 4)):
                with M.tuning(MIPGEMM_VARIANT=variant, MIPGEMM_SPLITK=splits):
                    warm = time_case_graph(M, case)
                    cold = time_case_graph(M, case, footprint=600 * 10 ** 6)
                cells.append("%.1f / %.1f" % (warm, cold))
            name = M.mipgemm_variant_name_for_mode(m, n, k, case.lda, 0, case.ldb, 0, case.ldc, 0, False, False,
                                                   True, mode)
            print("| %d | %d | %d | %s | %s | %s | %s | %s |" % (
                m, n, k, "overwrite" if mode == W.OVERWRITE else "accumulate", name, cells[0], cells[1],
                cells[2]), flush=True)


def run_ragged_table(M):
    """Aligned operands whose m or n is no multiple of the tile: the dispatcher's choice (the
    general forms of the kernel with 128-deep blocks) against the 64-deep tile kernels with
    masked edges (HIP graph replay, warm)."""
    print()
    print("Aligned operands, m or n no multiple of the tile, row-major, overwrite, us per call warm:")
    print()
    print("| m | n | k | entry | as dispatched | us | TOPS | 64-deep tiles | us | TOPS |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for (m, n, k) in ((4000, 4000, 1024), (4000, 4000, 4096), (4000, 4000, 8192), (8000, 8000, 4096),
                      (6000, 4000, 8192), (3000, 2000, 4096), (1000, 3072, 768)):
        for b_unsigned in (False, True):
            case = W.Case("ragged_%dx%dx%d_u%d" % (m, n, k, b_unsigned), 8, 0, m, n, k, b_unsigned=b_unsigned,
                          b_dist=("uniform", 0, 255) if b_unsigned else ("uniform", -128, 127), seed=3)
            calls = 4 if case.ops > 1e11 else 24
            cells = []
            for variant in (None, "dma256" if m * n >= 192 * 65536 and k >= 1024 else "dma128"):
                with M.tuning(MIPGEMM_VARIANT=variant):
                    name = M.mipgemm_variant_name(m, n, k, case.lda, 0, case.ldb, 0, case.ldc, 0, False,
                                                  b_unsigned, True)
                    us = time_case_graph(M, case, calls=calls)
                cells.append("%s | %.1f | %.0f" % (name, us, case.ops / us / 1e6))
            print("| %d | %d | %d | %s | %s | %s |" % (m, n, k, case.entry, cells[0], cells[1]), flush=True)


def run_conv_table(M):
    """The convolutions of the conv-as-GEMM workload, timed as convolutions (HIP graph
    replay, warm): the GEMM alone on a ready-made augmented matrix, the lowering written
    out (im2col kernel + GEMM, the paper's route: it counts the transform in its
    times), and the lowering gathered inside the GEMM kernel."""
    import torch

    def replay_us(fn, calls=16, replays=5):
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(calls):
                fn()
        graph.replay()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(replays):
            graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / (calls * replays) * 1e3

    print()
    print("Convolution by lowering (Section 7.2), u8 activations x s8 filters -> s32, us per call:")
    print()
    print("| b | image | filters | (m, n, k) | GEMM alone | im2col + GEMM | gathered in the GEMM kernel "
          "| path | GB/s of I + F + O |")
    print("|---|---|---|---|---|---|---|---|---|")
    for b in W.CONV_BATCHES:
        for geo in W.CONV_GEOMETRY + (W.CONV_FIRST_LAYER,):
            hi, ci, co, hf, stride, pad = geo
            image, filt = W.conv_tensors(b, geo)
            ho = (hi + 2 * pad - hf) // stride + 1
            n, k = b * ho * ho, hf * hf * ci
            dI, dF = torch.from_numpy(image).cuda(), torch.from_numpy(filt.view(np.uint8)).cuda()
            dO = torch.zeros(n * co, dtype=torch.int32, device="cuda")
            ldm = (k + 15) // 16 * 16
            dM = torch.zeros(n * ldm, dtype=torch.uint8, device="cuda")      # a ready-made matrix
            args = (b, hi, hi, ci, co, hf, hf, stride, pad)
            with M.tuning(MIPGEMM_CONV="im2col"):
                need = M.mipgemm_conv_workspace_size(*args)                # of the written-out route
            dW = torch.zeros(need, dtype=torch.uint8, device="cuda")

            def gemm_only():
                M.mipgemm_s8u8s32(co, n, k, dF, k, W.ROW_MAJOR, dM, ldm, W.COL_MAJOR, dO, co,
                                  W.COL_MAJOR, W.OVERWRITE)

            def conv():
                M.mipgemm_conv_s8u8s32(*args, dF, dI, dO, W.OVERWRITE, workspace=dW, workspace_bytes=need)

            t_gemm = replay_us(gemm_only)
            with M.tuning(MIPGEMM_CONV="im2col"):
                t_explicit = replay_us(conv)
            t_implicit = replay_us(conv)
            moved = image.size + filt.size + 4 * n * co
            print("| %d | %dx%dx%d | %d of %dx%d | (%d, %d, %d) | %.1f | %.1f | %.1f | %s | %.0f |" % (
                b, hi, hi, ci, co, hf, hf, co, n, k, t_gemm, t_explicit, t_implicit,
                M.mipgemm_conv_variant_name(*args), moved / t_implicit / 1e3), flush=True)


def run_network_table(M):
    """Every convolution of a ResNet-50-type network (the paper's first workload) through the
    lowering, all 53 captured into one HIP graph per batch size."""
    import torch
    print()
    print("All 53 convolutions of a ResNet-50 v1.5-type network on 224 x 224 images (23 distinct layers),")
    print("u8 activations x s8 filters -> s32, each layer on its own synthetic tensors:")
    print()
    print("| batch | us, all convolutions | of which the 7 x 7 stem (3 channels: row-segment kernel) | GMAC | TOPS "
          "| us with the filters' k-sums supplied (computed once) | TOPS "
          "| us with the sums and an int8 output (requantised for the next layer) | TOPS |")
    print("|---|---|---|---|---|---|---|---|---|")
    layers = W.resnet50_conv_layers()
    for b in W.CONV_BATCHES:
        calls, calls_sums, calls_q8, macs, stem_call = [], [], [], 0, None
        for name, geo, count in layers:
            hi, ci, co, hf, stride, pad = geo
            image, filt = W.conv_tensors(b, geo)
            ho = (hi + 2 * pad - hf) // stride + 1
            dI, dF = torch.from_numpy(image).cuda(), torch.from_numpy(filt.view(np.uint8)).cuda()
            dO = torch.zeros(b * ho * ho * co, dtype=torch.int32, device="cuda")
            args = (b, hi, hi, ci, co, hf, hf, stride, pad)
            need = M.mipgemm_conv_workspace_size(*args)
            ws = torch.zeros(need, dtype=torch.uint8, device="cuda") if need else None
            call = (lambda args=args, dF=dF, dI=dI, dO=dO, ws=ws, need=need:
                    M.mipgemm_conv_s8u8s32(*args, dF, dI, dO, W.OVERWRITE, workspace=ws,
                                           workspace_bytes=need))
            dS = torch.zeros(co, dtype=torch.int32, device="cuda")
            M.mipgemm_conv_filter_sums(co, hf * hf * ci, dF, dS)
            call_sums = (lambda args=args, dF=dF, dI=dI, dO=dO, ws=ws, need=need, dS=dS:
                         M.mipgemm_conv_s8u8s32_with_sums(*args, dF, dI, dO, W.OVERWRITE, dS, workspace=ws,
                                                          workspace_bytes=need))
            dQ = torch.zeros(b * ho * ho * co, dtype=torch.int8, device="cuda")
            call_q8 = (lambda args=args, dF=dF, dI=dI, dQ=dQ, ws=ws, need=need, dS=dS:
                       M.mipgemm_conv_s8u8s8(*args, dF, dI, dQ, W.OVERWRITE, dS, workspace=ws,
                                             workspace_bytes=need, scale=0.0004))
            calls += [call] * count
            calls_sums += [call_sums] * count
            calls_q8 += [call_q8] * count
            macs += count * b * ho * ho * co * ci * hf * hf
            if name == "stem":
                stem_call = call

        def timed(fns, repeats):
            for f in fns:
                f()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(repeats):
                    for f in fns:
                        f()
            graph.replay()
            torch.cuda.synchronize()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for _ in range(5):
                graph.replay()
            ev1.record()
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) / (5 * repeats) * 1e3

        total = timed(calls, 2)
        stem = timed([stem_call], 8)
        total_sums = timed(calls_sums, 2)
        total_q8 = timed(calls_q8, 2)
        print("| %d | %.0f | %.0f | %.2f | %.1f | %.0f | %.1f | %.0f | %.1f |" % (
            b, total, stem, macs / 1e9, 2 * macs / total / 1e6, total_sums, 2 * macs / total_sums / 1e6,
            total_q8, 2 * macs / total_q8 / 1e6), flush=True)


def run_pack_table(M):
    """Decode GEMMs on weights as stored (k x n, row-major) and on the same weights packed
    once with k contiguous (mipgemm_pack_b), cold (operand sets rotated over > 600 MB)."""
    import torch
    print()
    print("Weight pre-packing (Section 4.1 carried to constant weights), decode shapes, us per call, cold:")
    print()
    print("| m | n | k | row-major B as stored | packed once (k contiguous) | the packing itself (once) |")
    print("|---|---|---|---|---|---|")
    for (n, k) in W.DECODE_NK:
        for m in W.DECODE_M:
            plain = next(c for c in W.all_cases() if c.name == "c4_dec_%dx%dx%d" % (m, n, k))
            packed = next(c for c in W.all_cases() if c.name == "c4_dec_%dx%dx%d_Bc" % (m, n, k))
            t_plain = time_case_graph(M, plain, footprint=600 * 10 ** 6)
            t_packed = time_case_graph(M, packed, footprint=600 * 10 ** 6)
            dB = torch.zeros(k * n, dtype=torch.uint8, device="cuda")
            dP = torch.empty_like(dB)
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            M.mipgemm_pack_b(k, n, dB, n, W.ROW_MAJOR, dP, k)
            torch.cuda.synchronize()
            ev0.record()
            for _ in range(10):
                M.mipgemm_pack_b(k, n, dB, n, W.ROW_MAJOR, dP, k)
            ev1.record()
            torch.cuda.synchronize()
            print("| %d | %d | %d | %.1f | %.1f | %.1f |" % (m, n, k, t_plain, t_packed,
                                                        ev0.elapsed_time(ev1) / 10 * 1e3), flush=True)


def run_packed_weights_table(M):
    """Unsigned activations against signed weights: the weights as stored, and as a packed-weights
    object (mipgemm_pack_weights: k-contiguous, padded, with their k-sums), warm, graph replays."""
    import torch
    print()
    print("Packed weights with cached k-sums (Section 4.1 carried to constant weights), u8 activations x s8")
    print("weights -> s32, us per call (warm; 8192^3 as 60 launches per replay, the others 24):")
    print()
    print("| m | n | k | s8 x s8, B as stored (for reference) | u8 x s8, B row-major as stored | u8 x s8, B k-contiguous "
          "| u8 x s8 on packed weights | s8 x s8 on packed weights | packing (once) |")
    print("|---|---|---|---|---|---|---|---|---|")
    rng = np.random.default_rng(7)

    def replay_us(fn, calls, replays=6):
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(calls):
                fn()
        graph.replay()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(replays):
            graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / (replays * calls) * 1e3

    R, C_, OVW = W.ROW_MAJOR, W.COL_MAJOR, W.OVERWRITE
    for (m, n, k) in ((8192, 8192, 8192), (4096, 4096, 4096), (2048, 2048, 2048), (1024, 3072, 768),
                      (100352, 64, 576), (25088, 128, 1152), (6272, 256, 2304), (1568, 512, 4608),
                      (16, 11008, 4096), (1, 4096, 4096)):
        calls = 60 if m * n * k > 2e11 else 24
        dA = torch.from_numpy(rng.integers(0, 256, size=m * k, dtype=np.uint8)).cuda()
        dB = torch.from_numpy(rng.integers(-128, 128, size=k * n, dtype=np.int8).view(np.uint8)).cuda()
        dC = torch.zeros(m * n, dtype=torch.int32, device="cuda")
        dP = torch.zeros(M.mipgemm_packed_weights_bytes(k, n), dtype=torch.uint8, device="cuda")
        M.mipgemm_pack_weights(k, n, dB, n, R, dP)
        dBc = torch.zeros(k * n, dtype=torch.uint8, device="cuda")
        M.mipgemm_pack_b(k, n, dB, n, R, dBc, k)
        t = [replay_us(lambda: M.mipgemm_s8s8s32(m, n, k, dA, k, R, dB, n, R, dC, n, R, OVW), calls),
             replay_us(lambda: M.mipgemm_u8s8s32(m, n, k, dA, k, R, dB, n, R, dC, n, R, OVW), calls),
             replay_us(lambda: M.mipgemm_u8s8s32(m, n, k, dA, k, R, dBc, k, C_, dC, n, R, OVW), calls),
             replay_us(lambda: M.mipgemm_u8s8s32_packed(m, n, k, dA, k, R, dP, dC, n, R, OVW), calls),
             replay_us(lambda: M.mipgemm_s8s8s32_packed(m, n, k, dA, k, R, dP, dC, n, R, OVW), calls),
             replay_us(lambda: M.mipgemm_pack_weights(k, n, dB, n, R, dP), 8)]
        print("| %d | %d | %d | %s |" % (m, n, k, " | ".join("%.1f" % x for x in t)), flush=True)
        del dA, dB, dC, dP, dBc


def run_s16_table(M):
    """int16 x int16 -> int32 through byte planes against the 8-bit product of the same size."""
    import torch
    print()
    print("16-bit operands (int16 x int16 -> int32: byte planes, three s8 x s8 GEMMs and a combining pass),")
    print("us per call (warm, graph replays), TOPS counted as 2 m n k:")
    print()
    print("| m | n | k | s8 x s8 -> s32 | s16 x s16 -> s32 | ratio | TOPS (s16) |")
    print("|---|---|---|---|---|---|---|")
    rng = np.random.default_rng(11)
    R, OVW = W.ROW_MAJOR, W.OVERWRITE
    for (m, n, k) in ((4096, 4096, 4096), (2048, 2048, 2048), (1024, 3072, 768), (1024, 1024, 1024), (16, 4096, 4096)):
        dA8 = torch.from_numpy(rng.integers(-128, 128, size=m * k, dtype=np.int8).view(np.uint8)).cuda()
        dB8 = torch.from_numpy(rng.integers(-128, 128, size=k * n, dtype=np.int8).view(np.uint8)).cuda()
        dA = torch.from_numpy(rng.integers(-32768, 32768, size=m * k, dtype=np.int16)).cuda()
        dB = torch.from_numpy(rng.integers(-32768, 32768, size=k * n, dtype=np.int16)).cuda()
        dC = torch.zeros(m * n, dtype=torch.int32, device="cuda")
        need = M.mipgemm_workspace_size_s16(m, n, k)
        ws = torch.zeros(need, dtype=torch.uint8, device="cuda")

        def replay_us(fn, calls=12, replays=5):
            fn()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(calls):
                    fn()
            graph.replay()
            torch.cuda.synchronize()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for _ in range(replays):
                graph.replay()
            ev1.record()
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) / (replays * calls) * 1e3

        t8 = replay_us(lambda: M.mipgemm_s8s8s32(m, n, k, dA8, k, R, dB8, n, R, dC, n, R, OVW))
        t16 = replay_us(lambda: M.mipgemm_s16s16s32(m, n, k, dA, k, R, dB, n, R, dC, n, R, OVW,
                                                    workspace=ws, workspace_bytes=need))
        print("| %d | %d | %d | %.1f | %.1f | %.1f | %.0f |" % (m, n, k, t8, t16, t16 / t8,
                                                           2.0 * m * n * k / t16 / 1e6), flush=True)
        del dA8, dB8, dA, dB, dC, ws


def run_encoder_table(M):
    """The GEMMs of one transformer encoder block (the paper's second workload, Section 7.2),
    captured into one HIP graph in the order of the paper's table and replayed: once with
    the per-head attention products as separate calls (the paper's loop over heads), once
    with each of the two as one strided-batch call."""
    import torch
    print()
    print("One encoder block of a BERT-Large-type model (d = 1024, h = 16, f = 4096, b = 1), its GEMMs only,")
    print("s8 x s8 -> s32, us (warm):")
    print()
    print("| l | M1-M3 (each) | M5 (one head) | M7 (one head) | M9 | F11 | F13 | M5, all heads in one call "
          "| M7, all heads in one call | block, every GEMM its own call (38 calls) "
          "| block, M1-M3, M5 and M7 each one batched call (6 calls) "
          "| TOPS (batched) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|")

    def replay_us(fn, repeats, replays=6):
        """fn captured `repeats` times into one graph (the launch of a graph has a cost of its own)"""
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(repeats):
                fn()
        graph.replay()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(replays):
            graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / (replays * repeats) * 1e3

    h = W.ENCODER_H
    for l in W.ENCODER_TOKENS:
        block = W.encoder_block(l)
        each = [time_case_graph(M, case, calls=24) for (case, count) in block]
        looped, batched, ops = [], [], 0
        for (case, count) in block:
            o = W.materialize(case)
            per_head = count == h
            # a head's operands are slices of the full activation matrices: h copies, back to back
            dA = torch.from_numpy(np.tile(o.A.view(np.uint8), h if per_head else 1)).cuda()
            dB = torch.from_numpy(np.tile(o.B.view(np.uint8), h if per_head else 1)).cuda()
            dC = torch.zeros(o.C.size * (h if per_head else 1), dtype=torch.int32, device="cuda")
            ops += count * case.ops
            c = case
            if per_head:
                sa, sb, sc = o.A.size, o.B.size, o.C.size
                for z in range(h):
                    looped.append(lambda c=c, a=dA[z * sa:], b=dB[z * sb:], cc=dC[z * sc:]:
                                  M.mipgemm_s8s8s32(c.m, c.n, c.k, a, c.lda, c.orderA, b, c.ldb,
                                                    c.orderB, cc, c.ldc, c.orderC, c.mode))
                batched.append(lambda c=c, a=dA, b=dB, cc=dC, sa=sa, sb=sb, sc=sc:
                               M.mipgemm_s8s8s32_batched(c.m, c.n, c.k, a, c.lda, c.orderA, sa, b,
                                                         c.ldb, c.orderB, sb, cc, c.ldc, c.orderC,
                                                         sc, h, c.mode))
            elif count > 1:
                # M1-M3: three weight matrices against the same activations: looped, or one batch of
                # three with the B operand shared (stride 0)
                dA = torch.from_numpy(np.tile(o.A.view(np.uint8), count)).cuda()
                dC = torch.zeros(o.C.size * count, dtype=torch.int32, device="cuda")
                for z in range(count):
                    looped.append(lambda c=c, a=dA[z * o.A.size:], b=dB, cc=dC[z * o.C.size:]:
                                  M.mipgemm_s8s8s32(c.m, c.n, c.k, a, c.lda, c.orderA, b, c.ldb,
                                                    c.orderB, cc, c.ldc, c.orderC, c.mode))
                batched.append(lambda c=c, a=dA, b=dB, cc=dC, sa=o.A.size, sc=o.C.size, n3=count:
                               M.mipgemm_s8s8s32_batched(c.m, c.n, c.k, a, c.lda, c.orderA, sa, b,
                                                         c.ldb, c.orderB, 0, cc, c.ldc, c.orderC,
                                                         sc, n3, c.mode))
            else:
                call = (lambda c=c, a=dA, b=dB, cc=dC:
                        M.mipgemm_s8s8s32(c.m, c.n, c.k, a, c.lda, c.orderA, b, c.ldb, c.orderB,
                                          cc, c.ldc, c.orderC, c.mode))
                looped.append(call)
                batched.append(call)
        qkv, m5, m7 = [b for b in batched if b not in looped]
        t_m5 = replay_us(m5, 24)
        t_m7 = replay_us(m7, 24)
        t_looped = replay_us(lambda: [f() for f in looped], 4)
        t_batched = replay_us(lambda: [f() for f in batched], 8)
        del qkv
        print("| %d | %s | %.1f | %.1f | %.1f | %.1f | %.1f |" % (
            l, " | ".join("%.1f" % t for t in each), t_m5, t_m7, t_looped, t_batched,
            ops / t_batched / 1e6), flush=True)


def run_conv_layer(M, args):
    """One layer of the convolution workload through mipgemm_conv_s8u8s32: W untimed calls,
    K timed ones between two events on the launch stream, one JSON line."""
    import torch
    geo = None
    for name, g, _count in W.resnet50_conv_layers():
        if name == args.conv_layer:
            geo = g
    if geo is None:
        raise SystemExit("unknown layer %r" % args.conv_layer)
    b = args.batch
    hi, ci, co, hf, stride, pad = geo
    image, filt = W.conv_tensors(b, geo)
    ho = (hi + 2 * pad - hf) // stride + 1
    n, k = b * ho * ho, hf * hf * ci
    dI, dF = torch.from_numpy(image).cuda(), torch.from_numpy(filt.view(np.uint8)).cuda()
    dO = torch.zeros(n * co, dtype=torch.int32, device="cuda")
    geom = (b, hi, hi, ci, co, hf, hf, stride, pad)
    need = M.mipgemm_conv_workspace_size(*geom)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda") if need else None
    stream = torch.cuda.current_stream()

    def step():
        M.mipgemm_conv_s8u8s32(*geom, dF, dI, dO, W.OVERWRITE, workspace=ws, workspace_bytes=need,
                               stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / args.steps
    moved = image.size + filt.size + 4 * n * co
    print(json.dumps({
        "metric": "convolution by lowering, u8 x s8 -> s32", "value": 2.0 * n * k * co / (ms * 1e-3) / 1e12,
        "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "dtype": "u8*s8->s32", "data": "synthetic",
        "config": {"workload": "%s: b=%d image %dx%dx%d, %d filters %dx%d, stride %d, pad %d; "
                               "(m, n, k) = (%d, %d, %d)" % (args.conv_layer, b, hi, hi, ci, co, hf, hf,
                                                             stride, pad, co, n, k)},
        "roofline": {"bound": "hbm", "achieved": moved / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "kernel": M.mipgemm_conv_variant_name(*geom), "kernel_ms": ms,
                     "algorithmic_bytes": moved},
    }))


def run_timeline(step, stream, case, launches):
    """Every launch between its own pair of events, starting from a device that has done
    nothing yet: how long the device takes to reach its working clocks."""
    import torch
    events = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
    torch.cuda.synchronize()
    events[0].record(stream)
    for i in range(launches):
        step()
        events[i + 1].record(stream)
    torch.cuda.synchronize()
    us = [events[i].elapsed_time(events[i + 1]) * 1e3 for i in range(launches)]
    print(json.dumps({"workload": case.name, "launches": launches,
                      "us_per_launch": [round(x, 1) for x in us]}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (got --gpus %d)"
              % args.gpus, file=sys.stderr)
        raise SystemExit(2)

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("no GPU visible: bench.py needs an MI355X")
    import paper_2506_11728_amd as M
    M.load_library()

    if args.copy_calibration:
        copy_calibration()
        return
    if args.conv_layer:
        run_conv_layer(M, args)
        return
    if args.suite:
        run_suite(M, args)
        run_packed_table(M)
        run_deep_k_table(M)
        run_ragged_table(M)
        run_conv_table(M)
        run_network_table(M)
        run_pack_table(M)
        run_packed_weights_table(M)
        run_s16_table(M)
        run_encoder_table(M)
        return

    case = pick_case(args)
    ops = W.materialize(case)
    fn = getattr(M, "mipgemm_" + case.entry)
    dA = torch.from_numpy(ops.A.view(np.uint8)).cuda()
    dB = torch.from_numpy(ops.B.view(np.uint8)).cuda()
    dC = torch.from_numpy(ops.C).cuda()
    stream = torch.cuda.current_stream()

    def step():
        fn(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb, case.orderB,
           dC, case.ldc, case.orderC, case.mode, stream=stream)

    if args.timeline:
        run_timeline(step, stream, case, args.timeline)
        return

    ceiling = None
    if not args.no_ceiling:
        # What the matrix instruction itself sustains on this device with its operands in
        # registers, and the shader clock it ran at: the chip is power-limited and the rate
        # depends on the operand bits.  Run before the timed region: the probes (about 0.1 s
        # of matrix work) also bring the device out of its idle clocks, which the first tens
        # of milliseconds of any load otherwise run at (profiles/launch_timeline_*.txt).
        ceiling = {"unit": "TOPS"}
        # (keys without a suffix: v_mfma_i32_32x32x32_i8; "_16x16x64": the instruction the
        # kernel for large problems is built on)
        for key, pattern in (("near_zero_operands", 0), ("random_operands_rotated_by_valu", 1),
                             ("random_operands_two_sets", 2), ("random_operands_six_sets", 3),
                             ("near_zero_operands_16x16x64", 4), ("random_operands_16x16x64", 5)):
            tops_p, mhz_p = M.mipgemm_mfma_ceiling_clocked(pattern, 20000)
            ceiling[key] = tops_p
            ceiling[key + "_shader_mhz"] = mhz_p

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = ev0.elapsed_time(ev1) / args.steps     # one kernel launch per step
    ms_per_step = wall * 1e3 / args.steps

    variant = M.mipgemm_variant_name_for_mode(case.m, case.n, case.k, case.lda, case.orderA, case.ldb,
                                              case.orderB, case.ldc, case.orderC, case.a_unsigned,
                                              case.b_unsigned, True, case.mode)
    tops = case.ops / (ms_per_step * 1e-3) / 1e12
    kernel_tops = case.ops / (kernel_ms * 1e-3) / 1e12
    kernel_gbs = case.algorithmic_bytes / (kernel_ms * 1e-3) / 1e9
    t_mfma = case.ops / (INT8_MFMA_PEAK_TOPS * 1e12)
    t_hbm = case.algorithmic_bytes / (HBM_PEAK_GBS * 1e9)
    if t_mfma >= t_hbm:
        roofline = {"bound": "mfma", "achieved": kernel_tops, "peak": INT8_MFMA_PEAK_TOPS,
                    "unit": "TOP/s", "frac": kernel_tops / INT8_MFMA_PEAK_TOPS, "traffic": None}
    else:
        roofline = {"bound": "hbm", "achieved": kernel_gbs, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": kernel_gbs / HBM_PEAK_GBS, "traffic": None}
    roofline["kernel"] = variant
    roofline["kernel_ms"] = kernel_ms
    roofline["traffic"] = recorded_traffic(variant, case)
    roofline["algorithmic_bytes"] = case.algorithmic_bytes
    if variant == "mfma_dma256_k128" and case.entry == "s8s8s32":
        # the shader clock during the main loops of the same kernel, right after the timed steps
        tiles = -(-case.m // 256) * -(-case.n // 256)
        clocks = torch.zeros(2 * (-(-tiles // 8) * 8), dtype=torch.int64, device="cuda")
        for _ in range(3):
            M.mipgemm_s8s8s32_clocked(case.m, case.n, case.k, dA, case.lda, case.orderA, dB, case.ldb,
                                      case.orderB, dC, case.ldc, case.orderC, case.mode, clocks,
                                      clocks.numel() * 8, stream=stream)
        torch.cuda.synchronize()
        c = clocks.cpu().numpy().reshape(-1, 2).sum(axis=0)
        roofline["shader_mhz"] = float(c[0]) / float(c[1]) * 100.0 if c[1] else None
        # matrix instructions issue back to back at 32 clocks each: the share of the main
        # loops' clocks that the matrix pipe was busy
        # (per wave and tile k / 32 steps of 16 instructions of 32 clocks; three launches)
        roofline["mfma_busy_frac_of_main_loop"] = (
            3.0 * tiles * case.k * 16 / float(c[0]) if c[0] else None)

    out = {
        "metric": "int8 GEMM TOPS (int32 acc) at m=n=k=8192; % of MI355X int8 MFMA peak",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "s8*s8->s32", "data": "synthetic",
        "config": {"workload": "%s: %s m=%d n=%d k=%d, row-major, %s, seed %d" % (
            case.name, case.entry, case.m, case.n, case.k,
            "accumulate" if case.mode else "overwrite", case.seed)},
        "pct_of_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
        "roofline": roofline,
    }

    if ceiling is not None:
        best_random = max(ceiling["random_operands_two_sets"], ceiling["random_operands_six_sets"],
                          ceiling["random_operands_16x16x64"])
        ceiling["kernel_frac_of_random_ceiling"] = kernel_tops / best_random
        out["mfma_only_ceiling"] = ceiling

    check_rows = None
    if not args.no_cpu_baseline:
        base, C_rows = cpu_baseline(case, ops, args.cpu_sample_rows)
        out["cpu_baseline"] = base
        check_rows = C_rows
    if not args.no_check and check_rows is not None and case.mode == W.OVERWRITE \
            and case.orderC == W.ROW_MAJOR:
        got = dC.cpu().numpy()[:check_rows.size]
        mask = ~W.padding_mask(check_rows.size // case.ldc, case.n, case.orderC, case.ldc)
        out["parity_vs_oracle_sample"] = bool(np.array_equal(got[mask], check_rows[mask]))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
