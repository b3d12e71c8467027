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
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--size", type=int, default=8192, help="m = n = k of the square workload")
    ap.add_argument("--case", type=str, default=None, help="name of a workload case to run instead")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=4096)
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


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (got --gpus %d)"
              % args.gpus, file=sys.stderr)
        raise SystemExit(2)

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("no GPU visible: bench.py needs an MI355X")
    import paper_2506_11728_amd as M
    M.load_library()

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

    variant = M.mipgemm_variant_name(case.m, case.n, case.k, case.lda, case.orderA, case.ldb,
                                     case.orderB, case.ldc, case.orderC, case.a_unsigned,
                                     case.b_unsigned, True)
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
