#!/usr/bin/env python3
"""Benchmark of the hot path: generate -> emulate (two models) -> compare, on one MI355X.

Workload: bf16 A/B, fp32 C/D GEMM with
m = n = k = 1024; A, B ~ N(0,1) cast to bf16, C = 0; model 0 accumulates in fused groups of 8
products, each group added to the running fp32 sum with RNE (c_mode = C_AFTER_EXACT, F = 24);
model 1 is the fully fused model of the same shape (L = K = 1024, F = 24, RNE); the step ends
with the bitwise comparison of the two outputs.  One step = 2 * 1024^3 emulated MAC terms.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: the library runs on one GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT32_VALU_PEAK = 256 * 4 * 16 * 2.4e9      # lane-instructions / s: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
ALGO_OPS_PER_TERM = 8                       # accounting floor of INT32 VALU instructions per MAC term
# HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE counters (scaled by a copy kernel
# of known size; see profiles/emulate_tiled_bf16_gemm1024_hbm_counters.md).  Valid only for the kernel variant and
# problem size it was measured on: any other variant reports null.
MEASURED_TRAFFIC = {("tiled 32x32 r2x2 kc=32 L=8 c_mode=1 fold=0 vm=1", 1024): (11487.0 * 2.00 + 4096.0) * 1024.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--size", type=int, default=1024, help="m = n = k of the GEMM-shaped workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the timed region, run 5 plain device copies of 64 MiB (a kernel of known traffic, "
                         "to scale FETCH_SIZE / WRITE_SIZE counters collected under rocprofv3 --pmc)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target duration of the CPU-oracle sample")
    return ap.parse_args()


def cpu_baseline(size, target_seconds):
    """The C form of the CPU oracle, as it stands, timed on a bounded sample of the same workload:
    whole rows of D (all n columns, both models) on inputs from the oracle's own generator twin."""
    import numpy as np
    from oracle import o2lib, gen as ogen, formats as fm
    from oracle.fdpa import ModelParams, C_AFTER_EXACT
    m = n = k = size
    A = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=0), fm.BF16, m * k, 0, 1).reshape(m, k)
    B = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=1), fm.BF16, n * k, 0, 1).reshape(n, k)
    models = [ModelParams(group_len=8, frac_bits=24, c_mode=C_AFTER_EXACT), ModelParams(group_len=0, frac_bits=24)]
    rows, used, elapsed, terms = 2, 1, 0.0, 0
    while True:
        rows = min(rows, m)
        Cz = np.zeros((1, rows, n), dtype=np.uint32)
        t0 = time.perf_counter()
        for p in models:
            _, used = o2lib.emulate_mma(p, A[None, :rows], B[None], Cz, fm.BF16, fm.BF16)
        elapsed = time.perf_counter() - t0
        terms = 2 * rows * n * k
        if elapsed >= 0.5 * target_seconds or rows == m:
            break
        rows = int(min(m, max(rows * 2, rows * target_seconds / max(elapsed, 1e-3) * 0.9)))
    return dict(value=terms / elapsed, unit="terms/s", cores=used, kind="oracle",
                sample="rows 0..%d of D (all %d columns, both models): %d terms in %.2f s" % (rows - 1, n, terms, elapsed))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this benchmark runs on ONE GPU (tiles and D elements are independent, so the path would shard by "
              "tile range); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_2511_10909_amd import binding as mm

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    m = n = k = args.size
    dt = (mm.BF16, mm.BF16, mm.FP32, mm.FP32)
    A = torch.empty((m, k), dtype=torch.int16, device=dev)
    B = torch.empty((n, k), dtype=torch.int16, device=dev)
    C = torch.empty((m, n), dtype=torch.int32, device=dev)
    D0 = torch.empty((m, n), dtype=torch.int32, device=dev)
    D1 = torch.empty((m, n), dtype=torch.int32, device=dev)
    stats = torch.empty(mm.STATS_BYTES, dtype=torch.uint8, device=dev)
    chained = mm.model_create(group_len=8, frac_bits=24, c_mode=mm.C_AFTER_EXACT, out_round=mm.RNE)
    fused = mm.model_create(group_len=0, frac_bits=24, c_mode=mm.C_IN_GROUP, out_round=mm.RNE)
    kernels = {}

    def step(events=None):
        mm.generate(A, mm.BF16, m * k, 0, 1, mm.GEN_NORMAL, seed=0, operand=0)
        mm.generate(B, mm.BF16, n * k, 0, 1, mm.GEN_NORMAL, seed=0, operand=1)
        mm.generate(C, mm.FP32, m * n, 0, 1, mm.GEN_ZERO, seed=0, operand=2)
        mm.stats_reset(stats)
        if events is not None:
            events[0].record()
        mm.emulate_mma(chained, A, B, C, D0, m, n, k, 1, dt)
        kernels["chained"] = mm.last_kernel()
        if events is not None:
            events[1].record()
        mm.emulate_mma(fused, A, B, C, D1, m, n, k, 1, dt)
        kernels["fused"] = mm.last_kernel()
        if events is not None:
            events[2].record()
        mm.compare(D0, D1, m * n, stats)

    if args.copy_calibration:
        src = torch.arange(16 * 1024 * 1024, dtype=torch.int32, device=dev)       # 64 MiB read + 64 MiB written
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1, out=dst)                                             # one elementwise kernel per call
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    terms_per_model = m * n * k
    terms_per_step = 2 * terms_per_model
    t_chained = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps * 1e-3
    t_fused = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps * 1e-3
    dom_name, dom_t = ("chained", t_chained) if t_chained >= t_fused else ("fused", t_fused)
    achieved = ALGO_OPS_PER_TERM * terms_per_model / dom_t
    st = mm.read_stats(stats)
    out = {
        "metric": "bit-exact emulated MAC terms/sec on 1 MI355X",
        "value": terms_per_step * args.steps / elapsed,
        "unit": "terms/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i32",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: bf16 A/B, fp32 C/D GEMM m=n=k=%d; step = generate(A,B ~ N(0,1)->bf16, C=0) + "
                        "emulate(chained L=8, C_AFTER_EXACT, F=24, RNE) + emulate(fully fused L=%d, F=24, RNE) + compare"
                        % (m, k),
            "terms_per_step": terms_per_step,
            "kernels": kernels,
            "mismatch_count_chained_vs_fused": st["n_mismatch_bits"],
            "n_compared": st["n_compared"],
            "emulate_only_terms_per_s": terms_per_step / (t_chained + t_fused),
            "emulate_ms": {"chained": t_chained * 1e3, "fused": t_fused * 1e3},
        },
        "roofline": {
            "bound": "alu",
            "kernel": "%s (%s)" % (dom_name, kernels[dom_name]),
            "achieved": achieved / 1e12,
            "peak": INT32_VALU_PEAK / 1e12,
            "unit": "T INT32 lane-instr/s (8 algorithmic instr per MAC term)",
            "frac": achieved / INT32_VALU_PEAK,
            "traffic": MEASURED_TRAFFIC.get((kernels[dom_name], args.size)),
        },
    }
    mm.model_destroy(chained)
    mm.model_destroy(fused)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.size, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
