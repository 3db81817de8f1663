#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: the closed-loop scan (the largest of the five workloads).

One step = the whole scan: for each operand type (bf16 x bf16, e4m3 x e5m2), 2^24 random 16x16x16 tiles in chunks of
2^16: generate A, B, C on the device, run every tile through the native MFMA instruction, evaluate the sixteen
parameter sets (fused dot-product-add models of internal width 16..32, group length 4..16, RNE / RZ, flushes on / off)
and accumulate each set's bitwise comparison statistics against the instruction's output.  With the default fused
path the sets of one group length share a launch (mmaemu_emulate_compare_many): the operands are staged and decoded
once per chunk and group of sets, every output is compared in registers, D never reaches memory.  `--unfused` runs one
mmaemu_emulate_mma and one mmaemu_compare per set instead.

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
# Counter figures of the emulation kernels, from rocprofv3 --pmc runs of this program (see the named files under profiles/):
# vector-ALU lane-instructions per MAC term (SQ_INSTS_VALU x 64 / terms) and HBM bytes per launch (FETCH_SIZE + WRITE_SIZE,
# scaled by a copy kernel of known size).  Keyed by the kernel's name: a kernel that has changed since reports null.
COUNTERS = {
    "multi x16 tiled 16x16 r2x2 kc=16 any L vm=0": {"valu_instr_per_term": 10.71, "traffic": 184924024, "chunk": 1 << 16},
    "multi x16 tiled 16x16 r2x2 kc=16 any L vm=1": {"valu_instr_per_term": 11.52, "traffic": 338665326, "chunk": 1 << 16},
    "multi x3 tiled 32x32 r2x2 kc=8 any L vm=0, twins share sums": {"valu_instr_per_term": 10.15, "traffic": 1342820407, "chunk": 1 << 18},
}
COUNTERS_SOURCE = ("profiles/closed_loop_scan_trace_and_counters.md, profiles/subnormal_stress_trace_and_counters.md (rocprofv3 --pmc SQ_INSTS_VALU; "
                   "FETCH_SIZE, WRITE_SIZE scaled by a 64 MiB copy); traffic per launch")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", choices=("scan", "subnormal"), default="scan",
                    help="scan: the closed-loop scan (the headline); subnormal: the subnormal stress workload (2^26 fp16 32x32x8 "
                         "tiles, three flush variants) as the step, for its own profile")
    ap.add_argument("--tiles", type=int, default=0, help="tiles per operand type (default: the workload as stated, 2^24 / 2^26)")
    ap.add_argument("--chunk", type=int, default=0, help="tiles generated and evaluated at a time (default 2^16; 2^18 for the subnormal workload)")
    ap.add_argument("--unfused", action="store_true", help="one emulation launch and one comparison launch per parameter set")
    ap.add_argument("--time-every", type=int, default=16, help="HIP events around the emulation launches of every n-th chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the one-off runs of workloads 1-4 after the timed region")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the timed region, run 5 plain device copies of 64 MiB (a kernel of known traffic, "
                         "to scale FETCH_SIZE / WRITE_SIZE counters collected under rocprofv3 --pmc)")
    ap.add_argument("--issue-rates", action="store_true",
                    help="instead of the benchmark: time the library's issue-rate probes (one per hot-loop instruction) and "
                         "print their lane-instructions per second as one JSON line")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target duration of the CPU-oracle sample")
    return ap.parse_args()


def cpu_baseline(target_seconds):
    """The C form of the CPU oracle, as it stands, timed on a bounded sample of the same workload: the first tiles of
    the bf16 half of the scan (inputs from the oracle's own generator twin), all sixteen parameter sets."""
    import numpy as np
    from oracle import o2lib, gen as ogen, formats as fm
    from oracle.fdpa import ModelParams
    from paper_2511_10909_amd.configs import CONFIG5_MODELS
    models = [ModelParams(group_len=L, frac_bits=F, out_round=rho, ftz_in=bool(z), ftz_out=bool(z)) for F, L, rho, z in CONFIG5_MODELS]
    nt, used, elapsed, terms = 1 << 10, 1, 0.0, 0
    while True:
        A = ogen.generate(ogen.GenParams(family=ogen.GEN_FINITE_BITS, seed=0, operand=0), fm.BF16, 256, 0, nt).reshape(nt, 16, 16)
        B = ogen.generate(ogen.GenParams(family=ogen.GEN_FINITE_BITS, seed=0, operand=1), fm.BF16, 256, 0, nt).reshape(nt, 16, 16)
        C = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=2), fm.FP32, 256, 0, nt, threads=8).reshape(nt, 16, 16)
        t0 = time.perf_counter()
        for p in models:
            _, used = o2lib.emulate_mma(p, A, B, C, fm.BF16, fm.BF16)
        elapsed = time.perf_counter() - t0
        terms = len(models) * nt * 4096
        if elapsed >= 0.5 * target_seconds or nt >= (1 << 20):
            break
        nt = int(min(1 << 20, max(nt * 2, nt * target_seconds / max(elapsed, 1e-3) * 0.9)))
    return dict(value=terms / elapsed, unit="terms/s", cores=used, kind="oracle",
                sample="tiles 0..%d of the bf16 half, all 16 parameter sets (emulation only): %d terms in %.2f s" % (nt - 1, terms, elapsed))


def subnormal_stress(args, torch, mm, configs, fused):
    """The subnormal stress workload as the step (not the headline: it has fewer terms than the scan)."""
    n_tiles = args.tiles or (1 << 26)
    chunk = min(args.chunk or (1 << 18), n_tiles)
    timed = []

    def timer(name, terms, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        timed.append((name, terms, e0, e1))

    for _ in range(args.warmup):
        configs.config4(n_tiles=n_tiles, chunk=chunk, fused=fused)
    secs, r = 0.0, None
    for _ in range(args.steps):
        r = configs.config4(n_tiles=n_tiles, chunk=chunk, fused=fused, timer=timer, time_every=args.time_every * 4)
        secs += r["seconds"]
    ms = sum(e0.elapsed_time(e1) for _, _, e0, e1 in timed)
    terms = sum(t for _, t, _, _ in timed)
    ctr = COUNTERS.get(r["kernel"], {})
    ctr = ctr if chunk == ctr.get("chunk") else {}                           # (the counters were taken on launches of that many tiles)
    frac = ALGO_OPS_PER_TERM * terms / (ms * 1e-3) / INT32_VALU_PEAK
    return {
        "metric": "bit-exact emulated MAC terms/sec on 1 MI355X", "value": r["terms"] * args.steps / secs, "unit": "terms/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": secs / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32+i32 (exact binary32 products, int32 sums)", "data": "synthetic",
        "config": {"workload": "configs[3]: subnormal stress, 2^%d fp16 32x32x8 tiles, exponent fields uniform over the whole range, "
                               "variants none / ftz_in / ftz_out each compared with the first (%s)"
                               % (n_tiles.bit_length() - 1, "one fused launch per chunk" if fused else "one emulation and one comparison per variant"),
                   "terms_per_step": r["terms"], "chunk": chunk, "fused": fused, "kernel": r["kernel"],
                   "mismatches": {k: v["n_mismatch_bits"] for k, v in r["stats"].items()},
                   "emulation_launches_timed": len(timed), "avg_emulation_launch_ms": ms / max(len(timed), 1)},
        "roofline": {"bound": "alu", "kernel": r["kernel"], "achieved": frac * INT32_VALU_PEAK / 1e12, "peak": INT32_VALU_PEAK / 1e12,
                     "unit": "T INT32 lane-instr/s (8 algorithmic instr per MAC term)", "frac": frac,
                     "valu_instr_per_term": ctr.get("valu_instr_per_term"),
                     "valu_util": (ctr["valu_instr_per_term"] * terms / (ms * 1e-3) / INT32_VALU_PEAK) if ctr else None,
                     "traffic": ctr.get("traffic"), "traffic_source": COUNTERS_SOURCE if ctr else None},
    }


def issue_rates(torch, mm):
    """Lane-instructions per second of each probed instruction: 2048 workgroups x 256 lanes x 8 chains x 4096 iterations,
    best of five launches timed with events."""
    out = torch.zeros(256, dtype=torch.int32, device="cuda")
    iters, wgs = 4096, 2048
    rates = {}
    for op, name in enumerate(mm.issue_probe_names()):
        mm.issue_probe(op, 64, wgs, out)
        best = None
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            mm.issue_probe(op, iters, wgs, out)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None or ms < best else best
        rates[name] = wgs * 256 * 8 * iters / (best * 1e-3)
    return dict(unit="lane-instructions/s", peak_assumed=INT32_VALU_PEAK, rates=rates,
                frac_of_peak={k: v / INT32_VALU_PEAK for k, v in rates.items()})


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
    from paper_2511_10909_amd import binding as mm, configs

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.issue_rates:
        print(json.dumps(issue_rates(torch, mm)))
        return
    fused = not args.unfused
    if args.copy_calibration:
        src = torch.arange(16 * 1024 * 1024, dtype=torch.int32, device=dev)       # 64 MiB read + 64 MiB written
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1, out=dst)                                             # one elementwise kernel per call
        torch.cuda.synchronize()
    if args.workload == "subnormal":
        print(json.dumps(subnormal_stress(args, torch, mm, configs, fused)))
        return
    n_tiles = args.tiles or (1 << 24)
    chunk = min(args.chunk or (1 << 16), n_tiles)
    scans = [configs.ClosedLoopScan(kind, chunk, 0, "cuda", fused) for kind in ("bf16", "fp8")]
    n_sets = len(configs.CONFIG5_MODELS)
    timed = []                      # (kernel key, terms, start event, end event) of the emulation launches that carry events

    def step(collect):
        for scan in scans:
            scan.reset()
            for ci, t0 in enumerate(range(0, n_tiles, chunk)):
                nt = min(chunk, n_tiles - t0)
                timer = None
                if collect and ci % args.time_every == 0:
                    def timer(name, terms, fn, scan=scan):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        fn()
                        e1.record()
                        timed.append(((scan.kind, name), terms, e0, e1))
                scan.chunk_step(t0, nt, timer=timer)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    terms_per_step = 2 * n_sets * n_tiles * 4096
    # per emulation kernel: average launch duration and the fraction of the accounting roofline it reaches
    per = {}
    for key, terms, e0, e1 in timed:
        d = per.setdefault(key, dict(launches=0, ms=0.0, terms=0))
        d["launches"] += 1
        d["ms"] += e0.elapsed_time(e1)
        d["terms"] += terms
    kernels = {}
    for (kind, name), d in per.items():
        scan = scans[0] if kind == "bf16" else scans[1]
        idx = int(name.split()[1])
        kname = scan.kernels.get(idx, "?")
        kernels["%s %s: %s" % (kind, name, kname)] = dict(
            launches_timed=d["launches"], avg_ms=d["ms"] / d["launches"], terms_per_launch=d["terms"] // d["launches"],
            frac=ALGO_OPS_PER_TERM * d["terms"] / (d["ms"] * 1e-3) / INT32_VALU_PEAK, kernel=kname)
    dom_key = max(kernels, key=lambda k: kernels[k]["avg_ms"] * kernels[k]["launches_timed"])
    dom = kernels[dom_key]
    tot_ms = sum(v["avg_ms"] * v["launches_timed"] for v in kernels.values())
    tot_terms = sum(v["terms_per_launch"] * v["launches_timed"] for v in kernels.values())
    achieved = ALGO_OPS_PER_TERM * dom["terms_per_launch"] / (dom["avg_ms"] * 1e-3)
    ctr = COUNTERS.get(dom["kernel"], {})
    ctr = ctr if chunk == ctr.get("chunk") else {}                           # (the counters were taken on launches of that many tiles)
    stats = {scan.kind: scan.read() for scan in scans}
    agreement = {kind: [1.0 - s["n_mismatch_bits"] / max(s["n_compared"], 1) for s in st] for kind, st in stats.items()}
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
        "dtype": "f32+i32 (exact binary32 products, int32 / binary64 sums, binary64 group conversion)",
        "data": "synthetic",
        "config": {
            "workload": "configs[4]: closed-loop scan, 16 parameter sets x 2^%d tiles 16x16x16 x {bf16 finite bit patterns, "
                        "e4m3 x e5m2 N(0,1) scaled per tile}, C ~ N(0,1); step = per chunk of 2^%d tiles: generate A, B, C + "
                        "native MFMA + 16 sets emulated and compared with the instruction (%s)"
                        % (n_tiles.bit_length() - 1, chunk.bit_length() - 1,
                           "fused: statistics formed inside the emulation kernels" if fused else "one emulation and one comparison launch per set"),
            "terms_per_step": terms_per_step,
            "tiles_per_type": n_tiles,
            "chunk": chunk,
            "fused": fused,
            "n_compared_per_set": stats["bf16"][0]["n_compared"],
            "agreement_with_mfma": {kind: dict(min=min(a), max=max(a)) for kind, a in agreement.items()},
            "emulation_kernels": kernels,
            "emulation_only_terms_per_s": tot_terms / (tot_ms * 1e-3),
        },
        "roofline": {
            "bound": "alu",
            "kernel": dom_key,
            "achieved": achieved / 1e12,
            "peak": INT32_VALU_PEAK / 1e12,
            "unit": "T INT32 lane-instr/s (8 algorithmic instr per MAC term)",
            "frac": achieved / INT32_VALU_PEAK,
            "frac_time_weighted_all_emulation_kernels": ALGO_OPS_PER_TERM * tot_terms / (tot_ms * 1e-3) / INT32_VALU_PEAK,
            "valu_instr_per_term": ctr.get("valu_instr_per_term"),
            "valu_util": (ctr["valu_instr_per_term"] * dom["terms_per_launch"] / (dom["avg_ms"] * 1e-3) / INT32_VALU_PEAK) if ctr else None,
            "traffic": ctr.get("traffic"),
            "traffic_source": COUNTERS_SOURCE if ctr else None,
        },
    }
    for scan in scans:
        scan.close()
    if not args.no_other_workloads:
        # the other four workloads, once each, outside the timed region: end-to-end rates for context
        other = {}
        configs.config1(n_tiles=256)
        for name, fn in (("configs[0]", lambda: configs.config1()), ("configs[1]", lambda: configs.config2()),
                         ("configs[2]", lambda: configs.config3()), ("configs[3]", lambda: configs.config4(fused=fused))):
            fn()                                  # (first call of a workload: kernel loading and allocator warm-up)
            r = fn()
            other[name] = dict(terms=r["terms"], ms=r["seconds"] * 1e3, terms_per_s=r["terms"] / r["seconds"])
        # beside the five: Step 4 on sixteen TR-FDPA candidates at once (the fitted gfx950 set with other widths and group
        # lengths) against the native 16x16x16 instructions, three input families of 2^16 tiles each
        from paper_2511_10909_amd import presets
        for name, instr in (("tr_fdpa_candidates_fp16", mm.MFMA_F32_16X16X16_F16), ("tr_fdpa_candidates_bf16", mm.MFMA_F32_16X16X16_BF16)):
            fitted = presets.GFX950_MFMA[instr]
            cands = [dict(fitted, frac_bits=F, frac_bits2=F2, group_len=L) for F in (20, 24) for F2 in (27, 31) for L in (4, 8, 16, 8)][:16]
            cands[15] = dict(fitted)
            fams = ("normal", "finite_bits", "random_bits")
            configs.scan_against_mfma(instr, cands, n_tiles=1 << 12, families=fams)
            r = configs.scan_against_mfma(instr, cands, n_tiles=1 << 16, families=fams)
            other[name] = dict(terms=r["terms"], ms=r["seconds"] * 1e3, terms_per_s=r["terms"] / r["seconds"],
                               candidates_without_mismatch=sum(1 for t in r["total"] if t == 0))
        # the deviation histograms of Sec. 6.2.4 (TR-FDPA as printed, its truncating variant, the native instruction) on
        # 2^18 FP16 32x32x8 tiles, every output against its exact result
        configs.bias_experiment(n_tiles=1 << 12)
        r = configs.bias_experiment(n_tiles=1 << 18)
        other["bias_experiment_fp16"] = dict(terms=r["terms"], ms=r["seconds"] * 1e3, terms_per_s=r["terms"] / r["seconds"],
                                             mean_delta={k: h["sum"] / max(h["n_samples"], 1) for k, h in r["hists"].items()})
        out["config"]["other_workloads_end_to_end"] = other
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
