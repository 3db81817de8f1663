"""The five probing workloads, run through libmmaemu (device memory from PyTorch, every
computation inside the library).  Each runner returns a dict of results; tensors it leaves
on the device are returned under "dev" so that tests can check them against the CPU oracle.

Workloads (synthetic stand-ins for the randomized validation of the paper's Sec. 3.1 Step 4):
  config1  10,000 fp16 16x16x16 tiles, uniform finite bit patterns, C ~ N(0,1); F = 27, L = 16,
           RNE against RZ output
  config2  bf16 1024^3 GEMM, N(0,1) operands, C = 0; groups of 8 added exactly to the running
           sum (C_AFTER_EXACT) against the fully fused model
  config3  e4m3 x e5m2 4096^3 GEMM, N(0,1) scaled per tensor to the format maximum; F = 14,
           L = 32; error statistics against exact dot products on a 1 % sample
  config4  subnormal stress: fp16 32x32x8 tiles with uniform exponent fields; input-flush,
           output-flush and no-flush variants, histogram of each against the no-flush run
  config5  closed-loop scan: 16 parameter sets x {bf16, fp8} 16x16x16 tiles against the native
           MFMA instruction
"""
import bisect
import time

import torch

from . import binding as mm

_TORCH = {1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}


def _buf(shape, dtype_id, dev):
    return torch.empty(shape, dtype=_TORCH[mm.ELEM_BYTES[dtype_id]], device=dev)


def _stats_buf(dev):
    st = torch.empty(mm.STATS_BYTES, dtype=torch.uint8, device=dev)
    mm.stats_reset(st)
    return st


def _timed(fn):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = fn()
    torch.cuda.synchronize()
    return out, time.perf_counter() - t0


def _graph_of(fn):
    """`fn` (kernel launches of this library only: no allocation, no synchronisation) captured in a HIP graph; the
    captured launches run once here, on a side stream, before the capture."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            fn()
    torch.cuda.synchronize()
    return graph


def config1(n_tiles=10000, seed=0, dev="cuda", use_graph=False, fused=False):
    """`fused`: both models in one launch of the scan kernel, the first one's outputs being the reference (both models'
    outputs are still written, for the parity tests); otherwise two emulation launches and one comparison launch, which
    on these 10 000 tiles is the faster way (0.10 ms against 0.12 ms: with two models and every output written, the
    scan kernel has nothing to share).
    `use_graph`: the step is small enough to be bound by its launches; captured in a HIP graph it is replayed
    as one submission (the statistics are reset inside the step so that every replay stands alone)."""
    m = n = k = 16
    dt = (mm.FP16, mm.FP16, mm.FP32, mm.FP32)
    A, B = _buf((n_tiles, m, k), mm.FP16, dev), _buf((n_tiles, n, k), mm.FP16, dev)
    C, Dall = _buf((n_tiles, m, n), mm.FP32, dev), _buf((2, n_tiles, m, n), mm.FP32, dev)
    D0, D1 = Dall[0], Dall[1]
    st = _stats_array(2, dev) if fused else _stats_buf(dev)
    m0 = mm.model_create(group_len=16, frac_bits=27, out_round=mm.RNE)
    m1 = mm.model_create(group_len=16, frac_bits=27, out_round=mm.RZ)

    def run():
        mm.generate(A, mm.FP16, m * k, 0, n_tiles, mm.GEN_FINITE_BITS, seed=seed, operand=0)
        mm.generate(B, mm.FP16, n * k, 0, n_tiles, mm.GEN_FINITE_BITS, seed=seed, operand=1)
        mm.generate(C, mm.FP32, m * n, 0, n_tiles, mm.GEN_NORMAL, seed=seed, operand=2)
        if fused:
            mm.emulate_compare_many([m0, m1], A, B, C, None, Dall, m, n, k, n_tiles, dt, st)
            return mm.last_kernel()
        mm.emulate_mma(m0, A, B, C, D0, m, n, k, n_tiles, dt)
        k0 = mm.last_kernel()
        mm.emulate_mma(m1, A, B, C, D1, m, n, k, n_tiles, dt)
        mm.compare(D0, D1, n_tiles * m * n, st)
        return k0

    if use_graph:
        def step():
            mm.stats_reset(st)
            if fused:
                mm.stats_reset(st[mm.STATS_BYTES:])
            run()
        kernel = run()
        graph = _graph_of(step)
        _, secs = _timed(graph.replay)
    else:
        kernel, secs = _timed(run)
    mm.model_destroy(m0)
    mm.model_destroy(m1)
    # (fused: the statistics of the second model against the first)
    stats = mm.read_stats_array(st, 2)[1] if fused else mm.read_stats(st)
    return dict(terms=2 * n_tiles * m * n * k, seconds=secs, kernel=kernel, stats=stats,
                dev=dict(A=A, B=B, C=C, D0=D0, D1=D1))


def config2(size=1024, seed=0, dev="cuda"):
    m = n = k = size
    dt = (mm.BF16, mm.BF16, mm.FP32, mm.FP32)
    A, B = _buf((m, k), mm.BF16, dev), _buf((n, k), mm.BF16, dev)
    C, D0, D1 = (_buf((m, n), mm.FP32, dev) for _ in range(3))
    st = _stats_buf(dev)
    chained = mm.model_create(group_len=8, frac_bits=24, c_mode=mm.C_AFTER_EXACT)
    fused = mm.model_create(group_len=0, frac_bits=24, c_mode=mm.C_IN_GROUP)

    def run():
        mm.generate(A, mm.BF16, m * k, 0, 1, mm.GEN_NORMAL, seed=seed, operand=0)
        mm.generate(B, mm.BF16, n * k, 0, 1, mm.GEN_NORMAL, seed=seed, operand=1)
        mm.generate(C, mm.FP32, m * n, 0, 1, mm.GEN_ZERO, seed=seed, operand=2)
        mm.emulate_mma(chained, A, B, C, D0, m, n, k, 1, dt)
        k0 = mm.last_kernel()
        mm.emulate_mma(fused, A, B, C, D1, m, n, k, 1, dt)
        k1 = mm.last_kernel()
        mm.compare(D0, D1, m * n, st)
        return k0, k1

    kernels, secs = _timed(run)
    mm.model_destroy(chained)
    mm.model_destroy(fused)
    return dict(terms=2 * m * n * k, seconds=secs, kernels=kernels, stats=mm.read_stats(st),
                dev=dict(A=A, B=B, C=C, D0=D0, D1=D1))


def config3(size=4096, seed=0, stride=100, dev="cuda"):
    m = n = k = size
    dt = (mm.E4M3, mm.E5M2, mm.FP32, mm.FP32)
    A, B = _buf((m, k), mm.E4M3, dev), _buf((n, k), mm.E5M2, dev)
    C, D = _buf((m, n), mm.FP32, dev), _buf((m, n), mm.FP32, dev)
    ws = torch.empty(8, dtype=torch.uint8, device=dev)
    err = torch.empty(mm.ERR_STATS_BYTES, dtype=torch.uint8, device=dev)
    mm.err_stats_reset(err)
    model = mm.model_create(group_len=32, frac_bits=14, out_round=mm.RNE)

    def run():
        mm.generate(A, mm.E4M3, m * k, 0, 1, mm.GEN_NORMAL, seed=seed, operand=0, scale_scope=mm.SCALE_TENSOR,
                    scale_target=448.0, workspace=ws)
        mm.generate(B, mm.E5M2, n * k, 0, 1, mm.GEN_NORMAL, seed=seed, operand=1, scale_scope=mm.SCALE_TENSOR,
                    scale_target=57344.0, workspace=ws)
        mm.generate(C, mm.FP32, m * n, 0, 1, mm.GEN_ZERO, seed=seed, operand=2)
        mm.emulate_mma(model, A, B, C, D, m, n, k, 1, dt)
        kern = mm.last_kernel()
        mm.exact_dot_sample(A, B, D, m, n, k, dt, stride, err)
        return kern

    kernel, secs = _timed(run)
    mm.model_destroy(model)
    return dict(terms=m * n * k, seconds=secs, kernel=kernel, err_stats=mm.read_err_stats(err),
                dev=dict(A=A, B=B, C=C, D=D))


CONFIG4_VARIANTS = (("none", dict()), ("ftz_in", dict(ftz_in=True)), ("ftz_out", dict(ftz_out=True)))


def config4_generate(A, B, C, first_tile, n_tiles, seed=0):
    """fp16 A/B with sign, exponent field 0..30 and mantissa all uniform; fp32 C with exponent field
    uniform over {0} and 79..158 (zero/subnormal, or the span of fp16 products)."""
    mm.generate(A, mm.FP16, 32 * 8, first_tile, n_tiles, mm.GEN_UNIFORM_EXP, seed=seed, operand=0, exp_lo=0, exp_hi=30)
    mm.generate(B, mm.FP16, 32 * 8, first_tile, n_tiles, mm.GEN_UNIFORM_EXP, seed=seed, operand=1, exp_lo=0, exp_hi=30)
    mm.generate(C, mm.FP32, 32 * 32, first_tile, n_tiles, mm.GEN_UNIFORM_EXP, seed=seed, operand=2, exp_lo=79,
                exp_hi=158, exp_zero=True)


def _stats_array(count, dev):
    st = torch.empty(count * mm.STATS_BYTES, dtype=torch.uint8, device=dev)
    for i in range(count):
        mm.stats_reset(st[i * mm.STATS_BYTES:])
    return st


class _Sampler:
    """Keeps the operands and outputs of chosen tiles of a streamed run (device-side copies, no synchronisation)."""

    def __init__(self, tiles):
        self.tiles = sorted(int(t) for t in (tiles if tiles is not None else ()))
        self.kept = []

    def in_chunk(self, t0, nt):
        lo, hi = bisect.bisect_left(self.tiles, t0), bisect.bisect_left(self.tiles, t0 + nt)
        return [t - t0 for t in self.tiles[lo:hi]]

    def take(self, t0, local, **tensors):
        idx = torch.tensor(local, dtype=torch.int64, device=next(iter(tensors.values())).device)
        rec = {name: (t.index_select(1, idx) if name == "D" else t.index_select(0, idx)) for name, t in tensors.items()}
        rec["tiles"] = [t0 + i for i in local]
        self.kept.append(rec)


def config4(n_tiles=1 << 26, chunk=1 << 18, seed=0, dev="cuda", keep_first_chunk=False, fused=True, sample_tiles=None,
            first_tile=0, timer=None, time_every=64):
    """Tiles first_tile .. first_tile + n_tiles - 1 of the stream.  `timer`, if given, is called as timer(name, terms, fn)
    around the emulation launches of every `time_every`-th chunk (it must run fn).  `fused`: the three variants share one pass over each chunk (mmaemu_emulate_compare_many, the no-flush variant's
    outputs as the reference, D never written); otherwise one emulation and one comparison per variant.
    `keep_first_chunk` / `sample_tiles`: operands and all three outputs of the first chunk / of the given tiles are
    kept (those chunks also write D) and returned under "dev" / "samples"."""
    m = n = 32
    k = 8
    dt = (mm.FP16, mm.FP16, mm.FP32, mm.FP32)
    chunk = min(chunk, n_tiles)
    nv = len(CONFIG4_VARIANTS)
    A, B = _buf((chunk, m, k), mm.FP16, dev), _buf((chunk, n, k), mm.FP16, dev)
    C = _buf((chunk, m, n), mm.FP32, dev)
    Dall = _buf((nv, chunk, m, n), mm.FP32, dev) if (not fused or keep_first_chunk or sample_tiles is not None) else None
    stats = _stats_array(nv, dev)
    models = [mm.model_create(group_len=8, frac_bits=24, out_round=mm.RNE, **kw) for _, kw in CONFIG4_VARIANTS]
    kept = {}
    sampler = _Sampler(sample_tiles)

    def run():
        kern = None
        for ci, t0 in enumerate(range(first_tile, first_tile + n_tiles, chunk)):
            nt = min(chunk, first_tile + n_tiles - t0)
            run_ = (lambda name, terms, fn: fn()) if (timer is None or ci % time_every) else timer
            config4_generate(A, B, C, t0, nt, seed)
            local = sampler.in_chunk(t0, nt)
            keep = keep_first_chunk and t0 == first_tile
            want_d = (not fused) or keep or bool(local)
            # ([variant][tile][m][n] for this chunk's tile count: the layout mmaemu_emulate_compare_many writes)
            dump = Dall.reshape(-1)[: nv * nt * m * n].view(nv, nt, m, n) if want_d else None
            if fused:
                run_("variants", nv * nt * m * n * k,
                     lambda: mm.emulate_compare_many(models, A, B, C, None, dump, m, n, k, nt, dt, stats, index_base=t0 * m * n))
                kern = mm.last_kernel()
            else:
                for i, h in enumerate(models):
                    run_("variant %d" % i, nt * m * n * k, lambda: mm.emulate_mma(h, A, B, C, dump[i], m, n, k, nt, dt))
                kern = mm.last_kernel()
                for i in range(nv):
                    mm.compare(dump[i], dump[0], nt * m * n, stats[i * mm.STATS_BYTES:], index_base=t0 * m * n)
            if keep:
                kept.update(A=A.clone(), B=B.clone(), C=C.clone(), D=[dump[i].clone() for i in range(nv)])
            if local:
                sampler.take(t0, local, A=A[:nt], B=B[:nt], C=C[:nt], D=dump)
        return kern

    kernel, secs = _timed(run)
    for h in models:
        mm.model_destroy(h)
    res = mm.read_stats_array(stats, nv)
    return dict(terms=nv * n_tiles * m * n * k, seconds=secs, kernel=kernel,
                stats={name: st for (name, _), st in zip(CONFIG4_VARIANTS, res)}, dev=kept, samples=sampler.kept)


# (F, L_max, output rounding, flush both ways)
CONFIG5_MODELS = [(16, 4, mm.RNE, 0), (16, 8, mm.RZ, 1), (16, 16, mm.RNE, 1), (16, 64, mm.RZ, 0),
                  (20, 4, mm.RZ, 1), (20, 8, mm.RNE, 0), (20, 16, mm.RZ, 0), (20, 32, mm.RNE, 1),
                  (24, 4, mm.RNE, 1), (24, 8, mm.RZ, 0), (24, 16, mm.RNE, 0), (24, 32, mm.RZ, 1),
                  (28, 8, mm.RNE, 1), (32, 4, mm.RZ, 0), (32, 16, mm.RZ, 1), (32, 64, mm.RNE, 0)]


def config5_generate(kind, A, B, C, first_tile, n_tiles, seed=0):
    """kind "bf16": uniform finite bf16 bit patterns; kind "fp8": N(0,1) scaled per tile to the format
    maximum, A e4m3 and B e5m2.  C ~ N(0,1) fp32 for both."""
    if kind == "bf16":
        mm.generate(A, mm.BF16, 256, first_tile, n_tiles, mm.GEN_FINITE_BITS, seed=seed, operand=0)
        mm.generate(B, mm.BF16, 256, first_tile, n_tiles, mm.GEN_FINITE_BITS, seed=seed, operand=1)
    else:
        mm.generate(A, mm.E4M3, 256, first_tile, n_tiles, mm.GEN_NORMAL, seed=seed, operand=0,
                    scale_scope=mm.SCALE_TILE, scale_target=448.0)
        mm.generate(B, mm.E5M2, 256, first_tile, n_tiles, mm.GEN_NORMAL, seed=seed, operand=1,
                    scale_scope=mm.SCALE_TILE, scale_target=57344.0)
    mm.generate(C, mm.FP32, 256, first_tile, n_tiles, mm.GEN_NORMAL, seed=seed, operand=2)


class ClosedLoopScan:
    """Workload 5 for one operand type: the sixteen parameter sets over chunks of generated 16x16x16 tiles, each chunk
    also run through the native MFMA instruction, per-set statistics of model against instruction.

    `fused`: one mmaemu_emulate_compare_many call per class of sets that share launches (the statistics are formed
    inside the emulation kernels); otherwise one mmaemu_emulate_mma and one mmaemu_compare per set.  `timer`, if given,
    is called as timer(name, fn) around every emulation launch of a chunk whose index is a multiple of `time_every`
    (it must run fn); bench.py uses it for HIP events."""

    def __init__(self, kind, chunk=1 << 16, seed=0, dev="cuda", fused=True, with_dump=False):
        self.kind, self.chunk, self.seed, self.fused = kind, chunk, seed, fused
        self.ta, self.tb = (mm.BF16, mm.BF16) if kind == "bf16" else (mm.E4M3, mm.E5M2)
        self.instr = mm.MFMA_F32_16X16X16_BF16 if kind == "bf16" else mm.MFMA_F32_16X16X32_FP8_BF8
        self.dt = (self.ta, self.tb, mm.FP32, mm.FP32)
        nm = len(CONFIG5_MODELS)
        self.A, self.B = _buf((chunk, 16, 16), self.ta, dev), _buf((chunk, 16, 16), self.tb, dev)
        self.C, self.Dhw = _buf((chunk, 16, 16), mm.FP32, dev), _buf((chunk, 16, 16), mm.FP32, dev)
        self.D1 = None if fused else _buf((chunk, 16, 16), mm.FP32, dev)
        self.Dall = _buf((nm, chunk, 16, 16), mm.FP32, dev) if with_dump else None
        self.stats = _stats_array(nm, dev)
        self.models = [mm.model_create(group_len=L, frac_bits=F, out_round=rho, ftz_in=bool(ftz), ftz_out=bool(ftz))
                       for F, L, rho, ftz in CONFIG5_MODELS]
        cls = mm.compare_many_classes(self.models, 16, 16, 16, self.dt)
        self.groups = []                                   # lists of set indices; one launch each when fused
        for c in sorted(set(cls)):
            members = [i for i, x in enumerate(cls) if x == c]
            self.groups.extend([[i] for i in members] if c < 0 else [members])
        # the statistics array is laid out group by group, so that every group's structs are consecutive
        order = [i for g in self.groups for i in g]
        self.pos = {i: q for q, i in enumerate(order)}
        self.kernels = {}

    def close(self):
        for h in self.models:
            mm.model_destroy(h)
        self.models = []

    def reset(self):
        for i in range(len(CONFIG5_MODELS)):
            mm.stats_reset(self.stats[i * mm.STATS_BYTES:])

    def _slot(self, i):
        return self.stats[self.pos[i] * mm.STATS_BYTES:]

    def chunk_step(self, t0, nt, dump=False, timer=None):
        """Generate tiles t0 .. t0 + nt - 1, run the instruction and every set, accumulate the statistics.
        `dump`: every set's outputs of this chunk are also written to self.Dall[set]."""
        A, B, C, Dhw = self.A, self.B, self.C, self.Dhw
        config5_generate(self.kind, A, B, C, t0, nt, self.seed)
        mm.mfma_probe(self.instr, A, B, C, Dhw, 16, nt)              # fp8: k positions 16..31 are fed as zeros
        run = (lambda name, terms, fn: fn()) if timer is None else timer
        if self.fused and not dump:
            for gi, members in enumerate(self.groups):
                hs = [self.models[i] for i in members]
                run("group %d" % gi, len(members) * nt * 4096,
                    lambda: mm.emulate_compare_many(hs, A, B, C, Dhw, None, 16, 16, 16, nt, self.dt, self._slot(members[0]), index_base=t0 * 256))
                self.kernels.setdefault(gi, mm.last_kernel())
        elif self.fused:
            for i, h in enumerate(self.models):                      # (a set's dump area is its own slice of Dall)
                mm.emulate_compare_many([h], A, B, C, Dhw, self.Dall[i, :nt], 16, 16, 16, nt, self.dt, self._slot(i), index_base=t0 * 256)
        else:
            for i, h in enumerate(self.models):
                D = self.Dall[i, :nt] if dump else self.D1
                run("set %d" % i, nt * 4096, lambda: mm.emulate_mma(h, A, B, C, D, 16, 16, 16, nt, self.dt))
                self.kernels.setdefault(i, mm.last_kernel())
                mm.compare(D, Dhw, nt * 256, self._slot(i), index_base=t0 * 256)

    def read(self):
        """Per-set statistics, a list of dicts in the order of CONFIG5_MODELS."""
        res = mm.read_stats_array(self.stats, len(CONFIG5_MODELS))
        return [res[self.pos[i]] for i in range(len(CONFIG5_MODELS))]


def config5(n_tiles=1 << 24, chunk=1 << 16, seed=0, dev="cuda", kinds=("bf16", "fp8"), keep_first_chunk=False, fused=True,
            sample_tiles=None, first_tile=0):
    """Tiles first_tile .. first_tile + n_tiles - 1 of each operand type's stream; `keep_first_chunk` / `sample_tiles` as
    in config4 (the chunks concerned write every set's D)."""
    out = {}
    for kind in kinds:
        ch = min(chunk, n_tiles)
        need_dump = keep_first_chunk or sample_tiles is not None
        scan = ClosedLoopScan(kind, ch, seed, dev, fused, with_dump=need_dump)
        kept = {}
        sampler = _Sampler(sample_tiles)

        def run():
            for t0 in range(first_tile, first_tile + n_tiles, ch):
                nt = min(ch, first_tile + n_tiles - t0)
                local = sampler.in_chunk(t0, nt)
                keep = keep_first_chunk and t0 == first_tile
                scan.chunk_step(t0, nt, dump=bool(keep or local))
                if keep:
                    kept.update(A=scan.A.clone(), B=scan.B.clone(), C=scan.C.clone(), Dhw=scan.Dhw.clone(),
                                D=[scan.Dall[i, :nt].clone() for i in range(len(CONFIG5_MODELS))])
                if local:
                    sampler.take(t0, local, A=scan.A[:nt], B=scan.B[:nt], C=scan.C[:nt], Dhw=scan.Dhw[:nt], D=scan.Dall[:, :nt])

        _, secs = _timed(run)
        res = scan.read()
        kernels = [scan.kernels[key] for key in sorted(scan.kernels)]
        scan.close()
        out[kind] = dict(terms=len(CONFIG5_MODELS) * n_tiles * 256 * 16, seconds=secs, kernels=kernels, stats=res,
                         agreement=[1.0 - s["n_mismatch_bits"] / max(s["n_compared"], 1) for s in res], dev=kept,
                         samples=sampler.kept)
    return out


# ---------------------------------------------------------------------------------------------
# Randomised validation of a candidate model against the native instruction (paper Sec. 3, Step 4).

def bias_experiment_generate(A, B, C, first_tile, n_tiles, seed=0):
    """Sec. 6.2.4's inputs: A, B ~ 1000 x N(0,1) in FP16, C ~ N(0,1) in FP32, 32x32x8 tiles."""
    mm.generate(A, mm.FP16, 32 * 8, first_tile, n_tiles, mm.GEN_NORMAL, seed=seed, operand=0, scale_scope=mm.SCALE_FACTOR, scale_target=1000.0)
    mm.generate(B, mm.FP16, 32 * 8, first_tile, n_tiles, mm.GEN_NORMAL, seed=seed, operand=1, scale_scope=mm.SCALE_FACTOR, scale_target=1000.0)
    mm.generate(C, mm.FP32, 32 * 32, first_tile, n_tiles, mm.GEN_NORMAL, seed=seed, operand=2)


BIAS_BIN_EXP = -5        # bins of 1/32: outputs lie around 2^21 .. 2^23, one place of binary32 there is 1/4 .. 1/2


def bias_experiment(n_tiles=1 << 20, chunk=1 << 14, seed=0, stride=1, dev="cuda", keep_first_chunk=False, with_mfma=True):
    """The numerical-bias experiment of Sec. 6.2.4 as a device workload: the CDNA3 model of v_mfma_f32_32x32x8_f16
    (Algorithm "TR-FDPA", L = 8, F = 24, F2 = 31, RNE-FP32) and the hypothetical variant whose round-downs truncate
    toward zero instead, on the paper's inputs; per variant the distribution of delta = D - D_real with D_real exact
    (mmaemu_deviation_sample on every stride-th output), plus the same for this GPU's own instruction."""
    from . import presets
    m, n, k = 32, 32, 8
    dt = (mm.FP16, mm.FP16, mm.FP32, mm.FP32)
    A, B = _buf((chunk, m, k), mm.FP16, dev), _buf((chunk, n, k), mm.FP16, dev)
    C, D = _buf((chunk, m, n), mm.FP32, dev), _buf((chunk, m, n), mm.FP32, dev)
    base = presets.PAPER[("cdna3", "fp16")]
    variants = [("rd", mm.model_create(**base)), ("rz", mm.model_create(**dict(base, rd_toward_zero=True)))]
    names = [v[0] for v in variants] + (["mfma"] if with_mfma else [])
    hists = {name: torch.empty(mm.DEVIATION_HIST_BYTES, dtype=torch.uint8, device=dev) for name in names}
    for h in hists.values():
        mm.deviation_hist_reset(h)
    kernels, first = {}, {}

    def run():
        for t0 in range(0, n_tiles, chunk):
            nt = min(chunk, n_tiles - t0)
            bias_experiment_generate(A, B, C, t0, nt, seed)
            for name, h in variants:
                mm.emulate_mma(h, A, B, C, D, m, n, k, nt, dt)
                kernels[name] = mm.last_kernel()
                mm.deviation_sample(A, B, C, D, m, n, k, nt, dt, stride, BIAS_BIN_EXP, hists[name])
                if keep_first_chunk and t0 == 0:
                    first[name] = D.clone()
            if with_mfma:
                mm.mfma_probe(mm.MFMA_F32_32X32X8_F16, A, B, C, D, k, nt)
                mm.deviation_sample(A, B, C, D, m, n, k, nt, dt, stride, BIAS_BIN_EXP, hists["mfma"])
            if keep_first_chunk and t0 == 0:
                first.update(A=A.clone(), B=B.clone(), C=C.clone())

    _, secs = _timed(run)
    for _, h in variants:
        mm.model_destroy(h)
    out = dict(terms=len(variants) * n_tiles * m * n * k, seconds=secs, kernels=kernels,
               hists={name: mm.read_deviation_hist(h) for name, h in hists.items()}, first=first)
    return out


def validation_families(ta, tb):
    """Input families of Step 4: common distributions, all finite bit patterns, all bit patterns (NaN and infinities
    included: the paper calls this one the most important), and exponent ranges chosen to put the accumulator above,
    below and anywhere relative to the products.  Each entry: (name, generator arguments for A, for B, for C)."""
    cs = 896 if ta == mm.FP64 else 0           # exponent codes of the accumulator's format: binary64's bias is 1023, binary32's 127
    full = {mm.FP64: (1, 2046), mm.FP32: (1, 254), mm.FP16: (1, 30), mm.BF16: (1, 254), mm.E4M3: (0, 15), mm.E5M2: (0, 30), mm.E2M3: (0, 3), mm.E3M2: (0, 7), mm.E2M1: (0, 3)}
    mid = {mm.FP64: (1016, 1030), mm.FP32: (120, 134), mm.FP16: (11, 19), mm.BF16: (120, 134), mm.E4M3: (3, 11), mm.E5M2: (11, 19), mm.E2M3: (1, 2), mm.E3M2: (2, 5), mm.E2M1: (1, 2)}

    def ue(rng, zero=True):
        return dict(family=mm.GEN_UNIFORM_EXP, exp_lo=rng[0], exp_hi=rng[1], exp_zero=zero)

    simple = [("normal", mm.GEN_NORMAL), ("uniform", mm.GEN_UNIFORM), ("normal_outliers", mm.GEN_NORMAL_OUTLIERS),
              ("finite_bits", mm.GEN_FINITE_BITS), ("random_bits", mm.GEN_RANDOM_BITS)]
    fams = [(name, dict(family=f), dict(family=f), dict(family=f)) for name, f in simple]
    # adversarial sums: products cancelling pairwise up to last-place perturbations, accumulator near the residue
    canc = dict(family=mm.GEN_CANCELLING, exp_zero=False)
    if ta not in (mm.FP32, mm.FP64):       # (the generator does not build cancelling pairs of FP32 / FP64 values)
        fams.append(("cancelling", dict(canc, exp_lo=mid[ta][0], exp_hi=mid[ta][1]), dict(canc, exp_lo=mid[tb][0], exp_hi=mid[tb][1]),
                     ue((100, 135))))
    # zeros of both signs, +-1 and the smallest subnormals: exact zeros from zeros, whose sign a model must get right
    zs = dict(family=mm.GEN_SIGNED_ZEROS)
    fams.append(("signed_zeros", zs, zs, zs))
    fams.append(("mid_exp_c_above", ue(mid[ta]), ue(mid[tb]), ue((cs + 125, cs + 145), zero=False)))
    fams.append(("mid_exp_c_below", ue(mid[ta]), ue(mid[tb]), ue((cs + 80, cs + 129))))
    fams.append(("wide_exp_c_any", ue(full[ta]), ue(full[tb]), ue((1, 2046) if cs else (1, 254))))
    # every product at one exponent, the accumulator 20 to 32 binary places above it (where whole sums drop out)
    bias = {mm.FP64: 1023, mm.FP32: 127, mm.FP16: 15, mm.BF16: 127, mm.E4M3: 7, mm.E5M2: 15, mm.E2M3: 1, mm.E3M2: 3, mm.E2M1: 1}
    one = {mm.FP64: 1024, mm.FP32: 128, mm.FP16: 16, mm.BF16: 128, mm.E4M3: 8, mm.E5M2: 16, mm.E2M3: 2, mm.E3M2: 4, mm.E2M1: 2}
    e_prod = (one[ta] - bias[ta]) + (one[tb] - bias[tb])
    fams.append(("one_exp_c_far_above", ue((one[ta], one[ta]), zero=False), ue((one[tb], one[tb]), zero=False),
                 ue((cs + 127 + e_prod + (49 if cs else 20), cs + 127 + e_prod + (61 if cs else 32)), zero=False)))
    if ta == mm.FP64:
        # products around the bottom of binary64's subnormal range
        tiny = ue((483, 489))
        fams.append(("tiny_products_c_zero", tiny, tiny, dict(family=mm.GEN_ZERO)))
        fams.append(("tiny_products_c_subnormal", tiny, tiny, ue((0, 2))))
    if ta == tb and ta in (mm.BF16, mm.FP32):
        # products around the bottom of binary32's subnormal range, with a zero and with a subnormal accumulator
        tiny = ue((46, 52))
        fams.append(("tiny_products_c_zero", tiny, tiny, dict(family=mm.GEN_ZERO)))
        fams.append(("tiny_products_c_subnormal", tiny, tiny, ue((0, 2))))
    return fams


# ranges of E8M0 scale codes for the block-scaled instructions: (name, lowest code, highest code, zero accumulator)
SCALE_RANGES = [("unit", 127, 127, False), ("narrow", 120, 134, False), ("wide", 60, 190, False), ("all_codes", 0, 255, False),
                ("low", 0, 70, False), ("low_c_zero", 30, 70, True)]


def validate_scaled_against_mfma(instr, model_kwargs, n_tiles=1024, seeds=(0,), dev="cuda"):
    """The same loop for a block-scaled native instruction (MFMA_SCALE_* ids; one E8M0 scale per row and 32 values of
    k): every input family under every range of scale codes in SCALE_RANGES.  Returns {(range, family): stats dict}
    plus "seconds", "terms" and "kernel"."""
    info = mm.mfma_info(instr)
    m, n, k, ta, tb = info["m"], info["n"], info["k"], info["a"], info["b"]
    nblk = k // 32
    A, B = _buf((n_tiles, m, k), ta, dev), _buf((n_tiles, n, k), tb, dev)
    SA, SB = _buf((n_tiles, m, nblk), mm.E8M0, dev), _buf((n_tiles, n, nblk), mm.E8M0, dev)
    C, Dhw, D = (_buf((n_tiles, m, n), mm.FP32, dev) for _ in range(3))
    h = mm.model_create(**model_kwargs)
    fams = validation_families(ta, tb)
    stats = {(rname, name): _stats_buf(dev) for rname, _, _, _ in SCALE_RANGES for name, _, _, _ in fams}

    def run():
        for rname, lo, hi, c_zero in SCALE_RANGES:
            for name, ga, gb, gc in fams:
                for seed in seeds:
                    mm.generate(A, ta, m * k, 0, n_tiles, seed=seed, operand=0, **ga)
                    mm.generate(B, tb, n * k, 0, n_tiles, seed=seed, operand=1, **gb)
                    mm.generate(C, mm.FP32, m * n, 0, n_tiles, seed=seed, operand=2, **(dict(family=mm.GEN_ZERO) if c_zero else gc))
                    mm.generate(SA, mm.E8M0, m * nblk, 0, n_tiles, family=mm.GEN_UNIFORM_EXP, seed=seed, operand=3, exp_lo=lo, exp_hi=hi)
                    mm.generate(SB, mm.E8M0, n * nblk, 0, n_tiles, family=mm.GEN_UNIFORM_EXP, seed=seed, operand=4, exp_lo=lo, exp_hi=hi)
                    mm.mfma_probe_scaled(instr, A, B, C, Dhw, SA, SB, k, n_tiles)
                    mm.emulate_mma_scaled(h, A, B, C, D, SA, SB, 32, m, n, k, n_tiles, (ta, tb, mm.FP32, mm.FP32))
                    mm.compare(D, Dhw, n_tiles * m * n, stats[(rname, name)])

    _, secs = _timed(run)
    kernel = mm.last_kernel()
    mm.model_destroy(h)
    out = {key: mm.read_stats(st) for key, st in stats.items()}
    out["seconds"] = secs
    out["terms"] = len(SCALE_RANGES) * len(fams) * len(seeds) * n_tiles * m * n * k
    out["kernel"] = kernel
    return out


def validate_against_mfma(instr, model_kwargs, n_tiles=4096, seeds=(0,), dev="cuda", fused=True):
    """Runs the native instruction `instr` (one issue per tile, k = the instruction's K) and the model on the same
    generated tiles and compares bit for bit.  Returns {family: stats dict} plus "seconds" and "terms".
    `fused` = False: one emulation and one comparison launch also where the scan kernel would take the model."""
    info = mm.mfma_info(instr)
    m, n, k, ta, tb = info["m"], info["n"], info["k"], info["a"], info["b"]
    A, B = _buf((n_tiles, m, k), ta, dev), _buf((n_tiles, n, k), tb, dev)
    tc = mm.FP64 if ta == mm.FP64 else mm.FP32            # the binary64 forms accumulate in binary64
    C, Dhw, D = (_buf((n_tiles, m, n), tc, dev) for _ in range(3))
    h = mm.model_create(**model_kwargs)
    fams = validation_families(ta, tb)
    stats = {name: _stats_buf(dev) for name, _, _, _ in fams}
    # a model that the scan kernel takes is compared inside it, D never reaches memory: with a single model that pays on
    # 16x16x16 tiles (+45 % for the loop); on the other shapes the single-model kernels' larger register blocks make up
    # for their store and the comparison launch
    fused = (fused and tc == mm.FP32 and (m, n, k) == (16, 16, 16)
             and mm.compare_many_classes([h], m, n, k, (ta, tb, tc, tc))[0] >= 0)

    def run():
        for name, ga, gb, gc in fams:
            for seed in seeds:
                mm.generate(A, ta, m * k, 0, n_tiles, seed=seed, operand=0, **ga)
                mm.generate(B, tb, n * k, 0, n_tiles, seed=seed, operand=1, **gb)
                mm.generate(C, tc, m * n, 0, n_tiles, seed=seed, operand=2, **gc)
                mm.mfma_probe(instr, A, B, C, Dhw, k, n_tiles)
                if fused:
                    mm.emulate_compare_many([h], A, B, C, Dhw, None, m, n, k, n_tiles, (ta, tb, tc, tc), stats[name])
                else:
                    mm.emulate_mma(h, A, B, C, D, m, n, k, n_tiles, (ta, tb, tc, tc))
                    mm.compare(D, Dhw, n_tiles * m * n, stats[name], d=tc)

    _, secs = _timed(run)
    kernel = mm.last_kernel()
    mm.model_destroy(h)
    out = {name: mm.read_stats(st) for name, st in stats.items()}
    out["seconds"] = secs
    out["terms"] = len(fams) * len(seeds) * n_tiles * m * n * k
    out["kernel"] = kernel
    return out


def scan_against_mfma(instr, candidates, n_tiles=1 << 16, seeds=(0,), families=None, dev="cuda"):
    """Sec. 3.1 Step 4 for a list of candidate models at once: every input family (or the named ones) is generated,
    run through the native instruction `instr` and through all `candidates` (keyword dicts for model_create) in one
    mmaemu_emulate_compare_many call per family and seed, each candidate compared bit for bit with the instruction.
    Returns {"mismatches": [[per family] per candidate], "families": names, "total": [per candidate], "seconds",
    "terms", "classes": the launch class of each candidate (-1: one emulation and one comparison launch of its own)}.
    A candidate with total 0 reproduces the instruction on every input tried."""
    info = mm.mfma_info(instr)
    m, n, k, ta, tb = info["m"], info["n"], info["k"], info["a"], info["b"]
    dt = (ta, tb, mm.FP32, mm.FP32)
    A, B = _buf((n_tiles, m, k), ta, dev), _buf((n_tiles, n, k), tb, dev)
    C, Dhw = _buf((n_tiles, m, n), mm.FP32, dev), _buf((n_tiles, m, n), mm.FP32, dev)
    hs = [mm.model_create(**kw) for kw in candidates]
    try:
        classes = mm.compare_many_classes(hs, m, n, k, dt)
        # (only models outside the scan kernel need their outputs in memory; the call wants one array for all then)
        Dall = _buf((len(hs), n_tiles, m, n), mm.FP32, dev) if min(classes) < 0 else None
        fams = [f for f in validation_families(ta, tb) if families is None or f[0] in families]
        stats = {name: _stats_array(len(hs), dev) for name, _, _, _ in fams}

        def run():
            for name, ga, gb, gc in fams:
                for seed in seeds:
                    mm.generate(A, ta, m * k, 0, n_tiles, seed=seed, operand=0, **ga)
                    mm.generate(B, tb, n * k, 0, n_tiles, seed=seed, operand=1, **gb)
                    mm.generate(C, mm.FP32, m * n, 0, n_tiles, seed=seed, operand=2, **gc)
                    mm.mfma_probe(instr, A, B, C, Dhw, k, n_tiles)
                    mm.emulate_compare_many(hs, A, B, C, Dhw, Dall, m, n, k, n_tiles, dt, stats[name])

        _, secs = _timed(run)
        per = {name: mm.read_stats_array(st, len(hs)) for name, st in stats.items()}
    finally:
        for h in hs:
            mm.model_destroy(h)
    names = [f[0] for f in fams]
    mism = [[per[name][i]["n_mismatch_bits"] for name in names] for i in range(len(candidates))]
    return dict(mismatches=mism, families=names, total=[sum(row) for row in mism], seconds=secs, classes=classes,
                terms=len(candidates) * len(fams) * len(seeds) * n_tiles * m * n * k)


def _report(argv=None):
    """`python -m paper_2511_10909_amd.configs`: the five workloads end to end, one table row each."""
    import argparse
    ap = argparse.ArgumentParser(description="run the five benchmark workloads end to end and print their rates")
    ap.add_argument("--tiles4", type=int, default=1 << 26, help="tiles of workload 4 (the workload as stated: 2^26)")
    ap.add_argument("--tiles5", type=int, default=1 << 24, help="tiles of workload 5 per operand type (as stated: 2^24)")
    ap.add_argument("--unfused", action="store_true", help="workloads 4 and 5 with one emulation and one comparison per model")
    ap.add_argument("--size3", type=int, default=4096, help="m = n = k of workload 3")
    ap.add_argument("--tiles6", type=int, default=1 << 20, help="tiles of the bias experiment (Sec. 6.2.4)")
    args = ap.parse_args(argv)
    config1(n_tiles=256)                                  # (first call: library load and allocator warm-up)

    def row(name, r, note=""):
        print("| %s | %.3g | %.3f | %.3g | %s |" % (name, r["terms"], 1e3 * r["seconds"], r["terms"] / r["seconds"], note), flush=True)

    print("| workload | MAC terms | ms | terms/s end to end | |\n|---|---|---|---|---|")
    r = config1()
    row("1: fp16 16x16x16, 10 000 tiles, RNE against RZ", r, "%d of %d outputs differ" % (r["stats"]["n_mismatch_bits"], r["stats"]["n_compared"]))
    r = config1(use_graph=True)
    row("1: the same, replayed from a HIP graph", r, "%d of %d outputs differ" % (r["stats"]["n_mismatch_bits"], r["stats"]["n_compared"]))
    config2()
    r = config2()
    row("2: bf16 1024^3, chained against fused", r, "%d of %d outputs differ" % (r["stats"]["n_mismatch_bits"], r["stats"]["n_compared"]))
    r = config3(size=args.size3)
    row("3: e4m3 x e5m2 %d^3, exact dots on 1 %% of D" % args.size3, r)
    r = config4(n_tiles=args.tiles4, fused=not args.unfused)
    row("4: fp16 32x32x8, %d tiles, three flush variants" % args.tiles4, r,
        ", ".join("%s: %d differ" % (name, st["n_mismatch_bits"]) for name, st in r["stats"].items()))
    r = config5(n_tiles=args.tiles5, fused=not args.unfused)
    for kind, v in r.items():
        row("5 (%s): 16x16x16, %d tiles, 16 models against the native MFMA" % (kind, args.tiles5), v,
            "agreement %.4f .. %.4f" % (min(v["agreement"]), max(v["agreement"])))
    r = bias_experiment(n_tiles=args.tiles6)
    means = ", ".join("%s: mean delta %+.4f (%d below, %d above)" % (name, h["sum"] / max(h["n_samples"], 1), h["n_negative"], h["n_positive"])
                      for name, h in r["hists"].items())
    row("6: deviation from the exact result, fp16 32x32x8, %d tiles, TR-FDPA as printed (rd) / truncating (rz) / this GPU's instruction" % args.tiles6, r, means)
    # beside the five: the validation loop of Sec. 3.1 Step 4 on one FP16 and one FP32 instruction of this GPU
    from . import presets
    for instr, name in ((mm.MFMA_F32_32X32X8_F16, "v_mfma_f32_32x32x8_f16"), (mm.MFMA_F32_16X16X4_F32, "v_mfma_f32_16x16x4_f32")):
        r = validate_against_mfma(instr, presets.GFX950_MFMA[instr], n_tiles=1 << 16, seeds=(0, 1))
        bad = sum(st["n_mismatch_bits"] for st in r.values() if isinstance(st, dict))
        row("validation of the fitted model against %s, 2^16 tiles, every input family, two seeds" % name, r, "%d outputs differ; %s" % (bad, r["kernel"]))


if __name__ == "__main__":
    _report()
