"""The five probing workloads at their real shapes, GPU against the CPU oracle.

All five run at their stated sizes.  Configs 4 and 5 stream 2^26 and 2^24 tiles per run (config 5 is the
workload bench.py times, in the same launch configuration).  Everything the oracle can recompute in
seconds is compared bit for bit: generated operands, emulated outputs (all of them, or a sample for
config 3 and, for the streamed configs, a prefix plus tiles at hashed indices over the whole stream),
and comparison statistics; the streamed runs are checked against their whole-run invariants as well.
"""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib, gen as ogen, stats as ostats
from oracle.fdpa import ModelParams, emulate_element, C_AFTER_EXACT
from oracle.rounding import RNE, RZ
from gpu_utils import to_host
from test_gpu_parity import assert_same, mm  # noqa: F401

THREADS = 8


@pytest.fixture(scope="module")
def cfg(mm):
    from paper_2511_10909_amd import configs
    return configs


def host(t, np_dtype):
    return to_host(t, np_dtype)


@pytest.mark.parametrize("fused", [True, False])
def test_config1_full(cfg, mm, fused):
    nt = 10000
    r = cfg.config1(n_tiles=nt, seed=0, fused=fused)
    assert r["kernel"].startswith("multi x2 tiled 16x16" if fused else "tiled 16x16"), r["kernel"]
    A = ogen.generate(ogen.GenParams(family=ogen.GEN_FINITE_BITS, seed=0, operand=0), fm.FP16, 256, 0, nt)
    B = ogen.generate(ogen.GenParams(family=ogen.GEN_FINITE_BITS, seed=0, operand=1), fm.FP16, 256, 0, nt)
    C = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=2), fm.FP32, 256, 0, nt)
    assert_same(host(r["dev"]["A"], np.uint16).reshape(nt, 256), A.astype(np.uint16), "config1 A")
    assert_same(host(r["dev"]["B"], np.uint16).reshape(nt, 256), B.astype(np.uint16), "config1 B")
    assert_same(host(r["dev"]["C"], np.uint32).reshape(nt, 256), C, "config1 C")
    A, B, C = A.reshape(nt, 16, 16), B.reshape(nt, 16, 16), C.reshape(nt, 16, 16)
    w0, _ = o2lib.emulate_mma(ModelParams(group_len=16, frac_bits=27, out_round=RNE), A, B, C, fm.FP16, fm.FP16)
    w1, _ = o2lib.emulate_mma(ModelParams(group_len=16, frac_bits=27, out_round=RZ), A, B, C, fm.FP16, fm.FP16)
    assert_same(host(r["dev"]["D0"], np.uint32), w0, "config1 D (RNE)")        # all 2.56e6 outputs
    assert_same(host(r["dev"]["D1"], np.uint32), w1, "config1 D (RZ)")
    assert r["stats"] == ostats.compare(w0, w1)
    assert r["stats"]["n_compared"] == nt * 256 and 0 < r["stats"]["n_mismatch_bits"] < nt * 256


def test_config2_full(cfg, mm):
    size = 1024
    r = cfg.config2(size=size, seed=0)
    assert all(k.startswith("tiled") for k in r["kernels"])
    A = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=0), fm.BF16, size * size, 0, 1, threads=THREADS)
    B = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=1), fm.BF16, size * size, 0, 1, threads=THREADS)
    assert_same(host(r["dev"]["A"], np.uint16).reshape(1, -1), A.astype(np.uint16), "config2 A")
    assert_same(host(r["dev"]["B"], np.uint16).reshape(1, -1), B.astype(np.uint16), "config2 B")
    assert not host(r["dev"]["C"], np.uint32).any()
    A, B = A.reshape(size, size), B.reshape(size, size)
    Cz = np.zeros((size, size), dtype=np.uint32)
    p0 = ModelParams(group_len=8, frac_bits=24, c_mode=C_AFTER_EXACT)
    p1 = ModelParams(group_len=0, frac_bits=24)
    w0, _ = o2lib.emulate_mma(p0, A, B, Cz, fm.BF16, fm.BF16)                  # all 2^20 outputs, both models
    w1, _ = o2lib.emulate_mma(p1, A, B, Cz, fm.BF16, fm.BF16)
    g0, g1 = host(r["dev"]["D0"], np.uint32), host(r["dev"]["D1"], np.uint32)
    assert_same(g0, w0[0], "config2 chained")
    assert_same(g1, w1[0], "config2 fused")
    assert r["stats"] == ostats.compare(w0, w1)
    # the rational-arithmetic form of the oracle on a few outputs
    rng = np.random.default_rng(0)
    for idx in rng.choice(size * size, size=24, replace=False):
        i, j = divmod(int(idx), size)
        assert int(g0[i, j]) == emulate_element(p0, A[i].tolist(), B[j].tolist(), 0, fm.BF16, fm.BF16)
        assert int(g1[i, j]) == emulate_element(p1, A[i].tolist(), B[j].tolist(), 0, fm.BF16, fm.BF16)


def test_config3_full(cfg, mm):
    size, stride = 4096, 100
    r = cfg.config3(size=size, seed=0, stride=stride)
    assert r["kernel"].startswith("tiled 64x64")
    A = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=0, scale_scope=ogen.SCALE_TENSOR,
                                     scale_target=448.0), fm.E4M3, size * size, 0, 1, threads=THREADS)
    B = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=1, scale_scope=ogen.SCALE_TENSOR,
                                     scale_target=57344.0), fm.E5M2, size * size, 0, 1, threads=THREADS)
    assert_same(host(r["dev"]["A"], np.uint8).reshape(1, -1), A.astype(np.uint8), "config3 A")
    assert_same(host(r["dev"]["B"], np.uint8).reshape(1, -1), B.astype(np.uint8), "config3 B")
    assert (A & 0x7F).max() == 0x7E and (B & 0x7F).max() == 0x7B               # scaled to 448 / 57344
    A, B = A.reshape(size, size), B.reshape(size, size)
    Cz = np.zeros((size, size), dtype=np.uint32)
    p = ModelParams(group_len=32, frac_bits=14, out_round=RNE)
    G = host(r["dev"]["D"], np.uint32)
    idx = np.arange(0, size * size, stride, dtype=np.uint64)                    # the 1 % sample: 167,773 outputs
    assert idx.size == 167773
    want = o2lib.emulate_sample(p, A, B, Cz, idx, fm.E4M3, fm.E5M2)
    assert_same(G.ravel()[idx.astype(np.int64)], want, "config3 sampled outputs")
    rows = np.array([0, 1, 2047, 4095])                                          # plus whole rows (several tiles + last)
    wr, _ = o2lib.emulate_mma(p, A[rows], B, Cz[rows], fm.E4M3, fm.E5M2)
    assert_same(G[rows], wr[0], "config3 whole rows")
    # error statistics against exact dot products: expected values from the oracle's own outputs
    Dor = np.zeros((size, size), dtype=np.uint32)
    Dor.ravel()[idx.astype(np.int64)] = want
    ws = o2lib.exact_dot_stats(A, B, Dor, fm.E4M3, fm.E5M2, stride)
    gs = r["err_stats"]
    assert gs["n_skipped"] == 0
    for key in ("n_samples", "n_equal_rne", "n_above", "n_below", "ulp_hist"):
        assert gs[key] == ws[key], key
    for key in ("sum_abs_err", "max_abs_err", "sum_rel_err", "max_rel_err", "sum_signed_err"):
        assert gs[key] == pytest.approx(ws[key], rel=1e-9, abs=1e-300), key
    # rational-arithmetic oracle on a few sampled outputs
    for o in idx[:: idx.size // 12][:12]:
        i, j = divmod(int(o), size)
        assert int(G[i, j]) == emulate_element(p, A[i].tolist(), B[j].tolist(), 0, fm.E4M3, fm.E5M2)


def _config4_oracle_inputs(first_tile, nt):
    A = ogen.generate(ogen.GenParams(family=ogen.GEN_UNIFORM_EXP, seed=0, operand=0, exp_lo=0, exp_hi=30), fm.FP16, 256, first_tile, nt)
    B = ogen.generate(ogen.GenParams(family=ogen.GEN_UNIFORM_EXP, seed=0, operand=1, exp_lo=0, exp_hi=30), fm.FP16, 256, first_tile, nt)
    C = ogen.generate(ogen.GenParams(family=ogen.GEN_UNIFORM_EXP, seed=0, operand=2, exp_lo=79, exp_hi=158, exp_zero=True),
                      fm.FP32, 1024, first_tile, nt)
    return A.reshape(nt, 32, 8), B.reshape(nt, 32, 8), C.reshape(nt, 32, 32)


CONFIG4_ORACLE = [ModelParams(group_len=8, frac_bits=24), ModelParams(group_len=8, frac_bits=24, ftz_in=True),
                  ModelParams(group_len=8, frac_bits=24, ftz_out=True)]


def hashed_tiles(n_tiles, chunk, n_chunks, per_chunk, seed):
    """Tile indices scattered over the whole stream: `per_chunk` tiles in each of `n_chunks` chunks picked by a seeded
    generator, the last chunk always among them (with its last tile)."""
    rng = np.random.default_rng(seed)
    total_chunks = n_tiles // chunk
    chunks = set(int(c) for c in rng.choice(total_chunks - 1, size=n_chunks - 1, replace=False)) | {total_chunks - 1}
    tiles = []
    for c in sorted(chunks):
        local = set(int(x) for x in rng.choice(chunk, size=per_chunk, replace=False))
        if c == total_chunks - 1:
            local = set(list(local)[: per_chunk - 1]) | {chunk - 1}
        tiles.extend(c * chunk + x for x in sorted(local))
    return tiles


def test_config4_at_its_stated_size(cfg, mm):
    """All 2^26 tiles, three variants sharing one pass per chunk.  Whole-run invariants; the first chunk's operands and the
    first 2^12 tiles of every variant against the oracle; 2^10 tiles at hashed indices over the whole stream (the last
    chunk included) taken out of the run itself, operands and outputs against the oracle."""
    n_tiles, chunk = 1 << 26, 1 << 14
    samples = hashed_tiles(n_tiles, chunk, 64, 16, seed=4)
    r = cfg.config4(n_tiles=n_tiles, chunk=chunk, seed=0, keep_first_chunk=True, sample_tiles=samples)
    assert r["kernel"].startswith("multi x3 tiled 32x32"), r["kernel"]
    total = n_tiles * 1024                                                     # 2^36 outputs per variant
    for name, st in r["stats"].items():
        assert st["n_compared"] == total and sum(st["ulp_hist"]) == total, name
    none, fin, fout = (r["stats"][k] for k in ("none", "ftz_in", "ftz_out"))
    assert none["n_mismatch_bits"] == 0 and none["ulp_hist"][0] == total and none["first_mismatch_index"] == mm.NO_MISMATCH
    assert fin["n_mismatch_bits"] > total // 16 and fin["ulp_hist"][33] == 0
    assert fout["n_mismatch_bits"] == fout["n_mismatch_nan_equiv"] == 0         # (no result of these inputs is subnormal)
    # first chunk: operands, and the first 2^12 tiles of every variant
    A, B, C = _config4_oracle_inputs(0, chunk)
    assert_same(host(r["dev"]["A"], np.uint16), A.astype(np.uint16), "config4 A")
    assert_same(host(r["dev"]["B"], np.uint16), B.astype(np.uint16), "config4 B")
    assert_same(host(r["dev"]["C"], np.uint32), C, "config4 C")
    nchk = 1 << 12
    outs = []
    for p, Dg in zip(CONFIG4_ORACLE, r["dev"]["D"]):
        w, _ = o2lib.emulate_mma(p, A[:nchk], B[:nchk], C[:nchk], fm.FP16, fm.FP16)
        assert_same(host(Dg, np.uint32)[:nchk], w, "config4 %s" % (p,))
        outs.append(w)
    # the statistics of that prefix, formed inside the fused kernels, against the oracle's comparison of its own outputs;
    # the whole run's first mismatch lies in it
    pre = cfg.config4(n_tiles=nchk, chunk=chunk, seed=0)
    for name, w in zip(("none", "ftz_in", "ftz_out"), outs):
        assert pre["stats"][name] == ostats.compare(w, outs[0]), name
    assert fin["first_mismatch_index"] == pre["stats"]["ftz_in"]["first_mismatch_index"]
    # the sampled tiles of the run itself
    seen = []
    for rec in r["samples"]:
        nt = len(rec["tiles"])
        gA, gB, gC = host(rec["A"], np.uint16), host(rec["B"], np.uint16), host(rec["C"], np.uint32)
        gD = host(rec["D"], np.uint32)
        for q, t in enumerate(rec["tiles"]):
            Ah, Bh, Ch = _config4_oracle_inputs(t, 1)
            assert_same(gA[q:q + 1], Ah.astype(np.uint16), "config4 A of tile %d" % t)
            assert_same(gB[q:q + 1], Bh.astype(np.uint16), "config4 B of tile %d" % t)
            assert_same(gC[q:q + 1], Ch, "config4 C of tile %d" % t)
        for vi, p in enumerate(CONFIG4_ORACLE):
            w, _ = o2lib.emulate_mma(p, gA.astype(np.uint16), gB.astype(np.uint16), gC, fm.FP16, fm.FP16)
            assert_same(gD[vi], w, "config4 variant %d, tiles %s" % (vi, rec["tiles"][:3]))
        seen.extend(rec["tiles"])
    assert sorted(seen) == sorted(samples) and len(seen) == 1024 and max(seen) == n_tiles - 1
    # the rational form of the oracle on a few outputs of the last sampled tile
    last = r["samples"][-1]
    gA, gB, gC, gD = host(last["A"], np.uint16), host(last["B"], np.uint16), host(last["C"], np.uint32), host(last["D"], np.uint32)
    for vi, p in enumerate(CONFIG4_ORACLE):
        for (i, j) in ((0, 0), (5, 17), (31, 31)):
            assert int(gD[vi][-1, i, j]) == emulate_element(p, gA[-1, i].tolist(), gB[-1, j].tolist(), int(gC[-1, i, j]), fm.FP16, fm.FP16)
    # the end of the stream on its own: output indices beyond 2^32 in the statistics
    ntail = 1 << 10
    tail = cfg.config4(n_tiles=ntail, chunk=chunk, seed=0, first_tile=n_tiles - ntail)
    At, Bt, Ct = _config4_oracle_inputs(n_tiles - ntail, ntail)
    wt = [o2lib.emulate_mma(p, At, Bt, Ct, fm.FP16, fm.FP16)[0] for p in CONFIG4_ORACLE]
    base = (n_tiles - ntail) * 1024
    for name, w in zip(("none", "ftz_in", "ftz_out"), wt):
        assert tail["stats"][name] == ostats.compare(w, wt[0], index_base=base), name
    assert tail["stats"]["ftz_in"]["first_mismatch_index"] > (1 << 35)


def test_config4_unfused_path_agrees(cfg, mm):
    """One emulation and one comparison per variant (the other route through the library) gives the same statistics."""
    a = cfg.config4(n_tiles=1 << 16, chunk=1 << 14, fused=True)
    b = cfg.config4(n_tiles=1 << 16, chunk=1 << 14, fused=False)
    assert a["stats"] == b["stats"] and b["kernel"].startswith("tiled 32x32")


def _config5_oracle_inputs(kind, first_tile, nt):
    if kind == "bf16":
        A = ogen.generate(ogen.GenParams(family=ogen.GEN_FINITE_BITS, seed=0, operand=0), fm.BF16, 256, first_tile, nt)
        B = ogen.generate(ogen.GenParams(family=ogen.GEN_FINITE_BITS, seed=0, operand=1), fm.BF16, 256, first_tile, nt)
    else:
        A = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=0, scale_scope=ogen.SCALE_TILE,
                                         scale_target=448.0), fm.E4M3, 256, first_tile, nt, threads=THREADS)
        B = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=1, scale_scope=ogen.SCALE_TILE,
                                         scale_target=57344.0), fm.E5M2, 256, first_tile, nt, threads=THREADS)
    C = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=0, operand=2), fm.FP32, 256, first_tile, nt, threads=THREADS)
    return A.reshape(nt, 16, 16), B.reshape(nt, 16, 16), C.reshape(nt, 16, 16)


def test_config5_at_its_stated_size(cfg, mm):
    """Sixteen parameter sets x 2^24 tiles x two operand types, every tile through the native instruction.  Whole-run
    invariants; first chunk's operands and the first 2^10 tiles of every set against the oracle; 2^10 tiles at hashed
    indices over the whole stream (32 chunks, the last among them) out of the run itself; the statistics the fused
    kernels form, against the oracle's comparison on a prefix."""
    n_tiles, chunk = 1 << 24, 1 << 16
    samples = hashed_tiles(n_tiles, chunk, 32, 32, seed=5)
    r = cfg.config5(n_tiles=n_tiles, chunk=chunk, seed=0, keep_first_chunk=True, sample_tiles=samples)
    nchk = 1 << 10
    total = n_tiles * 256                                                      # 2^32 outputs per set and type
    for kind, (ta, tb) in (("bf16", (fm.BF16, fm.BF16)), ("fp8", (fm.E4M3, fm.E5M2))):
        res = r[kind]
        npdt = np.uint16 if kind == "bf16" else np.uint8
        plist = [ModelParams(group_len=L, frac_bits=F, out_round=rho, ftz_in=bool(ftz), ftz_out=bool(ftz)) for F, L, rho, ftz in cfg.CONFIG5_MODELS]
        assert all(k.startswith("multi x16") for k in res["kernels"]) and len(res["kernels"]) == 1, res["kernels"]     # one launch per chunk
        for st in res["stats"]:
            assert st["n_compared"] == total and sum(st["ulp_hist"]) == total
            assert 0 < st["n_mismatch_bits"] < total                             # (none of the sets is the instruction's arithmetic)
        for a in res["agreement"]:
            assert 0.0 < a < 1.0
        # generated operands of the first chunk
        A, B, C = _config5_oracle_inputs(kind, 0, chunk)
        assert_same(host(res["dev"]["A"], npdt), A.astype(npdt), "config5 %s A" % kind)
        assert_same(host(res["dev"]["B"], npdt), B.astype(npdt), "config5 %s B" % kind)
        assert_same(host(res["dev"]["C"], np.uint32), C, "config5 %s C" % kind)
        Dhw = host(res["dev"]["Dhw"], np.uint32)
        # every parameter set on the first 2^10 tiles
        want = []
        for p, Dg in zip(plist, res["dev"]["D"]):
            w, _ = o2lib.emulate_mma(p, A[:nchk], B[:nchk], C[:nchk], ta, tb)
            assert_same(host(Dg, np.uint32)[:nchk], w, "config5 %s %s" % (kind, p))
            want.append(w)
        # statistics of that prefix from the grouped launches (D never written), against the oracle's comparison of its own
        # outputs with the instruction's output as the run produced it
        pre = cfg.config5(n_tiles=nchk, chunk=chunk, seed=0, kinds=(kind,))[kind]
        for i, w in enumerate(want):
            assert pre["stats"][i] == ostats.compare(w, Dhw[:nchk]), (kind, i)
        # rational-arithmetic oracle on one tile row for two of the sets
        for mi in (0, 15):
            Dg = host(res["dev"]["D"][mi], np.uint32)
            for j in range(16):
                assert int(Dg[3, 5, j]) == emulate_element(plist[mi], A[3, 5].tolist(), B[3, j].tolist(), int(C[3, 5, j]), ta, tb)
        # the sampled tiles of the run itself
        seen = []
        for rec in res["samples"]:
            t_first = rec["tiles"][0]
            gA, gB, gC = host(rec["A"], npdt), host(rec["B"], npdt), host(rec["C"], np.uint32)
            gD = host(rec["D"], np.uint32)
            for q in (0, len(rec["tiles"]) - 1):                                # (operands: first and last sampled tile of the chunk)
                Ah, Bh, Ch = _config5_oracle_inputs(kind, rec["tiles"][q], 1)
                assert_same(gA[q:q + 1], Ah.astype(npdt), "config5 %s A of tile %d" % (kind, rec["tiles"][q]))
                assert_same(gB[q:q + 1], Bh.astype(npdt), "config5 %s B of tile %d" % (kind, rec["tiles"][q]))
                assert_same(gC[q:q + 1], Ch, "config5 %s C of tile %d" % (kind, rec["tiles"][q]))
            for mi, p in enumerate(plist):
                w, _ = o2lib.emulate_mma(p, gA, gB, gC, ta, tb)
                assert_same(gD[mi], w, "config5 %s set %d, tiles from %d" % (kind, mi, t_first))
            seen.extend(rec["tiles"])
        assert sorted(seen) == sorted(samples) and len(seen) == 1024 and max(seen) == n_tiles - 1


def test_config5_unfused_path_agrees(cfg, mm):
    a = cfg.config5(n_tiles=1 << 17, chunk=1 << 16, fused=True)
    b = cfg.config5(n_tiles=1 << 17, chunk=1 << 16, fused=False)
    for kind in ("bf16", "fp8"):
        assert a[kind]["stats"] == b[kind]["stats"], kind
        assert all(k.startswith("tiled 16x16") for k in b[kind]["kernels"])


def test_config1_replayed_from_a_hip_graph_gives_the_same_statistics():
    from paper_2511_10909_amd import configs
    eager = configs.config1(n_tiles=300)
    graph = configs.config1(n_tiles=300, use_graph=True)
    assert graph["stats"] == eager["stats"] and graph["stats"]["n_compared"] == 300 * 256
    import torch
    for name in ("D0", "D1"):
        assert torch.equal(graph["dev"][name], eager["dev"][name])
