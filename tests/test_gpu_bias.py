"""Sec. 6.2.4 on the GPU: the truncating variant of TR-FDPA (rd_toward_zero) in the general and in the tiled kernels
against the rational oracle, mmaemu_deviation_sample against oracle/exact.py (integers bit-exact, the three binary64
sums to 1e-9), the constant-factor generator against its CPU twin, and the experiment itself as a device workload."""
import dataclasses

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib, gen as ogen
from oracle.exact import deviation_hist
from oracle.fdpa import ModelParams, C_AFTER_RD, C_AFTER_RD_EVEN_ODD, SPLIT_HALVES, SPLIT_QUARTERS, SPLIT_EVEN_ODD
from paper_2511_10909_amd import synth
from gpu_utils import to_dev, to_host
from o1_jobs import run_pool
from test_gpu_parity import mm, gpu_emulate  # noqa: F401

TRZ = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD, rd_toward_zero=True)


def close(a, b):
    return abs(a - b) <= 1e-9 * max(abs(a), abs(b), 1e-300)


def same_hist(got, want, what):
    for key in ("n_samples", "n_skipped", "n_negative", "n_zero", "n_positive", "bins"):
        assert got[key] == want[key], (what, key, got[key], want[key])
    for key in ("sum", "sum_abs", "sum_sq"):
        assert close(got[key], want[key]), (what, key, got[key], want[key])


def test_truncating_variant_matches_the_rational_oracle(mm):
    rng = np.random.default_rng(777)
    cases = [("unsplit fp16, ragged (general)", TRZ, fm.FP16, (5, 12, 20, 16), "general"),
             ("unsplit bf16, ragged (general)", TRZ.with_(frac_bits=20, frac_bits2=27, out_round=1), fm.BF16, (5, 12, 20, 16), "general"),
             ("even/odd fp8 (general)", TRZ.with_(c_mode=C_AFTER_RD_EVEN_ODD, group_len=16), fm.E5M2, (5, 12, 20, 32), "general"),
             ("halves, F_m = 20 (general)", TRZ.with_(split=SPLIT_HALVES, frac_bits_merge=20, group_len=8), fm.FP16, (4, 16, 16, 16), "general"),
             ("quarters (general)", TRZ.with_(split=SPLIT_QUARTERS, frac_bits=13, group_len=16), fm.E4M3, (4, 16, 16, 32), "general"),
             ("leading-bit F2 rule, zero terms skipped (general)", TRZ.with_(f2_at_leading_bit=True, skip_zero_terms=True, zero_result_positive=True), fm.BF16, (4, 16, 16, 16), "general"),
             ("special truncation, drop distance (tiled)", TRZ.with_(acc_special_truncation=True, sum_drop_distance=28), fm.FP16, (2, 32, 32, 16), "tiled"),
             ("unsplit fp16 32x32x8 (tiled)", TRZ, fm.FP16, (2, 32, 32, 8), "tiled"),
             ("unsplit bf16 16x16x16 (tiled)", TRZ, fm.BF16, (6, 16, 16, 16), "tiled"),
             ("unsplit fp8 16x16x32 (tiled)", TRZ.with_(group_len=16, frac_bits=13, frac_bits2=24), fm.E4M3, (6, 16, 16, 32), "tiled")]
    gpu, jobs = [], []
    for idx, (name, p, t, (nb, m, n, k), route) in enumerate(cases):
        A = synth.narrow_exponent_bits(rng, (nb, m, k), t, *((8, 22) if t != fm.BF16 and t != fm.E4M3 else ((120, 134) if t == fm.BF16 else (3, 12))))
        B = synth.narrow_exponent_bits(rng, (nb, n, k), t, *((8, 22) if t != fm.BF16 and t != fm.E4M3 else ((120, 134) if t == fm.BF16 else (3, 12))))
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 110, 140)
        if idx % 2:
            A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[t], 0.01)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.01)
        got = gpu_emulate(mm, p, A, B, C, t, t)
        assert gpu_emulate.last_kernel.startswith(route), (name, gpu_emulate.last_kernel)
        gpu.append(got)
        jobs.append((dataclasses.asdict(p), A, B, C, t, t, None, None, 0))
        # the switch matters on these inputs: the printed algorithm differs somewhere
        rd = gpu_emulate(mm, p.with_(rd_toward_zero=False), A, B, C, t, t)
        assert (rd != got).any(), name
    want = run_pool(jobs, workers=12)
    for (name, *_), g, w in zip(cases, gpu, want):
        assert g.size >= 1000
        bad = np.argwhere(g != w)
        assert len(bad) == 0, "%s: %d of %d differ, first at %s: gpu %08x oracle %08x" % (name, len(bad), g.size, tuple(bad[0]), g[tuple(bad[0])], w[tuple(bad[0])])


def test_truncating_variant_block_scaled(mm):
    from test_gpu_scaled import gpu_emulate_scaled
    from oracle.fdpa import emulate_mma as o1
    rng = np.random.default_rng(778)
    p = TRZ.with_(group_len=16, frac_bits=13, frac_bits2=31, split=SPLIT_HALVES, frac_bits_merge=24, wide_products=True)
    nb, m, n, k, block = 2, 12, 11, 32, 32
    A, B = synth.random_bits(rng, (nb, m, k), fm.E4M3), synth.random_bits(rng, (nb, n, k), fm.E5M2)
    C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 100, 150)
    SA = rng.integers(110, 140, size=(nb, m, k // block)).astype(np.uint8)
    SB = rng.integers(110, 140, size=(nb, n, k // block)).astype(np.uint8)
    got = gpu_emulate_scaled(mm, p, A, B, C, SA, SB, block, fm.E4M3, fm.E5M2)
    want = o1(p, A, B, C, fm.E4M3, fm.E5M2, SA=SA, SB=SB, block=block)
    assert np.array_equal(got, want)


def test_constant_factor_generator_matches_cpu_twin(mm):
    import torch
    for dtype, np_t, ept, nt in ((fm.FP16, np.uint16, 256, 37), (fm.BF16, np.uint16, 100, 9), (fm.FP32, np.uint32, 1024, 5)):
        out = torch.empty(nt * ept, dtype={np.uint16: torch.int16, np.uint32: torch.int32}[np_t], device="cuda")
        mm.generate(out, dtype, ept, 3, nt, mm.GEN_NORMAL, seed=9, operand=1, scale_scope=mm.SCALE_FACTOR, scale_target=1000.0)
        want = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=9, operand=1, scale_scope=ogen.SCALE_FACTOR, scale_target=1000.0),
                             dtype, ept, 3, nt).ravel()
        assert np.array_equal(to_host(out, np_t).astype(np.uint32), want.astype(np.uint32))


def dev_hist(mm, A, B, C, D, ta, tb, stride, bin_exp, calls=1):
    import torch
    h = torch.empty(mm.DEVIATION_HIST_BYTES, dtype=torch.uint8, device="cuda")
    mm.deviation_hist_reset(h)
    nb, m, k = A.shape
    n = B.shape[1]
    dA, dB, dD = to_dev(A), to_dev(B), to_dev(D)
    dC = to_dev(C) if C is not None else None
    for _ in range(calls):
        mm.deviation_sample(dA, dB, dC, dD, m, n, k, nb, (ta, tb, fm.FP32, fm.FP32), stride, bin_exp, h)
    return mm.read_deviation_hist(h)


def test_deviation_sample_matches_oracle(mm):
    rng = np.random.default_rng(4)
    for idx, (ta, tb, shape, stride, bin_exp, with_c) in enumerate((
            (fm.FP16, fm.FP16, (5, 32, 32, 8), 1, -5, True), (fm.BF16, fm.BF16, (7, 16, 16, 16), 7, -12, False),
            (fm.E4M3, fm.E5M2, (3, 16, 16, 32), 3, -9, True), (fm.FP16, fm.BF16, (2, 9, 13, 5), 1, 2, True),
            (fm.E2M3, fm.E2M1, (4, 16, 16, 64), 5, -6, True), (fm.BF16, fm.BF16, (3, 16, 16, 8), 1, 0, True))):
        nb, m, n, k = shape
        lo_hi = {fm.FP16: (10, 24), fm.BF16: (118, 132), fm.E4M3: (3, 12), fm.E5M2: (10, 20), fm.E2M3: (0, 3), fm.E2M1: (0, 3)}
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *lo_hi[ta])
        B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *lo_hi[tb])
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 118, 132) if with_c else None
        if idx == 5:         # whole exponent range: many sums leave the pair of binary64 numbers for the wide accumulator
            A = synth.random_bits(rng, (nb, m, k), ta)
            B = synth.random_bits(rng, (nb, n, k), tb)
            C = synth.random_bits(rng, (nb, m, n), fm.FP32)
        if idx == 0:
            A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.003)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.01)
        p = ModelParams(group_len=k, frac_bits=[24, 10, 13, 6, 30, 24][idx], frac_bits2=31, c_mode=C_AFTER_RD)
        D = o2lib.emulate_mma(p, A, B, C if with_c else np.zeros((nb, m, n), np.uint32), ta, tb)[0]
        if idx == 1:
            D[0, 0, :4] = [0x7F800000, 0x7FC00000, 0x00000001, 0x80000001]        # skipped; tiny outputs, far off
        got = dev_hist(mm, A, B, C, D, ta, tb, stride, bin_exp, calls=2 if idx == 2 else 1)
        want = deviation_hist(A, B, C, D, ta, tb, stride, bin_exp)
        if idx == 2:
            want = deviation_hist(A, B, C, D, ta, tb, stride, bin_exp, hist=want)
        same_hist(got, want, (ta, tb, shape))
        assert got["n_samples"] + got["n_skipped"] == (2 if idx == 2 else 1) * ((nb * m * n + stride - 1) // stride)
        if idx == 0:
            assert got["n_skipped"] > 0 and len([b for b in got["bins"] if b]) > 8


def test_deviation_sample_extremes_and_errors(mm):
    import torch
    # the widest reach of the exact sum: BF16 products at both ends of the range next to binary32's smallest subnormal
    big, tiny = 0x7F7F, 0x0001
    A = np.array([[[big, tiny, big, tiny]]], dtype=np.uint16)
    B = np.array([[[big, tiny, 0xFF7F, 0x8001]]], dtype=np.uint16)         # everything cancels
    C = np.array([[[0x00000001]]], dtype=np.uint32)
    D = np.array([[[0x00000001]]], dtype=np.uint32)
    h = dev_hist(mm, A, B, C, D, fm.BF16, fm.BF16, 1, -149)
    assert h["n_zero"] == 1 and h["bins"][32] == 1
    same_hist(h, deviation_hist(A, B, C, D, fm.BF16, fm.BF16, 1, -149), "cancelling extremes")
    D[0, 0, 0] = 0x7F7FFFFF
    h = dev_hist(mm, A[:, :, :2], B[:, :, :2], C, D, fm.BF16, fm.BF16, 1, 250)
    same_hist(h, deviation_hist(A[:, :, :2], B[:, :, :2], C, D, fm.BF16, fm.BF16, 1, 250), "largest product")
    z = torch.zeros(64, dtype=torch.int32, device="cuda")
    hist = torch.empty(mm.DEVIATION_HIST_BYTES, dtype=torch.uint8, device="cuda")
    for kw, status in ((dict(stride=0), 3), (dict(bin_exp=-281), 1), (dict(dtypes=(mm.FP32, mm.FP32, mm.FP32, mm.FP32)), 2), (dict(k=0), 3)):
        args = dict(m=2, n=2, k=4, batch=1, dtypes=(mm.FP16, mm.FP16, mm.FP32, mm.FP32), stride=1, bin_exp=0)
        args.update(kw)
        with pytest.raises(mm.MmaemuError) as ei:
            mm.deviation_sample(z, z, z, z, args["m"], args["n"], args["k"], args["batch"], args["dtypes"], args["stride"], args["bin_exp"], hist)
        assert ei.value.status == status, kw


def test_bias_experiment_workload(mm):
    from paper_2511_10909_amd import configs
    nt, chunk = 1 << 16, 1 << 14
    r = configs.bias_experiment(n_tiles=nt, chunk=chunk, seed=2, stride=1, keep_first_chunk=True)
    assert r["kernels"]["rd"].startswith("tiled") and r["kernels"]["rz"].startswith("tiled")
    H = r["hists"]
    n = nt * 1024
    for name in ("rd", "rz", "mfma"):
        h = H[name]
        assert h["n_samples"] == n and h["n_skipped"] == 0 and sum(h["bins"]) == n
        assert h["n_negative"] + h["n_zero"] + h["n_positive"] == n
    mean = {k: h["sum"] / n for k, h in H.items()}
    sd_of_mean = {k: (h["sum_sq"] / n - mean[k] ** 2) ** 0.5 / n ** 0.5 for k, h in H.items()}
    assert mean["rd"] < -50 * sd_of_mean["rd"]                    # Sec. 6.2.4: shifted toward the negative side
    assert abs(mean["rz"]) < 5 * sd_of_mean["rz"]                 # the truncating variant is centred
    assert H["rd"]["n_negative"] > 1.2 * H["rd"]["n_positive"] and 0.98 < H["rz"]["n_negative"] / H["rz"]["n_positive"] < 1.02
    assert mean["mfma"] < -50 * sd_of_mean["mfma"]                # this GPU's FP16 instruction rounds down as well
    # a prefix against the oracle: generated inputs, both variants' outputs, and the histogram of that prefix
    f = r["first"]
    t = 3
    A = to_host(f["A"], np.uint16)[:t]; B = to_host(f["B"], np.uint16)[:t]; C = to_host(f["C"], np.uint32)[:t]
    gp = lambda op, **kw: ogen.GenParams(family=ogen.GEN_NORMAL, seed=2, operand=op, **kw)
    assert np.array_equal(A.ravel(), ogen.generate(gp(0, scale_scope=ogen.SCALE_FACTOR, scale_target=1000.0), fm.FP16, 256, 0, t).ravel())
    assert np.array_equal(C.ravel(), ogen.generate(gp(2), fm.FP32, 1024, 0, t).ravel())
    base = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)
    jobs = [(dataclasses.asdict(base.with_(rd_toward_zero=z)), A, B, C, fm.FP16, fm.FP16, None, None, 0) for z in (False, True)]
    for name, want in zip(("rd", "rz"), run_pool(jobs, workers=2)):
        got = to_host(f[name], np.uint32)[:t]
        assert np.array_equal(got, want), name
        same_hist(dev_hist(mm, A, B, C, got, fm.FP16, fm.FP16, 1, configs.BIAS_BIN_EXP), deviation_hist(A, B, C, want, fm.FP16, fm.FP16, 1, configs.BIAS_BIN_EXP), name)
