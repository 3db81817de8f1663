"""The C form of the oracle (oracle/o2) against the rational form (oracle/fdpa.py), against the
paper's printed values and against library arithmetic."""
import numpy as np
import pytest
import torch

from oracle import formats as fm, o2lib, exact as ex
from oracle.fdpa import ModelParams, emulate_mma, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD_EVEN_ODD
from oracle.rounding import RNE, RZ
from helpers import f32_bits, bits_f32, ENCODERS
from paper_2511_10909_amd import synth
from test_oracle_model import _rows, FMT_ID

PAIRS = [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3),
         (fm.E4M3, fm.E4M3), (fm.E5M2, fm.E5M2), (fm.FP16, fm.BF16), (fm.E4M3, fm.FP16)]


def _case(rng, ta, tb, nb, m, n, k, special_frac=0.0, c_exp=None):
    A = synth.random_bits(rng, (nb, m, k), ta)
    B = synth.random_bits(rng, (nb, n, k), tb)
    if c_exp is None:
        C = synth.random_bits(rng, (nb, m, n), fm.FP32)
    else:
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, *c_exp)
    if special_frac:
        A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], special_frac)
        B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], special_frac)
        C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], special_frac)
    return A, B, C


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_o2_equals_rational_oracle_random(ta, tb):
    rng = np.random.default_rng(100 + 8 * ta + tb)
    for trial in range(14):
        L = int(rng.choice([1, 2, 4, 8, 16, 0]))
        k = int(rng.choice([8, 16, 32])) if L == 0 else L * int(rng.integers(1, 4))
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([0, 3, 13, 14, 23, 24, 25, 27, 32, 38, 64])),
                        c_mode=int(rng.integers(0, 2)), out_round=int(rng.integers(0, 2)),
                        ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        nan_bits=0x7FFFFFFF if trial % 3 == 0 else 0x7FC00000)
        if p.c_mode == C_AFTER_EXACT and p.frac_bits > 32:
            p = p.with_(frac_bits=32)
        if p.out_round == RZ and trial % 2:
            p = p.with_(out_mant_bits=13)
        # accumulators near the products' range half of the time, anywhere otherwise
        c_exp = (90, 165) if trial % 2 else None
        A, B, C = _case(rng, ta, tb, 2, 3, 4, k, special_frac=0.02 if trial % 4 == 0 else 0.0, c_exp=c_exp)
        want = emulate_mma(p, A, B, C, ta, tb)
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        assert np.array_equal(got, want), (p, np.argwhere(got != want)[:3])


def test_o2_after_exact_wide_exponent_gaps():
    # bf16 products range over 2^-266 .. 2^255 while c is anywhere in FP32: exercises the far-apart branch
    rng = np.random.default_rng(7)
    for F in (8, 24, 30):
        for rho in (RNE, RZ):
            p = ModelParams(group_len=4, frac_bits=F, c_mode=C_AFTER_EXACT, out_round=rho)
            A, B, C = _case(rng, fm.BF16, fm.BF16, 3, 4, 4, 8)
            assert np.array_equal(o2lib.emulate_mma(p, A, B, C, fm.BF16, fm.BF16)[0], emulate_mma(p, A, B, C, fm.BF16, fm.BF16))
    # exponent gaps swept one by one across the near/far decision, with cancelling signs and ties
    p = ModelParams(group_len=1, frac_bits=24, c_mode=C_AFTER_EXACT)
    for gap in range(-70, 71):
        for csig in (0x000000, 0x000001, 0x7FFFFF, 0x400000):
            for sgn in (0, 1):
                ea = 127 + (gap // 2)
                eb = 127 + gap - (gap // 2)
                A = np.array([[[(ea << 7) | 0x55]]], dtype=np.uint16)
                B = np.array([[[(sgn << 15) | (eb << 7) | 0x2B]]], dtype=np.uint16)
                C = np.array([[[(127 << 23) | csig]]], dtype=np.uint32)
                for rho in (RNE, RZ):
                    q = p.with_(out_round=rho)
                    assert np.array_equal(o2lib.emulate_mma(q, A, B, C, fm.BF16, fm.BF16)[0], emulate_mma(q, A, B, C, fm.BF16, fm.BF16)), (gap, csig, sgn)


@pytest.mark.parametrize("row", _rows("table_d00.txt"), ids=lambda r: r[0])
def test_o2_table_d00(row):
    label, typ, lmax, F, rho, want = row
    enc, t = ENCODERS[typ], FMT_ID[typ]
    K = 32
    a = [enc(-2.0 ** 13), enc(-0.5), enc(-0.25), enc(-0.125)] + [0] * (K - 4)
    b = [enc(2.0 ** 10), enc(1.0), enc(1.0), enc(1.0)] + [0] * (K - 4)
    A, B = np.array([[a]]), np.array([[b]])
    C = np.array([[[f32_bits(2.0 ** 23)]]], dtype=np.uint32)
    p = ModelParams(group_len=int(lmax), frac_bits=64 if F == "exact" else (24 if F == "-" else int(F)), out_round=RZ if rho == "RZ" else RNE)
    if rho in ("TR", "GTR"):
        p = p.with_(frac_bits2=31, c_mode=C_AFTER_RD if rho == "TR" else C_AFTER_RD_EVEN_ODD)
    if rho == "ADDMUL":
        p = ModelParams(group_len=int(lmax), family=1)
    if rho == "FMA":
        p = ModelParams(group_len=1, frac_bits=24, c_mode=C_AFTER_EXACT)
    got, _ = o2lib.emulate_mma(p, A, B, C, t, t)
    assert bits_f32(got[0, 0, 0]) == float(want)


@pytest.mark.parametrize("ta,tb,tda,tdb", [
    (fm.E4M3, fm.E5M2, torch.float8_e4m3fn, torch.float8_e5m2),
    (fm.E4M3, fm.E4M3, torch.float8_e4m3fn, torch.float8_e4m3fn),
    (fm.E5M2, fm.E5M2, torch.float8_e5m2, torch.float8_e5m2)])
def test_o2_fp8_k2_closed_form(ta, tb, tda, tdb):
    # k = 2, all 65536 (a0, b0) pairs x random (a1, b1): a0 b0 + a1 b1 of FP8 values is exact in binary64.
    # F = 64 truncates nothing: e_max <= 30 (largest product exponent; c = +0 has Exp -126 and never
    # raises it) and no product has a bit below 2^-32, a span of at most 62.
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    va, vb = codes.view(tda).to(torch.float64).numpy(), codes.view(tdb).to(torch.float64).numpy()
    fa = np.isfinite(va); fb = np.isfinite(vb)
    rng = np.random.default_rng(21)
    x0, y0 = np.meshgrid(np.arange(256), np.arange(256), indexing="ij")
    x0, y0 = x0.ravel(), y0.ravel()
    p = ModelParams(group_len=2, frac_bits=64)
    for rep in range(16):
        x1 = rng.integers(0, 256, size=x0.size)
        y1 = rng.integers(0, 256, size=x0.size)
        ok = fa[x0] & fb[y0] & fa[x1] & fb[y1]
        A = np.stack([x0[ok], x1[ok]], axis=1).astype(np.uint8)[:, None, :]      # batch of 1x1x2 tiles
        B = np.stack([y0[ok], y1[ok]], axis=1).astype(np.uint8)[:, None, :]
        C = np.zeros((A.shape[0], 1, 1), dtype=np.uint32)
        exact = va[A[:, 0, 0]] * vb[B[:, 0, 0]] + va[A[:, 0, 1]] * vb[B[:, 0, 1]]
        want = np.where(exact == 0, 0, exact.astype(np.float32).view(np.uint32))
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        assert np.array_equal(got.ravel(), want)


def test_o2_wide_F_vs_double_arithmetic_fp16():
    # exponent fields restricted so that the exact sum fits binary64; numpy's float64 dot of exact products,
    # summed in any order, is then exact, and astype(float32) is one correct rounding
    rng = np.random.default_rng(22)
    nb, m, n, k = 64, 4, 4, 16
    A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.FP16, 11, 19)
    B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.FP16, 11, 19)
    C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 122, 132)
    av = A.view(np.float16).astype(np.float64)
    bv = B.view(np.float16).astype(np.float64)
    exact = np.einsum("bik,bjk->bij", av, bv) + C.view(np.float32).astype(np.float64)
    want = exact.astype(np.float32).view(np.uint32)
    want = np.where(exact == 0, 0, want)
    got, _ = o2lib.emulate_mma(ModelParams(frac_bits=64), A, B, C, fm.FP16, fm.FP16)
    assert np.array_equal(got, want)


def test_o2_sample_matches_full_and_threads():
    rng = np.random.default_rng(23)
    A, B, C = _case(rng, fm.FP16, fm.FP16, 5, 8, 8, 16, c_exp=(100, 150))
    p = ModelParams(group_len=8, frac_bits=24)
    full, used = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16, nthreads=3)
    assert used == 3
    one, used1 = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16, nthreads=1)
    assert used1 == 1 and np.array_equal(full, one)
    idx = rng.choice(full.size, size=50, replace=False)
    assert np.array_equal(o2lib.emulate_sample(p, A, B, C, idx, fm.FP16, fm.FP16), full.ravel()[idx])


def test_o2_rejects_bad_arguments():
    rng = np.random.default_rng(24)
    A, B, C = _case(rng, fm.FP16, fm.FP16, 1, 2, 2, 12)
    with pytest.raises(ValueError):
        o2lib.emulate_mma(ModelParams(group_len=8), A, B, C, fm.FP16, fm.FP16)
    with pytest.raises(ValueError):
        o2lib.emulate_mma(ModelParams(group_len=4, frac_bits=65), A, B, C, fm.FP16, fm.FP16)


def test_o2_exact_dot_stats_against_rational():
    rng = np.random.default_rng(25)
    m, n, k = 12, 10, 64
    A = synth.random_bits(rng, (m, k), fm.E4M3)
    B = synth.random_bits(rng, (n, k), fm.E5M2)
    p = ModelParams(group_len=32, frac_bits=14)
    D, _ = o2lib.emulate_mma(p, A, B, np.zeros((m, n), dtype=np.uint32), fm.E4M3, fm.E5M2)
    D = D[0]
    want = ex.error_stats(A, B, D, fm.E4M3, fm.E5M2, stride=7)
    got = o2lib.exact_dot_stats(A, B, D, fm.E4M3, fm.E5M2, 7)
    for key in ("n_samples", "n_equal_rne", "n_above", "n_below", "ulp_hist"):
        assert got[key] == want[key], key
    for key in ("sum_abs_err", "max_abs_err", "sum_rel_err", "max_rel_err", "sum_signed_err"):
        assert got[key] == pytest.approx(want[key], rel=1e-12, abs=1e-300), key
    assert want["n_samples"] == len(range(0, m * n, 7)) and want["n_equal_rne"] < want["n_samples"]


def test_o2_longest_groups():
    # one group over k = 2^20 (the longest dot product the entry points take), on several threads: against the rational
    # form on one output, and against a closed form (2^20 equal products: the exact sum is a power of two times k)
    from oracle.fdpa import emulate_element
    rng = np.random.default_rng(2020)
    k = 1 << 20
    A = synth.narrow_exponent_bits(rng, (1, 3, k), fm.FP16, 12, 18)
    B = synth.narrow_exponent_bits(rng, (1, 2, k), fm.FP16, 12, 18)
    C = synth.narrow_exponent_bits(rng, (1, 3, 2), fm.FP32, 120, 140)
    full, _ = o2lib.emulate_mma(ModelParams(group_len=0, frac_bits=24), A, B, C, fm.FP16, fm.FP16)
    q = k // 8                                                  # (the rational form on an eighth: it takes seconds per 10^5 terms)
    p = ModelParams(group_len=q, frac_bits=24, c_mode=C_AFTER_EXACT)
    got, _ = o2lib.emulate_mma(p, A[:, :, :q], B[:, :, :q], C, fm.FP16, fm.FP16)
    assert int(got[0, 2, 1]) == emulate_element(p, A[0, 2, :q].tolist(), B[0, 1, :q].tolist(), int(C[0, 2, 1]), fm.FP16, fm.FP16)
    # the whole length in one group with nothing cut (F wide, three-bit values on two exponents): binary64's dot product,
    # exact here, rounded once
    wide = ModelParams(group_len=0, frac_bits=40)
    Cz = np.zeros((1, 3, 2), dtype=np.uint32)
    Ah, Bh = synth.narrow_exponent_bits(rng, (1, 3, k), fm.FP16, 15, 16) & 0xFF00, synth.narrow_exponent_bits(rng, (1, 2, k), fm.FP16, 15, 16) & 0xFF00
    d1, _ = o2lib.emulate_mma(wide, Ah, Bh, Cz, fm.FP16, fm.FP16)
    exact = (Ah.view(np.float16).astype(np.float64)[0] @ Bh.view(np.float16).astype(np.float64)[0].T).astype(np.float32).view(np.uint32)
    assert np.array_equal(d1[0], exact) and full.shape == (1, 3, 2)
    ones = np.full((1, 1, k), ENCODERS["fp16"](1.5), dtype=np.uint16)
    got, _ = o2lib.emulate_mma(ModelParams(group_len=0, frac_bits=24), ones, ones, np.zeros((1, 1, 1), dtype=np.uint32), fm.FP16, fm.FP16)
    assert bits_f32(int(got[0, 0, 0])) == 2.25 * k
