"""Pins for the oracle's generators, Philox, and comparison statistics."""
import numpy as np
import pytest
import torch

from oracle import formats as fm, gen, stats
from oracle.philox import philox4x32_10
from helpers import f32_bits


def test_philox_known_answers():
    # known-answer vectors distributed with the reference implementation of
    # Salmon et al., "Parallel random numbers: as easy as 1, 2, 3" (SC'11), Philox-4x32-10
    kat = [((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
           ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
           ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
            (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1))]
    for ctr, key, want in kat:
        assert tuple(int(x) for x in philox4x32_10(*ctr, *key)) == want


def test_philox_vectorised_equals_scalar():
    c0 = np.arange(10, dtype=np.uint64)
    out = philox4x32_10(c0, 7, 1, 0, 123, 456)
    for i in range(10):
        assert tuple(int(x[i]) for x in out) == tuple(int(x) for x in philox4x32_10(i, 7, 1, 0, 123, 456))


def test_word_stream_is_chunk_independent():
    gp = gen.GenParams(family=gen.GEN_FINITE_BITS, seed=5, operand=1)
    whole = gen.generate(gp, fm.FP16, 256, 0, 8)
    parts = np.concatenate([gen.generate(gp, fm.FP16, 256, 0, 3), gen.generate(gp, fm.FP16, 256, 3, 5)])
    assert np.array_equal(whole, parts)
    other = gen.generate(gen.GenParams(family=gen.GEN_FINITE_BITS, seed=5, operand=0), fm.FP16, 256, 0, 8)
    assert not np.array_equal(whole, other)


@pytest.mark.parametrize("fmt,ncodes", [(fm.FP16, 63488), (fm.BF16, 65280), (fm.E5M2, 248), (fm.E4M3, 254)])
def test_finite_bits_family(fmt, ncodes):
    gp = gen.GenParams(family=gen.GEN_FINITE_BITS, seed=0, operand=0)
    out = gen.generate(gp, fmt, 4096, 0, 64).ravel()
    cls = [fm.decode(int(b), fmt).cls for b in np.unique(out)]
    assert fm.NAN not in cls and fm.INF not in cls
    if ncodes <= 256:
        assert len(np.unique(out)) == ncodes       # every finite pattern appears
        counts = np.unique(out, return_counts=True)[1]
        assert counts.min() > 0.8 * out.size / ncodes and counts.max() < 1.2 * out.size / ncodes
    else:
        assert len(np.unique(out)) > 0.9 * ncodes
    f = fm.FORMATS[fmt]
    assert abs(((out >> (f.width - 1)) & 1).mean() - 0.5) < 0.01


def test_uniform_exp_family_fp16():
    gp = gen.GenParams(family=gen.GEN_UNIFORM_EXP, seed=0, operand=0, exp_lo=0, exp_hi=30)
    out = gen.generate(gp, fm.FP16, 256, 0, 2048).ravel()
    E = (out >> 10) & 31
    counts = np.bincount(E, minlength=32)
    assert counts[31] == 0
    assert counts[:31].min() > 0.95 * out.size / 31 and counts[:31].max() < 1.05 * out.size / 31
    assert abs((out >> 15).mean() - 0.5) < 0.01
    assert len(np.unique(out & 0x3FF)) == 1024


def test_uniform_exp_family_fp32_with_zero_choice():
    gp = gen.GenParams(family=gen.GEN_UNIFORM_EXP, seed=3, operand=2, exp_lo=79, exp_hi=158, exp_zero=True)
    out = gen.generate(gp, fm.FP32, 1024, 0, 512).ravel()
    E = (out >> 23) & 255
    vals, counts = np.unique(E, return_counts=True)
    assert set(vals.tolist()) == {0} | set(range(79, 159))
    assert counts.min() > 0.9 * out.size / 81 and counts.max() < 1.1 * out.size / 81
    # mantissa bits come from an independent word
    assert abs(np.corrcoef((out & 0x7FFFFF).astype(np.float64), E.astype(np.float64))[0, 1]) < 0.01


def test_normal_family_moments_and_tails():
    gp = gen.GenParams(family=gen.GEN_NORMAL, seed=0, operand=0)
    z = gen.normal_values(gp, 1 << 20, 0, 1).ravel()
    n = z.size
    assert abs(z.mean()) < 4 / np.sqrt(n)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs((z ** 3).mean()) < 4 * np.sqrt(15 / n)
    assert abs((z ** 4).mean() - 3) < 4 * np.sqrt(96 / n)
    # tail mass beyond 3 sigma: 2.6998e-3
    assert abs((np.abs(z) > 3).mean() - 2.6998e-3) < 4 * np.sqrt(2.7e-3 / n)
    # the two outputs of a pair are uncorrelated
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 4 / np.sqrt(n / 2)


def test_uniform_family():
    gp = gen.GenParams(family=gen.GEN_UNIFORM, seed=3, operand=1)
    u = gen.normal_values(gp, 1 << 20, 0, 1).ravel()
    n = u.size
    assert u.min() >= -1.0 and u.max() < 1.0
    assert abs(u.mean()) < 4 * np.sqrt(1 / 3 / n)
    assert abs(u.var() - 1 / 3) < 4 * np.sqrt(4 / 45 / n)
    # every value is (r + 0.5) 2^-31 - 1 for an integer r below 2^32
    r = (u + 1.0) * 2147483648.0 - 0.5
    assert np.array_equal(r, np.floor(r)) and r.max() < 2 ** 32


def test_normal_outliers_family():
    # Sec. 3.1 Step 4: N(0,1) + Bernoulli(0.001) * N(0,100)
    gp = gen.GenParams(family=gen.GEN_NORMAL_OUTLIERS, seed=5, operand=0)
    x = gen.normal_values(gp, 1 << 21, 0, 1).ravel()
    z = gen.normal_values(gen.GenParams(family=gen.GEN_NORMAL, seed=5, operand=0), 1 << 21, 0, 1).ravel()
    hit = x != z
    n = x.size
    assert abs(hit.mean() - 0.001) < 4 * np.sqrt(0.001 / n)
    extra = (x - z)[hit] / 10.0                      # the second normal, where it was added
    assert abs(extra.std() - 1.0) < 5 / np.sqrt(2 * hit.sum())
    assert abs(np.corrcoef(extra, z[hit])[0, 1]) < 5 / np.sqrt(hit.sum())
    # variance of the mixture: 1 + 0.001 * 100
    assert abs(x.var() - 1.1) < 0.02


def test_cancelling_family_has_large_condition_numbers():
    # Sec. 3.1 Step 4, second input type: sum |p_k| / |sum p_k| >> 1
    K, rows = 16, 4096
    ga = gen.GenParams(family=gen.GEN_CANCELLING, seed=1, operand=0, exp_lo=10, exp_hi=20)
    gb = gen.GenParams(family=gen.GEN_CANCELLING, seed=1, operand=1, exp_lo=10, exp_hi=20)
    A = gen.generate(ga, fm.FP16, K, 0, rows).astype(np.uint16)
    B = gen.generate(gb, fm.FP16, K, 0, rows).astype(np.uint16)
    assert np.array_equal(A[:, 1::2], A[:, 0::2] ^ 0x8000)
    same = B[:, 1::2] == B[:, 0::2]
    assert np.array_equal(B[:, 1::2][~same], B[:, 0::2][~same] ^ 1)
    assert abs((~same).mean() - 1 / 16) < 0.01
    p = A.view(np.float16).astype(np.float64) * B.view(np.float16).astype(np.float64)
    cond = np.abs(p).sum(axis=1) / np.maximum(np.abs(p.sum(axis=1)), 1e-300)
    assert np.median(cond) > 1e3
    with pytest.raises(ValueError):
        gen.generate(ga, fm.FP32, K, 0, 1)


def test_elementary_functions_against_libm():
    r = np.random.default_rng(1).integers(0, 1 << 32, size=20000, dtype=np.uint64).astype(np.uint32)
    want = np.log((r.astype(np.float64) + 0.5) / 2.0 ** 32)
    assert np.abs(gen._ln_unit(r) - want).max() < 1e-12
    # the square root is the correctly rounded one: its square brackets x within one last place, exactly checked in integers
    from fractions import Fraction
    x = np.exp(np.random.default_rng(2).uniform(np.log(1e-10), np.log(50), 2000))
    for xv, yv in zip(x.tolist(), gen._sqrt(x).tolist()):
        y, half_ulp = Fraction(yv), Fraction(np.spacing(yv)) / 2
        assert (y - half_ulp) ** 2 <= Fraction(xv) <= (y + half_ulp) ** 2
    th = np.linspace(0, np.pi / 2, 10001)
    s, c = gen._sincos_quarter(th)
    assert np.abs(s - np.sin(th)).max() < 1e-15 and np.abs(c - np.cos(th)).max() < 1e-15


def test_cast_against_library_casts():
    b = np.random.default_rng(0).integers(0, 1 << 32, 300000, dtype=np.uint64).astype(np.uint32)
    b = b[((b >> 23) & 0xFF) != 255]
    f = b.view(np.float32)
    t32 = torch.from_numpy(f.copy())
    ok = np.abs(f) < 65504
    assert np.array_equal(gen.cast_from_fp32(b[ok], fm.FP16), f[ok].astype(np.float16).view(np.uint16))
    ok = np.abs(f) < 3e38
    assert np.array_equal(gen.cast_from_fp32(b, fm.BF16)[ok], t32.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)[ok])
    for fmt, tdt, mx in ((fm.E4M3, torch.float8_e4m3fn, 448.0), (fm.E5M2, torch.float8_e5m2, 57344.0)):
        ok = np.abs(f) <= mx
        assert ok.sum() > 50000
        assert np.array_equal(gen.cast_from_fp32(b[ok], fmt), t32[torch.from_numpy(ok)].to(tdt).view(torch.uint8).numpy())
    # dense sweep of small magnitudes (subnormal targets) for FP8/FP16
    x = (np.random.default_rng(1).standard_normal(200000) * np.exp(np.random.default_rng(2).uniform(-25, 6, 200000))).astype(np.float32)
    xb = x.view(np.uint32)
    assert np.array_equal(gen.cast_from_fp32(xb, fm.FP16), x.astype(np.float16).view(np.uint16))
    tx = torch.from_numpy(x.copy())
    ok = np.abs(x) <= 448
    assert np.array_equal(gen.cast_from_fp32(xb[ok], fm.E4M3), tx[torch.from_numpy(ok)].to(torch.float8_e4m3fn).view(torch.uint8).numpy())
    # saturation
    assert gen.cast_from_fp32(np.array([f32_bits(1e6)], dtype=np.uint32), fm.E4M3)[0] == 0x7E
    assert gen.cast_from_fp32(np.array([f32_bits(-1e9)], dtype=np.uint32), fm.E5M2)[0] == 0xFB
    assert gen.cast_from_fp32(np.array([f32_bits(1e9)], dtype=np.uint32), fm.FP16)[0] == 0x7BFF


def test_normal_scaled_hits_target_maximum():
    for scope in (gen.SCALE_TENSOR, gen.SCALE_TILE):
        for fmt, target in ((fm.E4M3, 448.0), (fm.E5M2, 57344.0)):
            gp = gen.GenParams(family=gen.GEN_NORMAL, seed=0, operand=0, scale_scope=scope, scale_target=target)
            out = gen.generate(gp, fmt, 256, 0, 16)
            mags = out & 0x7F
            top = gen.max_finite_code(fm.FORMATS[fmt])
            if scope == gen.SCALE_TILE:
                assert (mags.max(axis=1) == top).all()
            else:
                assert mags.max() == top and (mags.max(axis=1) == top).sum() == 1
            assert not any(fm.decode(int(b), fmt).cls in (fm.NAN, fm.INF) for b in np.unique(out))


def test_compare_stats_definition():
    one = f32_bits(1.0)
    d0 = np.array([one, one, one, 0x00000000, 0x7FC00000, 0x7FC00000, one, 0x00000001, 0x7F7FFFFF], dtype=np.uint32)
    d1 = np.array([one, one + 1, one + 5, 0x80000000, 0x7FC00001, one, 0x7FFFFFFF, 0x80000001, 0xFF7FFFFF], dtype=np.uint32)
    st = stats.compare(d0, d1, index_base=100)
    assert st["n_compared"] == 9
    assert st["n_mismatch_bits"] == 8
    assert st["n_mismatch_nan_equiv"] == 1
    assert st["first_mismatch_index"] == 101
    h = st["ulp_hist"]
    assert h[0] == 3            # equal, +0 vs -0, NaN vs NaN
    assert h[1] == 1            # distance 1
    assert h[2] == 1            # 1 vs -1 denormal steps: distance 2
    assert h[3] == 1            # distance 5
    assert h[33] == 2           # NaN against a number, both directions
    assert h[32] == 1 and st["max_ulp_dist"] == 2 * 0x7F7FFFFF
    assert sum(h) == 9
    st2 = stats.compare(d0, d0, stats=st, index_base=200)
    assert st2["n_compared"] == 18 and st2["first_mismatch_index"] == 101 and st2["ulp_hist"][0] == 12
    empty = stats.compare(d0[:0], d0[:0])
    assert empty["first_mismatch_index"] == stats.NO_MISMATCH and empty["n_compared"] == 0


def test_ordered_distance_matches_float_neighbours():
    x = np.array([1.0, -1.0, 1e-40, 0.0], dtype=np.float32)
    up = np.nextafter(x, np.float32(np.inf))
    d = np.abs(stats.ordered_key(x.view(np.uint32)) - stats.ordered_key(up.view(np.uint32)))
    assert (d == 1).all()


def test_scale_code_generation():
    # E8M0 codes: UNIFORM_EXP draws every code of the range about equally often and nothing else; RANDOM_BITS gives
    # all 256 codes; chunks compose
    from oracle import gen as ogen
    gp = ogen.GenParams(family=ogen.GEN_UNIFORM_EXP, seed=5, operand=3, exp_lo=120, exp_hi=134)
    x = ogen.generate(gp, ogen.E8M0, 64, 0, 512).ravel()
    counts = np.bincount(x, minlength=256)
    assert counts[:120].sum() == 0 and counts[135:].sum() == 0
    assert counts[120:135].min() > 0.8 * x.size / 15 and counts[120:135].max() < 1.2 * x.size / 15
    gz = ogen.GenParams(family=ogen.GEN_UNIFORM_EXP, seed=5, operand=3, exp_lo=200, exp_hi=203, exp_zero=True)
    assert set(np.unique(ogen.generate(gz, ogen.E8M0, 64, 0, 64))) == {0, 200, 201, 202, 203}
    gr = ogen.GenParams(family=ogen.GEN_RANDOM_BITS, seed=1, operand=4)
    r = ogen.generate(gr, ogen.E8M0, 256, 0, 256)
    assert len(np.unique(r)) == 256 and r.max() == 255
    assert np.array_equal(ogen.generate(gr, ogen.E8M0, 256, 100, 7), r[100:107])
    assert not ogen.generate(ogen.GenParams(family=ogen.GEN_ZERO), ogen.E8M0, 16, 0, 4).any()
    with pytest.raises(ValueError):
        ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL), ogen.E8M0, 16, 0, 4)


def test_fp6_fp4_generation():
    # FP6 / FP4 codes stay inside their 6 / 4 bits; FINITE_BITS reaches every code; NORMAL saturates at the largest
    # finite value and rounds to nearest (checked against the decoded values)
    from oracle import gen as ogen
    for t, width in ((fm.E2M1, 4), (fm.E2M3, 6), (fm.E3M2, 6)):
        x = ogen.generate(ogen.GenParams(family=ogen.GEN_FINITE_BITS, seed=3, operand=0), t, 64, 0, 64).ravel()
        assert x.max() < (1 << width) and len(np.unique(x)) == (1 << width)
        z = ogen.generate(ogen.GenParams(family=ogen.GEN_NORMAL, seed=3, operand=1), t, 256, 0, 16).ravel()
        assert z.max() < (1 << width)
        vals = np.array([float(fm.decode(int(c), t).value) for c in range(1 << width)])
        zs = ogen.normal_values(ogen.GenParams(family=ogen.GEN_NORMAL, seed=3, operand=1), 256, 0, 16).ravel()
        got = vals[z]
        big = float(vals.max())
        want_mag = np.minimum(np.abs(zs.astype(np.float32).astype(np.float64)), big)
        # nearest representable magnitude (ties aside): the error is at most half the local spacing
        grid = np.sort(np.unique(np.abs(vals)))
        nearest = grid[np.abs(grid[None, :] - want_mag[:, None]).argmin(axis=1)]
        tie = np.isclose(np.abs(np.abs(got) - want_mag), np.abs(nearest - want_mag))
        assert np.all((np.abs(got) == nearest) | tie)
        assert np.all((np.sign(got) == np.sign(zs)) | (got == 0))


def test_compare_stats_fp16_patterns():
    # the same definition on binary16 patterns (outputs of the models with FP16 accumulators): hand-counted
    one = 0x3C00
    d0 = np.array([one, one, one, 0x0000, 0x7E00, 0x7E00, one, 0x0001, 0x7BFF, 0x7C00], dtype=np.uint16)
    d1 = np.array([one, one + 1, one + 5, 0x8000, 0x7E01, one, 0x7FFF, 0x8001, 0xFBFF, 0x7BFF], dtype=np.uint16)
    st = stats.compare(d0, d1, index_base=7, width=16)
    assert st["n_compared"] == 10 and st["n_mismatch_bits"] == 9 and st["n_mismatch_nan_equiv"] == 1
    assert st["first_mismatch_index"] == 8
    h = st["ulp_hist"]
    assert h[0] == 3 and h[1] == 2 and h[2] == 1 and h[3] == 1 and h[33] == 2      # (inf vs largest finite: distance 1)
    assert h[16] == 1 and st["max_ulp_dist"] == 2 * 0x7BFF and sum(h) == 10
    # neighbours in binary16 are at distance 1, across zero too
    x = np.array([1.0, -1.0, 6e-8, 0.0, -6e-8, 65504.0], dtype=np.float16)
    with np.errstate(over="ignore"):                    # (the neighbour of 65504 is infinity)
        up = np.nextafter(x, np.float16(np.inf))
    d = np.abs(stats.ordered_key(x.view(np.uint16), 16) - stats.ordered_key(up.view(np.uint16), 16))
    assert (d == 1).all()
    # a 16-bit pattern is never taken for a binary32 one: 0x7E00 is a NaN at width 16 and a small number at width 32
    assert stats.is_nan(np.array([0x7E00]), 16)[0] and not stats.is_nan(np.array([0x7E00]), 32)[0]


@pytest.mark.parametrize("fmt,one,neg", [(fm.FP32, 0x3F800000, 0x80000000), (fm.FP16, 0x3C00, 0x8000), (fm.BF16, 0x3F80, 0x8000),
                                         (fm.E4M3, 0x38, 0x80), (fm.E5M2, 0x3C, 0x80), (fm.E2M3, 0x08, 0x20), (fm.E3M2, 0x0C, 0x20),
                                         (fm.E2M1, 0x2, 0x8)])
def test_signed_zeros_family(fmt, one, neg):
    # eight equally likely values: +-0 twice, +-1.0, +- the smallest subnormal; 1.0 written out per format
    gp = gen.GenParams(family=gen.GEN_SIGNED_ZEROS, seed=5, operand=1)
    x = gen.generate(gp, fmt, 4096, 3, 4).ravel()
    values, counts = np.unique(x, return_counts=True)
    assert set(values.tolist()) == {0, neg, one, one | neg, 1, 1 | neg}
    freq = dict(zip(values.tolist(), (counts / x.size).tolist()))
    for v, p in ((0, 0.25), (neg, 0.25), (one, 0.125), (one | neg, 0.125), (1, 0.125), (1 | neg, 0.125)):
        assert abs(freq[v] - p) < 0.02, (hex(v), freq[v])
    assert fm.decode(one, fmt).value == 1 and fm.decode(one | neg, fmt).value == -1
    assert fm.decode(1, fmt).cls == fm.SUBNORMAL and fm.decode(neg, fmt).cls == fm.ZERO and fm.decode(neg, fmt).sign == 1
    # chunk independence, like every family
    y = gen.generate(gp, fmt, 4096, 5, 1).ravel()
    assert np.array_equal(y, x[2 * 4096:3 * 4096])
