"""mmaemu_emulate_compare_many (several models per pass, compared with a reference inside the kernel) against the CPU
oracle: every model's outputs (written on request) bit for bit, and every model's statistics equal to the oracle's
comparison of the oracle's outputs with the same reference."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib, stats as ostats
from oracle.fdpa import ModelParams, emulate_mma as o1_emulate, C_AFTER_RD
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from gpu_utils import to_dev, dev_empty, to_host
from test_gpu_parity import assert_same, mm, make_case, NP  # noqa: F401

# the sixteen parameter sets of the closed-loop scan: (F, L_max, output rounding, both flushes)
SETS16 = [(16, 4, RNE, 0), (16, 8, RZ, 1), (16, 16, RNE, 1), (16, 64, RZ, 0), (20, 4, RZ, 1), (20, 8, RNE, 0), (20, 16, RZ, 0),
          (20, 32, RNE, 1), (24, 4, RNE, 1), (24, 8, RZ, 0), (24, 16, RNE, 0), (24, 32, RZ, 1), (28, 8, RNE, 1), (32, 4, RZ, 0),
          (32, 16, RZ, 1), (32, 64, RNE, 0)]


def _handles(mm, plist):
    return [mm.model_create(group_len=p.group_len, frac_bits=p.frac_bits, frac_bits2=p.frac_bits2, c_mode=p.c_mode, out_round=p.out_round,
                            ftz_in=p.ftz_in, ftz_out=p.ftz_out, nan_bits=p.nan_bits, out_mant_bits=p.out_mant_bits, split=p.split,
                            acc_special_truncation=p.acc_special_truncation, frac_bits_merge=p.frac_bits_merge,
                            frac_bits_acc=p.frac_bits_acc, f2_at_leading_bit=p.f2_at_leading_bit,
                            skip_zero_terms=p.skip_zero_terms, zero_result_positive=p.zero_result_positive,
                            sum_drop_distance=p.sum_drop_distance, wide_products=p.wide_products, rd_toward_zero=p.rd_toward_zero)
            for p in plist]


def run_many(mm, plist, A, B, C, ta, tb, ref=None, dump=True, index_base=0, stats=None):
    """Returns (list of statistics dicts, dumped outputs [n_models][nb][m][n] or None, kernel name)."""
    import torch
    nb, m, k = A.shape
    n = B.shape[1]
    hs = _handles(mm, plist)
    try:
        dA, dB, dC = to_dev(A.astype(NP[ta])), to_dev(B.astype(NP[tb])), to_dev(C.astype(np.uint32))
        dR = None if ref is None else to_dev(ref.astype(np.uint32))
        dD = dev_empty((len(plist), nb, m, n), np.uint32) if dump else None
        if dump:
            dD.fill_(0x5A5A5A5A)
        if stats is None:
            stats = torch.empty(len(plist) * mm.STATS_BYTES, dtype=torch.uint8, device="cuda")
            for i in range(len(plist)):
                mm.stats_reset(stats[i * mm.STATS_BYTES:])
        mm.emulate_compare_many(hs, dA, dB, dC, dR, dD, m, n, k, nb, (ta, tb, fm.FP32, fm.FP32), stats, index_base=index_base)
        kern = mm.last_kernel()
        out = to_host(dD, np.uint32) if dump else None
        return mm.read_stats_array(stats, len(plist)), out, kern, stats
    finally:
        for h in hs:
            mm.model_destroy(h)


def oracle_outputs(plist, A, B, C, ta, tb):
    return [o2lib.emulate_mma(p, A, B, C, ta, tb)[0] for p in plist]


def sets16():
    return [ModelParams(group_len=L, frac_bits=F, out_round=rho, ftz_in=bool(z), ftz_out=bool(z)) for F, L, rho, z in SETS16]


@pytest.mark.parametrize("ta,tb", [(fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.FP16, fm.FP16)])
def test_sixteen_sets_against_a_reference_array(mm, ta, tb):
    rng = np.random.default_rng(100 + ta)
    nb = 301                                                    # not a multiple of the tiles per workgroup (16 and 4)
    A, B, C = make_case(rng, ta, tb, nb, 16, 16, 16, c_exp=(100, 140))
    if ta == fm.BF16:                                           # half the tiles inside binary32's comfortable range, half anywhere
        A[: nb // 2] = synth.narrow_exponent_bits(rng, (nb // 2, 16, 16), ta, 110, 140)
        B[: nb // 2] = synth.narrow_exponent_bits(rng, (nb // 2, 16, 16), tb, 110, 140)
    plist = sets16()
    want = oracle_outputs(plist, A, B, C, ta, tb)
    # a reference that agrees with set 10 mostly: some entries moved by a few places, some NaNs of two patterns, a -0
    ref = want[10].copy()
    flat = ref.reshape(-1)
    idx = rng.choice(flat.size, size=flat.size // 50, replace=False)
    flat[idx] += rng.integers(1, 200, size=idx.size).astype(np.uint32)
    flat[rng.choice(flat.size, size=40, replace=False)] = 0x7FC00000
    flat[rng.choice(flat.size, size=40, replace=False)] = 0xFFC00001
    flat[rng.choice(flat.size, size=10, replace=False)] = 0x80000000
    got_stats, got_D, kern, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, index_base=5_000_000_000)
    assert kern.startswith("multi"), kern
    for i, p in enumerate(plist):
        assert_same(got_D[i], want[i], "set %d %s" % (i, p))
        assert got_stats[i] == ostats.compare(want[i], ref, index_base=5_000_000_000), (i, p)


@pytest.mark.parametrize("ta,tb,m,k", [(fm.BF16, fm.BF16, 16, 32), (fm.E4M3, fm.E5M2, 16, 32), (fm.FP16, fm.FP16, 16, 32),
                                       (fm.FP16, fm.FP16, 32, 16), (fm.BF16, fm.BF16, 32, 16), (fm.E5M2, fm.E4M3, 32, 16)])
def test_sixteen_sets_on_the_longer_tile_shapes(mm, ta, tb, m, k):
    # 16x16x32 and 32x32x16 (the shapes of the newer MFMA instructions): the whole k of a tile staged at once, groups of up to 32
    rng = np.random.default_rng(300 + 8 * ta + k)
    nb = 53
    A, B, C = make_case(rng, ta, tb, nb, m, m, k, c_exp=(100, 140))
    if ta == fm.BF16:
        A[: nb // 2] = synth.narrow_exponent_bits(rng, (nb // 2, m, k), ta, 110, 140)
        B[: nb // 2] = synth.narrow_exponent_bits(rng, (nb // 2, m, k), tb, 110, 140)
    A[-6:] = synth.sprinkle(rng, A[-6:], synth.SPECIAL_CODES[ta], 0.02)        # NaN and infinities in the last tiles
    plist = sets16()
    want = oracle_outputs(plist, A, B, C, ta, tb)
    ref = want[6].copy()
    flat = ref.reshape(-1)
    idx = rng.choice(flat.size, size=flat.size // 40, replace=False)
    flat[idx] += rng.integers(1, 1000, size=idx.size).astype(np.uint32)
    got_stats, got_D, kern, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, index_base=77)
    assert kern.startswith("multi x16 tiled %dx%d r2x2 kc=%d" % (m, m, k)), kern
    for i, p in enumerate(plist):
        assert_same(got_D[i], want[i], "set %d %s" % (i, p))
        assert got_stats[i] == ostats.compare(want[i], ref, index_base=77), (i, p)
    # the rational form of the oracle on the first tile
    for i in (1, 7, 12, 15):
        assert_same(got_D[i][:1], o1_emulate(plist[i], A[:1], B[:1], C[:1], ta, tb), "rational oracle, set %d" % i)


def test_sets_without_dump_give_the_same_statistics_and_accumulate(mm):
    rng = np.random.default_rng(7)
    ta, tb = fm.E4M3, fm.E5M2
    A, B, C = make_case(rng, ta, tb, 128, 16, 16, 16, c_exp=(110, 135))
    plist = sets16()
    want = oracle_outputs(plist, A, B, C, ta, tb)
    ref = want[3]
    st1, _, kern, dev = run_many(mm, plist, A, B, C, ta, tb, ref=ref, dump=False)
    assert kern.startswith("multi")
    expect = [ostats.compare(w, ref) for w in want]
    assert st1 == expect
    # second call on the same device structs: counters add up, the first index stays
    st2, _, _, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, dump=False, index_base=1 << 33, stats=dev)
    for i, w in enumerate(want):
        assert st2[i] == ostats.compare(w, ref, stats=ostats.compare(w, ref), index_base=1 << 33), i


@pytest.mark.parametrize("lead_flushes", [False, True])
def test_first_model_as_reference_flush_variants(mm, lead_flushes):
    """Subnormal stress shape: fp16 32x32x8 tiles, exponent fields over the whole range; no reference array, the
    first model's outputs are the reference and never leave the kernel."""
    rng = np.random.default_rng(11)
    nb = 77
    A = synth.narrow_exponent_bits(rng, (nb, 32, 8), fm.FP16, 0, 30)
    B = synth.narrow_exponent_bits(rng, (nb, 32, 8), fm.FP16, 0, 30)
    C = synth.narrow_exponent_bits(rng, (nb, 32, 32), fm.FP32, 79, 158)
    C[rng.random(C.shape) < 0.1] &= 0x807FFFFF                  # zeros and subnormals
    plist = [ModelParams(group_len=8, frac_bits=24), ModelParams(group_len=8, frac_bits=24, ftz_in=True),
             ModelParams(group_len=8, frac_bits=24, ftz_out=True)]
    if lead_flushes:
        plist = [plist[1], plist[0], plist[2]]
    want = oracle_outputs(plist, A, B, C, fm.FP16, fm.FP16)
    if not lead_flushes:
        st, _, kern, _ = run_many(mm, plist, A, B, C, fm.FP16, fm.FP16, ref=None, dump=False)
        assert kern.startswith("multi x3"), kern
        assert st == [ostats.compare(w, want[0]) for w in want]
        assert st[0]["n_mismatch_bits"] == 0 and st[1]["n_mismatch_bits"] > 0
    else:
        # the flushing set leads: the others cannot share its launch, so the call needs D_out
        with pytest.raises(mm.MmaemuError) as ei:
            run_many(mm, plist, A, B, C, fm.FP16, fm.FP16, ref=None, dump=False)
        assert ei.value.status == 2 and "D_out" in mm.last_error()
    st, D, kern, _ = run_many(mm, plist, A, B, C, fm.FP16, fm.FP16, ref=None, dump=True)
    for i in range(3):
        assert_same(D[i], want[i], "variant %d" % i)
    assert st == [ostats.compare(w, want[0]) for w in want]


def test_special_values_and_wide_bf16_inside_the_fused_kernels(mm):
    rng = np.random.default_rng(21)
    for ta, tb in ((fm.BF16, fm.BF16), (fm.E5M2, fm.E5M2), (fm.FP16, fm.E4M3)):
        A, B, C = make_case(rng, ta, tb, 65, 16, 16, 16, special_frac=0.02)
        A2 = synth.random_bits(rng, A.shape, ta, finite=False)   # all bit patterns in a third of the tiles
        A[:20] = A2[:20]
        plist = [ModelParams(group_len=8, frac_bits=24, nan_bits=0x7FFFFFFF), ModelParams(group_len=8, frac_bits=20, out_round=RZ, ftz_in=True),
                 ModelParams(group_len=8, frac_bits=16, ftz_out=True, out_round=RZ, out_mant_bits=13)]
        want = oracle_outputs(plist, A, B, C, ta, tb)
        ref = want[0]
        st, D, kern, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref)
        assert kern.startswith("multi")
        for i in range(3):
            assert_same(D[i], want[i], "types %s set %d" % ((ta, tb), i))
            assert st[i] == ostats.compare(want[i], ref)
    # the rational form of the oracle on the first tiles of one case
    A, B, C = make_case(rng, fm.BF16, fm.BF16, 3, 16, 16, 16, c_exp=(100, 140))
    plist = sets16()
    st, D, _, _ = run_many(mm, plist, A, B, C, fm.BF16, fm.BF16, ref=C)
    for i, p in enumerate(plist):
        assert_same(D[i], o1_emulate(p, A, B, C, fm.BF16, fm.BF16), "rational oracle, set %d" % i)


def rd_sets(rng, k, count):
    """TR-FDPA sets (unsplit groups) with the variation switches drawn at random, group lengths the fused kernel takes."""
    from test_gpu_tiled_rd import random_rd_params
    out = []
    while len(out) < count:
        p = random_rd_params(rng, k).with_(group_len=int(rng.choice([L for L in (4, 8, 16, 32) if L <= k])))
        if p.f2_at_leading_bit and rng.integers(0, 3) == 0:
            p = p.with_(f2_at_leading_bit=False, rd_toward_zero=True)          # Sec. 6.2.4's truncating variant
        out.append(p)
    return out


@pytest.mark.parametrize("ta,tb,m,k", [(fm.BF16, fm.BF16, 16, 16), (fm.FP16, fm.FP16, 32, 8), (fm.E4M3, fm.E5M2, 16, 32), (fm.FP16, fm.FP16, 16, 16),
                                       (fm.BF16, fm.BF16, 32, 16), (fm.E5M2, fm.E5M2, 16, 16), (fm.BF16, fm.FP16, 16, 32)])
def test_tr_fdpa_sets_in_the_fused_kernel(mm, ta, tb, m, k):
    # Alg. "TR-FDPA" and its variations, sixteen sets per call: zero terms in or out of the maxima and input flushes make
    # up to three launches; operands over the whole format (BF16: finite products of 2^128 and more, Sec. 4.2's rule),
    # NaN and infinities sprinkled in, zeros among operands and accumulators
    rng = np.random.default_rng(400 + 8 * ta + tb + k)
    nb = 41
    A, B, C = make_case(rng, ta, tb, nb, m, m, k, special_frac=0.004)
    half = nb // 2
    A[:half] = synth.narrow_exponent_bits(rng, (half, m, k), ta, *((110, 140) if ta == fm.BF16 else (1, 14)))
    B[:half] = synth.narrow_exponent_bits(rng, (half, m, k), tb, *((110, 140) if tb == fm.BF16 else (1, 14)))
    C[:half] = synth.narrow_exponent_bits(rng, (half, m, m), fm.FP32, 100, 150)
    A = synth.sprinkle(rng, A, np.array([0, 1 << (A.dtype.itemsize * 8 - 1)], dtype=A.dtype), 0.1)
    A[1, 0, :] = 0
    C = np.where(rng.random(C.shape) < 0.1, np.uint32(0x80000000), C).astype(np.uint32)
    plist = rd_sets(rng, k, 16)
    want = oracle_outputs(plist, A, B, C, ta, tb)
    ref = want[5].copy()
    flat = ref.reshape(-1)
    idx = rng.choice(flat.size, size=flat.size // 30, replace=False)
    flat[idx] += rng.integers(1, 300, size=idx.size).astype(np.uint32)
    hs = _handles(mm, plist)
    cls = mm.compare_many_classes(hs, m, m, k, (ta, tb, fm.FP32, fm.FP32))
    for h in hs:
        mm.model_destroy(h)
    assert min(cls) >= 1 and max(cls) <= 3, cls
    got_stats, got_D, kern, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, index_base=1 << 34)
    assert kern.startswith("multi") and kern.endswith(" rd"), kern
    for i, p in enumerate(plist):
        assert_same(got_D[i], want[i], "set %d %s" % (i, p))
        assert got_stats[i] == ostats.compare(want[i], ref, index_base=1 << 34), (i, p)
    # without the dump: the same statistics
    st2, _, _, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, dump=False, index_base=1 << 34)
    assert st2 == got_stats
    # the rational form of the oracle on the first tile and on one of the wide-range tiles
    for i in (0, 3, 9, 14):
        for t in (0, nb - 1):
            assert_same(got_D[i][t:t + 1, :4], o1_emulate(plist[i], A[t:t + 1, :4], B[t:t + 1], C[t:t + 1, :4], ta, tb), "rational oracle, set %d tile %d" % (i, t))


@pytest.mark.parametrize("ta,tb,m,k", [(fm.FP16, fm.FP16, 16, 16), (fm.E4M3, fm.E5M2, 16, 32), (fm.FP16, fm.FP16, 32, 8), (fm.E5M2, fm.E5M2, 32, 16),
                                       (fm.E4M3, fm.E4M3, 16, 16), (fm.FP16, fm.E5M2, 16, 32)])
def test_split_group_sets_in_the_fused_kernel(mm, ta, tb, m, k):
    # groups split in halves or quarters (Alg. "GTR-FDPA", steps 3 to 5, on consecutive sub-groups) with the variation
    # switches drawn at random; whole sub-groups of zero products, NaN and infinities, zero accumulators
    from oracle.fdpa import SPLIT_HALVES, SPLIT_QUARTERS
    from test_gpu_tiled_rd import random_rd_params
    rng = np.random.default_rng(500 + 8 * ta + tb + k)
    nb = 37
    A, B, C = make_case(rng, ta, tb, nb, m, m, k, special_frac=0.004)
    half = nb // 2
    A[:half] = synth.narrow_exponent_bits(rng, (half, m, k), ta, 1, 14)
    B[:half] = synth.narrow_exponent_bits(rng, (half, m, k), tb, 1, 14)
    C[:half] = synth.narrow_exponent_bits(rng, (half, m, m), fm.FP32, 100, 150)
    A = synth.sprinkle(rng, A, np.array([0, 1 << (A.dtype.itemsize * 8 - 1)], dtype=A.dtype), 0.15)
    A[0, 1, : k // 2] = 0                       # one whole half without a live term
    A[1, 3, : 3 * (k // 4)] = 0                 # three quarters of a row
    A[2, 0, :] = 0
    C = np.where(rng.random(C.shape) < 0.1, np.uint32(0x80000000), C).astype(np.uint32)
    plist = []
    while len(plist) < 16:
        L = int(rng.choice([L for L in (8, 16, 32) if L <= k]))
        split = int(rng.choice([SPLIT_HALVES] + ([SPLIT_QUARTERS] * 2 if L >= 16 else [])))
        p = random_rd_params(rng, k).with_(group_len=L, split=split, frac_bits=int(rng.choice([5, 13, 20, 24])),
                                           frac_bits_merge=int(rng.choice([0, 13, 24, 28])))
        fc = p.frac_bits_acc or p.frac_bits
        plist.append(p.with_(frac_bits2=min(p.frac_bits2, fc + 40)))
    want = oracle_outputs(plist, A, B, C, ta, tb)
    ref = want[2].copy()
    flat = ref.reshape(-1)
    idx = rng.choice(flat.size, size=flat.size // 30, replace=False)
    flat[idx] += rng.integers(1, 300, size=idx.size).astype(np.uint32)
    hs = _handles(mm, plist)
    cls = mm.compare_many_classes(hs, m, m, k, (ta, tb, fm.FP32, fm.FP32))
    for h in hs:
        mm.model_destroy(h)
    assert min(cls) >= 4 and max(cls) <= 6, cls
    got_stats, got_D, kern, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, index_base=123)
    assert kern.startswith("multi") and kern.endswith(" rd split"), kern
    for i, p in enumerate(plist):
        assert_same(got_D[i], want[i], "set %d %s" % (i, p))
        assert got_stats[i] == ostats.compare(want[i], ref, index_base=123), (i, p)
    st2, _, _, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, dump=False, index_base=123)
    assert st2 == got_stats
    for i in (0, 5, 11):
        for t in (0, 1, nb - 1):
            assert_same(got_D[i][t:t + 1, :4], o1_emulate(plist[i], A[t:t + 1, :4], B[t:t + 1], C[t:t + 1, :4], ta, tb), "rational oracle, set %d tile %d" % (i, t))


@pytest.mark.parametrize("ta,tb,m,k", [(fm.E4M3, fm.E5M2, 16, 32), (fm.FP16, fm.FP16, 16, 16), (fm.E5M2, fm.E4M3, 32, 16), (fm.FP16, fm.FP16, 32, 8)])
def test_even_odd_sets_in_the_fused_kernel(mm, ta, tb, m, k):
    # Alg. "GTR-FDPA": the even and the odd products of a group summed at their own maxima, then merged
    from oracle.fdpa import SPLIT_EVEN_ODD, C_AFTER_RD_EVEN_ODD
    from test_gpu_tiled_rd import random_rd_params
    rng = np.random.default_rng(600 + 8 * ta + tb + k)
    nb = 35
    A, B, C = make_case(rng, ta, tb, nb, m, m, k, special_frac=0.004)
    half = nb // 2
    A[:half] = synth.narrow_exponent_bits(rng, (half, m, k), ta, 1, 14)
    B[:half] = synth.narrow_exponent_bits(rng, (half, m, k), tb, 1, 14)
    C[:half] = synth.narrow_exponent_bits(rng, (half, m, m), fm.FP32, 100, 150)
    A = synth.sprinkle(rng, A, np.array([0, 1 << (A.dtype.itemsize * 8 - 1)], dtype=A.dtype), 0.15)
    A[0, 2, 0::2] = 0                           # all even products zero
    A[1, 5, 1::2] = 0                           # all odd products zero
    A[2, 0, :] = 0
    C = np.where(rng.random(C.shape) < 0.1, np.uint32(0x80000000), C).astype(np.uint32)
    plist = [ModelParams(group_len=min(16, k), frac_bits=13, frac_bits2=31, c_mode=C_AFTER_RD_EVEN_ODD)]       # the CDNA3 FP8 shape of the model
    while len(plist) < 16:
        L = int(rng.choice([L for L in (4, 8, 16, 32) if L <= k]))
        p = random_rd_params(rng, k).with_(group_len=L, split=SPLIT_EVEN_ODD, frac_bits=int(rng.choice([5, 13, 20, 24])),
                                           frac_bits_merge=int(rng.choice([0, 13, 24, 28])))
        fc = p.frac_bits_acc or p.frac_bits
        plist.append(p.with_(frac_bits2=min(p.frac_bits2, fc + 40)))
    want = oracle_outputs(plist, A, B, C, ta, tb)
    ref = want[0]
    hs = _handles(mm, plist)
    cls = mm.compare_many_classes(hs, m, m, k, (ta, tb, fm.FP32, fm.FP32))
    for h in hs:
        mm.model_destroy(h)
    assert min(cls) >= 7 and max(cls) <= 9, cls
    got_stats, got_D, kern, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref)
    assert kern.startswith("multi") and kern.endswith(" rd even/odd"), kern
    for i, p in enumerate(plist):
        assert_same(got_D[i], want[i], "set %d %s" % (i, p))
        assert got_stats[i] == ostats.compare(want[i], ref), (i, p)
    for i in (0, 4, 13):
        for t in (0, 1, nb - 1):
            assert_same(got_D[i][t:t + 1, :6], o1_emulate(plist[i], A[t:t + 1, :6], B[t:t + 1], C[t:t + 1, :6], ta, tb), "rational oracle, set %d tile %d" % (i, t))


@pytest.mark.parametrize("ta,tb,m,k", [(fm.FP16, fm.FP16, 16, 16), (fm.BF16, fm.BF16, 16, 16), (fm.FP16, fm.FP16, 32, 8), (fm.E4M3, fm.E5M2, 16, 32),
                                       (fm.BF16, fm.BF16, 32, 16), (fm.E5M2, fm.E5M2, 32, 8)])
def test_twins_share_their_sums(mm, ta, tb, m, k):
    # tiles of one group: sets that differ only in the output conversion (rounding, E8M13, output flush, NaN pattern) are
    # evaluated in pairs that share the group's maximum and sum; every set's outputs and statistics as if alone
    rng = np.random.default_rng(700 + 8 * ta + tb + k)
    nb = 45
    A, B, C = make_case(rng, ta, tb, nb, m, m, k, special_frac=0.003)
    half = nb // 2
    A[:half] = synth.narrow_exponent_bits(rng, (half, m, k), ta, *((110, 140) if ta == fm.BF16 else (1, 14)))
    B[:half] = synth.narrow_exponent_bits(rng, (half, m, k), tb, *((110, 140) if tb == fm.BF16 else (1, 14)))
    C[:half] = synth.narrow_exponent_bits(rng, (half, m, m), fm.FP32, 100, 150)
    C[half:half + 4] = synth.narrow_exponent_bits(rng, (4, m, m), fm.FP32, 0, 3)          # subnormal accumulators and results
    a = ModelParams(group_len=k, frac_bits=16)
    b = ModelParams(group_len=k, frac_bits=24 if k <= 16 else 20, nan_bits=0x7FFFFFFF)
    c = ModelParams(group_len=k, frac_bits=20, ftz_in=True)
    w = ModelParams(group_len=k, frac_bits=32)                                             # binary64 sums
    plist = [a, b, a.with_(out_round=RZ), c, a.with_(out_round=RZ, out_mant_bits=13), b.with_(out_round=RZ, nan_bits=0xFFC00000),
             c.with_(ftz_out=True, out_round=RZ), a.with_(ftz_out=True), w, w.with_(out_round=RZ, ftz_out=True),
             ModelParams(group_len=k // 2, frac_bits=16), ModelParams(group_len=k // 2, frac_bits=16, out_round=RZ)]   # (two groups per tile: no twins)
    want = oracle_outputs(plist, A, B, C, ta, tb)
    ref = want[1].copy()
    flat = ref.reshape(-1)
    idx = rng.choice(flat.size, size=flat.size // 25, replace=False)
    flat[idx] += rng.integers(1, 500, size=idx.size).astype(np.uint32)
    got_stats, got_D, kern, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref, index_base=9)
    assert kern.startswith("multi x12") and kern.endswith("twins share sums"), kern
    for i, p in enumerate(plist):
        assert_same(got_D[i], want[i], "set %d %s" % (i, p))
        assert got_stats[i] == ostats.compare(want[i], ref, index_base=9), (i, p)
    # the first set as the reference, its twin compared with it; no outputs written
    pl2 = [plist[1], plist[5], plist[3], plist[6], plist[7]]
    w2 = [want[1], want[5], want[3], want[6], want[7]]
    st, _, kern, _ = run_many(mm, pl2, A, B, C, ta, tb, ref=None, dump=False)
    assert kern.endswith("twins share sums"), kern
    assert st == [ostats.compare(x, w2[0]) for x in w2]
    assert st[1]["n_mismatch_bits"] > 0


def test_t_fdpa_and_tr_fdpa_sets_in_one_call(mm):
    # a list that mixes both families and a set outside the fused kernels; the first model is the reference
    rng = np.random.default_rng(55)
    ta = tb = fm.FP16
    A, B, C = make_case(rng, ta, tb, 29, 16, 16, 16, c_exp=(100, 140))
    rd = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)
    plist = [rd, ModelParams(group_len=8, frac_bits=24), rd.with_(out_round=RZ), rd.with_(skip_zero_terms=True, zero_result_positive=True),
             ModelParams(group_len=16, frac_bits=27, out_round=RZ), rd.with_(group_len=2), rd.with_(frac_bits2=24, ftz_in=True)]
    want = oracle_outputs(plist, A, B, C, ta, tb)
    for ref in (None, want[4]):
        st, D, _, _ = run_many(mm, plist, A, B, C, ta, tb, ref=ref)
        base = want[0] if ref is None else ref
        for i in range(len(plist)):
            assert_same(D[i], want[i], "set %d" % i)
            assert st[i] == ostats.compare(want[i], base), i
    # TR-FDPA sets of one class alone need no output array, with the first as the reference too
    same = [rd, rd.with_(out_round=RZ), rd.with_(frac_bits=20), rd.with_(group_len=4, frac_bits2=27)]
    w = oracle_outputs(same, A, B, C, ta, tb)
    st, _, kern, _ = run_many(mm, same, A, B, C, ta, tb, ref=None, dump=False)
    assert kern == "multi x4 tiled 16x16 r2x2 kc=16 any L vm=0 rd", kern
    assert st == [ostats.compare(x, w[0]) for x in w]


def test_models_outside_the_fused_kernels_fall_back(mm):
    """A TR-FDPA set and a ragged shape run through the ordinary kernels; statistics and outputs are the same."""
    rng = np.random.default_rng(31)
    A, B, C = make_case(rng, fm.FP16, fm.FP16, 40, 16, 16, 16, c_exp=(100, 140))
    plist = [ModelParams(group_len=8, frac_bits=24), ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD),
             ModelParams(group_len=16, frac_bits=27, out_round=RZ), ModelParams(group_len=2, frac_bits=24)]
    want = oracle_outputs(plist, A, B, C, fm.FP16, fm.FP16)
    for ref in (None, want[2]):
        st, D, _, _ = run_many(mm, plist, A, B, C, fm.FP16, fm.FP16, ref=ref)
        base = want[0] if ref is None else ref
        for i in range(len(plist)):
            assert_same(D[i], want[i], "set %d" % i)
            assert st[i] == ostats.compare(want[i], base), i
    with pytest.raises(mm.MmaemuError) as ei:
        run_many(mm, plist, A, B, C, fm.FP16, fm.FP16, ref=want[2], dump=False)
    assert ei.value.status == 2
    # a shape the fused kernels do not take (20 x 20 x 8)
    A, B, C = make_case(rng, fm.FP16, fm.FP16, 9, 20, 20, 8, c_exp=(100, 140))
    want = oracle_outputs(plist[:1], A, B, C, fm.FP16, fm.FP16)
    st, D, _, _ = run_many(mm, plist[:1], A, B, C, fm.FP16, fm.FP16, ref=C)
    assert_same(D[0], want[0], "ragged shape")
    assert st[0] == ostats.compare(want[0], C)


def test_argument_checks(mm):
    h = mm.model_create(group_len=8, frac_bits=24)
    ok = 0x1000
    dt = (mm.FP16, mm.FP16, mm.FP32, mm.FP32)
    for kw, status in ((dict(models=[]), 1), (dict(stats=None), 1), (dict(m=0), 3), (dict(dt=(mm.FP16, mm.FP16, mm.FP16, mm.FP16)), 2),
                       (dict(A=None), 1), (dict(C=ok + 2), 1), (dict(models=[h] * 65), 1)):
        a = dict(models=[h], A=ok, B=ok, C=ok, Dref=ok, D_out=None, m=16, n=16, k=16, batch=4, dt=dt, stats=ok)
        a.update(kw)
        with pytest.raises(mm.MmaemuError) as ei:
            mm.emulate_compare_many(a["models"], a["A"], a["B"], a["C"], a["Dref"], a["D_out"], a["m"], a["n"], a["k"], a["batch"], a["dt"], a["stats"], stream=0)
        assert ei.value.status == status, (kw, mm.last_error())
    mm.emulate_compare_many([h], None, None, None, None, None, 16, 16, 16, 0, dt, ok, stream=0)       # no tiles: nothing to do
    mm.model_destroy(h)
