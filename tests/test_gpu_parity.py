"""GPU parity: every C-ABI entry point of libmmaemu against the CPU oracle, bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib, gen as ogen, stats as ostats
from oracle.fdpa import ModelParams, emulate_mma as o1_emulate, C_IN_GROUP, C_AFTER_EXACT
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth


@pytest.fixture(scope="module")
def mm():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_10909_amd import binding
    return binding


from gpu_utils import to_dev, dev_empty, to_host

NP = synth.NP_DTYPE
PAIRS = [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3),
         (fm.E4M3, fm.E4M3), (fm.E5M2, fm.E5M2), (fm.FP16, fm.BF16), (fm.E4M3, fm.FP16), (fm.BF16, fm.E5M2)]


def gpu_emulate(mm, p, A, B, C, ta, tb, tc=fm.FP32, in_place=False):
    nb, m, k = A.shape
    n = B.shape[1]
    h = mm.model_create(group_len=p.group_len, frac_bits=p.frac_bits, frac_bits2=p.frac_bits2, c_mode=p.c_mode, out_round=p.out_round,
                        ftz_in=p.ftz_in, ftz_out=p.ftz_out, nan_bits=p.nan_bits, split=p.split,
                        acc_special_truncation=p.acc_special_truncation, frac_bits_merge=p.frac_bits_merge,
                        frac_bits_acc=p.frac_bits_acc, f2_at_leading_bit=p.f2_at_leading_bit,
                        skip_zero_terms=p.skip_zero_terms, zero_result_positive=p.zero_result_positive,
                        sum_drop_distance=p.sum_drop_distance, family=p.family, out_mant_bits=p.out_mant_bits,
                        wide_products=p.wide_products, nan_propagate=p.nan_propagate, rd_toward_zero=p.rd_toward_zero)
    try:
        dA, dB, dC = to_dev(A.astype(NP[ta])), to_dev(B.astype(NP[tb])), to_dev(C.astype(NP[tc]))
        dD = dC if in_place else dev_empty((nb, m, n), NP[tc])      # (D may be C itself)
        mm.emulate_mma(h, dA, dB, dC, dD, m, n, k, nb, (ta, tb, tc, tc))
        gpu_emulate.last_kernel = mm.last_kernel()
        return to_host(dD, NP[tc]).astype(np.uint32)
    finally:
        mm.model_destroy(h)


def make_case(rng, ta, tb, nb, m, n, k, special_frac=0.0, c_exp=None):
    A = synth.random_bits(rng, (nb, m, k), ta)
    B = synth.random_bits(rng, (nb, n, k), tb)
    C = synth.random_bits(rng, (nb, m, n), fm.FP32) if c_exp is None else synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, *c_exp)
    if special_frac:
        A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], special_frac)
        B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], special_frac)
        C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], special_frac)
    return A, B, C


def assert_same(got, want, what):
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d differ; first at %s: got %08x want %08x" %
                             (what, len(bad), got.size, i, got[i], want[i]))


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_emulate_random_parameters(mm, ta, tb):
    rng = np.random.default_rng(1000 + 8 * ta + tb)
    for trial in range(16):
        L = int(rng.choice([1, 2, 4, 8, 16, 32, 0]))
        k = int(rng.choice([8, 24, 64])) if L == 0 else L * int(rng.integers(1, 5))
        F = int(rng.choice([0, 3, 13, 14, 23, 24, 25, 27, 29, 30, 32, 36, 40]))
        p = ModelParams(group_len=L, frac_bits=F, c_mode=int(rng.integers(0, 2)), out_round=int(rng.integers(0, 2)),
                        ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        nan_bits=0x7FFFFFFF if trial % 3 == 0 else 0x7FC00000)
        if p.out_round == RZ and trial % 2:
            p = p.with_(out_mant_bits=13)
        if p.c_mode == C_AFTER_EXACT and F > 30:
            p = p.with_(frac_bits=30)       # limit of the C oracle for this mode
        m, n = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        nb = int(rng.integers(1, 6))
        c_exp = (90, 165) if trial % 2 else None
        A, B, C = make_case(rng, ta, tb, nb, m, n, k, special_frac=0.02 if trial % 4 == 0 else 0.0, c_exp=c_exp)
        print("case", ta, tb, trial, p, (nb, m, n, k), flush=True)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert_same(got, want, "emulate %s" % (p,))


def test_emulate_against_rational_oracle_directly(mm):
    rng = np.random.default_rng(5)
    for ta, tb in PAIRS[:4]:
        for p in (ModelParams(group_len=4, frac_bits=24), ModelParams(group_len=8, frac_bits=13, out_round=RZ),
                  ModelParams(group_len=2, frac_bits=30, c_mode=C_AFTER_EXACT, ftz_out=True)):
            A, B, C = make_case(rng, ta, tb, 2, 5, 6, 8, special_frac=0.03)
            assert_same(gpu_emulate(mm, p, A, B, C, ta, tb), o1_emulate(p, A, B, C, ta, tb), "vs rational oracle")


def test_emulate_worked_example_of_the_paper(mm):
    # Sec. 5, Table "divergent results": same input, F = 23 / 24 / 25 / wide
    from helpers import fp16_bits, f32_bits, bits_f32
    a = [fp16_bits(-2.0 ** 13), fp16_bits(-0.5), fp16_bits(-0.25), fp16_bits(-0.125)] + [0] * 12
    b = [fp16_bits(2.0 ** 10), fp16_bits(1.0), fp16_bits(1.0), fp16_bits(1.0)] + [0] * 12
    A, B = np.array([[a]], dtype=np.uint16), np.array([[b]], dtype=np.uint16)
    C = np.array([[[f32_bits(2.0 ** 23)]]], dtype=np.uint32)
    for L, F, want in ((4, 23, 0.0), (8, 24, -0.5), (16, 25, -0.75), (16, 26, -0.875), (4, 40, -0.875)):
        got = gpu_emulate(mm, ModelParams(group_len=L, frac_bits=F, out_round=RZ), A, B, C, fm.FP16, fm.FP16)
        assert bits_f32(got[0, 0, 0]) == want


def test_emulate_in_place_and_empty(mm):
    rng = np.random.default_rng(6)
    A, B, C = make_case(rng, fm.FP16, fm.FP16, 3, 16, 16, 16, c_exp=(100, 150))
    p = ModelParams(group_len=8, frac_bits=24)
    want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16)
    h = mm.model_create(group_len=8, frac_bits=24)
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    mm.emulate_mma(h, dA, dB, dC, dC, 16, 16, 16, 3, (fm.FP16, fm.FP16, fm.FP32, fm.FP32))     # D aliases C
    assert_same(to_host(dC, np.uint32), want, "in place")
    mm.emulate_mma(h, None, None, None, None, 16, 16, 16, 0, (fm.FP16, fm.FP16, fm.FP32, fm.FP32))  # batch 0: no-op
    mm.model_destroy(h)


def test_emulate_argument_errors(mm):
    h = mm.model_create(group_len=8)
    dt = (fm.FP16, fm.FP16, fm.FP32, fm.FP32)
    x = dev_empty(4096)
    for args, status in (((h, x, x, x, x, 4, 4, 12, 1, dt), 3),          # K % L != 0
                         ((h, x, x, x, x, 0, 4, 8, 1, dt), 3),
                         ((h, x, x, x, x, 4, 4, 8, 1, (fm.FP32, fm.FP16, fm.FP32, fm.FP32)), 2),
                         ((h, x, x, x, x, 4, 4, 8, 1, (fm.FP16, fm.FP16, fm.FP16, fm.FP32)), 2),
                         ((h, x, x, x, x, 4, 4, 8, 1, (11, fm.FP16, fm.FP32, fm.FP32)), 1),
                         ((h, x, x, x, x, 4, 4, 8, 1, (10, fm.FP16, fm.FP32, fm.FP32)), 2),      # binary64 goes with the FMA family only
                         ((h, x, x, x, x, 4, 4, 8, 1, (fm.TF32, fm.FP16, fm.FP32, fm.FP32)), 2),   # TF32 pairs with itself only
                         ((h, None, x, x, x, 4, 4, 8, 1, dt), 1)):
        with pytest.raises(mm.MmaemuError) as ei:
            mm.emulate_mma(*args)
        assert ei.value.status == status
    mm.model_destroy(h)


GEN_CASES = [
    (ogen.GEN_FINITE_BITS, fm.FP16, {}), (ogen.GEN_FINITE_BITS, fm.BF16, {}), (ogen.GEN_FINITE_BITS, fm.E4M3, {}),
    (ogen.GEN_FINITE_BITS, fm.E5M2, {}), (ogen.GEN_FINITE_BITS, fm.FP32, {}),
    (ogen.GEN_RANDOM_BITS, fm.FP16, {}), (ogen.GEN_RANDOM_BITS, fm.E4M3, {}), (ogen.GEN_RANDOM_BITS, fm.FP32, {}),
    (ogen.GEN_UNIFORM_EXP, fm.FP16, dict(exp_lo=0, exp_hi=30)),
    (ogen.GEN_UNIFORM_EXP, fm.BF16, dict(exp_lo=100, exp_hi=140, exp_zero=True)),
    (ogen.GEN_UNIFORM_EXP, fm.E5M2, dict(exp_lo=1, exp_hi=30)),
    (ogen.GEN_UNIFORM_EXP, fm.FP32, dict(exp_lo=79, exp_hi=158, exp_zero=True)),
    (ogen.GEN_ZERO, fm.FP32, {}), (ogen.GEN_ZERO, fm.E4M3, {}),
    (ogen.GEN_NORMAL, fm.FP32, {}), (ogen.GEN_NORMAL, fm.BF16, {}), (ogen.GEN_NORMAL, fm.FP16, {}),
    (ogen.GEN_NORMAL, fm.E4M3, dict(scale_scope=ogen.SCALE_TENSOR, scale_target=448.0)),
    (ogen.GEN_NORMAL, fm.E5M2, dict(scale_scope=ogen.SCALE_TENSOR, scale_target=57344.0)),
    (ogen.GEN_NORMAL, fm.E4M3, dict(scale_scope=ogen.SCALE_TILE, scale_target=448.0)),
    (ogen.GEN_NORMAL, fm.E5M2, dict(scale_scope=ogen.SCALE_TILE, scale_target=57344.0)),
    (ogen.GEN_NORMAL, fm.BF16, dict(scale_scope=ogen.SCALE_TILE, scale_target=3.0)),
    (ogen.GEN_UNIFORM, fm.FP32, {}), (ogen.GEN_UNIFORM, fm.FP16, {}),
    (ogen.GEN_UNIFORM, fm.E4M3, dict(scale_scope=ogen.SCALE_TENSOR, scale_target=448.0)),
    (ogen.GEN_NORMAL_OUTLIERS, fm.FP32, {}), (ogen.GEN_NORMAL_OUTLIERS, fm.BF16, {}), (ogen.GEN_NORMAL_OUTLIERS, fm.FP16, {}),
    (ogen.GEN_NORMAL_OUTLIERS, fm.E5M2, dict(scale_scope=ogen.SCALE_TILE, scale_target=57344.0)),
    (ogen.GEN_CANCELLING, fm.FP16, dict(exp_lo=5, exp_hi=25)), (ogen.GEN_CANCELLING, fm.BF16, dict(exp_lo=100, exp_hi=150, exp_zero=True)),
    (ogen.GEN_CANCELLING, fm.E4M3, dict(exp_lo=0, exp_hi=14)), (ogen.GEN_CANCELLING, fm.E5M2, dict(exp_lo=1, exp_hi=30)),
    (ogen.GEN_UNIFORM_EXP, ogen.E8M0, dict(exp_lo=60, exp_hi=190)), (ogen.GEN_UNIFORM_EXP, ogen.E8M0, dict(exp_lo=0, exp_hi=255, exp_zero=True)),
    (ogen.GEN_RANDOM_BITS, ogen.E8M0, {}), (ogen.GEN_ZERO, ogen.E8M0, {}),
    (ogen.GEN_FINITE_BITS, fm.E2M1, {}), (ogen.GEN_FINITE_BITS, fm.E2M3, {}), (ogen.GEN_FINITE_BITS, fm.E3M2, {}),
    (ogen.GEN_RANDOM_BITS, fm.E2M1, {}), (ogen.GEN_RANDOM_BITS, fm.E3M2, {}),
    (ogen.GEN_UNIFORM_EXP, fm.E2M1, dict(exp_lo=0, exp_hi=3)), (ogen.GEN_UNIFORM_EXP, fm.E2M3, dict(exp_lo=1, exp_hi=3, exp_zero=True)),
    (ogen.GEN_UNIFORM_EXP, fm.E3M2, dict(exp_lo=0, exp_hi=7)),
    (ogen.GEN_NORMAL, fm.E2M1, dict(scale_scope=ogen.SCALE_TILE, scale_target=6.0)), (ogen.GEN_NORMAL, fm.E2M3, {}),
    (ogen.GEN_NORMAL, fm.E3M2, dict(scale_scope=ogen.SCALE_TENSOR, scale_target=28.0)),
    (ogen.GEN_CANCELLING, fm.E2M1, dict(exp_lo=0, exp_hi=3)), (ogen.GEN_CANCELLING, fm.E3M2, dict(exp_lo=1, exp_hi=6)),
    (ogen.GEN_ZERO, fm.E2M1, {}),
    (ogen.GEN_SIGNED_ZEROS, fm.FP32, {}), (ogen.GEN_SIGNED_ZEROS, fm.FP16, {}), (ogen.GEN_SIGNED_ZEROS, fm.BF16, {}),
    (ogen.GEN_SIGNED_ZEROS, fm.E4M3, {}), (ogen.GEN_SIGNED_ZEROS, fm.E5M2, {}), (ogen.GEN_SIGNED_ZEROS, fm.E2M3, {}),
    (ogen.GEN_SIGNED_ZEROS, fm.E3M2, {}), (ogen.GEN_SIGNED_ZEROS, fm.E2M1, {}),
]


@pytest.mark.parametrize("family,fmt,kw", GEN_CASES)
def test_generate_matches_cpu_twin(mm, family, fmt, kw):
    ws = dev_empty(8)
    for ept, first, nt, seed, operand in ((256, 0, 9, 0, 0), (256, 1000003, 5, 7, 1), (1024, 17, 3, 1 << 40, 2),
                                          (37, 5, 11, 3, 0), (4096 + 2, 1, 2, 9, 1), (1, 3, 7, 2, 2)):
        if family == ogen.GEN_CANCELLING and operand == 2:
            operand = 1              # (the family is meant for the two multiplicands)
        gp = ogen.GenParams(family=family, seed=seed, operand=operand, **kw)
        want = ogen.generate(gp, fmt, ept, first, nt).astype(NP[fmt])
        out = dev_empty((nt, ept), NP[fmt])
        out.fill_(0x55)
        print("gen", family, fmt, kw, (ept, first, nt, seed, operand), flush=True)
        mm.generate(out, fmt, ept, first, nt, family, seed=seed, operand=operand, workspace=ws, **kw)
        assert_same(to_host(out, NP[fmt]), want, "generate")


def test_generate_chunks_compose(mm):
    whole = dev_empty((64, 256), np.uint16)
    parts = dev_empty((64, 256), np.uint16)
    mm.generate(whole, fm.BF16, 256, 0, 64, ogen.GEN_NORMAL, seed=4, operand=1)
    mm.generate(parts[:20], fm.BF16, 256, 0, 20, ogen.GEN_NORMAL, seed=4, operand=1)
    mm.generate(parts[20:], fm.BF16, 256, 20, 44, ogen.GEN_NORMAL, seed=4, operand=1)
    assert_same(to_host(parts, np.uint16), to_host(whole, np.uint16), "chunked generation")


def test_compare_matches_oracle(mm):
    rng = np.random.default_rng(8)
    for count, misalign in ((1, 0), (1000, 0), (100003, 0), (4099, 1), (1 << 20, 0)):
        x = synth.random_bits(rng, count + misalign, fm.FP32, finite=False)
        y = x.copy()
        flip = rng.random(count + misalign) < 0.3
        y[flip] ^= (np.uint32(1) << rng.integers(0, 32, size=int(flip.sum())).astype(np.uint32))
        y[rng.random(count + misalign) < 0.01] = 0x7FC00001
        x[rng.random(count + misalign) < 0.01] = 0x7FC00000
        dx, dy = to_dev(x), to_dev(y)
        st = dev_empty(mm.STATS_BYTES)
        mm.stats_reset(st)
        mm.compare(dx[misalign:], dy[misalign:], count, st, index_base=10)
        want = ostats.compare(x[misalign:], y[misalign:], index_base=10)
        assert mm.read_stats(st) == want
        # accumulation over a second chunk
        mm.compare(dx[misalign:], dx[misalign:], count, st, index_base=10 + count)
        want = ostats.compare(x[misalign:], x[misalign:], stats=want, index_base=10 + count)
        assert mm.read_stats(st) == want
    st = dev_empty(mm.STATS_BYTES)
    mm.stats_reset(st)
    mm.compare(None, None, 0, st)
    assert mm.read_stats(st) == ostats.empty_stats()


def test_compare_fp16_outputs_matches_oracle(mm):
    rng = np.random.default_rng(81)
    for count, misalign in ((1, 0), (7, 0), (1000, 0), (100003, 0), (4099, 1), (4099, 3), (1 << 20, 0)):
        x = synth.random_bits(rng, count + misalign, fm.FP16, finite=False)
        y = x.copy()
        flip = rng.random(count + misalign) < 0.3
        y[flip] ^= (np.uint16(1) << rng.integers(0, 16, size=int(flip.sum())).astype(np.uint16))
        y[rng.random(count + misalign) < 0.01] = 0x7E01
        x[rng.random(count + misalign) < 0.01] = 0x7E00
        dx, dy = to_dev(x), to_dev(y)
        st = dev_empty(mm.STATS_BYTES)
        mm.stats_reset(st)
        mm.compare(dx[misalign:], dy[misalign:], count, st, index_base=10, d=mm.FP16)
        want = ostats.compare(x[misalign:], y[misalign:], index_base=10, width=16)
        assert mm.read_stats(st) == want, (count, misalign)
        mm.compare(dx[misalign:], dx[misalign:], count, st, index_base=10 + count, d=mm.FP16)
        want = ostats.compare(x[misalign:], x[misalign:], stats=want, index_base=10 + count, width=16)
        assert mm.read_stats(st) == want
    with pytest.raises(mm.MmaemuError) as ei:
        mm.compare(dx, dy, 4, st, d=mm.BF16)
    assert ei.value.status == 2


MFMA_TYPES = {0: (fm.FP16, fm.FP16), 1: (fm.BF16, fm.BF16), 2: (fm.FP16, fm.FP16), 3: (fm.BF16, fm.BF16),
              4: (fm.FP16, fm.FP16), 5: (fm.BF16, fm.BF16), 6: (fm.E4M3, fm.E4M3), 7: (fm.E4M3, fm.E5M2),
              8: (fm.E5M2, fm.E4M3), 9: (fm.E5M2, fm.E5M2),
              35: (fm.FP16, fm.FP16), 36: (fm.BF16, fm.BF16), 37: (fm.E4M3, fm.E4M3), 38: (fm.E4M3, fm.E5M2),
              39: (fm.E5M2, fm.E4M3), 40: (fm.E5M2, fm.E5M2), 41: (fm.FP32, fm.FP32), 42: (fm.FP32, fm.FP32),
              # multi-block forms (2, 4 or 16 tiles per issue; seven tiles: the last issue is a partial one)
              68: (fm.FP16, fm.FP16), 69: (fm.FP16, fm.FP16), 70: (fm.FP16, fm.FP16), 71: (fm.BF16, fm.BF16), 72: (fm.BF16, fm.BF16),
              73: (fm.BF16, fm.BF16), 74: (fm.FP32, fm.FP32), 75: (fm.FP32, fm.FP32), 76: (fm.FP32, fm.FP32)}


def _small_int_codes(rng, shape, t):
    """Bit patterns of random integers in -4..4 (exactly representable in every format)."""
    vals = rng.integers(-4, 5, size=shape)
    f = fm.FORMATS[t]
    out = np.zeros(shape, dtype=np.uint32)
    for v in range(1, 5):
        e = int(np.floor(np.log2(v)))
        man = int((v / 2 ** e - 1) * (1 << f.mbits))
        code = ((e + f.bias) << f.mbits) | man
        out[vals == v] = code
        out[vals == -v] = code | (1 << (f.width - 1))
    return out.astype(NP[t]), vals


@pytest.mark.parametrize("instr", sorted(MFMA_TYPES))
def test_mfma_probe_register_layout(mm, instr):
    # with small-integer operands every arithmetic is exact, so D = A B^T + C exactly whatever the
    # instruction's internal behaviour: any mistake in the operand/result register layout shows
    info = mm.mfma_info(instr)
    ta, tb = MFMA_TYPES[instr]
    assert (info["a"], info["b"]) == (ta, tb)
    M, N, KN = info["m"], info["n"], info["k"]
    rng = np.random.default_rng(instr)
    for k in sorted({q for q in (KN, KN // 2, 3) if 1 <= q <= KN}):
        nb = 7 if instr < 68 else 37
        A, av = _small_int_codes(rng, (nb, M, k), ta)
        B, bv = _small_int_codes(rng, (nb, N, k), tb)
        cv = rng.integers(-100, 100, size=(nb, M, N))
        C = cv.astype(np.float32).view(np.uint32)
        want = (np.einsum("bik,bjk->bij", av, bv) + cv).astype(np.float32).view(np.uint32)
        dD = dev_empty((nb, M, N), np.uint32)
        print("mfma", instr, k, flush=True)
        mm.mfma_probe(instr, to_dev(A), to_dev(B), to_dev(C), dD, k, nb)
        got = to_host(dD, np.uint32)
        # an exact-zero result may come out as -0 or +0 depending on the unit; compare values
        assert_same(np.where(got == 0x80000000, 0, got), want, "mfma layout")


def test_exact_dot_sample_matches_oracle(mm):
    rng = np.random.default_rng(9)
    for ta, tb in ((fm.E4M3, fm.E5M2), (fm.E5M2, fm.E5M2), (fm.E4M3, fm.E4M3), (fm.E5M2, fm.E4M3)):
        m, n, k = 48, 40, 192
        A = synth.random_bits(rng, (m, k), ta)
        B = synth.random_bits(rng, (n, k), tb)
        p = ModelParams(group_len=32, frac_bits=14)
        D, _ = o2lib.emulate_mma(p, A, B, np.zeros((m, n), dtype=np.uint32), ta, tb)
        D = D[0]
        want = o2lib.exact_dot_stats(A, B, D, ta, tb, 7)
        Dnan = D.copy()
        Dnan[0, 0] = 0x7FC00000                    # a NaN at a sampled place is skipped and counted
        st = dev_empty(mm.ERR_STATS_BYTES)
        mm.err_stats_reset(st)
        mm.exact_dot_sample(to_dev(A), to_dev(B), to_dev(Dnan), m, n, k, (ta, tb, fm.FP32, fm.FP32), 7, st)
        got = mm.read_err_stats(st)
        assert got["n_skipped"] == 1 and got["n_samples"] == want["n_samples"] - 1
        full = dev_empty(mm.ERR_STATS_BYTES)
        mm.err_stats_reset(full)
        mm.exact_dot_sample(to_dev(A), to_dev(B), to_dev(D), m, n, k, (ta, tb, fm.FP32, fm.FP32), 7, full)
        got = mm.read_err_stats(full)
        assert got["n_skipped"] == 0
        for key in ("n_samples", "n_equal_rne", "n_above", "n_below", "ulp_hist"):
            assert got[key] == want[key], key
        for key in ("sum_abs_err", "max_abs_err", "sum_rel_err", "max_rel_err", "sum_signed_err"):
            assert got[key] == pytest.approx(want[key], rel=1e-9, abs=1e-300), key


def test_exact_dot_every_pair_of_codes(mm):
    # every pair of FP8 codes as the one non-zero product of a dot product of four: D holds the exact product (every one is
    # a binary32 number), so each finite pair must be counted as equal, and each pair with a NaN or an infinity as skipped
    from fractions import Fraction
    for ta, tb in ((fm.E4M3, fm.E5M2), (fm.E5M2, fm.E5M2), (fm.E4M3, fm.E4M3), (fm.E5M2, fm.E4M3)):
        A = np.zeros((256, 4), dtype=np.uint8)
        B = np.zeros((256, 4), dtype=np.uint8)
        A[:, 1] = np.arange(256)
        B[:, 1] = np.arange(256)
        B[:, 3] = 0x80                             # (a negative zero elsewhere in the row changes nothing)
        da = [fm.decode(c, ta) for c in range(256)]
        db = [fm.decode(c, tb) for c in range(256)]
        D = np.zeros((256, 256), dtype=np.uint32)
        finite = 0
        for i in range(256):
            for j in range(256):
                if da[i].finite and db[j].finite:
                    finite += 1
                    D[i, j] = np.float32(float(da[i].value * db[j].value)).view(np.uint32)
                    assert Fraction(float(np.uint32(D[i, j]).view(np.float32))) == da[i].value * db[j].value
                    if D[i, j] == 0x80000000:
                        D[i, j] = 0                # (an exact zero is +0.0)
        st = dev_empty(mm.ERR_STATS_BYTES)
        mm.err_stats_reset(st)
        mm.exact_dot_sample(to_dev(A), to_dev(B), to_dev(D), 256, 256, 4, (ta, tb, fm.FP32, fm.FP32), 1, st)
        got = mm.read_err_stats(st)
        assert got["n_samples"] == finite and got["n_skipped"] == 65536 - finite, (ta, tb, got["n_samples"], got["n_skipped"], finite)
        assert got["n_equal_rne"] == finite and got["max_abs_err"] == 0.0, (ta, tb, got["n_equal_rne"], got["max_abs_err"])
        assert 0 < 65536 - finite < 6000


@pytest.mark.parametrize("ta,tb,L,cm", [(fm.FP16, fm.FP16, 0, C_IN_GROUP), (fm.BF16, fm.BF16, 8, C_AFTER_EXACT), (fm.E4M3, fm.E5M2, 32, C_IN_GROUP),
                                        (fm.FP16, fm.FP16, 1 << 20, C_AFTER_EXACT)])
def test_emulate_longest_dot_products(mm, ta, tb, L, cm):
    # k at the entry point's limit (2^20), one group spanning all of it and chains of short groups; k one above: refused
    rng = np.random.default_rng(77 + L % 97)
    k = 1 << 20
    A = synth.narrow_exponent_bits(rng, (1, 3, k), ta, *((12, 18) if ta != fm.BF16 else (120, 134)))
    B = synth.narrow_exponent_bits(rng, (1, 2, k), tb, *((12, 18) if tb != fm.BF16 else (120, 134)))
    if ta == fm.E4M3:
        A, B = synth.random_bits(rng, (1, 3, k), ta), synth.random_bits(rng, (1, 2, k), tb)
    C = synth.narrow_exponent_bits(rng, (1, 3, 2), fm.FP32, 120, 140)
    p = ModelParams(group_len=L, frac_bits=24, c_mode=cm)
    want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
    got = gpu_emulate(mm, p, A, B, C, ta, tb)
    assert_same(got, want, "k = 2^20, L = %d" % L)
    h = mm.model_create(group_len=1)
    x = dev_empty(64)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, x, x, x, x, 1, 1, k + 1, 1, (ta, tb, fm.FP32, fm.FP32))
    assert ei.value.status == 3
    mm.model_destroy(h)
