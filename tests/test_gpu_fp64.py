"""GPU parity on binary64 (Algorithms "FMA" / "Phi_FMA" with F = FP64; Sec. 5: every FP64 instruction behaves as the
chain): the generators, the FMA family and the comparison element by element against the oracle, the register layout of
the two binary64 MFMA forms by exact small-integer products, and those instructions against the model."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, fma as ofma, gen as ogen, stats as ostats
from gpu_utils import to_dev, dev_empty, to_host
from test_gpu_parity import assert_same, mm                                     # noqa: F401  (mm is a fixture)

FP64 = 10
INF = 0x7FF0000000000000


def gpu_fma64(mm, A, B, C, nan_bits=0x7FC00000, nan_propagate=False, offset_words=0):
    nb, m, k = A.shape
    n = B.shape[1]
    h = mm.model_create(family=mm.FAMILY_FMA, nan_bits=nan_bits, nan_propagate=nan_propagate)
    try:
        def shifted(x):
            buf = np.zeros(x.size + offset_words, dtype=np.uint64)
            buf[offset_words:] = x.reshape(-1)
            return to_dev(buf)
        bA, bB = shifted(A), shifted(B)
        dC = to_dev(C)
        dD = dev_empty((nb, m, n), np.uint64)
        mm.emulate_mma(h, bA.data_ptr() + 8 * offset_words, bB.data_ptr() + 8 * offset_words, dC, dD, m, n, k, nb, (FP64,) * 4)
        gpu_fma64.last_kernel = mm.last_kernel()
        return to_host(dD, np.uint64)
    finally:
        mm.model_destroy(h)


def fp64_case(rng, nb, m, n, k, trial):
    """Input families of the chain: ordinary values; cancelling first step; the bottom of the range; all bit patterns
    (NaN and infinity included); zeros, units and smallest subnormals of both signs."""
    shp = ((nb, m, k), (nb, n, k), (nb, m, n))
    if trial == 0:
        A, B, C = (rng.standard_normal(s) for s in shp)
    elif trial == 1:
        A, B = rng.standard_normal(shp[0]), rng.standard_normal(shp[1])
        C = -np.einsum("tik,tjk->tij", A[:, :, :1], B[:, :, :1])
    elif trial == 2:
        A, B, C = rng.standard_normal(shp[0]) * 2.0 ** -520, rng.standard_normal(shp[1]) * 2.0 ** -520, rng.standard_normal(shp[2]) * 2.0 ** -1060
    elif trial == 3:
        return tuple(rng.integers(0, 1 << 64, size=s, dtype=np.uint64) for s in shp)
    else:
        Z = np.array([0, 1 << 63, 1, (1 << 63) | 1, 0x3FF0000000000000, 0xBFF0000000000000, INF, INF | (1 << 63), 0x7FF0000000012345], dtype=np.uint64)
        return tuple(Z[rng.integers(0, len(Z) - (3 if trial == 4 else 0), s)] for s in shp)
    return tuple(np.ascontiguousarray(x, dtype=np.float64).view(np.uint64) for x in (A, B, C))


SHAPES = [  # (tiles, m, n, k, offset_words, kernel)
    (3, 16, 16, 4, 0, "fma chain fp64, 16x16 blocks, 128-bit loads, 4 blocks in flight"),
    (1, 32, 16, 6, 0, "fma chain fp64, 16x16 blocks, 128-bit loads"),
    (20, 4, 4, 4, 0, "fma chain fp64, 128-bit loads"),
    (2, 16, 32, 3, 0, "fma chain fp64, 16x16 blocks"),
    (3, 5, 7, 3, 0, "fma chain fp64"),
    (2, 16, 16, 6, 1, "fma chain fp64, 16x16 blocks"),              # rows off the 16-byte alignment
    (2, 9, 13, 8, 0, "fma chain fp64, 128-bit loads"),
    (1, 32, 16, 21, 0, "fma chain fp64, 16x16 blocks"),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_fma_family_on_binary64_matches_the_oracle(mm, shape):
    nb, m, n, k, off, kernel = shape
    rng = np.random.default_rng(6400 + 7 * m + k)
    for trial in range(6):
        print("case", shape, trial, flush=True)
        A, B, C = fp64_case(rng, nb, m, n, k, trial)
        for propagate, nan_bits in ((False, 0x7FC00000), (True, 0xFFC00000), (False, 0x7FFFFFFF)):
            want = ofma.emulate_mma(A, B, C, nan_bits=nan_bits, nan_propagate=propagate, fmt=fm.FP64)
            got = gpu_fma64(mm, A, B, C, nan_bits=nan_bits, nan_propagate=propagate, offset_words=off)
            assert gpu_fma64.last_kernel == (kernel.replace("fp64", "fp64, payloads") if propagate else kernel), gpu_fma64.last_kernel
            assert_same(got, want, "fma family fp64 %s trial %d propagate %d" % (shape, trial, propagate))
        if trial == 4:
            assert np.count_nonzero(want == 1 << 63) > 0          # the case does reach the sign rule


def test_binary64_argument_errors(mm):
    h = mm.model_create(family=mm.FAMILY_FMA)
    g = mm.model_create(group_len=4)
    x = dev_empty(4096, np.uint64)
    try:
        with pytest.raises(mm.MmaemuError):
            mm.emulate_mma(g, x, x, x, x, 4, 4, 4, 1, (FP64,) * 4)                 # FDPA family on binary64
        with pytest.raises(mm.MmaemuError):
            mm.emulate_mma(h, x, x, x, x, 4, 4, 4, 1, (FP64, FP64, mm.FP32, mm.FP32))   # mixed widths
        with pytest.raises(mm.MmaemuError):
            mm.emulate_mma(h, x.data_ptr() + 4, x, x, x, 4, 4, 4, 1, (FP64,) * 4)    # misaligned
        with pytest.raises(mm.MmaemuError):
            mm.generate(x, FP64, 16, 0, 4, mm.GEN_CANCELLING, exp_lo=1, exp_hi=5)
        with pytest.raises(mm.MmaemuError):
            mm.generate(x, FP64, 16, 0, 4, mm.GEN_NORMAL, scale_scope=mm.SCALE_TILE, scale_target=2.0)
        with pytest.raises(mm.MmaemuError):
            mm.generate(x, FP64, 16, 0, 4, mm.GEN_UNIFORM_EXP, exp_lo=1, exp_hi=2048)
        mm.emulate_mma(h, x, x, x, x, 4, 4, 4, 0, (FP64,) * 4)                    # an empty batch is fine
    finally:
        mm.model_destroy(h)
        mm.model_destroy(g)


GEN_CASES = [
    (ogen.GEN_ZERO, {}), (ogen.GEN_NORMAL, {}), (ogen.GEN_UNIFORM, {}), (ogen.GEN_NORMAL_OUTLIERS, {}),
    (ogen.GEN_NORMAL, dict(scale_scope=ogen.SCALE_FACTOR, scale_target=1000.0)),
    (ogen.GEN_NORMAL_OUTLIERS, dict(scale_scope=ogen.SCALE_FACTOR, scale_target=2.0 ** -600)),
    (ogen.GEN_RANDOM_BITS, {}), (ogen.GEN_FINITE_BITS, {}), (ogen.GEN_SIGNED_ZEROS, {}),
    (ogen.GEN_UNIFORM_EXP, dict(exp_lo=1000, exp_hi=1040, exp_zero=True)), (ogen.GEN_UNIFORM_EXP, dict(exp_lo=0, exp_hi=2047)),
]


@pytest.mark.parametrize("family,kw", GEN_CASES)
def test_generate_binary64_matches_cpu_twin(mm, family, kw):
    for ept, first, nt, seed, operand in ((256, 0, 9, 0, 0), (256, 1000003, 5, 7, 1), (1024, 17, 3, 1 << 40, 2),
                                          (37, 5, 11, 3, 0), (4096 + 1, 1, 2, 9, 1), (1, 3, 7, 2, 2)):
        gp = ogen.GenParams(family=family, seed=seed, operand=operand, **kw)
        want = ogen.generate(gp, fm.FP64, ept, first, nt)
        out = dev_empty((nt, ept), np.uint64)
        out.fill_(0x55)
        print("gen fp64", family, kw, (ept, first, nt, seed, operand), flush=True)
        mm.generate(out, FP64, ept, first, nt, family, seed=seed, operand=operand, **kw)
        assert_same(to_host(out, np.uint64), want, "generate fp64")


def test_normal_stream_in_binary64_at_size(mm):
    # 2^23 values of the N(0,1) series as binary64 numbers, before any narrowing hides a last place: the series' square
    # root is the IEEE-754 operation on both sides, so a device routine that were not correctly rounded would show here
    ept, nt = 4096, 2048
    gp = ogen.GenParams(family=ogen.GEN_NORMAL, seed=5, operand=1)
    out = dev_empty((nt, ept), np.uint64)
    mm.generate(out, FP64, ept, 0, nt, ogen.GEN_NORMAL, seed=5, operand=1)
    got = to_host(out, np.uint64)
    step = 256
    for t0 in range(0, nt, step):
        want = ogen.generate(gp, fm.FP64, ept, t0, step, threads=8)
        assert_same(got[t0:t0 + step], want, "N(0,1) in binary64, tiles %d.." % t0)


def test_compare_binary64_matches_oracle(mm):
    rng = np.random.default_rng(18)
    for count, misalign in ((1, 0), (1000, 0), (100003, 0), (4099, 1), (1 << 19, 0)):
        x = rng.integers(0, 1 << 64, size=count + misalign, dtype=np.uint64)
        y = x.copy()
        flip = rng.random(count + misalign) < 0.3
        y[flip] ^= (np.uint64(1) << rng.integers(0, 64, size=int(flip.sum())).astype(np.uint64))
        y[rng.random(count + misalign) < 0.01] = 0x7FF8000000000001
        x[rng.random(count + misalign) < 0.01] = 0x7FF8000000000000
        dx, dy = to_dev(x), to_dev(y)
        st = dev_empty(mm.STATS_BYTES)
        mm.stats_reset(st)
        mm.compare(dx[misalign:], dy[misalign:], count, st, index_base=(1 << 40) + 10, d=FP64)
        want = ostats.compare(x[misalign:], y[misalign:], index_base=(1 << 40) + 10, width=64)
        assert mm.read_stats(st) == want
        mm.compare(dx[misalign:], dx[misalign:], count, st, index_base=10 + count, d=FP64)
        want = ostats.compare(x[misalign:], x[misalign:], stats=want, index_base=10 + count, width=64)
        assert mm.read_stats(st) == want


F64_FORMS = ((77, 16), (78, 4))


def run_probe(mm, instr, A, B, C, k):
    nb, m = A.shape[0], A.shape[1]
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    dD = dev_empty((nb, m, m), np.uint64)
    dD.fill_(0x33)
    mm.mfma_probe(instr, dA, dB, dC, dD, k, nb)
    return to_host(dD, np.uint64)


@pytest.mark.parametrize("instr,m", F64_FORMS)
def test_binary64_mfma_layout_by_exact_integer_products(mm, instr, m):
    info = mm.mfma_info(instr)
    assert (info["m"], info["n"], info["k"], info["a"], info["b"]) == (m, m, 4, FP64, FP64)
    rng = np.random.default_rng(77 + m)
    for nb in (1, 3, 4, 9, 130):
        for k in (4, 3, 1):
            Av, Bv, Cv = rng.integers(-9, 10, (nb, m, k)), rng.integers(-9, 10, (nb, m, k)), rng.integers(-50, 51, (nb, m, m))
            want = (np.einsum("tik,tjk->tij", Av, Bv) + Cv).astype(np.float64)
            got = run_probe(mm, instr, *(x.astype(np.float64).view(np.uint64) for x in (Av, Bv, Cv)), k)
            assert np.array_equal(got.view(np.float64), want), (instr, nb, k)


@pytest.mark.parametrize("instr,m", F64_FORMS)
def test_binary64_mfma_is_the_fma_chain(mm, instr, m):
    """Sec. 5: the FP64 instructions behave as Phi_FMA; here for gfx950's two forms, on every input family, bit for bit
    (finite results and infinities; NaN results compared as NaN, the hardware's payload is its own)."""
    rng = np.random.default_rng(640 + m)
    nb = 64
    for trial in range(6):
        A, B, C = fp64_case(rng, nb, m, m, 4, trial)
        got = run_probe(mm, instr, A, B, C, 4)
        model = gpu_fma64(mm, A, B, C)
        gn, mn = (got & np.uint64(0x7FFFFFFFFFFFFFFF)) > INF, (model & np.uint64(0x7FFFFFFFFFFFFFFF)) > INF
        assert np.array_equal(gn, mn), (instr, trial)
        assert np.array_equal(got[~gn], model[~mn]), (instr, trial, int(np.count_nonzero(got[~gn] != model[~mn])))
    # the oracle itself on a slice of the last family and of the cancelling one
    for trial in (1, 3):
        A, B, C = fp64_case(rng, 2, m, m, 4, trial)
        got = run_probe(mm, instr, A, B, C, 4)
        want = ofma.emulate_mma(A, B, C, fmt=fm.FP64)
        gn = (got & np.uint64(0x7FFFFFFFFFFFFFFF)) > INF
        assert np.array_equal(gn, (want & np.uint64(0x7FFFFFFFFFFFFFFF)) > INF)
        assert np.array_equal(got[~gn], want[~gn])
