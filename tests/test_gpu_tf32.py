"""GPU parity for TF32 operands (Require lines of Algorithms "T-FDPA" and "TR-FDPA"): binary32 words whose low 13
mantissa bits do not count."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, SPLIT_HALVES
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from test_gpu_parity import gpu_emulate, assert_same, mm                                     # noqa: F401  (mm is a fixture)


def tf32_case(rng, nb, m, n, k, trial):
    if trial % 3 == 0:
        A = synth.random_bits(rng, (nb, m, k), fm.TF32, finite=trial % 2 == 0)
        B = synth.random_bits(rng, (nb, n, k), fm.TF32)
    else:
        A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.TF32, 100, 150)
        B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.TF32, 100, 150)
    C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 80, 170)
    if trial % 4 == 1:
        A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[fm.TF32], 0.03)
        B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[fm.TF32], 0.03)
        C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.03)
    return A, B, C


def test_tf32_random_parameters(mm):
    rng = np.random.default_rng(9001)
    for trial in range(24):
        L = int(rng.choice([1, 2, 4, 8, 16]))
        k = L * int(rng.integers(1, 5))
        cm = int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD]))
        F = int(rng.choice([0, 13, 23, 24, 25, 27, 30]))
        p = ModelParams(group_len=L, frac_bits=F, c_mode=cm, out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)),
                        ftz_out=bool(rng.integers(0, 2)), nan_bits=0x7FFFFFFF if trial % 2 else 0x7FC00000)
        if cm == C_AFTER_RD:
            p = p.with_(frac_bits2=int(rng.choice([24, 31])), f2_at_leading_bit=bool(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)), zero_result_positive=bool(rng.integers(0, 2)))
            if L >= 2 and trial % 2:
                p = p.with_(split=SPLIT_HALVES, frac_bits_merge=max(F, 24))
        nb, m, n = int(rng.integers(1, 5)), int(rng.integers(1, 36)), int(rng.integers(1, 36))
        A, B, C = tf32_case(rng, nb, m, n, k, trial)
        print("case", trial, p, (nb, m, n, k), flush=True)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.TF32, fm.TF32)
        got = gpu_emulate(mm, p, A, B, C, fm.TF32, fm.TF32)
        assert gpu_emulate.last_kernel == "general" or "vm=4" in gpu_emulate.last_kernel
        assert_same(got, want, "tf32 %s" % (p,))


def test_tf32_worked_example_and_paper_parameter_sets(mm):
    # Sec. 5, Table "divergent results", column "TF32/BF16 Instr.": Ampere / Ada -0.5, Hopper / Blackwell -0.75, CDNA3 -0.5
    from helpers import f32_bits, bits_f32
    from paper_2511_10909_amd import presets
    a = [f32_bits(-2.0 ** 13), f32_bits(-0.5), f32_bits(-0.25), f32_bits(-0.125)] + [0] * 4
    b = [f32_bits(2.0 ** 10), f32_bits(1.0), f32_bits(1.0), f32_bits(1.0)] + [0] * 4
    A, B = np.array([[a]], dtype=np.uint32), np.array([[b]], dtype=np.uint32)
    C = np.array([[[f32_bits(2.0 ** 23)]]], dtype=np.uint32)
    for arch, want in (("ampere", -0.5), ("ada", -0.5), ("hopper", -0.75), ("blackwell", -0.75), ("cdna3", -0.5)):
        h = mm.model_create(**presets.PAPER[(arch, "tf32")])
        try:
            from gpu_utils import to_dev, dev_empty, to_host
            dD = dev_empty((1, 1, 1), np.uint32)
            mm.emulate_mma(h, to_dev(A), to_dev(B), to_dev(C), dD, 1, 1, 8, 1, (mm.TF32, mm.TF32, mm.FP32, mm.FP32))
            assert bits_f32(int(to_host(dD, np.uint32)[0, 0, 0])) == want, arch
        finally:
            mm.model_destroy(h)


def test_tf32_low_bits_do_not_count(mm):
    rng = np.random.default_rng(9002)
    p = ModelParams(group_len=4, frac_bits=24, out_round=RZ)
    A, B, C = tf32_case(rng, 3, 17, 19, 16, 2)
    clean = gpu_emulate(mm, p, A & np.uint32(0xFFFFE000), B & np.uint32(0xFFFFE000), C, fm.TF32, fm.TF32)
    assert_same(gpu_emulate(mm, p, A, B, C, fm.TF32, fm.TF32), clean, "low bits")


TILED_SHAPES = [(9, 16, 16, 8), (3, 16, 16, 24), (5, 16, 16, 16), (3, 16, 16, 32), (2, 32, 32, 8), (2, 32, 32, 24), (1, 64, 32, 64), (1, 96, 64, 32), (70, 16, 16, 16)]


@pytest.mark.parametrize("shape", TILED_SHAPES)
def test_tf32_tiled_kernels(mm, shape):
    # the tiled kernels' value mode for 32-bit words: every accumulation mode, both flushes, special values, the full
    # exponent range (products beyond binary32: the binary64 pass; 2^128 and more in the RD mode: the integer routine)
    nb, m, n, k = shape
    rng = np.random.default_rng(9100 + m + k + nb)
    for trial in range(9):
        L = int(rng.choice([4, 8]))
        cm = [C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD][trial % 3]
        F = int(rng.choice([0, 13, 23, 24, 25, 27, 29]))
        p = ModelParams(group_len=L, frac_bits=F, c_mode=cm, out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)),
                        ftz_out=bool(rng.integers(0, 2)), nan_bits=0x7FFFFFFF if trial % 2 else 0x7FC00000)
        if cm == C_AFTER_RD:
            p = p.with_(frac_bits2=int(rng.choice([24, 31])), f2_at_leading_bit=bool(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)), zero_result_positive=bool(rng.integers(0, 2)))
        A, B, C = tf32_case(rng, nb, m, n, k, trial)
        if trial == 7:          # subnormal operands next to ordinary ones
            A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.TF32, 0, 3)
            B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.TF32, 120, 250)
        print("case", shape, trial, p, flush=True)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.TF32, fm.TF32)
        got = gpu_emulate(mm, p, A, B, C, fm.TF32, fm.TF32)
        assert gpu_emulate.last_kernel.startswith("tiled") and gpu_emulate.last_kernel.endswith("vm=4"), gpu_emulate.last_kernel
        assert_same(got, want, "tf32 tiled %s %s" % (shape, p))


def test_tf32_tiled_equals_general_kernel_on_the_paper_sets(mm):
    # the same problem through both routes: F = 30 sends TF32 to the general kernel, and with products of a few bits
    # F = 29 and F = 30 give the same sums
    from paper_2511_10909_amd import presets
    rng = np.random.default_rng(9200)
    nb, m, n, k = 4, 32, 32, 32
    A, B, C = tf32_case(rng, nb, m, n, k, 2)
    for arch in ("ampere", "hopper", "cdna3"):
        kw = presets.PAPER[(arch, "tf32")]
        p = ModelParams(group_len=kw["group_len"], frac_bits=kw["frac_bits"], c_mode=kw.get("c_mode", C_IN_GROUP), out_round=kw["out_round"],
                        frac_bits2=kw.get("frac_bits2", 0))
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.TF32, fm.TF32)
        got = gpu_emulate(mm, p, A, B, C, fm.TF32, fm.TF32)
        assert "vm=4" in gpu_emulate.last_kernel, gpu_emulate.last_kernel
        assert_same(got, want, "paper set %s" % arch)
        # off the 16-byte alignment the general kernel takes over, with the same result
        from gpu_utils import to_dev, dev_empty, to_host
        h = mm.model_create(**kw)
        buf = np.zeros(A.size + 2, dtype=np.uint32); buf[2:] = A.reshape(-1)
        dA, dB, dC, dD = to_dev(buf), to_dev(B), to_dev(C), dev_empty((nb, m, n), np.uint32)
        mm.emulate_mma(h, dA.data_ptr() + 8, dB, dC, dD, m, n, k, nb, (mm.TF32, mm.TF32, mm.FP32, mm.FP32))
        assert mm.last_kernel() == "general"
        assert_same(to_host(dD, np.uint32), want, "general route %s" % arch)
        mm.model_destroy(h)
