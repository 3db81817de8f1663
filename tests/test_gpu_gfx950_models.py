"""The parameter sets in presets.GFX950_MFMA against the native v_mfma_f32_* instructions of the GPU the tests run
on: bit-for-bit agreement on every validation family (paper Sec. 3, Step 4: randomised validation of a model against
the MMA interface; Eq. 2).  This is not a parity test of the library (those compare with the CPU oracle): it checks a
*model* against silicon, and it ties the oracle-checked emulation to something outside this repository."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_10909_amd import binding, configs, presets
    return binding, configs, presets


@pytest.mark.parametrize("instr", list(range(10)) + list(range(35, 41)) + list(range(68, 74)))
def test_gfx950_preset_reproduces_the_instruction(env, instr):
    mm, configs, presets = env
    res = configs.validate_against_mfma(instr, presets.GFX950_MFMA[instr], n_tiles=1024, seeds=(0, 1))
    for fam, st in res.items():
        if not isinstance(st, dict):
            continue
        assert st["n_compared"] > 0
        assert st["n_mismatch_bits"] == 0, (instr, fam, st["n_mismatch_bits"], st["first_mismatch_index"])


@pytest.mark.parametrize("instr", [41, 42, 74, 75, 76, 77, 78])
def test_gfx950_fp32_instructions_are_fma_chains(env, instr):
    # Sec. 4.1.2 / Sec. 5: FP32 and FP64 instructions are chains of standard FMAs (the FMA family); here one that passes NaN
    # payloads on (`nan_propagate`).  Every output agrees bit for bit, NaN patterns included.  With the paper's one NaN
    # pattern instead, all mismatches are NaN against NaN.  A flushing variant and a single fused sum of the exact
    # products do not reproduce it.
    mm, configs, presets = env
    res = configs.validate_against_mfma(instr, presets.GFX950_MFMA[instr], n_tiles=1024, seeds=(0, 1))
    assert res["kernel"].startswith("fma chain fp64, payloads" if instr >= 77 else "fma chain, payloads")
    for fam, st in res.items():
        if not isinstance(st, dict):
            continue
        assert st["n_compared"] > 0
        assert st["n_mismatch_bits"] == 0, (instr, fam, st["n_mismatch_bits"], st["first_mismatch_index"])
    one_pattern = configs.validate_against_mfma(instr, dict(presets.GFX950_MFMA[instr], nan_propagate=False), n_tiles=256)
    st = one_pattern["random_bits"]
    assert st["n_mismatch_bits"] > 0 and st["n_mismatch_bits"] == st["n_mismatch_nan_equiv"] and st["ulp_hist"][33] == 0
    if instr >= 77:
        return                                                                 # (the FDPA family takes no binary64 operands)
    chain = dict(presets.PAPER[("fma_chain", "fp32")], nan_bits=0xFFC00000, nan_propagate=True)      # the same chain in the FDPA family
    flushed = configs.validate_against_mfma(instr, dict(chain, ftz_in=True, ftz_out=True), n_tiles=256)
    assert flushed["tiny_products_c_subnormal"]["n_mismatch_bits"] > 0         # subnormals are kept, not flushed
    if mm.mfma_info(instr)["k"] > 1:
        fused = configs.validate_against_mfma(instr, dict(group_len=0, frac_bits=48, c_mode=mm.C_AFTER_EXACT, nan_bits=0x7FC00000), n_tiles=256)
        assert fused["normal"]["n_mismatch_bits"] > 0                          # one rounding per product, not one per dot product


@pytest.mark.parametrize("instr", [41, 42, 74, 75, 76])
def test_gfx950_fp32_instructions_keep_the_standard_signs_of_zero(env, instr):
    # operands drawn from zeros of both signs, +-1 and the smallest subnormals: many exact zeros.  The FMA family
    # (IEEE-754: a zero product and a zero accumulator of one sign keep it) agrees on every output; the chain expressed
    # in the FDPA family, where every exact zero is +0.0, differs exactly where the instruction returns -0.0.
    import numpy as np
    from gpu_utils import to_dev, dev_empty, to_host
    mm, configs, presets = env
    info = mm.mfma_info(instr)
    m, n, k, nb = info["m"], info["n"], info["k"], 64
    rng = np.random.default_rng(900 + instr)
    vals = np.array([0, 0x80000000, 0, 0x80000000, 0x3F800000, 0xBF800000, 0x00000001, 0x80000001], dtype=np.uint32)
    A, B, C = (to_dev(vals[rng.integers(0, len(vals), shp)]) for shp in ((nb, m, k), (nb, n, k), (nb, m, n)))
    Dhw, Dfma, Dchain = (dev_empty((nb, m, n), np.uint32) for _ in range(3))
    mm.mfma_probe(instr, A, B, C, Dhw, k, nb)
    f32 = (mm.FP32,) * 4
    h = mm.model_create(**presets.GFX950_MFMA[instr])
    mm.emulate_mma(h, A, B, C, Dfma, m, n, k, nb, f32)
    mm.model_destroy(h)
    h = mm.model_create(**dict(presets.PAPER[("fma_chain", "fp32")], nan_bits=0xFFC00000, nan_propagate=True))
    mm.emulate_mma(h, A, B, C, Dchain, m, n, k, nb, f32)
    mm.model_destroy(h)
    hw, fma, chain = (to_host(x, np.uint32) for x in (Dhw, Dfma, Dchain))
    assert np.array_equal(hw, fma)
    d = hw != chain
    assert np.count_nonzero(d) > 0 and np.all(hw[d] == 0x80000000) and np.all(chain[d] == 0)


@pytest.mark.parametrize("instr", list(range(10)) + list(range(35, 41)) + list(range(68, 74)))
def test_gfx950_16bit_and_fp8_presets_on_zeros_of_both_signs(env, instr):
    # the same directed family in the instruction's own operand types (zeros of both signs, +-1, the smallest
    # subnormals; accumulators from the same values, then zeros only): exact zeros from zeros, which the random
    # families almost never produce.  These instructions never return -0.0 there, and the presets agree on every output.
    import numpy as np
    from gpu_utils import to_dev, dev_empty, to_host
    mm, configs, presets = env
    codes = {mm.FP16: ([0, 0x8000, 0, 0x8000, 0x3C00, 0xBC00, 1, 0x8001], np.uint16), mm.BF16: ([0, 0x8000, 0, 0x8000, 0x3F80, 0xBF80, 1, 0x8001], np.uint16),
             mm.E4M3: ([0, 0x80, 0, 0x80, 0x38, 0xB8, 1, 0x81], np.uint8), mm.E5M2: ([0, 0x80, 0, 0x80, 0x3C, 0xBC, 1, 0x81], np.uint8)}
    info = mm.mfma_info(instr)
    m, n, k, ta, tb, nb = info["m"], info["n"], info["k"], info["a"], info["b"], 32
    rng = np.random.default_rng(950 + instr)
    va, vb = np.array(codes[ta][0], dtype=codes[ta][1]), np.array(codes[tb][0], dtype=codes[tb][1])
    vc = np.array([0, 0x80000000, 0, 0x80000000, 0x3F800000, 0xBF800000, 1, 0x80000001], dtype=np.uint32)
    h = mm.model_create(**presets.GFX950_MFMA[instr])
    for nc in (8, 2):
        A, B, C = to_dev(va[rng.integers(0, 8, (nb, m, k))]), to_dev(vb[rng.integers(0, 8, (nb, n, k))]), to_dev(vc[rng.integers(0, nc, (nb, m, n))])
        Dhw, Dm = dev_empty((nb, m, n), np.uint32), dev_empty((nb, m, n), np.uint32)
        mm.mfma_probe(instr, A, B, C, Dhw, k, nb)
        mm.emulate_mma(h, A, B, C, Dm, m, n, k, nb, (ta, tb, mm.FP32, mm.FP32))
        hw, md = to_host(Dhw, np.uint32), to_host(Dm, np.uint32)
        assert np.array_equal(hw, md), (instr, nc, int(np.count_nonzero(hw != md)))
        assert np.count_nonzero(hw == 0x80000000) == 0 and np.count_nonzero(hw == 0) > 0
    mm.model_destroy(h)


@pytest.mark.parametrize("instr", [10, 16, 22, 28, 34, 11, 29, 43, 55, 67])
def test_gfx950_block_scaled_presets_on_zeros_of_both_signs(env, instr):
    # the directed zero family on the block-scaled instructions (unit scales, then a spread of scale codes)
    import numpy as np
    from gpu_utils import to_dev, dev_empty, to_host
    mm, configs, presets = env
    codes = {mm.E4M3: [0, 0x80, 0, 0x80, 0x38, 0xB8, 1, 0x81], mm.E5M2: [0, 0x80, 0, 0x80, 0x3C, 0xBC, 1, 0x81],
             mm.E2M3: [0, 0x20, 0, 0x20, 0x08, 0x28, 1, 0x21], mm.E3M2: [0, 0x20, 0, 0x20, 0x0C, 0x2C, 1, 0x21],
             mm.E2M1: [0, 0x8, 0, 0x8, 0x2, 0xA, 1, 0x9]}
    info = mm.mfma_info(instr)
    m, n, k, ta, tb, nb = info["m"], info["n"], info["k"], info["a"], info["b"], 16
    rng = np.random.default_rng(980 + instr)
    va, vb = np.array(codes[ta], dtype=np.uint8), np.array(codes[tb], dtype=np.uint8)
    vc = np.array([0, 0x80000000, 0, 0x80000000, 0x3F800000, 0xBF800000, 1, 0x80000001], dtype=np.uint32)
    h = mm.model_create(**presets.GFX950_MFMA[instr])
    for nc, (lo, hi) in ((8, (127, 128)), (2, (127, 128)), (2, (100, 150))):
        A, B, C = to_dev(va[rng.integers(0, 8, (nb, m, k))]), to_dev(vb[rng.integers(0, 8, (nb, n, k))]), to_dev(vc[rng.integers(0, nc, (nb, m, n))])
        SA = to_dev(rng.integers(lo, hi, (nb, m, k // 32)).astype(np.uint8))
        SB = to_dev(rng.integers(lo, hi, (nb, n, k // 32)).astype(np.uint8))
        Dhw, Dm = dev_empty((nb, m, n), np.uint32), dev_empty((nb, m, n), np.uint32)
        mm.mfma_probe_scaled(instr, A, B, C, Dhw, SA, SB, k, nb)
        mm.emulate_mma_scaled(h, A, B, C, Dm, SA, SB, 32, m, n, k, nb, (ta, tb, mm.FP32, mm.FP32))
        hw, md = to_host(Dhw, np.uint32), to_host(Dm, np.uint32)
        assert np.array_equal(hw, md), (instr, nc, lo, hi, int(np.count_nonzero(hw != md)))
        assert np.count_nonzero(hw == 0) > 0
    mm.model_destroy(h)


def test_paper_cdna3_models_differ_from_gfx950(env):
    # the published CDNA3 parameter sets are close to, but not the same as, what gfx950 computes
    mm, configs, presets = env
    res = configs.validate_against_mfma(mm.MFMA_F32_16X16X32_FP8_FP8, dict(presets.PAPER[("cdna3", "fp8")], nan_bits=0xFFC00000),
                                        n_tiles=512)
    assert res["normal"]["n_mismatch_bits"] > 0
    res = configs.validate_against_mfma(mm.MFMA_F32_32X32X8_F16, dict(presets.PAPER[("cdna3", "fp16")], nan_bits=0xFFC00000),
                                        n_tiles=512)
    assert res["normal"]["n_mismatch_bits"] == 0            # indistinguishable on common distributions ...
    assert res["wide_exp_c_any"]["n_mismatch_bits"] > 0     # ... but not once zero operands carry large exponents


@pytest.mark.parametrize("instr", list(range(10, 35)) + list(range(43, 68)))
def test_gfx950_preset_reproduces_the_block_scaled_instruction(env, instr):
    # Algorithm "ST-FDPA" on the FP8 instructions' structure, against v_mfma_scale_f32_16x16x128_f8f6f4 (ids 10 .. 34)
    # and v_mfma_scale_f32_32x32x64_f8f6f4 (ids 43 .. 67): every input
    # family under every range of scale codes (unit, narrow, wide, all codes with NaN, and the bottom of binary32)
    mm, configs, presets = env
    res = configs.validate_scaled_against_mfma(instr, presets.GFX950_MFMA[instr], n_tiles=256 if instr < 43 else 64)
    assert res["kernel"].startswith("tiled") and "vm=3" in res["kernel"]
    for key, st in res.items():
        if not isinstance(st, dict):
            continue
        assert st["n_compared"] > 0
        assert st["n_mismatch_bits"] == 0, (instr, key, st["n_mismatch_bits"], st["first_mismatch_index"])


def test_block_scaled_model_needs_its_switches(env):
    mm, configs, presets = env
    instr = mm.MFMA_SCALE_F32_16X16X128_FP8_FP8
    good = presets.GFX950_MFMA[instr]
    # a single product of 2^128 and more is no infinity there: the overflow rule of Sec. 4.2 breaks agreement once
    # the scales are large
    res = configs.validate_scaled_against_mfma(instr, dict(good, wide_products=False), n_tiles=256)
    assert sum(res[("narrow", f)]["n_mismatch_bits"] for f in ("normal", "random_bits", "wide_exp_c_any")) == 0
    assert res[("all_codes", "normal")]["n_mismatch_bits"] > 0


@pytest.mark.parametrize("instr", [0, 1, 5, 7, 35])
def test_candidate_scan_singles_out_the_fitted_model(env, instr):
    # Step 4 on several candidates at once (one scan-kernel launch per family of inputs and class of candidates): the
    # fitted set reproduces the instruction on every input family; the paper's CDNA3 sets, T-FDPA sets and the fitted set
    # with a longer group fail somewhere, as does one or another of the fitted set with one switch taken away; and every count equals what the candidate gives on its own through
    # the plain emulation and comparison calls.
    mm, configs, presets = env
    fitted = presets.GFX950_MFMA[instr]
    fp8 = instr == 7
    cdna3 = presets.PAPER[("cdna3", "fp8" if fp8 else ("bf16" if instr in (1, 5) else "fp16"))]
    cands = [fitted, cdna3, dict(group_len=fitted["group_len"], frac_bits=24), dict(group_len=4, frac_bits=fitted["frac_bits"], out_round=mm.RZ),
             dict(fitted, skip_zero_terms=False), dict(fitted, f2_at_leading_bit=False), dict(fitted, sum_drop_distance=0),
             dict(fitted, group_len=2 * fitted["group_len"])]
    res = configs.scan_against_mfma(instr, cands, n_tiles=512, seeds=(0,))
    assert res["classes"][0] >= 1, res["classes"]                   # the fitted sets run in the scan kernel
    assert res["total"][0] == 0, (instr, res["mismatches"][0])
    assert all(res["total"][i] > 0 for i in (1, 2, 3, 7)), (instr, res["total"])
    assert sum(res["total"][4:7]) > 0, (instr, res["total"])         # (a single switch may need more inputs than these to show)
    for i in (0, 1, 4, 7):
        alone = configs.validate_against_mfma(instr, cands[i], n_tiles=512, seeds=(0,), fused=False)
        assert [alone[name]["n_mismatch_bits"] for name in res["families"]] == res["mismatches"][i], (instr, i)
