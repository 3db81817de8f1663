"""The probing steps of paper Sec. 3.1 (Steps 1 to 3) run against the native MFMA instructions of the GPU and
against the parameter sets fitted to them, through the library: both sides must give the same observations (the
model-side ones are in turn checked against the CPU oracle by the parity tests)."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_10909_amd import binding, presets, probes
    return binding, presets, probes


@pytest.mark.parametrize("instr,scales", [(i, None) for i in list(range(10)) + [35, 36, 37, 40, 68, 69, 70, 73]] + [(10, (127, 127)), (11, (100, 154)), (15, (150, 104)), (16, (127, 127)), (43, (127, 127)), (49, (110, 144))])
def test_probes_agree_between_instruction_and_model(env, instr, scales):
    mm, presets, probes = env
    if scales is None:
        hw = probes.hardware(instr)
        md = probes.model(presets.GFX950_MFMA[instr], hw.m, hw.n, hw.k, hw.ta, hw.tb)
    else:       # the block-scaled instruction, all scales of A and of B at one code each (the two cancel: the probes
                # build products and accumulator on one scale)
        hw = probes.hardware_scaled(instr, *scales)
        md = probes.model_scaled(presets.GFX950_MFMA[instr], hw.m, hw.n, hw.k, hw.ta, hw.tb, *scales)
    assert probes.independence(hw, trials=16)
    assert probes.independence(md, trials=16)
    t_hw, t_md = probes.summation_table(hw), probes.summation_table(md)
    assert t_hw == t_md
    tree = probes.infer_tree(t_hw)
    text = probes.tree_to_string(tree)
    L = min(presets.GFX950_MFMA[instr]["group_len"], hw.k)      # (the multi-block forms have K = 4: one group of four)
    # chained swamped fused sums of L products and the running accumulator
    inner = "p%d" % hw.k
    for g in range(hw.k // L):
        inner = "F[" + ", ".join((["%s" % inner] if g else []) + ["p%d" % q for q in range(g * L, (g + 1) * L)] + ([] if g else [inner])) + "]"
    assert text.replace(" ", "") == inner.replace(" ", ""), text
    # precision among products of one sub-group (F), and across the two halves of an FP8 group (F_m)
    assert probes.fused_precision(hw, 0, 1, 2) == probes.fused_precision(md, 0, 1, 2) == presets.GFX950_MFMA[instr]["frac_bits"]
    across = presets.GFX950_MFMA[instr].get("frac_bits_merge") or presets.GFX950_MFMA[instr]["frac_bits"]
    if L > 2:
        assert probes.fused_precision(hw, 0, 1, L - 1) == probes.fused_precision(md, 0, 1, L - 1) == across
    assert probes.fused_precision(hw, 0, hw.k, 1) == probes.fused_precision(md, 0, hw.k, 1)
    assert probes.rounding_mode(hw, 0, 1, 23) == probes.rounding_mode(md, 0, 1, 23)
    assert probes.rounding_mode(hw, 0, hw.k, 23) == probes.rounding_mode(md, 0, hw.k, 23)


@pytest.mark.parametrize("instr,tree", [(41, "((((p0 + p4) + p1) + p2) + p3)"), (42, "((p0 + p2) + p1)")])
def test_probes_on_the_fp32_instructions_find_a_chain_of_fmas(env, instr, tree):
    # Sec. 4.1.2 and Figure "Examples of summation trees": one product joins the running sum per step (p_K = c)
    mm, presets, probes = env
    hw = probes.hardware(instr)
    md = probes.model(presets.GFX950_MFMA[instr], hw.m, hw.n, hw.k, hw.ta, hw.tb)
    assert probes.independence(hw, trials=16) and probes.independence(md, trials=16)
    t_hw, t_md = probes.summation_table(hw), probes.summation_table(md)
    assert t_hw == t_md
    assert probes.tree_to_string(probes.infer_tree(t_hw)).replace(" ", "") == tree.replace(" ", "")
    assert probes.fused_precision(hw, 0, 1, hw.k) == probes.fused_precision(md, 0, 1, hw.k) == 23      # each step rounds to binary32
    assert probes.rounding_mode(hw, 0, hw.k, 23) == probes.rounding_mode(md, 0, hw.k, 23) == "RNE"
