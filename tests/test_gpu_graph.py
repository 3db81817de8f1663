"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset nodes), so one
closed-loop step -- generate, native MFMA, model, compare (Sec. 3.1 Step 4) -- can be captured in a HIP graph.  Every
replay, with eager work and synchronisations in between, must reproduce the eager result."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_closed_loop_step_replays_from_a_hip_graph():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_10909_amd import binding as mm, presets
    from gpu_utils import dev_empty, to_host
    instr = mm.MFMA_F32_16X16X32_FP8_BF8
    info = mm.mfma_info(instr)
    m, n, k, ta, tb = info["m"], info["n"], info["k"], info["a"], info["b"]
    nt = 512
    A, B = dev_empty((nt, m, k)), dev_empty((nt, n, k))
    C, Dhw, D0, D1 = (dev_empty((nt, m, n), np.uint32) for _ in range(4))
    st0, st1 = dev_empty(mm.STATS_BYTES), dev_empty(mm.STATS_BYTES)
    good = mm.model_create(**presets.GFX950_MFMA[instr])
    other = mm.model_create(**dict(presets.PAPER[("cdna3", "fp8")], nan_bits=0xFFC00000))
    dt = (ta, tb, mm.FP32, mm.FP32)

    def step():
        mm.generate(A, ta, m * k, 0, nt, mm.GEN_RANDOM_BITS, seed=3, operand=0)
        mm.generate(B, tb, n * k, 0, nt, mm.GEN_RANDOM_BITS, seed=3, operand=1)
        mm.generate(C, mm.FP32, m * n, 0, nt, mm.GEN_UNIFORM_EXP, seed=3, operand=2, exp_lo=100, exp_hi=140)
        mm.mfma_probe(instr, A, B, C, Dhw, k, nt)
        mm.emulate_mma(good, A, B, C, D0, m, n, k, nt, dt)
        mm.emulate_mma(other, A, B, C, D1, m, n, k, nt, dt)
        mm.stats_reset(st0)
        mm.stats_reset(st1)
        mm.compare(D0, Dhw, nt * m * n, st0)
        mm.compare(D1, Dhw, nt * m * n, st1)

    step()
    torch.cuda.synchronize()
    eager0, eager1, eager_d = mm.read_stats(st0), mm.read_stats(st1), to_host(D0, np.uint32).copy()
    assert eager0["n_compared"] == nt * m * n and eager0["n_mismatch_bits"] == 0 and eager1["n_mismatch_bits"] > 0

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                      # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(4):
        for t in (A, B, C, Dhw, D0, D1, st0, st1):  # eager work between the replays: wipe everything the graph writes
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert mm.read_stats(st0) == eager0, replay
        assert mm.read_stats(st1) == eager1, replay
        assert np.array_equal(to_host(D0, np.uint32), eager_d), replay
    mm.model_destroy(good)
    mm.model_destroy(other)
