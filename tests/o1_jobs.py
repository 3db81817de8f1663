"""Worker side of the tests that evaluate the rational-arithmetic form of the oracle in a process pool (it is pure
Python on exact fractions: about a thousand outputs a second on one core).  Imports the oracle only."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def o1_case(job):
    """job = (params as a dict of oracle.fdpa.ModelParams fields, A, B, C, ta, tb, SA, SB, block) -> D (uint32 bits)."""
    from oracle.fdpa import ModelParams, emulate_mma
    kw, A, B, C, ta, tb, SA, SB, block = job
    p = ModelParams(**kw)
    if SA is None:
        return emulate_mma(p, A, B, C, ta, tb)
    return emulate_mma(p, A, B, C, ta, tb, SA=SA, SB=SB, block=block)


def run_pool(jobs, workers=8):
    """Evaluates the jobs in spawned worker processes (spawned, not forked: the caller holds a GPU context)."""
    import multiprocessing as mp
    ctx = mp.get_context("spawn")
    with ctx.Pool(min(workers, max(1, len(jobs)))) as pool:
        return pool.map(o1_case, jobs, chunksize=1)
