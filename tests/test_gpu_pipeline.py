"""GPU parity of the five-stage pipeline at reduced sizes (same code paths as the full shape): three layer
stacks sharing one slot pair, merger MLP, pooling, prefill + greedy decode, 10 Euler steps of the
cross-attending action head, trajectory projection — against oracle/pipeline.py."""
import numpy as np
import pytest

from oracle import pipeline as PL
from paper_2605_11678_amd import binding as B
from paper_2605_11678_amd import configs as CFG
from paper_2605_11678_amd.harness import Engine, VlaPipeline
from tests import parity_cases as PC

pytestmark = pytest.mark.gpu
TOL = 2e-2


def test_vla_pipeline_small_vs_oracle_and_residency_invariance():
    vit, dec, act = PC.pipe_small_modules()
    P = PC.PIPE_SMALL
    n_decode = P["n_decode"]
    eng = Engine(1 << 30, device=0)
    try:
        pipe = VlaPipeline(eng, vit, dec, act, n_patches=P["n_patches"], n_text=P["n_text"], n_actions=P["n_actions"],
                           matrix_gain=P["gain"])
        pipe.run(n_decode)
        got = pipe.results(n_decode)
        want = PC.pipeline_oracle()
        # each measure in units of its bound (tests/test_parity_discriminates.py shows that removing any sub-block
        # of any of the three stacks from the oracle moves one of them past 10)
        m = PC.pipeline_measures(got, want)
        print("pipeline measures / bound:", {k: "%.3f" % v for k, v in m.items()}, flush=True)
        assert max(m.values()) <= 1.0, m
        # integer ids are compared away from near-ties: with the default head seed (8) the oracle's smallest
        # top-1/top-2 logit gap over the 4 steps must be far above the bf16-level logit error
        srt = np.sort(want["logits"], axis=1)
        assert float(np.min(srt[:, -1] - srt[:, -2])) > 0.05
        assert got["tokens"] == want["tokens"], (got["tokens"], want["tokens"])
        # every module streamed / mixed / resident, sequential or pipelined, prefetch across passes or not:
        # the trajectory never changes by a bit (Table IX is stated on exactly this output: 64 waypoints x 3)
        ref = got["trajectory"].view(np.uint32).copy()
        ref_tok = got["tokens"]
        plans = [([0], [1], [0]), ([0, 1, 2], [0, 1, 2], [0, 1]), ([], [0, 2], [1]), ([], [], [])]
        for (rv, rd, ra), (mode, wrap) in zip(plans, [(0, 1), (0, 0), (1, 0), (0, 1)]):
            eng.ctx.set_residency(pipe.m_vit, rv)
            eng.ctx.set_residency(pipe.m_dec, rd)
            eng.ctx.set_residency(pipe.m_act, ra)
            eng.ctx.set_mode(mode, wrap)
            pipe.run(n_decode)
            out = pipe.results(n_decode)
            assert np.array_equal(out["trajectory"].view(np.uint32), ref), (rv, rd, ra, mode, wrap)
            assert out["tokens"] == ref_tok
    finally:
        eng.close()
