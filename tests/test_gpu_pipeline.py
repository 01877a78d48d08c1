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


def test_vla_pipeline_full_shape_vs_stored_oracle():
    """The five-stage pipeline at the shape bench.py times (27-layer encoder on 4096 patches, merger, 36-layer decoder
    over 1024 + 2048 positions, 8-layer action head cross-attending to the 3072 final-normed states, 10 Euler steps,
    64 x 3 trajectory) under the 16e9-byte arena, everything streamed, against oracle values stored by
    tests/golden/make_full_depth.py (part vla_full; the float64 oracle needs a quarter of an hour for it).  No decode
    steps: the generated tokens feed neither the action head nor the trajectory, and full-size single-token steps
    are compared in tests/test_gpu_fullsize.py.  Every measure is held to the stated 2e-2 (observed: final-normed
    decoder states 1.2e-2, action tokens 1.4e-3, trajectory 2.3e-3).  Which sub-block each measure can see is shown
    on the reduced pipeline and on the full-shape action head (tests/test_parity_discriminates.py); the oracle is
    too slow at this size to be run once more per removed sub-block.  A partially resident plan reproduces the
    bits (Table IX)."""
    import json
    import os
    gold = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    with open(os.path.join(gold, "full_depth_meta.json")) as f:
        meta = json.load(f)
    arrays = np.load(os.path.join(gold, "full_depth.npz"))
    m = meta["vla_full"]
    vit, dec, act = CFG.vit_encoder(), CFG.decoder_8b(), CFG.action_head()
    eng = Engine(16_000_000_000, device=0)
    try:
        pipe = VlaPipeline(eng, vit, dec, act, n_patches=m["n_patches"], n_text=m["n_text"], n_actions=m["n_actions"])
        pipe.run(0, m["n_euler"])
        got = pipe.results(0)
        rows = arrays["vla_full_hidden_ctx_rows"]
        e_ctx = float(np.max(np.abs(got["hidden_ctx"][rows].astype(np.float64) - arrays["vla_full_hidden_ctx_want"])))
        e_act = float(np.max(np.abs(got["actions"].astype(np.float64) - arrays["vla_full_actions"])))
        e_traj = float(np.max(np.abs(got["trajectory"].astype(np.float64) - arrays["vla_full_trajectory"])))
        measures = {
            "hidden_ctx": e_ctx / meta["vla_full_hidden_ctx"]["max_abs"] / TOL,
            "actions": e_act / m["actions_max_abs"] / TOL,
            "actions_contrib": e_act / m["actions_max_abs_contrib"] / PC.TOL_CONTRIB,
            "trajectory": e_traj / m["trajectory_max_abs"] / TOL,
        }
        print("full-shape pipeline, measures / bound:", {k: "%.3f" % v for k, v in measures.items()}, flush=True)
        assert max(measures.values()) <= 1.0, measures
        ref = got["trajectory"].view(np.uint32).copy()
        ref_act = got["actions"].view(np.uint32).copy()
        eng.ctx.set_residency(pipe.m_act, list(range(act.n_layers)))
        eng.ctx.set_residency(pipe.m_dec, B.place_interleaved(dec.n_layers, 18))
        pipe.run(0, m["n_euler"])
        out = pipe.results(0)
        assert np.array_equal(out["trajectory"].view(np.uint32), ref)
        assert np.array_equal(out["actions"].view(np.uint32), ref_act)
    finally:
        eng.close()
