"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same seeded inputs.

Tolerance (stated by the benchmark spec): max |gpu - oracle| / max |oracle| <= 2e-2 on final hidden states.
Integer results (greedy token ids) must be identical; streamed, partially resident and fully
resident runs must agree bit for bit (the paper's Table IX)."""
import itertools

import numpy as np
import pytest

from oracle import forward as F
from paper_2605_11678_amd import binding as B
from paper_2605_11678_amd import configs as CFG
from tests import parity_cases as PC
from tests.gpu_common import GpuStack, oracle_cfg, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
TINY_HEAD_SEED = 12


def oracle_stack(c, weights, x, pos0=0, kv=None, ctx=None, final=None):
    h = F.stack_forward(oracle_cfg(c), weights, x, pos0, kv, ctx)
    if final is not None:
        return F.final_norm(oracle_cfg(c), h, final[CFG.R_FINAL_NORM_G], final.get(CFG.R_FINAL_NORM_B))
    return h


def test_tiny_decoder_prefill_parity_and_bit_identity():
    c = CFG.tiny_decoder()
    T = 128
    x = CFG.make_tokens(T, c.d_model, seed=7)
    g = GpuStack(c, max_tokens=T)
    try:
        want = oracle_stack(c, g.weights, x, final=g.head)
        got = g.forward(x, final_norm=True)
        assert rel_err(got, want) <= TOL, rel_err(got, want)
        print("tiny decoder, final-normed hidden states: %.3e" % rel_err(got, want), flush=True)
        ref_bits = g.forward_bits(x)
        # every residency set, both modes, both prefetch settings, one to four slots: identical bits (Table IX)
        for n_slots in (2, 1, 3, 4):
            g.eng.ctx.set_residency(g.mid, [])
            g.eng.ctx.set_slot_count(n_slots)
            for mask in itertools.product([0, 1], repeat=c.n_layers):
                g.eng.ctx.set_residency(g.mid, [i for i in range(c.n_layers) if mask[i]])
                for mode, wrap in ((B.DL_MODE_PIPELINED, 0), (B.DL_MODE_PIPELINED, 1), (B.DL_MODE_SEQUENTIAL, 0)):
                    g.eng.ctx.set_mode(mode, wrap)
                    for rep in range(2):
                        assert np.array_equal(g.forward_bits(x), ref_bits), (n_slots, mask, mode, wrap, rep)
    finally:
        g.close()


def test_tiny_decoder_greedy_ids_identical():
    c = CFG.tiny_decoder()
    T, steps = 128, 8
    x = CFG.make_tokens(T, c.d_model, seed=7)
    # head seed 12: of seeds 8..19 the one whose oracle top-1/top-2 margin over the 8 steps is widest (0.026);
    # chosen on the oracle alone, so that integer ids are compared away from near-ties
    g = GpuStack(c, max_tokens=T, head=CFG.make_head(c, seed=TINY_HEAD_SEED))
    try:
        toks, logits, hs = F.generate_greedy(oracle_cfg(c), g.weights, g.head, x, steps)
        for k in (0, 2, 4):
            g.eng.ctx.set_residency(g.mid, B.place_interleaved(c.n_layers, k))
            g.eng.ctx.set_mode(B.DL_MODE_PIPELINED, 1)
            g.eng.upload(g.xv[:T * c.d_model], x)
            g.eng.ctx.forward(g.mid, g.xp, g.yp, T, 0)
            h_ptr = g.yp + 4 * (T - 1) * c.d_model
            got_toks, worst_logit_err = [], 0.0
            lg = np.empty(c.vocab, np.float32)
            for s in range(steps):
                t = g.eng.ctx.logits_argmax(g.mid, h_ptr, lg)
                got_toks.append(t)
                worst_logit_err = max(worst_logit_err, float(np.max(np.abs(lg - logits[s]))))
                g.eng.ctx.embed_token(g.mid, t, g.xp)
                g.eng.ctx.forward(g.mid, g.xp, g.yp, 1, T + s)
                h_ptr = g.yp
            # the oracle's own top-1 / top-2 margin must dominate the observed logit error, else the
            # comparison of integer ids would rest on a near-tie
            srt = np.sort(logits, axis=1)
            margin = float(np.min(srt[:, -1] - srt[:, -2]))
            assert margin > 10 * worst_logit_err, (margin, worst_logit_err)
            assert got_toks == toks, (k, got_toks, toks)
            h_last = g.eng.download(g.yv[:c.d_model])
            assert rel_err(h_last, hs[-1]) <= TOL
        # device-side feedback (no host round trip per token) gives the same ids
        g.eng.upload(g.xv[:T * c.d_model], x)
        g.eng.ctx.forward(g.mid, g.xp, g.yp, T, 0)
        tp, tv = g.eng.alloc_f32(steps)
        h_ptr = g.yp + 4 * (T - 1) * c.d_model
        for s in range(steps):
            g.eng.ctx.greedy_step(g.mid, h_ptr, tp + 4 * s, g.xp)
            g.eng.ctx.forward(g.mid, g.xp, g.yp, 1, T + s)
            h_ptr = g.yp
        assert g.eng.download(tv).view(np.int32).tolist() == toks
        # the workspace shrunk to single-token passes between the prefill and the decode steps: the KV cache
        # survives, the ids are the same, and the freed bytes are there for one more resident layer
        g.eng.ctx.set_residency(g.mid, [])
        g.eng.upload(g.xv[:T * c.d_model], x)
        g.eng.ctx.forward(g.mid, g.xp, g.yp, T, 0)
        h_ptr = g.yp + 4 * (T - 1) * c.d_model
        prefill_out = g.eng.download(g.yv[:T * c.d_model])
        used_long = g.eng.ctx.arena_stats()["used"]
        g.eng.ctx.module_set_max_tokens(g.mid, 1)
        assert g.eng.ctx.arena_stats()["used"] < used_long
        g.eng.ctx.set_residency(g.mid, [1, 3])
        g.eng.upload(tv, np.zeros(steps, np.float32))
        for s in range(steps):
            g.eng.ctx.greedy_step(g.mid, h_ptr, tp + 4 * s, g.xp)
            g.eng.ctx.forward(g.mid, g.xp, g.yp, 1, T + s)
            h_ptr = g.yp
        assert g.eng.download(tv).view(np.int32).tolist() == toks
        with pytest.raises(B.DLError):
            g.eng.ctx.forward(g.mid, g.xp, g.yp, 2, 0)
        # grown back, the prefill runs again and reproduces its earlier output bit for bit
        g.eng.ctx.set_residency(g.mid, [])
        g.eng.ctx.module_set_max_tokens(g.mid, T)
        g.eng.upload(g.xv[:T * c.d_model], x)
        g.eng.ctx.forward(g.mid, g.xp, g.yp, T, 0)
        again = g.eng.download(g.yv[:T * c.d_model])
        assert np.array_equal(again.view(np.uint32), prefill_out.view(np.uint32))
    finally:
        g.close()


@pytest.mark.parametrize("case", PC.CASES, ids=[c.name for c in PC.CASES])
def test_case_vs_oracle(case):
    """Every pass of every parity case (tests/parity_cases.py: ragged encoder shapes with a padded head dimension,
    chunked GQA prefill over a cache followed by single-token passes, a decoder without a cache, cross-attention
    with and without the key-range split) against the oracle, on both error measures.  Each case is shown to be
    able to fail by tests/test_parity_discriminates.py."""
    c = case.cfg
    x, ctx = case.x(), case.ctx()
    want = PC.oracle_passes(case)
    g = GpuStack(c, max_tokens=case.max_tokens, max_ctx=case.n_ctx, weights=case.weights())
    try:
        for (p, t), w in zip(case.passes, want):
            got = g.forward(x[p:p + t], p, ctx=ctx)
            PC.check(got, w, x[p:p + t], "%s pos0=%d T=%d" % (case.name, p, t))
    finally:
        g.close()


def small_gqa(dh):
    return CFG.ModuleConfig("gqa_small", 2, 8 * dh, 8, 2, dh, 1056, CFG.NORM_RMS, CFG.ACT_SWIGLU, 0, 1, 1e6,
                            max_seq=384, seed_base=4200 + dh, vocab=0)


def test_identity_layer_is_exact():
    """A block whose output projections are zero must return its input bit for bit."""
    c = small_gqa(64)
    c.max_seq = 0
    c.causal = 1

    def weights(l):
        w = CFG.make_layer_weights(c, l)
        w[CFG.T_WO] = np.zeros_like(w[CFG.T_WO])
        w[CFG.T_W_DOWN] = np.zeros_like(w[CFG.T_W_DOWN])
        return w
    T = 130
    x = CFG.make_tokens(T, c.d_model, seed=41)
    g = GpuStack(c, max_tokens=T, weights=weights)
    try:
        assert np.array_equal(g.forward(x), x)
    finally:
        g.close()


def test_enqueuing_calls_are_refused_before_the_streams_are_set():
    """A device context without streams must return DL_ERR_BAD_STATE from every call that would launch a kernel,
    not fall back to the null stream."""
    import torch
    ctx = B.Context(0)
    try:
        arena = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
        ctx.set_arena(arena.data_ptr(), arena.numel(), keep=arena)
        a = ctx.arena_alloc(4096)
        b = ctx.arena_alloc(4096)
        for call in (lambda: ctx.axpy(a, 0.5, b, 16),
                     lambda: ctx.mean_pool(a, b, 4, 2, 8),
                     lambda: ctx.add_time_embedding(a, b, 0.3, 4, 8)):
            with pytest.raises(B.DLError) as e:
                call()
            assert e.value.code == B.DL_ERR_BAD_STATE
    finally:
        ctx.destroy()
