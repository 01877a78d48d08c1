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
        ref_bits = g.forward_bits(x)
        # every residency set, both modes, both prefetch settings, two slots and one: identical bits (Table IX)
        for n_slots in (2, 1):
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


def small_encoder():
    # head dim 72 (padded to 96 inside the attention kernel), d_ff not a multiple of 32, biases, LayerNorm
    return CFG.ModuleConfig("enc_small", 2, 144, 2, 2, 72, 536, CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, seed_base=4100)


def small_gqa(dh):
    return CFG.ModuleConfig("gqa_small", 2, 8 * dh, 8, 2, dh, 1056, CFG.NORM_RMS, CFG.ACT_SWIGLU, 0, 1, 1e6,
                            max_seq=384, seed_base=4200 + dh, vocab=0)


@pytest.mark.parametrize("T", [1, 77, 333])
def test_encoder_ragged_shapes(T):
    c = small_encoder()
    x = CFG.make_tokens(T, c.d_model, seed=17)
    g = GpuStack(c, max_tokens=T)
    try:
        want = oracle_stack(c, g.weights, x)
        got = g.forward(x)
        assert rel_err(got, want) <= TOL, rel_err(got, want)
    finally:
        g.close()


@pytest.mark.parametrize("dh", [64, 128])
def test_gqa_decoder_prefill_chunks_and_decode(dh):
    c = small_gqa(dh)
    T0, T1, T2, steps = 200, 70, 13, 3
    x = CFG.make_tokens(T0 + T1 + T2 + steps, c.d_model, seed=23)
    g = GpuStack(c, max_tokens=T0)
    try:
        kv = F.new_kv_cache(oracle_cfg(c))
        want0 = oracle_stack(c, g.weights, x[:T0], 0, kv)
        got0 = g.forward(x[:T0], 0)
        assert rel_err(got0, want0) <= TOL
        # a second chunk at pos0 > 0 attends over the cache of the first
        want1 = oracle_stack(c, g.weights, x[T0:T0 + T1], T0, kv)
        got1 = g.forward(x[T0:T0 + T1], T0)
        assert rel_err(got1, want1) <= TOL
        # a third chunk whose first position is not a multiple of 8 (the transposed-V append falls back to 2-byte stores)
        want2 = oracle_stack(c, g.weights, x[T0 + T1:T0 + T1 + T2], T0 + T1, kv)
        got2 = g.forward(x[T0 + T1:T0 + T1 + T2], T0 + T1)
        assert rel_err(got2, want2) <= TOL
        for s in range(steps):
            p = T0 + T1 + T2 + s
            want = oracle_stack(c, g.weights, x[p:p + 1], p, kv)
            got = g.forward(x[p:p + 1], p)      # single-token kernels
            assert rel_err(got, want) <= TOL, (s, rel_err(got, want))
    finally:
        g.close()


@pytest.mark.parametrize("T,n_ctx,heads,dh", [(64, 150, 2, 128), (64, 700, 2, 128), (20, 1100, 4, 64), (128, 515, 3, 72)],
                         ids=["short-context", "split-ragged-last-run", "split-gqa-wavefronts", "split-padded-head-dim"])
def test_cross_attention_module(T, n_ctx, heads, dh):
    """Cross-attention to a context.  From 512 context positions on (and at most 128 queries) the key range is split
    over several workgroups and merged by a second launch; the cases cover a ragged last run (700 = 10 tiles + 60
    positions), four query heads per KV head (the wavefronts of a workgroup are heads) and a padded head dimension."""
    c = CFG.ModuleConfig("cross_small", 2, 256, heads, 1 if heads == 4 else heads, dh, 512,
                         CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, d_ctx=384, seed_base=4300)
    x = CFG.make_tokens(T, c.d_model, seed=31)
    ctx = CFG.make_tokens(n_ctx, c.d_ctx, seed=32)
    g = GpuStack(c, max_tokens=T, max_ctx=n_ctx)
    try:
        want = oracle_stack(c, g.weights, x, ctx=ctx.astype(np.float64))
        got = g.forward(x, ctx=ctx)
        assert rel_err(got, want) <= TOL, rel_err(got, want)
    finally:
        g.close()


def test_decoder_without_cache_rotates_k_in_place():
    """No KV cache: K is rotated inside the QKV rows and attention reads it from there (ragged T)."""
    c = small_gqa(64)
    c.max_seq = 0
    T = 130
    x = CFG.make_tokens(T, c.d_model, seed=43)
    g = GpuStack(c, max_tokens=T)
    try:
        want = oracle_stack(c, g.weights, x)
        got = g.forward(x)
        assert rel_err(got, want) <= TOL, rel_err(got, want)
    finally:
        g.close()


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
