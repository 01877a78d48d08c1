"""GPU parity at the benchmark's full shapes, in the launch configuration bench.py times.

(a) one layer of the 8B-class shape against the oracle run live (every kernel at its real tile counts and grid), once
    as stated and once with the feed-forward zeroed so that the attention kernels are judged alone;
(b) the full-depth stacks, the 27-layer encoder at 4096 tokens and the 36-layer decoder at 3072 tokens followed by 8
    greedy steps through the 4096 x 32768 head, against oracle values stored by tests/golden/make_full_depth.py (a
    script that calls only the oracle: the float64 oracle needs ~10 minutes per 36-layer pass), at sampled rows (every
    61st / 83rd and the last, all columns), the maxima the error measures divide by taken over the whole output;
(c) properties that hold at any size: streamed, partially resident and fully resident passes agree bit for bit
    (Table IX), and so do repeated passes;
(d) a 16384-token prompt (the length at which a layer of this part executes longer than its copy takes, the regime
    of Sec. IV-C / Table IV that bench.py's long-prefill leg measures) through one 8B-class layer, against the oracle
    on three chunks of rows that it computes on their own."""
import json
import os

import numpy as np
import pytest

from paper_2605_11678_amd import binding as B
from paper_2605_11678_amd import configs as CFG
from tests import parity_cases as PC
from tests.gpu_common import GpuStack

pytestmark = pytest.mark.gpu
GOLD_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden():
    with open(os.path.join(GOLD_DIR, "full_depth_meta.json")) as f:
        meta = json.load(f)
    return np.load(os.path.join(GOLD_DIR, "full_depth.npz")), meta


def check_sampled(got, arrays, meta, key, what, contrib=True, tol=PC.TOL):
    """Both error measures on the stored rows; the denominators are the stored maxima over the whole oracle output."""
    rows = arrays[key + "_rows"]
    diff = np.abs(got[rows].astype(np.float64) - arrays[key + "_want"])
    want = np.abs(arrays[key + "_want"].astype(np.float64))
    err = float(np.max(diff))
    r, c_ = np.unravel_index(np.argmax(diff), diff.shape)
    print("  %s: worst element at row %d col %d (|want| there %.3f, row max %.3f); rms error / rms value %.3e; "
          "worst row-relative error %.3e" % (key, rows[r], c_, want[r, c_], want[r].max(),
                                            float(np.sqrt(np.mean(diff ** 2)) / np.sqrt(np.mean(want ** 2))),
                                            float(np.max(diff.max(axis=1) / want.max(axis=1)))), flush=True)
    s = err / meta[key]["max_abs"]
    c = err / meta[key]["max_abs_contrib"] if contrib else 0.0
    print("parity %s (%d sampled rows): stated %.3e (<= %.0e)  contrib %.3e (<= %.0e)" %
          (what, len(rows), s, tol, c, tol), flush=True)
    assert s <= tol, (what, "stated", s)
    assert c <= tol, (what, "contrib", c)


@pytest.mark.parametrize("name", ["dec8b_L1", "dec8b_L1_attn", "act_L8", "act_L8_cross", "vit_L1_T8192", "vit_L1_T8192_attn"])
def test_full_shape_case_vs_oracle_live(name):
    """Oracle run live.  dec8b_*: one 8B-class layer, 3072-token prefill, then two single-token passes over the
    3072-entry cache.  act_*: the 8-layer action head, 64 tokens cross-attending to a 3072 x 4096 context (the split
    cross-attention path).  vit_L1_T8192: one encoder layer over 8192 patches.  The *_attn / *_cross variants zero the
    other sub-blocks so that the attention kernels are judged alone (tests/parity_cases.py says why)."""
    case = PC.full_cases()[name]
    x, ctx = case.x(), case.ctx()
    g = GpuStack(case.cfg, max_tokens=case.max_tokens, max_ctx=case.n_ctx, cap_bytes=3 << 30, weights=case.weights())
    try:
        want = PC.oracle_passes(case)
        bits = None
        for (p, t), w in zip(case.passes, want):
            got = g.forward(x[p:p + t], p, ctx=ctx)
            PC.check(got, w, x[p:p + t], "%s pos0=%d T=%d" % (name, p, t))
            if p == 0:
                bits = got.view(np.uint32).copy()
        g.eng.ctx.set_residency(g.mid, [0])
        p0, t0 = case.passes[0]
        assert np.array_equal(g.forward_bits(x[:t0], ctx=ctx), bits)
    finally:
        g.close()


@pytest.mark.parametrize("attention_alone", [False, True])
def test_long_prompt_one_layer_sampled_chunks_vs_oracle(attention_alone):
    """16384 tokens through one 8B-class layer (64 x 96 GEMM tiles of 256 x 256 in the gate/up product, 512 query
    blocks per head, causal jobs of up to 256 K/V tiles), against the oracle on three chunks of rows (the first rows,
    a ragged chunk across the middle, the last rows: tests/parity_cases.py says how the oracle gets them without
    running the whole pass).  Both measures divide by maxima over the sampled rows only (smaller than over the whole
    output: stricter).  tests/test_parity_discriminates.py shows which sub-block each variant can see."""
    case = PC.long_prompt_case(attention_alone)
    x = case.x()
    g = GpuStack(case.cfg, max_tokens=PC.LONG_T, cap_bytes=6 << 30, weights=case.weights())
    try:
        got = g.forward(x)
        rows, want = PC.long_prompt_oracle(case, x=x)
        PC.check(got[rows], want, x[rows], "%s, %d sampled rows" % (case.name, len(rows)))
        bits = got.view(np.uint32).copy()
        g.eng.ctx.set_residency(g.mid, [0])
        assert np.array_equal(g.forward_bits(x), bits)
    finally:
        g.close()


def test_vit_full_depth_vs_stored_oracle():
    """27 layers, 4096 tokens, head dimension 72: streamed, against the stored oracle output; then k = 13 (Eq. 8
    placement) and k = 27 reproduce the bits."""
    arrays, meta = golden()
    case = PC.full_cases()["vit_L27"]
    x = case.x()
    g = GpuStack(case.cfg, max_tokens=4096, cap_bytes=2 << 30, weights=case.weights())
    try:
        got = g.forward(x)
        check_sampled(got, arrays, meta, "vit_L27", "27-layer encoder T=4096")
        ref = got.view(np.uint32)
        for k in (13, 27):
            g.eng.ctx.set_residency(g.mid, B.place_interleaved(27, k))
            assert np.array_equal(g.forward_bits(x), ref), k
    finally:
        g.close()


def test_decoder_8b_full_depth_prefill_greedy_and_bit_identity_under_16e9_cap():
    """All 36 layers, 3072 tokens, 16e9-byte arena.  The prefill output (raw and final-normed) and 8 greedy steps
    (token ids, the 32768 logits of every step, the hidden state after every step) against the stored oracle values;
    k = 0, 18 (Eq. 8 placement), 36, sequential mode and a repeat agree bit for bit."""
    arrays, meta = golden()
    case = PC.full_cases()["dec8b_L36"]
    c = case.cfg
    gm = meta["greedy"]
    head = CFG.make_head(c, seed=gm["head_seed"])
    T, L, d = 3072, c.n_layers, c.d_model
    x = case.x()
    g = GpuStack(c, max_tokens=T, cap_bytes=16_000_000_000, weights=case.weights(), head=head)
    try:
        got = g.forward(x)
        ref = got.view(np.uint32).copy()
        g.eng.ctx.final_norm(g.mid, g.yp, g.np_, T)
        fin = g.eng.download(g.nv[:T * d]).reshape(T, d)
        D36 = PC.TOL_DEPTH36       # BF16 operands alone cost 2.2e-2 at this depth under the stated recipe: see parity_cases.py
        check_sampled(fin, arrays, meta, "dec8b_L36_final", "36-layer decoder, final-normed hidden states", contrib=False, tol=D36)
        check_sampled(got, arrays, meta, "dec8b_L36", "36-layer decoder prefill T=3072", tol=D36)
        # greedy steps, streamed (k = 0): ids identical, logits and hidden states within tolerance
        toks, logits, hs = arrays["greedy_tokens"], arrays["greedy_logits"], arrays["greedy_hidden"]
        E = B_bits_to_f32(head[CFG.R_EMBED])
        h_ptr = g.yp + 4 * (T - 1) * d
        lg = np.empty(c.vocab, np.float32)
        worst_logit, worst_sigma = 0.0, 0.0
        for s in range(gm["steps"]):
            t = g.eng.ctx.logits_argmax(g.mid, h_ptr, lg)
            dl = lg.astype(np.float64) - logits[s]
            e_logit = float(np.max(np.abs(dl)))
            worst_logit = max(worst_logit, e_logit)
            # Integer ids are compared away from near-ties.  An id flips when the error of the DIFFERENCE of the two
            # leading logits exceeds the oracle's gap between them; the error of one given logit is of the size of the
            # RMS over the 32768 (the maximum over all of them is an extreme value), so the gap is held to three
            # standard deviations of that difference.
            sigma = float(np.sqrt(np.mean(dl ** 2)))
            worst_sigma = max(worst_sigma, sigma)
            assert gm["margins"][s] > 3.0 * np.sqrt(2.0) * sigma, (s, gm["margins"][s], sigma)
            assert e_logit <= PC.TOL_DEPTH36 * float(np.max(np.abs(logits[s]))), (s, e_logit)
            assert t == int(toks[s]), (s, t, int(toks[s]))
            g.eng.ctx.embed_token(g.mid, t, g.xp)
            g.eng.ctx.forward(g.mid, g.xp, g.yp, 1, T + s)
            h = g.eng.download(g.yv[:d])
            PC.check(h[None, :], hs[s][None, :].astype(np.float64), E[t][None, :],
                     "greedy step %d (token %d, logit err %.2e)" % (s, t, e_logit), tol=D36, tol_contrib=D36)
            h_ptr = g.yp
        print("logits: worst abs error %.3e, worst RMS error %.3e, smallest oracle margin %.3f" %
              (worst_logit, worst_sigma, min(gm["margins"])), flush=True)
        # residency never changes a bit
        for k in (18, 36, 0):
            g.eng.ctx.set_residency(g.mid, B.place_interleaved(L, k))
            assert np.array_equal(g.forward_bits(x), ref), k
        g.eng.ctx.set_mode(B.DL_MODE_SEQUENTIAL, 0)
        assert np.array_equal(g.forward_bits(x), ref)
        # the arena is the cap: a block larger than what is left is refused
        left = g.eng.ctx.arena_stats()
        with pytest.raises(B.DLError) as e:
            g.eng.ctx.arena_alloc(left["capacity"] - left["used"] + 4096)
        assert e.value.code == B.DL_ERR_BUDGET_EXCEEDED
    finally:
        g.close()


def B_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
