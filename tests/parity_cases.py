"""The GPU parity cases as data, shared by the GPU tests (which run them through the C ABI) and by the CPU
test that checks each case can fail (tests/test_parity_discriminates.py).

Two error measures are asserted on every compared stack output y for input x:
  stated  = max|gpu - oracle| / max|oracle|        <= TOL          (the tolerance the benchmark spec states)
  contrib = max|gpu - oracle| / max|oracle - x|    <= TOL_CONTRIB  (error relative to what the stack ADDED to
            its input: the fp32 residual stream carries x through exactly, so `stated` alone cannot see a
            sub-block whose contribution is small next to x)
A case is discriminating when removing any of its sub-blocks from the ORACLE moves one of the two measures to at
least 10x its bound (DISCRIMINATION), i.e. a GPU kernel that returned zeros for that sub-block would fail the case
by an order of magnitude.  Nothing here touches the HIP path; inputs come from the seeded generators only."""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

from oracle import forward as F
from paper_2605_11678_amd import configs as CFG

TOL = 2e-2
TOL_CONTRIB = 2e-2
DISCRIMINATION = 10.0
# gain of one linear map at the 8B-class shape under the stated N(0, 0.02) recipe: 0.02 * sqrt(4096)
GAIN_8B = 1.28


def stated_err(got, want):
    return float(np.max(np.abs(np.asarray(got, np.float64) - want)) / np.max(np.abs(want)))


def contrib_err(got, want, x):
    return float(np.max(np.abs(np.asarray(got, np.float64) - want)) / np.max(np.abs(want - np.asarray(x, np.float64))))


# The 36-layer 8B-class decoder under the stated recipe amplifies perturbations from layer to layer (a gain of 1.28
# per linear map): rounding the operands of every matrix product to BF16, which is the arithmetic the method is stated
# in, puts ANY implementation 2.1e-2 .. 2.2e-2 from the exact result at that depth (tests/test_bf16_depth_error.py shows
# it in numpy alone, no GPU involved).  Full-depth decoder outputs are therefore held to 3e-2; every other case, the
# 27-layer encoder included, to the stated 2e-2.
TOL_DEPTH36 = 3e-2


def check(got, want, x, what="", tol=TOL, tol_contrib=TOL_CONTRIB):
    """Asserts both measures; returns them (the tests print them)."""
    s, c = stated_err(got, want), contrib_err(got, want, x)
    print("parity %s: stated %.3e (<= %.0e)  contrib %.3e (<= %.0e)" % (what, s, tol, c, tol_contrib), flush=True)
    assert s <= tol, (what, "stated", s)
    assert c <= tol_contrib, (what, "contrib", c)
    return s, c


@dataclass
class Case:
    name: str
    cfg: CFG.ModuleConfig
    passes: List[Tuple[int, int]]          # (pos0, n_tokens) in order; pos0 > 0 needs a KV cache
    x_seed: int
    gain: float = GAIN_8B                  # 0: the stated N(0, 0.02) recipe
    n_ctx: int = 0
    ctx_seed: int = 0
    blind: Tuple[str, ...] = ()            # mutations this case cannot see (must be seen by `covered_by`)
    covered_by: str = ""
    zero: Tuple[int, ...] = ()             # tensor ids set to zero in the case's own weights (GPU and oracle alike)

    @property
    def max_tokens(self):
        return max(t for _, t in self.passes)

    def weights(self):
        gen = lambda l: CFG.make_layer_weights(self.cfg, l, self.gain)
        return zeroed(gen, self.zero) if self.zero else gen

    def x(self):
        n = max(p + t for p, t in self.passes)
        return CFG.make_tokens(n, self.cfg.d_model, seed=self.x_seed)

    def ctx(self):
        return CFG.make_tokens(self.n_ctx, self.cfg.d_ctx, seed=self.ctx_seed) if self.n_ctx else None


def oracle_passes(case: Case, weights=None, cfg_over=None):
    """Oracle output of every pass of the case (optionally with mutated weights / descriptor)."""
    cfg = case.cfg.as_dict()
    if cfg_over:
        cfg.update(cfg_over)
    gen = weights or case.weights()
    x = case.x()
    ctx = case.ctx()
    ctx = None if ctx is None else ctx.astype(np.float64)
    kv = F.new_kv_cache(cfg) if case.cfg.max_seq > 0 else None
    return [F.stack_forward(cfg, gen, x[p:p + t], p, kv, ctx) for p, t in case.passes]


def zeroed(gen, tids):
    def g(l):
        w = dict(gen(l))
        for t in tids:
            if t in w:
                w[t] = np.zeros_like(w[t])
        return w
    return g


# name -> (applies(case), lambda case: (weights, cfg_over)): every mutation removes one sub-block from the oracle
MUTATIONS = {
    "self_attention": (lambda c: CFG.T_WO not in c.zero, lambda c: (zeroed(c.weights(), [CFG.T_WO, CFG.T_BO]), None)),
    "cross_attention": (lambda c: c.cfg.d_ctx > 0, lambda c: (zeroed(c.weights(), [CFG.T_WO_C, CFG.T_BO_C]), None)),
    "ffn": (lambda c: CFG.T_W_DOWN not in c.zero, lambda c: (zeroed(c.weights(), [CFG.T_W_DOWN, CFG.T_B_DOWN]), None)),
    "rope": (lambda c: c.cfg.rope_theta > 0, lambda c: (None, dict(rope_theta=0.0))),
    "causal_mask": (lambda c: bool(c.cfg.causal), lambda c: (None, dict(causal=0))),
}


def mutation_ratio(case: Case, mutation: str, base=None):
    """Per pass: how far the mutated oracle sits from the oracle, in units of the asserted bounds
    (max over the two measures).  A single-token pass has no mask to drop: causal_mask gives None there."""
    _, make = MUTATIONS[mutation]
    w, over = make(case)
    base = base if base is not None else oracle_passes(case)
    mut = oracle_passes(case, w, over)
    x = case.x()
    out = []
    for (p, t), b, m in zip(case.passes, base, mut):
        if mutation == "causal_mask" and t == 1:
            out.append(None)
            continue
        out.append(max(stated_err(m, b) / TOL, contrib_err(m, b, x[p:p + t]) / TOL_CONTRIB))
    return out


def _enc_small():
    # head dim 72 (padded inside the attention kernel), d_ff not a multiple of 32, biases, LayerNorm
    return CFG.ModuleConfig("enc_small", 2, 144, 2, 2, 72, 536, CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, seed_base=4100)


def _enc_dh(dh):
    # two heads of an odd width: the attention kernel's other score / output paddings (40 -> 64 x 64 with a denominator
    # row, 88 -> 96 x 96 with one, 96 -> 96 x 96 without, 112 -> 128 x 128 with one)
    return CFG.ModuleConfig("enc_dh%d" % dh, 2, 2 * dh, 2, 2, dh, 536, CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, seed_base=4500 + dh)


def _gqa_small(dh, max_seq=384):
    return CFG.ModuleConfig("gqa_small", 2, 8 * dh, 8, 2, dh, 1056, CFG.NORM_RMS, CFG.ACT_SWIGLU, 0, 1, 1e6,
                            max_seq=max_seq, seed_base=4200 + dh, vocab=0)


def _cross_small(heads, dh):
    return CFG.ModuleConfig("cross_small", 2, 256, heads, 1 if heads == 4 else heads, dh, 512,
                            CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, d_ctx=384, seed_base=4300)


# chunks of the GQA decoder cases: a prefill, a second chunk that attends over the first one's cache, a third whose
# first position (217) is not a multiple of 8 (the transposed-V append falls back to 2-byte stores), then three
# single-token passes (decode kernels).  Chunk sizes are comparable with the positions before them so that the
# causal mask matters in every multi-token pass.
GQA_PASSES = [(0, 100), (100, 117), (217, 66), (283, 1), (284, 1), (285, 1)]

TINY_PASSES = [(0, 128)] + [(128 + s, 1) for s in range(8)]

CASES = [
    # the tiny workload exactly as stated (N(0, 0.02) matrices at d = 256: a gain of 0.32 per map)
    # (its 8 decode steps appear here as single-token passes over seeded N(0, 1) rows, the distribution of the
    # embedding table's rows; the greedy test feeds the oracle's own tokens back)
    Case("tiny_stated", CFG.tiny_decoder(), TINY_PASSES, 7, gain=0.0, blind=("rope",), covered_by="tiny_gain"),
    Case("tiny_gain", CFG.tiny_decoder(), TINY_PASSES, 7),
    Case("enc_T1", _enc_small(), [(0, 1)], 17),
    Case("enc_T77", _enc_small(), [(0, 77)], 17),
    Case("enc_T333", _enc_small(), [(0, 333)], 17),
    Case("gqa_dh64", _gqa_small(64), GQA_PASSES, 23),
    Case("gqa_dh128", _gqa_small(128), GQA_PASSES, 23),
    Case("gqa_nocache", _gqa_small(64, max_seq=0), [(0, 130)], 43),
    # head widths between the attention kernel's paddings, causal with a cache (prefill, chunk over the cache, single tokens)
    Case("gqa_dh88", _gqa_small(88), GQA_PASSES, 23),
    Case("gqa_dh96", _gqa_small(96), GQA_PASSES, 23),
    Case("gqa_dh112", _gqa_small(112), GQA_PASSES, 23),
    # and bidirectional, four 32-query slices of one head per workgroup, ragged token counts
    Case("enc_dh40_T150", _enc_dh(40), [(0, 150)], 19),
    Case("enc_dh96_T200", _enc_dh(96), [(0, 200)], 19),
    Case("enc_dh112_T131", _enc_dh(112), [(0, 131)], 19),
    # edges: 32 query heads on ONE KV head (the most the single-token attention kernel's tile takes), head dimension 8,
    # passes that end exactly at the cache's last position, a single context row
    Case("gqa_group32_dh8", CFG.ModuleConfig("g32", 2, 256, 32, 1, 8, 512, CFG.NORM_RMS, CFG.ACT_SWIGLU, 0, 1, 1e4,
                                             max_seq=72, seed_base=4400, vocab=0), [(0, 67), (67, 1), (68, 3), (71, 1)], 47),
    Case("cross_one_context_row", _cross_small(2, 128), [(0, 5)], 31, n_ctx=1, ctx_seed=32),
    Case("cross_short", _cross_small(2, 128), [(0, 64)], 31, n_ctx=150, ctx_seed=32),
    Case("cross_split_ragged", _cross_small(2, 128), [(0, 64)], 31, n_ctx=700, ctx_seed=32),
    Case("cross_split_gqa", _cross_small(4, 64), [(0, 20)], 31, n_ctx=1100, ctx_seed=32),
    Case("cross_split_dh72", _cross_small(3, 72), [(0, 128)], 31, n_ctx=515, ctx_seed=32),
]
CASE = {c.name: c for c in CASES}


# ---- the five-stage pipeline at reduced size (tests/test_gpu_pipeline.py) -----------------------------------
def pipe_small_modules():
    vit = CFG.ModuleConfig("vit_s", 3, 144, 2, 2, 72, 536, CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, seed_base=6100)
    dec = CFG.ModuleConfig("dec_s", 3, 512, 8, 2, 64, 1024, CFG.NORM_RMS, CFG.ACT_SWIGLU, 0, 1, 1e6, max_seq=160,
                           seed_base=6200, vocab=512)
    act = CFG.ModuleConfig("act_s", 2, 256, 2, 2, 128, 512, CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, d_ctx=512,
                           seed_base=6300)
    return vit, dec, act


PIPE_SMALL = dict(n_patches=256, n_text=40, n_actions=64, n_decode=4, gain=GAIN_8B)
# (module, mutation): every sub-block of every stack of the pipeline
PIPE_MUTATIONS = [("vit", "self_attention"), ("vit", "ffn"),
                  ("dec", "self_attention"), ("dec", "ffn"), ("dec", "rope"), ("dec", "causal_mask"),
                  ("act", "self_attention"), ("act", "cross_attention"), ("act", "ffn")]


def pipeline_oracle(mutate=None):
    """oracle.pipeline.vla_pipeline on the reduced pipeline; mutate = (module name, mutation name) or None."""
    from oracle import pipeline as PL
    vit, dec, act = pipe_small_modules()
    P = PIPE_SMALL
    inp = CFG.make_pipeline_inputs(vit, dec, act, P["n_patches"], P["n_text"], P["n_actions"], matrix_gain=P["gain"])
    mods = {"vit": vit, "dec": dec, "act": act}
    gens, cfgs = {}, {}
    for name, c in mods.items():
        gens[name] = (lambda cc: (lambda l: CFG.make_layer_weights(cc, l, P["gain"])))(c)
        cfgs[name] = c.as_dict()
    if mutate is not None:
        name, mutation = mutate
        stand_in = Case(name, mods[name], [(0, 1)], 0, gain=P["gain"])
        w, over = MUTATIONS[mutation][1](stand_in)
        if w is not None:
            gens[name] = w
        if over:
            cfgs[name].update(over)
    out = PL.vla_pipeline(cfgs["vit"], gens["vit"], inp["proj_w"], cfgs["dec"], gens["dec"], CFG.make_head(dec),
                          cfgs["act"], gens["act"], (inp["out_w"][2], inp["out_w"][3]),
                          inp["patches"], inp["text"], inp["a0"], P["n_decode"])
    out["a0"] = inp["a0"]
    return out


def pipeline_measures(got, want):
    """The measures the pipeline test asserts, each divided by its bound: the decoder's final-normed prefill
    states, the action tokens (also relative to what the ten Euler steps added to the noise), the trajectory."""
    a0 = want["a0"]
    return {
        "hidden_ctx": stated_err(got["hidden_ctx"], want["hidden_ctx"]) / TOL,
        "actions": stated_err(got["actions"], want["actions"]) / TOL,
        "actions_contrib": contrib_err(got["actions"], want["actions"], a0) / TOL_CONTRIB,
        "trajectory": stated_err(got["trajectory"], want["trajectory"]) / TOL,
    }


# ---- a 16384-token prompt through one 8B-class layer: the oracle computes three chunks of rows on their own -------
LONG_T = 16384
LONG_CHUNKS = [(0, 64), (8192 - 39, 77), (LONG_T - 128, 128)]      # first rows, a ragged chunk across the middle, last rows


def long_prompt_case(attention_alone):
    """attention_alone: the feed-forward's output projection zeroed, so that y - x is the attention sub-block only (next
    to the feed-forward, an average over thousands of keys is a tenth of the contribution)."""
    return Case("dec8b_L1_T%d%s" % (LONG_T, "_attn" if attention_alone else ""),
                CFG.decoder_8b(n_layers=1, max_seq=LONG_T, vocab=0), [(0, LONG_T)], 7, gain=0.0,
                zero=(CFG.T_W_DOWN,) if attention_alone else ())


def long_prompt_oracle(case, weights=None, cfg_over=None, x=None):
    """(rows, oracle output at those rows).  The whole pass would cost the oracle minutes (its attention alone one):
    the keys and values of all positions come from oracle.forward.project_kv, and layer_forward then computes
    LONG_CHUNKS at their positions over that cache, which tests/test_oracle_forward.py shows to equal those rows of the
    full pass."""
    cfg = case.cfg.as_dict()
    if cfg_over:
        cfg.update(cfg_over)
    gen = weights or case.weights()
    W = {t: (F.widen(a) if a.dtype == np.uint16 else np.asarray(a, np.float64)) for t, a in gen(0).items()}
    x64 = (case.x() if x is None else x).astype(np.float64)
    kv = F.new_kv_cache(cfg, 1)[0]
    kv["k"][:LONG_T], kv["v"][:LONG_T] = F.project_kv(cfg, W, x64, 0)
    want = np.concatenate([F.layer_forward(cfg, W, x64[p:p + t], p, kv) for p, t in LONG_CHUNKS])
    rows = np.concatenate([np.arange(p, p + t) for p, t in LONG_CHUNKS])
    return rows, want


# ---- full-shape cases: expected values and mutation ratios come from tests/golden/make_full_depth.py ---------
def full_cases():
    return {
        # one layer of the 8B-class decoder: 3072-token prefill, then two single-token passes over the cache
        "dec8b_L1": Case("dec8b_L1", CFG.decoder_8b(n_layers=1, max_seq=3136, vocab=0),
                         [(0, 3072), (3072, 1), (3073, 1)], 7, gain=0.0),
        # the same with the feed-forward's output projection zeroed: y - x is then the attention sub-block alone.
        # Over 3072 cached keys a single-token attention output is an average of thousands of values and adds ten
        # times less to the residual stream than the feed-forward does, so next to it the single-token attention
        # kernels would be judged at only ~7x their bound; alone they are judged at 50x.
        "dec8b_L1_attn": Case("dec8b_L1_attn", CFG.decoder_8b(n_layers=1, max_seq=3136, vocab=0),
                              [(0, 3072), (3072, 1), (3073, 1)], 7, gain=0.0, zero=(CFG.T_W_DOWN,)),
        # the action head at its full shape: 8 layers, 64 action tokens cross-attending to a 3072 x 4096 context
        # (seeded N(0, 1) rows standing in for the decoder's final-normed hidden states), stated N(0, 0.02) recipe
        "act_L8": Case("act_L8", CFG.action_head(), [(0, 64)], 61, gain=0.0, n_ctx=3072, ctx_seed=62),
        # the same with self-attention and feed-forward zeroed: y - x is the cross-attention alone (over 3072 context rows
        # it adds a tenth of what the feed-forward adds; next to it, it is judged at only ~5x its bound)
        "act_L8_cross": Case("act_L8_cross", CFG.action_head(), [(0, 64)], 61, gain=0.0, n_ctx=3072, ctx_seed=62,
                             zero=(CFG.T_WO, CFG.T_BO, CFG.T_W_DOWN, CFG.T_B_DOWN)),
        # the 27-layer encoder at 4096 tokens and the 36-layer decoder at 3072 tokens, as the workloads state them
        "vit_L27": Case("vit_L27", CFG.vit_encoder(), [(0, 4096)], 7, gain=0.0),
        # one encoder layer over 8192 patches: the length at which its execution outlasts its copy (bench.py's
        # execution-intensive leg); 128 K/V tiles per query block, 64 query blocks per head
        "vit_L1_T8192": Case("vit_L1_T8192", CFG.vit_encoder(n_layers=1), [(0, 8192)], 7, gain=0.0),
        # the same with the feed-forward zeroed: a bidirectional average over 8192 keys adds a twentieth of what the
        # feed-forward adds (judged at 2.3x its bound next to it), alone it is judged at 50x
        "vit_L1_T8192_attn": Case("vit_L1_T8192_attn", CFG.vit_encoder(n_layers=1), [(0, 8192)], 7, gain=0.0,
                                  zero=(CFG.T_W_DOWN, CFG.T_B_DOWN)),
        "dec8b_L36": Case("dec8b_L36", CFG.decoder_8b(max_seq=3136, vocab=32768), [(0, 3072)], 7, gain=0.0),
    }


def sample_rows(n_rows, step):
    """The rows of a full-shape output that are stored and compared: every `step`-th and the last."""
    rows = list(range(0, n_rows, step))
    if rows[-1] != n_rows - 1:
        rows.append(n_rows - 1)
    return np.array(rows, dtype=np.int64)
