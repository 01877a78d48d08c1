"""The synthetic workloads (shapes and seeded input recipes).

Shapes follow the paper's model description (Sec. II-A: a 27-layer d=1152
vision encoder, a 36-layer GQA 32Q/8KV decoder run as prefill then decode, a
10-step action head) with seeded random values standing in for the trained
weights.  Everything here is input description/generation: no forward-pass or
planner arithmetic.

Matrices use the [out_features, in_features] row-major convention; a linear
map is y = x @ W.T (+ b).
"""
from dataclasses import dataclass, field, asdict
from typing import Dict, List, Tuple

import numpy as np

from . import synth

# ---- tensor ids (mirrors include/demand_layering.h) ------------------------
T_NORM1_G, T_NORM1_B = 0, 1
T_WQ, T_WK, T_WV, T_BQ, T_BK, T_BV = 2, 3, 4, 5, 6, 7
T_WO, T_BO = 8, 9
T_NORM2_G, T_NORM2_B = 10, 11
T_W_GATE, T_W_UP, T_B_UP, T_W_DOWN, T_B_DOWN = 12, 13, 14, 15, 16
T_NORMC_G, T_NORMC_B = 17, 18
T_WQ_C, T_WK_C, T_WV_C, T_BQ_C, T_BK_C, T_BV_C, T_WO_C, T_BO_C = 19, 20, 21, 22, 23, 24, 25, 26

TENSOR_NAMES = {
    T_NORM1_G: "norm1_g", T_NORM1_B: "norm1_b", T_WQ: "wq", T_WK: "wk", T_WV: "wv",
    T_BQ: "bq", T_BK: "bk", T_BV: "bv", T_WO: "wo", T_BO: "bo",
    T_NORM2_G: "norm2_g", T_NORM2_B: "norm2_b", T_W_GATE: "w_gate", T_W_UP: "w_up",
    T_B_UP: "b_up", T_W_DOWN: "w_down", T_B_DOWN: "b_down",
    T_NORMC_G: "normc_g", T_NORMC_B: "normc_b", T_WQ_C: "wq_c", T_WK_C: "wk_c", T_WV_C: "wv_c",
    T_BQ_C: "bq_c", T_BK_C: "bk_c", T_BV_C: "bv_c", T_WO_C: "wo_c", T_BO_C: "bo_c",
}

NORM_RMS, NORM_LN = 0, 1
ACT_SWIGLU, ACT_GELU = 0, 1

# resident (non-layer) tensor ids
R_EMBED, R_HEAD, R_FINAL_NORM_G, R_FINAL_NORM_B = 0, 1, 2, 3


@dataclass
class ModuleConfig:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    d_ff: int
    norm: int            # NORM_RMS | NORM_LN
    act: int             # ACT_SWIGLU | ACT_GELU
    has_bias: int        # biases on every linear map (and LN bias)
    causal: int
    rope_theta: float    # 0 = no positional rotation
    norm_eps: float = 1e-6
    d_ctx: int = 0       # > 0: a cross-attention sub-block whose K/V come from a [n_ctx, d_ctx] source
    max_seq: int = 0     # > 0: keeps a KV cache of this many positions (decoders)
    seed_base: int = 1000
    vocab: int = 0       # > 0: has embedding table [vocab, d] and head [vocab, d]

    def as_dict(self):
        return asdict(self)


def layer_tensors(c: ModuleConfig) -> List[Tuple[int, Tuple[int, ...], str]]:
    """(tensor id, shape, kind) for every parameter tensor of one layer; kind in gain|bias|matrix."""
    d, dq, dkv, f = c.d_model, c.n_q_heads * c.d_head, c.n_kv_heads * c.d_head, c.d_ff
    ln, b = c.norm == NORM_LN, bool(c.has_bias)
    out = [(T_NORM1_G, (d,), "gain")]
    if ln:
        out.append((T_NORM1_B, (d,), "bias"))
    out += [(T_WQ, (dq, d), "matrix"), (T_WK, (dkv, d), "matrix"), (T_WV, (dkv, d), "matrix")]
    if b:
        out += [(T_BQ, (dq,), "bias"), (T_BK, (dkv,), "bias"), (T_BV, (dkv,), "bias")]
    out.append((T_WO, (d, dq), "matrix"))
    if b:
        out.append((T_BO, (d,), "bias"))
    if c.d_ctx > 0:
        out.append((T_NORMC_G, (d,), "gain"))
        if ln:
            out.append((T_NORMC_B, (d,), "bias"))
        out += [(T_WQ_C, (dq, d), "matrix"), (T_WK_C, (dkv, c.d_ctx), "matrix"), (T_WV_C, (dkv, c.d_ctx), "matrix")]
        if b:
            out += [(T_BQ_C, (dq,), "bias"), (T_BK_C, (dkv,), "bias"), (T_BV_C, (dkv,), "bias")]
        out.append((T_WO_C, (d, dq), "matrix"))
        if b:
            out.append((T_BO_C, (d,), "bias"))
    out.append((T_NORM2_G, (d,), "gain"))
    if ln:
        out.append((T_NORM2_B, (d,), "bias"))
    if c.act == ACT_SWIGLU:
        out.append((T_W_GATE, (f, d), "matrix"))
    out.append((T_W_UP, (f, d), "matrix"))
    if b:
        out.append((T_B_UP, (f,), "bias"))
    out.append((T_W_DOWN, (d, f), "matrix"))
    if b:
        out.append((T_B_DOWN, (d,), "bias"))
    return out


def layer_param_count(c: ModuleConfig) -> int:
    return sum(int(np.prod(s)) for _, s, _ in layer_tensors(c))


def make_layer_weights(c: ModuleConfig, layer: int, matrix_gain: float = 0.0) -> Dict[int, np.ndarray]:
    """BF16 bit patterns (uint16) per tensor id.  Matrices and biases ~ N(0, 0.02);
    norm gains ~ 1 + N(0, 0.02) so that every block contributes at full scale.
    matrix_gain > 0: matrices ~ N(0, matrix_gain / sqrt(in_features)) instead.  At the 8B-class shape the
    stated 0.02 is a gain of 0.02 * sqrt(4096) = 1.28 per linear map; a small test shape (d = 144 .. 1024) with
    std 0.02 has a gain of 0.24 .. 0.64 and its sub-blocks add almost nothing to the residual stream, so small
    parity cases ask for the 8B shape's gain to keep every sub-block visible in the output."""
    out = {}
    for tid, shape, kind in layer_tensors(c):
        n = int(np.prod(shape))
        mean = 1.0 if kind == "gain" else 0.0
        std = matrix_gain / float(np.sqrt(shape[1])) if (kind == "matrix" and matrix_gain > 0) else 0.02
        out[tid] = synth.normal_bf16(n, c.seed_base + layer, tid, mean, std).reshape(shape)
    return out


def make_tokens(n_tokens: int, d: int, seed: int = 7, stream: int = 0) -> np.ndarray:
    """[n_tokens, d] float32, values ~ N(0,1) rounded to BF16 (exactly representable)."""
    return synth.normal_bf16_as_f32(n_tokens * d, seed, stream, 0.0, 1.0).reshape(n_tokens, d)


def make_head(c: ModuleConfig, seed: int = 8) -> Dict[int, np.ndarray]:
    """Always-resident non-layer parts: embedding table ~ N(0,1), output head ~ N(0,0.02),
    final-norm gain ~ 1 + N(0,0.02) (and bias for LayerNorm)."""
    out = {
        R_EMBED: synth.normal_bf16(c.vocab * c.d_model, seed + 1, 0, 0.0, 1.0).reshape(c.vocab, c.d_model),
        R_HEAD: synth.normal_bf16(c.vocab * c.d_model, seed, 0, 0.0, 0.02).reshape(c.vocab, c.d_model),
        R_FINAL_NORM_G: synth.normal_bf16(c.d_model, seed, 1, 1.0, 0.02),
    }
    if c.norm == NORM_LN:
        out[R_FINAL_NORM_B] = synth.normal_bf16(c.d_model, seed, 2, 0.0, 0.02)
    return out


def make_mlp(d_in: int, d_hidden: int, d_out: int, seed: int, matrix_gain: float = 0.0):
    """(w1 [d_hidden, d_in], b1, w2 [d_out, d_hidden or d_in], b2) as BF16 bits ~ N(0, 0.02); w1, b1 None if d_hidden == 0.
    matrix_gain > 0: matrices ~ N(0, matrix_gain / sqrt(in_features)), as in make_layer_weights."""
    k2 = d_hidden if d_hidden > 0 else d_in
    s1 = matrix_gain / float(np.sqrt(d_in)) if matrix_gain > 0 else 0.02
    s2 = matrix_gain / float(np.sqrt(k2)) if matrix_gain > 0 else 0.02
    w1 = synth.normal_bf16(d_hidden * d_in, seed, 0, 0.0, s1).reshape(d_hidden, d_in) if d_hidden > 0 else None
    b1 = synth.normal_bf16(d_hidden, seed, 1, 0.0, 0.02) if d_hidden > 0 else None
    w2 = synth.normal_bf16(d_out * k2, seed, 2, 0.0, s2).reshape(d_out, k2)
    b2 = synth.normal_bf16(d_out, seed, 3, 0.0, 0.02)
    return w1, b1, w2, b2


def make_pipeline_inputs(vit: ModuleConfig, dec: ModuleConfig, act: ModuleConfig, n_patches: int, n_text: int,
                         n_actions: int = 64, out_dim: int = 3, seeds=(11, 12, 13, 14, 15), matrix_gain: float = 0.0):
    """Seeded non-layer inputs of the five-stage pipeline: merger MLP (vit.d -> dec.d -> dec.d), output projection
    (act.d -> out_dim), patch tokens, text embeddings and the initial action noise, all ~ N(0, 1) / N(0, 0.02)."""
    return dict(proj_w=make_mlp(vit.d_model, dec.d_model, dec.d_model, seeds[0], matrix_gain),
                out_w=make_mlp(act.d_model, 0, out_dim, seeds[1], matrix_gain),
                patches=make_tokens(n_patches, vit.d_model, seed=seeds[2]),
                text=make_tokens(n_text, dec.d_model, seed=seeds[3]),
                a0=make_tokens(n_actions, act.d_model, seed=seeds[4]))


# ---- the workloads ---------------------------------------------------------
def tiny_decoder() -> ModuleConfig:
    return ModuleConfig("tiny_decoder", 4, 256, 4, 4, 64, 768, NORM_RMS, ACT_SWIGLU, 0, 1, 1e4,
                        max_seq=160, seed_base=1000, vocab=1024)


def vit_encoder(n_layers: int = 27) -> ModuleConfig:
    return ModuleConfig("vit_encoder", n_layers, 1152, 16, 16, 72, 4304, NORM_LN, ACT_GELU, 1, 0, 0.0,
                        seed_base=2000)


def decoder_8b(n_layers: int = 36, max_seq: int = 3136, vocab: int = 32768) -> ModuleConfig:
    return ModuleConfig("decoder_8b", n_layers, 4096, 32, 8, 128, 12288, NORM_RMS, ACT_SWIGLU, 0, 1, 1e6,
                        max_seq=max_seq, seed_base=3000, vocab=vocab)


def action_head(n_layers: int = 8) -> ModuleConfig:
    return ModuleConfig("action_head", n_layers, 1024, 8, 8, 128, 4096, NORM_LN, ACT_GELU, 1, 0, 0.0,
                        d_ctx=4096, seed_base=5000)


WORKLOADS = {
    "tiny_decoder": dict(module=tiny_decoder, prefill=128, decode_steps=8),
    "vit_encoder": dict(module=vit_encoder, tokens=4096),
    "decoder_8b_prefill": dict(module=decoder_8b, prefill=3072, cap_bytes=16_000_000_000),
    "decoder_8b_decode": dict(module=decoder_8b, prefill=3072, decode_steps=64,
                              cap_bytes=(12_000_000_000, 16_000_000_000)),
}
