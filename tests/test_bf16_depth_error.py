"""Why the full-depth 8B-class decoder is held to 3e-2 instead of the stated 2e-2 (tests/parity_cases.py TOL_DEPTH36).

The method is stated in BF16 (Sec. V-A): the operands of every matrix product are BF16 values.  This test rounds
exactly those operands in a numpy forward pass that is otherwise float64 (no GPU, no product code) and compares with
the unrounded pass on a narrower stack of the same depth and recipe (36 layers, N(0, 0.02 sqrt(4096/d)) matrices, i.e.
the 8B shape's gain of 1.28 per linear map, which amplifies a perturbation from layer to layer): the rounding alone puts
the final-normed hidden states 2.1e-2 from the exact result at depth 36 (1.2e-2 at depth 8: the error grows with depth).
An implementation with BF16 operands cannot be closer than that to the exact oracle; the GPU path measures 2.1e-2 on
the real shape, the same figure."""
import math

import numpy as np
import pytest

from oracle import forward as F
from paper_2605_11678_amd import configs as CFG


def bf16_round(x):
    """Round-to-nearest-even to BF16 precision, returned as float64."""
    u = np.asarray(x, np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + 0x7FFF
    return ((u + r) & 0xFFFF0000).view(np.float32).astype(np.float64)


def layer(cfg, W, x, rnd):
    """The decoder block of oracle/forward.py with `rnd` applied to every matrix-product operand that is an
    activation (weights are BF16 already): normed inputs, q / k / v, rotated q / k, probabilities, attention output,
    feed-forward intermediate."""
    T = x.shape[0]
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["d_head"]
    n1 = rnd(F.rmsnorm(x, W[F.T_NORM1_G], cfg["norm_eps"]))
    pos = np.arange(T)
    q = rnd(F.rope(rnd(n1 @ W[F.T_WQ].T).reshape(T, Hq, dh), pos, cfg["rope_theta"]))
    k = rnd(F.rope(rnd(n1 @ W[F.T_WK].T).reshape(T, Hkv, dh), pos, cfg["rope_theta"]))
    v = rnd(n1 @ W[F.T_WV].T).reshape(T, Hkv, dh)
    out = np.empty_like(q)
    for h in range(Hq):
        g = h // (Hq // Hkv)
        s = (q[:, h] @ k[:, g].T) / math.sqrt(dh)
        s = np.where(pos[None, :] <= pos[:, None], s, -np.inf)
        p = np.exp(s - s.max(-1, keepdims=True))
        out[:, h] = (rnd(p) @ v[:, g]) / p.sum(-1, keepdims=True)
    h_ = x + rnd(out.reshape(T, Hq * dh)) @ W[F.T_WO].T
    n2 = rnd(F.rmsnorm(h_, W[F.T_NORM2_G], cfg["norm_eps"]))
    mid = rnd(F.silu(n2 @ W[F.T_W_GATE].T) * (n2 @ W[F.T_W_UP].T))
    return h_ + mid @ W[F.T_W_DOWN].T


def test_bf16_operands_alone_cost_two_percent_at_depth_36():
    c = CFG.ModuleConfig("narrow_8b", 36, 512, 4, 1, 128, 1536, CFG.NORM_RMS, CFG.ACT_SWIGLU, 0, 1, 1e6, seed_base=9000)
    cfg = c.as_dict()
    T = 128
    x0 = CFG.make_tokens(T, c.d_model, seed=7).astype(np.float64)
    exact, rounded = x0, x0
    ident = lambda a: a
    err = {}
    for l in range(c.n_layers):
        W = {t: F.widen(a) for t, a in CFG.make_layer_weights(c, l, 1.28).items()}
        # the plain block must be the oracle's own block (this file re-states it only to place the roundings)
        nxt = layer(cfg, W, exact, ident)
        if l == 0:
            assert np.allclose(nxt, F.layer_forward(cfg, W, exact), rtol=1e-12, atol=1e-12)
        exact, rounded = nxt, layer(cfg, W, rounded, bf16_round)
        if l + 1 in (8, 36):
            a = F.rmsnorm(exact, np.ones(c.d_model), 1e-6)
            b = F.rmsnorm(rounded, np.ones(c.d_model), 1e-6)
            err[l + 1] = float(np.max(np.abs(a - b)) / np.max(np.abs(a)))
    print("BF16-operand rounding alone: depth 8 -> %.3e, depth 36 -> %.3e" % (err[8], err[36]))
    assert err[8] < 1.6e-2 and err[8] < err[36]
    assert 1.6e-2 < err[36] < 3e-2
