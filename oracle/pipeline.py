"""CPU oracle for the multi-module (VLA-shaped) pipeline — TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use this file.  It imports
nothing from the product.  float64 numpy, built on oracle/forward.py.

Stages follow the paper's five-stage description of the model (Sec. II-A): vision encoder, patch
merger, VLM prefill, VLM decode, and a flow-matching action generator whose denoiser is called once
per Euler step (10 steps, 64 waypoints x 3).  What the paper leaves open is fixed here (readings):
  * merger: per-token 2-layer MLP gelu_tanh(x W1^T + b1) W2^T + b2, then the mean of every 4
    consecutive tokens (stand-in for the 2x2 patch merge);
  * decoder input: merged visual tokens followed by seeded text embeddings;
  * the action head cross-attends to the final-normed hidden states of the prefill positions;
  * flow time t = s/10 enters as a sinusoidal embedding added to every action token:
    e_i = sin(1000 t w_i) (i < d/2), cos(1000 t w_{i-d/2}) otherwise, w_j = 10000^(-j/(d/2));
  * velocity = output of the action stack; Euler: a <- a + (1/10) * velocity;
  * trajectory = a W_out^T + b_out.
Pins (tests/test_oracle_forward.py::test_pipeline_*): hand-computed pooling / embedding values,
Euler against the closed form for a linear velocity field, scalar re-derivation of the MLP, and the
composition of the five stages (which states feed what, in which order) re-derived with scalar loops on a
hand-sized case.
"""
import math

import numpy as np

from . import forward as F


def _f64(a):
    return F.widen(a) if getattr(a, "dtype", None) == np.uint16 else np.asarray(a, np.float64)


def mlp(x, w1, b1, w2, b2):
    """w1 None: plain linear map."""
    x = np.asarray(x, np.float64)
    if w1 is not None:
        x = F.gelu_tanh(x @ _f64(w1).T + (0.0 if b1 is None else _f64(b1)))
    return x @ _f64(w2).T + (0.0 if b2 is None else _f64(b2))


def mean_pool(x, group):
    T, d = x.shape
    return x.reshape(T // group, group, d).mean(axis=1)


def time_embedding(t, d):
    half = d // 2
    w = 10000.0 ** (-np.arange(half, dtype=np.float64) / half)
    ang = 1000.0 * t * w
    return np.concatenate([np.sin(ang), np.cos(ang)])


def euler_actions(cfg, layer_weights, a0, ctx, n_steps=10):
    """a <- a + (1/n_steps) * stack(a + e(t)), t = s / n_steps."""
    a = np.asarray(a0, np.float64).copy()
    for s in range(n_steps):
        t = s / n_steps
        v = F.stack_forward(cfg, layer_weights, a + time_embedding(t, a.shape[1])[None, :], ctx=ctx)
        a = a + v / n_steps
    return a


def vla_pipeline(vit_cfg, vit_w, proj, dec_cfg, dec_w, dec_head, act_cfg, act_w, out_proj, patches, text, a0,
                 n_decode, n_euler=10, pool=4):
    """proj = (w1, b1, w2, b2); out_proj = (w, b).  Returns dict(tokens, logits, hidden_ctx, actions, trajectory)."""
    v = F.stack_forward(vit_cfg, vit_w, patches)
    p = mlp(v, *proj)
    vis = mean_pool(p, pool)
    seq = np.vstack([vis, np.asarray(text, np.float64)])
    kv = F.new_kv_cache(dec_cfg)
    h = F.stack_forward(dec_cfg, dec_w, seq, 0, kv)
    hctx = F.final_norm(dec_cfg, h, dec_head[2], dec_head.get(3))
    E = _f64(dec_head[0])
    toks, logits = [], []
    h_last, pos = h[-1], seq.shape[0]
    for _ in range(n_decode):
        lg = F.head_logits(dec_cfg, h_last, dec_head[2], dec_head[1], dec_head.get(3))
        tok = F.greedy_token(lg)
        toks.append(tok)
        logits.append(lg)
        h_last = F.stack_forward(dec_cfg, dec_w, E[tok][None, :], pos, kv)[0]
        pos += 1
    a = euler_actions(act_cfg, act_w, a0, hctx, n_euler)
    traj = mlp(a, None, None, out_proj[0], out_proj[1])
    return dict(tokens=toks, logits=np.array(logits), hidden_ctx=hctx, actions=a, trajectory=traj)
