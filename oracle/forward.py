"""CPU oracle for the layer-stack forward pass — TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
this file.  It shares no code with the HIP path and imports nothing from it.

What it computes.  Demand Layering moves parameters; it never changes what a
layer computes: the paper's Table IX reports a maximum absolute error of zero
against full preloading for every residency count.  The result of the hot
path therefore has a plain definition — the ordinary forward pass of the layer
stack with all weights in place — and this file is that definition written
out in float64 with numpy, one library matmul per linear map, no blocking,
no fusion, no reordering.  The paper runs an off-the-shelf model (Sec. II-A)
and does not spell the layer out; the block structure below is the standard
pre-norm transformer block named by the workload descriptions:

    h = x + Attn(Norm1(x))            (+ CrossAttn(NormC(h), ctx) when d_ctx > 0)
    y = h + FFN(Norm2(h))

Conventions (all are readings where the paper is silent):
  * matrices are [out_features, in_features]; a linear map is x @ W.T (+ b);
  * RMSNorm: x / sqrt(mean(x^2) + eps) * g;  LayerNorm: (x-mean)/sqrt(var+eps)*g + b
    with the biased variance;
  * RoPE pairs element i with i + dh/2 inside a head, angle = pos * theta^(-2i/dh);
  * attention scores are scaled by 1/sqrt(dh); query head h reads KV head
    h // (Hq/Hkv); causal means key position <= query position;
  * SwiGLU FFN: (silu(n @ Wg.T) * (n @ Wu.T)) @ Wd.T;
    GELU FFN: gelu_tanh(n @ W1.T + b1) @ W2.T + b2;
  * greedy head: logits = FinalNorm(h) @ W_head.T, token = lowest index of the maximum.

Parity pins (tests/test_oracle_forward.py): brute-force attention with an
explicit score matrix and mask, closed forms for the norms and RoPE
invariants, identity layer when Wo = Wdown = 0, prefill/decode consistency,
hand-computed 2x2 cases.  Exact layer output values for the synthetic
workloads are not printed anywhere in the paper: parity unpinned by the paper
for those, pinned only by the checks above.
"""
import math

import numpy as np

# tensor ids: the integers of the public header, repeated here so that the
# oracle does not import the product package
T_NORM1_G, T_NORM1_B = 0, 1
T_WQ, T_WK, T_WV, T_BQ, T_BK, T_BV = 2, 3, 4, 5, 6, 7
T_WO, T_BO = 8, 9
T_NORM2_G, T_NORM2_B = 10, 11
T_W_GATE, T_W_UP, T_B_UP, T_W_DOWN, T_B_DOWN = 12, 13, 14, 15, 16
T_NORMC_G, T_NORMC_B = 17, 18
T_WQ_C, T_WK_C, T_WV_C, T_BQ_C, T_BK_C, T_BV_C, T_WO_C, T_BO_C = 19, 20, 21, 22, 23, 24, 25, 26
NORM_RMS, NORM_LN = 0, 1
ACT_SWIGLU, ACT_GELU = 0, 1


def widen(bits):
    """BF16 bit patterns (uint16) -> float64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rmsnorm(x, g, eps):
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def layernorm(x, g, b, eps):
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def norm(cfg, x, g, b):
    if cfg["norm"] == NORM_RMS:
        return rmsnorm(x, g, cfg["norm_eps"])
    return layernorm(x, g, b, cfg["norm_eps"])


def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def rope(x, positions, theta):
    """x: [T, H, dh]; positions: [T] absolute positions.  Rotates the pair (i, i+dh/2)."""
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]          # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def attention(q, k, v, causal, q_pos0=0):
    """q: [T, Hq, dh]; k, v: [S, Hkv, dh].  Query t sits at absolute position q_pos0 + t,
    key j at position j.  Returns [T, Hq, dh]."""
    T, Hq, dh = q.shape
    S, Hkv, _ = k.shape
    group = Hq // Hkv
    out = np.empty_like(q)
    qpos = q_pos0 + np.arange(T)[:, None]
    kpos = np.arange(S)[None, :]
    for h in range(Hq):
        kv = h // group
        s = (q[:, h, :] @ k[:, kv, :].T) / math.sqrt(dh)                      # [T, S]
        if causal:
            s = np.where(kpos <= qpos, s, -np.inf)
        s = s - np.max(s, axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / np.sum(p, axis=-1, keepdims=True)
        out[:, h, :] = p @ v[:, kv, :]
    return out


def _w(W, tid):
    return W[tid] if tid in W else 0.0


def layer_forward(cfg, W, x, pos0=0, kv=None, ctx=None):
    """One pre-norm block.  W: {tensor id: float64 array}.  x: [T, d] float64.
    kv: None, or a dict {'k': [max_seq, Hkv, dh], 'v': ...} that receives this call's keys and
    values at positions pos0..pos0+T-1 and supplies positions 0..pos0+T-1 to attention.
    ctx: [n_ctx, d_ctx] source of the cross-attention sub-block (when cfg['d_ctx'] > 0)."""
    T = x.shape[0]
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["d_head"]
    n1 = norm(cfg, x, W[T_NORM1_G], _w(W, T_NORM1_B))
    q = (n1 @ W[T_WQ].T + _w(W, T_BQ)).reshape(T, Hq, dh)
    k = (n1 @ W[T_WK].T + _w(W, T_BK)).reshape(T, Hkv, dh)
    v = (n1 @ W[T_WV].T + _w(W, T_BV)).reshape(T, Hkv, dh)
    if cfg["rope_theta"] > 0:
        pos = pos0 + np.arange(T)
        q, k = rope(q, pos, cfg["rope_theta"]), rope(k, pos, cfg["rope_theta"])
    if kv is not None:
        kv["k"][pos0:pos0 + T] = k
        kv["v"][pos0:pos0 + T] = v
        k_all, v_all = kv["k"][:pos0 + T], kv["v"][:pos0 + T]
    else:
        assert pos0 == 0
        k_all, v_all = k, v
    a = attention(q, k_all, v_all, bool(cfg["causal"]), q_pos0=pos0).reshape(T, Hq * dh)
    h = x + a @ W[T_WO].T + _w(W, T_BO)
    if cfg.get("d_ctx", 0) > 0:
        nc = norm(cfg, h, W[T_NORMC_G], _w(W, T_NORMC_B))
        n_ctx = ctx.shape[0]
        qc = (nc @ W[T_WQ_C].T + _w(W, T_BQ_C)).reshape(T, Hq, dh)
        kc = (ctx @ W[T_WK_C].T + _w(W, T_BK_C)).reshape(n_ctx, Hkv, dh)
        vc = (ctx @ W[T_WV_C].T + _w(W, T_BV_C)).reshape(n_ctx, Hkv, dh)
        ac = attention(qc, kc, vc, False).reshape(T, Hq * dh)
        h = h + ac @ W[T_WO_C].T + _w(W, T_BO_C)
    n2 = norm(cfg, h, W[T_NORM2_G], _w(W, T_NORM2_B))
    if cfg["act"] == ACT_SWIGLU:
        mid = silu(n2 @ W[T_W_GATE].T) * (n2 @ W[T_W_UP].T)
    else:
        mid = gelu_tanh(n2 @ W[T_W_UP].T + _w(W, T_B_UP))
    return h + mid @ W[T_W_DOWN].T + _w(W, T_B_DOWN)


def project_kv(cfg, W, x, pos0=0):
    """The keys and values layer_forward derives from rows x at positions pos0.. (the same definition, on its
    own): k, v = Norm1(x) Wk^T (+ bk), Norm1(x) Wv^T (+ bv), keys rotated when the module uses RoPE.  Lets a test
    fill a KV cache for a long prefix without paying for that prefix's attention and feed-forward, and then ask
    layer_forward for a few chunks of rows only.  Pinned against the cache rows layer_forward itself writes."""
    T = x.shape[0]
    Hkv, dh = cfg["n_kv_heads"], cfg["d_head"]
    n1 = norm(cfg, x, W[T_NORM1_G], _w(W, T_NORM1_B))
    k = (n1 @ W[T_WK].T + _w(W, T_BK)).reshape(T, Hkv, dh)
    v = (n1 @ W[T_WV].T + _w(W, T_BV)).reshape(T, Hkv, dh)
    if cfg["rope_theta"] > 0:
        k = rope(k, pos0 + np.arange(T), cfg["rope_theta"])
    return k, v


def new_kv_cache(cfg, n_layers=None):
    n = cfg["n_layers"] if n_layers is None else n_layers
    shape = (cfg["max_seq"], cfg["n_kv_heads"], cfg["d_head"])
    return [{"k": np.zeros(shape), "v": np.zeros(shape)} for _ in range(n)]


def stack_forward(cfg, layer_weights, x, pos0=0, kv_cache=None, ctx=None):
    """Runs layers 0..n-1 in order.  layer_weights: callable layer -> {tid: BF16 bits or float array}
    (called once per layer so that a large stack is widened one layer at a time)."""
    x = np.asarray(x, dtype=np.float64)
    for l in range(cfg["n_layers"]):
        W = {t: (widen(a) if a.dtype == np.uint16 else np.asarray(a, np.float64))
             for t, a in layer_weights(l).items()}
        x = layer_forward(cfg, W, x, pos0, None if kv_cache is None else kv_cache[l], ctx)
    return x


def final_norm(cfg, h, g, b=None):
    g = widen(g) if g.dtype == np.uint16 else g
    if b is not None and getattr(b, "dtype", None) == np.uint16:
        b = widen(b)
    return norm(cfg, np.asarray(h, np.float64), g, 0.0 if b is None else b)


def head_logits(cfg, h_last, g_final, w_head, b_final=None):
    """h_last: [d].  Returns logits [vocab] in float64."""
    w = widen(w_head) if w_head.dtype == np.uint16 else w_head
    return final_norm(cfg, h_last[None, :], g_final, b_final)[0] @ w.T


def greedy_token(logits):
    return int(np.argmax(logits))   # numpy returns the first (lowest) index of the maximum


def generate_greedy(cfg, layer_weights, head, x_prefill, n_steps):
    """Prefill on x_prefill [T, d], then n_steps decode steps.  Step s: token_s = greedy(head(h)),
    then h = stack(E[token_s]) at the next position.  head: {0: E[vocab,d], 1: W_head[vocab,d],
    2: final-norm gain, (3: bias)} as BF16 bits.  Returns (token ids [n_steps], logits [n_steps, vocab],
    hidden [n_steps+1, d]: hidden[0] is the last prefill row, hidden[s+1] the output of decode step s)."""
    E = widen(head[0]) if head[0].dtype == np.uint16 else np.asarray(head[0], np.float64)
    kv = new_kv_cache(cfg)
    h = stack_forward(cfg, layer_weights, x_prefill, 0, kv)
    pos = x_prefill.shape[0]
    h_last = h[-1]
    toks, all_logits, hs = [], [], [h_last]
    for _ in range(n_steps):
        logits = head_logits(cfg, h_last, head[2], head[1], head.get(3))
        t = greedy_token(logits)
        toks.append(t)
        all_logits.append(logits)
        h_last = stack_forward(cfg, layer_weights, E[t][None, :], pos, kv)[0]
        hs.append(h_last)
        pos += 1
    return toks, np.array(all_logits), np.array(hs)
