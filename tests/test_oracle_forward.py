"""Pins for oracle/forward.py: scalar-loop brute force on tiny inputs, closed forms, invariants.
None of these re-use the oracle's own expressions: the brute force below is written with explicit
Python loops over tokens, heads and features."""
import math

import numpy as np
import pytest

from oracle import forward as F


def cfg_decoder(**kw):
    c = dict(n_layers=2, d_model=8, n_q_heads=4, n_kv_heads=2, d_head=4, d_ff=12, norm=F.NORM_RMS,
             act=F.ACT_SWIGLU, has_bias=0, causal=1, rope_theta=100.0, norm_eps=1e-6, d_ctx=0, max_seq=16)
    c.update(kw)
    return c


def cfg_encoder(**kw):
    c = dict(n_layers=2, d_model=6, n_q_heads=3, n_kv_heads=3, d_head=2, d_ff=10, norm=F.NORM_LN,
             act=F.ACT_GELU, has_bias=1, causal=0, rope_theta=0.0, norm_eps=1e-6, d_ctx=0, max_seq=0)
    c.update(kw)
    return c


def rand_weights(c, rng, scale=0.5):
    d, dq, dkv, f = c["d_model"], c["n_q_heads"] * c["d_head"], c["n_kv_heads"] * c["d_head"], c["d_ff"]
    W = {F.T_NORM1_G: 1 + 0.1 * rng.standard_normal(d), F.T_NORM2_G: 1 + 0.1 * rng.standard_normal(d),
         F.T_WQ: scale * rng.standard_normal((dq, d)), F.T_WK: scale * rng.standard_normal((dkv, d)),
         F.T_WV: scale * rng.standard_normal((dkv, d)), F.T_WO: scale * rng.standard_normal((d, dq)),
         F.T_W_UP: scale * rng.standard_normal((f, d)), F.T_W_DOWN: scale * rng.standard_normal((d, f))}
    if c["act"] == F.ACT_SWIGLU:
        W[F.T_W_GATE] = scale * rng.standard_normal((f, d))
    if c["norm"] == F.NORM_LN:
        W[F.T_NORM1_B] = 0.1 * rng.standard_normal(d)
        W[F.T_NORM2_B] = 0.1 * rng.standard_normal(d)
    if c["has_bias"]:
        for t, n in ((F.T_BQ, dq), (F.T_BK, dkv), (F.T_BV, dkv), (F.T_BO, d), (F.T_B_UP, f), (F.T_B_DOWN, d)):
            W[t] = 0.1 * rng.standard_normal(n)
    if c["d_ctx"] > 0:
        W[F.T_NORMC_G] = 1 + 0.1 * rng.standard_normal(d)
        W[F.T_WQ_C] = scale * rng.standard_normal((dq, d))
        W[F.T_WK_C] = scale * rng.standard_normal((dkv, c["d_ctx"]))
        W[F.T_WV_C] = scale * rng.standard_normal((dkv, c["d_ctx"]))
        W[F.T_WO_C] = scale * rng.standard_normal((d, dq))
        if c["norm"] == F.NORM_LN:
            W[F.T_NORMC_B] = 0.1 * rng.standard_normal(d)
        if c["has_bias"]:
            for t, n in ((F.T_BQ_C, dq), (F.T_BK_C, dkv), (F.T_BV_C, dkv), (F.T_BO_C, d)):
                W[t] = 0.1 * rng.standard_normal(n)
    return W


# ---------------- scalar brute force (independent re-derivation from the definitions) --------------
def b_linear(x, W, b=None):
    T, n_out, n_in = len(x), len(W), len(W[0])
    y = [[0.0] * n_out for _ in range(T)]
    for t in range(T):
        for o in range(n_out):
            acc = 0.0
            for i in range(n_in):
                acc += x[t][i] * W[o][i]
            y[t][o] = acc + (b[o] if b is not None else 0.0)
    return y


def b_norm(c, x, g, b):
    out = []
    for row in x:
        d = len(row)
        if c["norm"] == F.NORM_RMS:
            ms = sum(v * v for v in row) / d
            out.append([v / math.sqrt(ms + c["norm_eps"]) * g[i] for i, v in enumerate(row)])
        else:
            mu = sum(row) / d
            var = sum((v - mu) ** 2 for v in row) / d
            out.append([(v - mu) / math.sqrt(var + c["norm_eps"]) * g[i] + b[i] for i, v in enumerate(row)])
    return out


def b_rope_vec(vec, pos, theta):
    dh = len(vec)
    half = dh // 2
    out = [0.0] * dh
    for i in range(half):
        ang = pos * theta ** (-2.0 * i / dh)
        out[i] = vec[i] * math.cos(ang) - vec[i + half] * math.sin(ang)
        out[i + half] = vec[i] * math.sin(ang) + vec[i + half] * math.cos(ang)
    return out


def b_attention(q, k, v, Hq, Hkv, dh, causal, q_pos0):
    """q: T x (Hq*dh) lists; k, v: S x (Hkv*dh) lists; explicit score matrix and mask."""
    T, S = len(q), len(k)
    out = [[0.0] * (Hq * dh) for _ in range(T)]
    for h in range(Hq):
        g = h // (Hq // Hkv)
        for t in range(T):
            scores = []
            for j in range(S):
                if causal and j > q_pos0 + t:
                    scores.append(None)
                    continue
                scores.append(sum(q[t][h * dh + e] * k[j][g * dh + e] for e in range(dh)) / math.sqrt(dh))
            m = max(s for s in scores if s is not None)
            w = [0.0 if s is None else math.exp(s - m) for s in scores]
            z = sum(w)
            for e in range(dh):
                out[t][h * dh + e] = sum(w[j] / z * v[j][g * dh + e] for j in range(S))
    return out


def b_layer(c, W, x, pos0=0, k_hist=None, v_hist=None, ctx=None):
    Wl = {t: a.tolist() for t, a in W.items()}
    Hq, Hkv, dh = c["n_q_heads"], c["n_kv_heads"], c["d_head"]
    x = [list(r) for r in x]
    T = len(x)
    n1 = b_norm(c, x, Wl[F.T_NORM1_G], Wl.get(F.T_NORM1_B))
    q = b_linear(n1, Wl[F.T_WQ], Wl.get(F.T_BQ))
    k = b_linear(n1, Wl[F.T_WK], Wl.get(F.T_BK))
    v = b_linear(n1, Wl[F.T_WV], Wl.get(F.T_BV))
    if c["rope_theta"] > 0:
        for t in range(T):
            for h in range(Hq):
                q[t][h * dh:(h + 1) * dh] = b_rope_vec(q[t][h * dh:(h + 1) * dh], pos0 + t, c["rope_theta"])
            for h in range(Hkv):
                k[t][h * dh:(h + 1) * dh] = b_rope_vec(k[t][h * dh:(h + 1) * dh], pos0 + t, c["rope_theta"])
    k_all = (k_hist or []) + k
    v_all = (v_hist or []) + v
    a = b_attention(q, k_all, v_all, Hq, Hkv, dh, bool(c["causal"]), pos0)
    o = b_linear(a, Wl[F.T_WO], Wl.get(F.T_BO))
    h_ = [[x[t][i] + o[t][i] for i in range(len(x[0]))] for t in range(T)]
    if c["d_ctx"] > 0:
        nc = b_norm(c, h_, Wl[F.T_NORMC_G], Wl.get(F.T_NORMC_B))
        qc = b_linear(nc, Wl[F.T_WQ_C], Wl.get(F.T_BQ_C))
        kc = b_linear([list(r) for r in ctx], Wl[F.T_WK_C], Wl.get(F.T_BK_C))
        vc = b_linear([list(r) for r in ctx], Wl[F.T_WV_C], Wl.get(F.T_BV_C))
        ac = b_attention(qc, kc, vc, Hq, Hkv, dh, False, 0)
        oc = b_linear(ac, Wl[F.T_WO_C], Wl.get(F.T_BO_C))
        h_ = [[h_[t][i] + oc[t][i] for i in range(len(x[0]))] for t in range(T)]
    n2 = b_norm(c, h_, Wl[F.T_NORM2_G], Wl.get(F.T_NORM2_B))
    if c["act"] == F.ACT_SWIGLU:
        gte = b_linear(n2, Wl[F.T_W_GATE])
        up = b_linear(n2, Wl[F.T_W_UP])
        mid = [[(g / (1 + math.exp(-g))) * u for g, u in zip(gr, ur)] for gr, ur in zip(gte, up)]
    else:
        up = b_linear(n2, Wl[F.T_W_UP], Wl.get(F.T_B_UP))
        mid = [[0.5 * u * (1 + math.tanh(math.sqrt(2 / math.pi) * (u + 0.044715 * u ** 3))) for u in ur] for ur in up]
    dn = b_linear(mid, Wl[F.T_W_DOWN], Wl.get(F.T_B_DOWN))
    y = [[h_[t][i] + dn[t][i] for i in range(len(x[0]))] for t in range(T)]
    return y, k_all, v_all


# ---------------- tests ----------------------------------------------------------------------------
def test_hand_values():
    # RMSNorm of (3,4): mean square 12.5
    y = F.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0)
    assert y[0] == pytest.approx([3 / math.sqrt(12.5), 8 / math.sqrt(12.5)])
    # LayerNorm of (1,3): mean 2, biased variance 1
    y = F.layernorm(np.array([[1.0, 3.0]]), np.array([2.0, 2.0]), np.array([0.5, 0.5]), 0.0)
    assert y[0] == pytest.approx([-1.5, 2.5])
    # textbook activation values
    assert F.silu(np.array([0.0, 1.0]))[0] == 0.0
    assert F.silu(np.array([1.0]))[0] == pytest.approx(0.7310585786300049)
    assert F.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert F.gelu_tanh(np.array([1.0]))[0] == pytest.approx(0.8411919906082768)
    assert F.gelu_tanh(np.array([-1.0]))[0] == pytest.approx(-0.15880800939172324)
    # RoPE with dh = 2 is a plane rotation by pos radians: a quarter turn maps (a, b) to (-b, a)
    x = np.array([[[2.0, 5.0]]])
    assert F.rope(x, np.array([math.pi / 2]), 10.0)[0, 0] == pytest.approx([-5.0, 2.0])
    assert F.rope(x, np.array([0]), 10.0)[0, 0] == pytest.approx([2.0, 5.0])
    # widening of BF16 bits: 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1001
    assert F.widen(np.array([0x3F80, 0xC000, 0x3DCD], np.uint16)).tolist() == [1.0, -2.0, 0.10009765625]


def test_norm_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64)) * 3 + 1
    y = F.rmsnorm(x, np.ones(64), 0.0)
    assert np.mean(y * y, axis=-1) == pytest.approx(np.ones(5))
    assert F.rmsnorm(7.0 * x, np.ones(64), 0.0) == pytest.approx(y)          # scale invariance
    z = F.layernorm(x, np.ones(64), np.zeros(64), 0.0)
    assert np.mean(z, axis=-1) == pytest.approx(np.zeros(5), abs=1e-12)
    assert np.var(z, axis=-1) == pytest.approx(np.ones(5))
    assert F.layernorm(3 * x + 11, np.ones(64), np.zeros(64), 0.0) == pytest.approx(z)   # shift and scale invariance


def test_rope_invariants():
    rng = np.random.default_rng(1)
    dh = 8
    q, k = rng.standard_normal((1, 1, dh)), rng.standard_normal((1, 1, dh))
    half = dh // 2
    for m, n in ((3, 1), (10, 8), (105, 103)):
        qm, kn = F.rope(q, np.array([m]), 1e4), F.rope(k, np.array([n]), 1e4)
        # each (i, i+dh/2) pair keeps its norm
        assert qm[0, 0, :half] ** 2 + qm[0, 0, half:] ** 2 == pytest.approx(q[0, 0, :half] ** 2 + q[0, 0, half:] ** 2)
        # the inner product depends on m - n only
        ref = np.sum(F.rope(q, np.array([2]), 1e4) * F.rope(k, np.array([0]), 1e4))
        assert np.sum(qm * kn) == pytest.approx(ref)


@pytest.mark.parametrize("causal,Hq,Hkv,T,S,pos0", [(True, 4, 2, 5, 5, 0), (False, 3, 3, 4, 4, 0),
                                                     (False, 4, 1, 3, 7, 0), (True, 4, 2, 1, 6, 5),
                                                     (True, 2, 2, 3, 7, 4)])
def test_attention_vs_brute_force(causal, Hq, Hkv, T, S, pos0):
    rng = np.random.default_rng(2)
    dh = 4
    q = rng.standard_normal((T, Hq, dh))
    k = rng.standard_normal((S, Hkv, dh))
    v = rng.standard_normal((S, Hkv, dh))
    got = F.attention(q, k, v, causal, q_pos0=pos0).reshape(T, Hq * dh)
    want = b_attention(q.reshape(T, -1).tolist(), k.reshape(S, -1).tolist(), v.reshape(S, -1).tolist(),
                       Hq, Hkv, dh, causal, pos0)
    assert got == pytest.approx(np.array(want), rel=1e-12, abs=1e-14)


@pytest.mark.parametrize("kind", ["decoder", "encoder", "cross", "decoder_mha_bias_ln"])
def test_layer_vs_scalar_brute_force(kind):
    rng = np.random.default_rng(3)
    ctx = None
    if kind == "decoder":
        c = cfg_decoder()
    elif kind == "encoder":
        c = cfg_encoder()
    elif kind == "cross":
        c = cfg_encoder(d_ctx=5)
        ctx = rng.standard_normal((7, 5))
    else:
        c = cfg_decoder(norm=F.NORM_LN, has_bias=1, n_kv_heads=4, act=F.ACT_GELU)
    W = rand_weights(c, rng)
    x = rng.standard_normal((5, c["d_model"]))
    got = F.layer_forward(c, W, x, ctx=ctx)
    want, _, _ = b_layer(c, W, x.tolist(), ctx=None if ctx is None else ctx.tolist())
    assert got == pytest.approx(np.array(want), rel=1e-11, abs=1e-13)


def test_decode_over_cache_vs_brute_force_and_prefill_consistency():
    rng = np.random.default_rng(4)
    c = cfg_decoder()
    Ws = [rand_weights(c, rng) for _ in range(c["n_layers"])]
    T = 6
    x = rng.standard_normal((T, c["d_model"]))
    full = F.stack_forward(c, lambda l: Ws[l], x)
    # prefill 4 tokens, then 2 single-token steps: rows must equal the full causal prefill
    kv = F.new_kv_cache(c)
    h4 = F.stack_forward(c, lambda l: Ws[l], x[:4], 0, kv)
    assert h4 == pytest.approx(full[:4], rel=1e-12)
    for t in (4, 5):
        ht = F.stack_forward(c, lambda l: Ws[l], x[t:t + 1], t, kv)
        assert ht[0] == pytest.approx(full[t], rel=1e-11)
    # single-layer decode step against the scalar brute force with an explicit key/value history
    y3, k_hist, v_hist = b_layer(c, Ws[0], x[:3].tolist())
    y_step, _, _ = b_layer(c, Ws[0], x[3:4].tolist(), pos0=3, k_hist=k_hist, v_hist=v_hist)
    kv1 = F.new_kv_cache(c, 1)
    F.layer_forward(c, Ws[0], x[:3], 0, kv1[0])
    got = F.layer_forward(c, Ws[0], x[3:4], 3, kv1[0])
    assert got == pytest.approx(np.array(y_step), rel=1e-11)
    # T = 1 prefill equals decode at position 0
    a = F.stack_forward(c, lambda l: Ws[l], x[:1])
    b = F.stack_forward(c, lambda l: Ws[l], x[:1], 0, F.new_kv_cache(c))
    assert a == pytest.approx(b, rel=1e-14)


def test_project_kv_is_what_layer_forward_caches_and_chunks_reproduce_the_full_pass():
    """project_kv against the cache rows layer_forward writes (RMSNorm + RoPE decoder, LayerNorm + bias module), and
    the use the long-prompt GPU test makes of it: a cache filled by project_kv for the whole prompt, then
    layer_forward on a chunk of rows at its position, reproduces those rows of the full causal pass."""
    rng = np.random.default_rng(41)
    for c in (cfg_decoder(), cfg_decoder(norm=F.NORM_LN, has_bias=1, n_kv_heads=4, act=F.ACT_GELU)):
        W = rand_weights(c, rng)
        T = 11
        x = rng.standard_normal((T, c["d_model"]))
        kv = F.new_kv_cache(c, 1)[0]
        full = F.layer_forward(c, W, x, 0, kv)
        k, v = F.project_kv(c, W, x, 0)
        assert np.array_equal(k, kv["k"][:T]) and np.array_equal(v, kv["v"][:T])
        # positions matter for the keys of a module with rotary embedding
        k3, v3 = F.project_kv(c, W, x[3:7], 3)
        assert np.array_equal(k3, kv["k"][3:7]) and np.array_equal(v3, kv["v"][3:7])
        if c["rope_theta"] > 0:
            assert not np.allclose(F.project_kv(c, W, x[3:7], 0)[0], k3)
        kv2 = F.new_kv_cache(c, 1)[0]
        kv2["k"][:T], kv2["v"][:T] = k, v
        for p0, t in ((0, 2), (4, 3), (9, 2)):
            got = F.layer_forward(c, W, x[p0:p0 + t], p0, kv2)
            assert got == pytest.approx(full[p0:p0 + t], rel=1e-12, abs=1e-14)


def test_structure_invariants():
    rng = np.random.default_rng(5)
    c = cfg_decoder()
    W = rand_weights(c, rng)
    x = rng.standard_normal((5, c["d_model"]))
    # a block whose two output projections are zero is the identity
    W0 = dict(W)
    W0[F.T_WO] = np.zeros_like(W[F.T_WO])
    W0[F.T_W_DOWN] = np.zeros_like(W[F.T_W_DOWN])
    assert np.array_equal(F.layer_forward(c, W0, x), x)
    # causality: later tokens never influence earlier outputs
    x2 = x.copy()
    x2[3:] += 1.0
    y, y2 = F.layer_forward(c, W, x), F.layer_forward(c, W, x2)
    assert np.array_equal(y[:3], y2[:3]) and not np.allclose(y[3:], y2[3:])
    # an encoder block without positional terms is permutation-equivariant
    e = cfg_encoder()
    We = rand_weights(e, rng)
    xe = rng.standard_normal((6, e["d_model"]))
    perm = rng.permutation(6)
    assert F.layer_forward(e, We, xe)[perm] == pytest.approx(F.layer_forward(e, We, xe[perm]), rel=1e-12)
    # grouped-query attention equals multi-head attention with each KV head repeated
    g = cfg_decoder()
    m = cfg_decoder(n_kv_heads=4)
    Wg = rand_weights(g, rng)
    Wm = dict(Wg)
    dh = g["d_head"]
    Wm[F.T_WK] = np.repeat(Wg[F.T_WK].reshape(2, dh, -1), 2, axis=0).reshape(4 * dh, -1)
    Wm[F.T_WV] = np.repeat(Wg[F.T_WV].reshape(2, dh, -1), 2, axis=0).reshape(4 * dh, -1)
    assert F.layer_forward(g, Wg, x) == pytest.approx(F.layer_forward(m, Wm, x), rel=1e-12)


def test_softmax_shift_invariance_and_uniform_case():
    # identical keys give a uniform softmax: the output is the mean of the values
    q = np.ones((2, 1, 4))
    k = np.ones((5, 1, 4))
    v = np.arange(20.0).reshape(5, 1, 4)
    out = F.attention(q, k, v, False)
    assert out[0, 0] == pytest.approx(v[:, 0].mean(axis=0))
    # causal row 0 sees only key 0
    out = F.attention(q, k[:2], v[:2], True)
    assert out[0, 0] == pytest.approx(v[0, 0]) and out[1, 0] == pytest.approx(v[:2, 0].mean(axis=0))
    # large scores do not overflow (row max subtracted)
    out = F.attention(1e3 * q, k, v, False)
    assert np.all(np.isfinite(out))


def test_greedy_head():
    c = cfg_decoder()
    rng = np.random.default_rng(6)
    h = rng.standard_normal(c["d_model"])
    g = 1 + 0.1 * rng.standard_normal(c["d_model"])
    Wh = rng.standard_normal((11, c["d_model"]))
    logits = F.head_logits(c, h, g, Wh)
    n = [v / math.sqrt(sum(u * u for u in h) / len(h) + c["norm_eps"]) * g[i] for i, v in enumerate(h)]
    want = [sum(n[i] * Wh[o][i] for i in range(len(n))) for o in range(11)]
    assert logits == pytest.approx(want)
    assert F.greedy_token(np.array([1.0, 3.0, 3.0, 2.0])) == 1          # lowest index on ties


def test_generate_greedy_consistency():
    """Tokens from the cached generation equal tokens from re-running a full prefill each step."""
    rng = np.random.default_rng(8)
    c = cfg_decoder(max_seq=12)
    Ws = [rand_weights(c, rng) for _ in range(c["n_layers"])]
    V = 9
    head = {0: rng.standard_normal((V, c["d_model"])), 1: rng.standard_normal((V, c["d_model"])),
            2: 1 + 0.1 * rng.standard_normal(c["d_model"])}
    x = rng.standard_normal((4, c["d_model"]))

    toks, logits, hs = F.generate_greedy(c, lambda l: Ws[l], head, x, 3)
    seq = x.copy()
    for s in range(3):
        full = F.stack_forward(c, lambda l: Ws[l], seq)
        lg = F.head_logits(c, full[-1], head[2], head[1])
        assert int(np.argmax(lg)) == toks[s]
        assert lg == pytest.approx(logits[s], rel=1e-10)
        seq = np.vstack([seq, head[0][toks[s]][None, :]])
    assert hs.shape == (4, c["d_model"])


# ---------------- pipeline oracle (oracle/pipeline.py) ----------------------------------------------
def test_pipeline_small_pieces_hand_values():
    from oracle import pipeline as PL
    x = np.arange(16.0).reshape(8, 2)
    assert PL.mean_pool(x, 4).tolist() == [[3.0, 4.0], [11.0, 12.0]]
    # t = 0: sines vanish, cosines are one
    assert PL.time_embedding(0.0, 6).tolist() == [0.0, 0.0, 0.0, 1.0, 1.0, 1.0]
    e = PL.time_embedding(0.001 * math.pi / 2, 4)          # 1000 t = pi/2: first frequency is 1
    assert e[0] == pytest.approx(1.0) and e[2] == pytest.approx(0.0, abs=1e-15)
    assert e[1] == pytest.approx(math.sin(math.pi / 2 * 10000.0 ** -0.5))
    # MLP against scalar loops
    rng = np.random.default_rng(0)
    w1, b1, w2, b2 = rng.standard_normal((5, 3)), rng.standard_normal(5), rng.standard_normal((2, 5)), rng.standard_normal(2)
    xin = rng.standard_normal((4, 3))
    got = PL.mlp(xin, w1, b1, w2, b2)
    for t in range(4):
        hid = [sum(xin[t][i] * w1[o][i] for i in range(3)) + b1[o] for o in range(5)]
        hid = [0.5 * u * (1 + math.tanh(math.sqrt(2 / math.pi) * (u + 0.044715 * u ** 3))) for u in hid]
        for o in range(2):
            assert got[t][o] == pytest.approx(sum(hid[i] * w2[o][i] for i in range(5)) + b2[o])
    assert PL.mlp(xin, None, None, w2[:, :3], None) == pytest.approx(xin @ w2[:, :3].T)


def test_pipeline_euler_closed_form():
    """With zero output projections the action stack is the identity, so the velocity is a + e(t) and
    ten Euler steps have the closed form a_10 = 1.1^10 a_0 + sum_s 1.1^(9-s) * 0.1 * e(s/10)."""
    from oracle import pipeline as PL
    rng = np.random.default_rng(1)
    c = cfg_encoder(d_ctx=4, n_layers=1)
    W = rand_weights(c, rng)
    for t in (F.T_WO, F.T_W_DOWN, F.T_WO_C):
        W[t] = np.zeros_like(W[t])
    for t in (F.T_BO, F.T_B_DOWN, F.T_BO_C):
        W[t] = np.zeros_like(W[t])
    a0 = rng.standard_normal((3, c["d_model"]))
    ctx = rng.standard_normal((5, 4))
    got = PL.euler_actions(c, lambda l: W, a0, ctx, 10)
    want = 1.1 ** 10 * a0
    for s in range(10):
        want = want + 1.1 ** (9 - s) * 0.1 * PL.time_embedding(s / 10, c["d_model"])[None, :]
    assert got == pytest.approx(want, rel=1e-12)


def test_pipeline_wiring_against_scalar_loops():
    """The composition of the five stages, re-derived with scalar loops from the written reading (Sec. II-A names the
    stages; the arithmetic between them is this build's reading): encoder -> per-token 2-layer GELU MLP -> mean of
    every `pool` consecutive tokens -> [visual tokens ; text embeddings] -> causal decoder with a KV cache ->
    FINAL-NORMED hidden states of the prefill positions become the cross-attention context -> greedy steps from the
    last prefill row (un-normed state into the head, which normalises itself) -> Euler loop a += v(a + e(s/n))/n with
    the context fixed -> linear trajectory head.  Swapping two stages, pooling before the MLP, feeding un-normed
    states to the cross-attention or the embedding instead of the hidden state to the next step all change these
    numbers."""
    from oracle import pipeline as PL
    rng = np.random.default_rng(21)
    vit = cfg_encoder(n_layers=1, d_model=4, n_q_heads=2, d_head=2, d_ff=6)
    vit["n_kv_heads"] = 2
    dec = cfg_decoder(n_layers=1, d_model=6, n_q_heads=2, n_kv_heads=1, d_head=2, d_ff=8, max_seq=12)
    act = cfg_encoder(n_layers=1, d_model=4, n_q_heads=2, d_head=2, d_ff=6, d_ctx=6)
    act["n_kv_heads"] = 2
    Wv, Wd, Wa = rand_weights(vit, rng), rand_weights(dec, rng), rand_weights(act, rng)
    proj = (0.5 * rng.standard_normal((6, 4)), 0.1 * rng.standard_normal(6), 0.5 * rng.standard_normal((6, 6)),
            0.1 * rng.standard_normal(6))
    vocab = 5
    head = {0: rng.standard_normal((vocab, 6)), 1: rng.standard_normal((vocab, 6)), 2: 1 + 0.1 * rng.standard_normal(6)}
    out_proj = (rng.standard_normal((3, 4)), rng.standard_normal(3))
    patches, text, a0 = rng.standard_normal((4, 4)), rng.standard_normal((2, 6)), rng.standard_normal((3, 4))
    n_decode, n_euler, pool = 2, 3, 2
    got = PL.vla_pipeline(vit, lambda l: Wv, proj, dec, lambda l: Wd, head, act, lambda l: Wa, out_proj,
                          patches, text, a0, n_decode, n_euler=n_euler, pool=pool)

    gelu = lambda u: 0.5 * u * (1 + math.tanh(math.sqrt(2 / math.pi) * (u + 0.044715 * u ** 3)))
    # stage 1: encoder
    v, _, _ = b_layer(vit, Wv, patches.tolist())
    # stage 2: merger = MLP per token, THEN the mean of `pool` consecutive tokens
    p = b_linear([[gelu(u) for u in row] for row in b_linear(v, proj[0].tolist(), proj[1].tolist())],
                 proj[2].tolist(), proj[3].tolist())
    vis = [[sum(p[t * pool + j][i] for j in range(pool)) / pool for i in range(6)] for t in range(len(p) // pool)]
    # stage 3: prefill over [visual ; text]
    seq = vis + text.tolist()
    h, k_hist, v_hist = b_layer(dec, Wd, seq)
    g = head[2].tolist()
    rms = lambda row: [x / math.sqrt(sum(y * y for y in row) / len(row) + dec["norm_eps"]) * g[i] for i, x in enumerate(row)]
    hctx = [rms(row) for row in h]
    assert got["hidden_ctx"] == pytest.approx(np.array(hctx), rel=1e-10)
    # stage 4: greedy steps
    toks, h_last, pos = [], h[-1], len(seq)
    for s in range(n_decode):
        n = rms(h_last)
        logits = [sum(n[i] * head[1][o][i] for i in range(6)) for o in range(vocab)]
        assert got["logits"][s] == pytest.approx(logits, rel=1e-10)
        tok = max(range(vocab), key=lambda o: (logits[o], -o))
        toks.append(tok)
        y, k_hist, v_hist = b_layer(dec, Wd, [head[0][tok].tolist()], pos0=pos, k_hist=k_hist, v_hist=v_hist)
        h_last, pos = y[0], pos + 1
    assert got["tokens"] == toks
    # stage 5: Euler steps of the action stack, cross-attending to the final-normed prefill states
    a = a0.tolist()
    half = 2
    for s in range(n_euler):
        t = s / n_euler
        e = [math.sin(1000.0 * t * 10000.0 ** (-j / half)) for j in range(half)] + \
            [math.cos(1000.0 * t * 10000.0 ** (-j / half)) for j in range(half)]
        vel, _, _ = b_layer(act, Wa, [[a[r][i] + e[i] for i in range(4)] for r in range(3)], ctx=hctx)
        a = [[a[r][i] + vel[r][i] / n_euler for i in range(4)] for r in range(3)]
    assert got["actions"] == pytest.approx(np.array(a), rel=1e-9)
    traj = [[sum(a[r][i] * out_proj[0][o][i] for i in range(4)) + out_proj[1][o] for o in range(3)] for r in range(3)]
    assert got["trajectory"] == pytest.approx(np.array(traj), rel=1e-9)
    # and the wiring matters on this case: un-normed states as context, or pooling before the MLP, move the result
    wrong_ctx = PL.euler_actions(act, lambda l: Wa, a0, np.array(h), n_euler)
    assert np.max(np.abs(wrong_ctx - got["actions"])) > 1e-3
    wrong_merge = PL.mlp(PL.mean_pool(np.array(v), pool), *proj)
    assert np.max(np.abs(wrong_merge - np.array(vis))) > 1e-3
