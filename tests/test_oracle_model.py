"""Pins for oracle/model.py: things the mathematics fixes, not the oracle itself."""
import math
from types import SimpleNamespace

import numpy as np
import pytest

import april_inputs as ai
from oracle import model as om


def tiny_shape(**kw):
    d = dict(n_layers=2, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=6, d_ffn=24, vocab=20,
             n_experts=0, experts_per_tok=0, d_expert_ffn=0, dtype=ai.DTYPE_FP32,
             rope_theta=10000.0, rms_eps=1e-6)
    d.update(kw)
    return ai.ModelShape(**d)


# ---------------------------------------------------------------------------
# brute force: scalar loops, no cache, full recompute of the whole prefix
# ---------------------------------------------------------------------------
def scalar_forward(s, w, tokens):
    """Logits of the LAST position of `tokens`, recomputing everything with python
    scalars (written separately from the oracle; lists and math.* only)."""
    T = len(tokens)
    d, dh, Hq, Hkv = s.d_model, s.head_dim, s.n_q_heads, s.n_kv_heads

    def matvec(W, x):
        return [sum(float(W[i][j]) * x[j] for j in range(len(x))) for i in range(len(W))]

    def norm(x, g):
        ms = sum(v * v for v in x) / len(x)
        return [x[i] * float(g[i]) / math.sqrt(ms + s.rms_eps) for i in range(len(x))]

    def rot(vec, p):
        out = list(vec)
        half = dh // 2
        for i in range(half):
            ang = p * s.rope_theta ** (-2.0 * i / dh)
            a, b = vec[i], vec[i + half]
            out[i] = a * math.cos(ang) - b * math.sin(ang)
            out[i + half] = a * math.sin(ang) + b * math.cos(ang)
        return out

    xs = [[float(v) for v in w["tok_emb"][t]] for t in tokens]
    for l in range(s.n_layers):
        hs = [norm(x, w[f"attn_norm.{l}"]) for x in xs]
        qs = [matvec(w[f"wq.{l}"], h) for h in hs]
        ks = [matvec(w[f"wk.{l}"], h) for h in hs]
        vs = [matvec(w[f"wv.{l}"], h) for h in hs]
        new_xs = []
        for t in range(T):
            o = []
            for a in range(Hq):
                kvh = a // (Hq // Hkv)
                qa = rot(qs[t][a * dh:(a + 1) * dh], t)
                sc = []
                for j in range(t + 1):
                    kj = rot(ks[j][kvh * dh:(kvh + 1) * dh], j)
                    sc.append(sum(qa[i] * kj[i] for i in range(dh)) / math.sqrt(dh))
                m = max(sc)
                e = [math.exp(v - m) for v in sc]
                z = sum(e)
                for i in range(dh):
                    o.append(sum(e[j] / z * vs[j][kvh * dh + i] for j in range(t + 1)))
            y = matvec(w[f"wo.{l}"], o)
            x = [xs[t][i] + y[i] for i in range(d)]
            h = norm(x, w[f"mlp_norm.{l}"])
            g = matvec(w[f"w_gate.{l}"], h)
            u = matvec(w[f"w_up.{l}"], h)
            act = [g[i] / (1.0 + math.exp(-g[i])) * u[i] for i in range(len(g))]
            y = matvec(w[f"w_down.{l}"], act)
            new_xs.append([x[i] + y[i] for i in range(d)])
        xs = new_xs
    return matvec(w["lm_head"], norm(xs[-1], w["final_norm"]))


def test_cached_decode_equals_scalar_full_recompute():
    s = tiny_shape()
    w = ai.make_weights(s, seed=3)
    dec = om.Decoder(s, w)
    rng = np.random.default_rng(0)
    toks = rng.integers(0, s.vocab, size=7).tolist()
    cache = dec.new_cache()
    for t in range(len(toks)):
        got = dec.decode_step(toks[t], cache)
        want = np.array(scalar_forward(s, w, toks[:t + 1]))
        assert np.max(np.abs(got - want)) < 1e-10
        assert int(np.argmax(got)) == int(np.argmax(want))


def test_block_prefill_equals_token_by_token_and_mixed():
    s = tiny_shape(n_q_heads=4, n_kv_heads=4)
    w = ai.make_weights(s, seed=4)
    dec = om.Decoder(s, w)
    toks = np.random.default_rng(1).integers(0, s.vocab, size=11)
    c1 = dec.new_cache()
    one = np.stack([dec.decode_step(t, c1) for t in toks])
    c2 = dec.new_cache()
    blk = dec.forward_block(toks, c2)
    assert np.max(np.abs(one - blk)) < 1e-10
    c3 = dec.new_cache()
    a = dec.forward_block(toks[:4], c3)
    b = dec.forward_block(toks[4:9], c3)
    c = np.stack([dec.decode_step(t, c3) for t in toks[9:]])
    assert np.max(np.abs(np.concatenate([a, b, c]) - one)) < 1e-10
    for l in range(s.n_layers):
        assert np.max(np.abs(c1.k[l][:11] - c3.k[l][:11])) < 1e-12
        assert np.max(np.abs(c1.v[l][:11] - c3.v[l][:11])) < 1e-12


# ---------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------
def test_rmsnorm_constant_input_and_scaling():
    g = np.array([0.5, -2.0, 3.0, 1.0])
    y = om.rmsnorm(np.full(4, -7.0), g, 0.0)
    assert np.allclose(y, -g, atol=1e-15)
    x = np.array([1.0, 2.0, -3.0, 0.5])
    assert np.allclose(om.rmsnorm(x, g, 0.0), om.rmsnorm(10 * x, g, 0.0), atol=1e-14)
    # eps enters under the root, next to the mean square
    assert np.allclose(om.rmsnorm(np.array([3.0, 4.0]), np.ones(2), 0.5),
                       np.array([3.0, 4.0]) / math.sqrt(12.5 + 0.5))


def test_rope_identity_norm_and_relative_position():
    rng = np.random.default_rng(5)
    q, k = rng.standard_normal(8), rng.standard_normal(8)
    assert np.allclose(om.rope(q, 0, 10000.0), q, atol=0)
    assert np.isclose(np.linalg.norm(om.rope(q, 123, 10000.0)), np.linalg.norm(q))
    d1 = om.rope(q, 17, 10000.0) @ om.rope(k, 5, 10000.0)
    d2 = om.rope(q, 112, 10000.0) @ om.rope(k, 100, 10000.0)
    assert np.isclose(d1, d2, atol=1e-12)
    # head_dim 2, theta anything: a plain rotation by `pos` radians, counter-clockwise
    r = om.rope(np.array([1.0, 0.0]), 0.5 * math.pi / 1.0, 10000.0)
    assert np.allclose(r, [0.0, 1.0], atol=1e-15)
    # pair (i, i + half) uses frequency theta^(-2i/d): second pair of d=4 turns 100x slower
    r = om.rope(np.array([0.0, 1.0, 0.0, 0.0]), 100.0 * 0.5 * math.pi, 10000.0)
    assert np.allclose(r, [0.0, 0.0, 0.0, 1.0], atol=1e-12)


def test_attention_equal_keys_gives_mean_of_values():
    """With every key projection zero all scores tie, so each head's output is the
    running mean of the values; with W_o = W_v = identity-like maps the residual
    update is that mean."""
    s = tiny_shape(n_layers=1, d_model=8, n_q_heads=2, n_kv_heads=2, head_dim=4, d_ffn=8, vocab=11)
    w = ai.make_weights(s, seed=6)
    w["wk.0"] = np.zeros_like(w["wk.0"])
    w["wv.0"] = np.eye(8, dtype=np.float32)
    w["wo.0"] = np.eye(8, dtype=np.float32)
    w["w_down.0"] = np.zeros_like(w["w_down.0"])
    w["attn_norm.0"] = np.ones(8, dtype=np.float32)
    dec = om.Decoder(s, w)
    toks = [3, 7, 1, 7, 9]
    logits = dec.forward_block(toks, dec.new_cache())
    E = w["tok_emb"].astype(np.float64)
    hs = np.stack([om.rmsnorm(E[t], np.ones(8), s.rms_eps) for t in toks])
    for t in range(len(toks)):
        x = E[toks[t]] + hs[:t + 1].mean(axis=0)
        want = w["lm_head"].astype(np.float64) @ om.rmsnorm(x, w["final_norm"], s.rms_eps)
        assert np.max(np.abs(logits[t] - want)) < 1e-12


def test_gqa_with_repeated_kv_heads_equals_mha():
    s_g = tiny_shape(n_q_heads=4, n_kv_heads=2)
    s_m = tiny_shape(n_q_heads=4, n_kv_heads=4)
    w = ai.make_weights(s_g, seed=7)
    wm = dict(w)
    dh = s_g.head_dim
    for l in range(s_g.n_layers):
        for nm in ("wk", "wv"):
            a = w[f"{nm}.{l}"].reshape(2, dh, -1)
            wm[f"{nm}.{l}"] = np.repeat(a, 2, axis=0).reshape(4 * dh, -1)   # q head a uses kv head a//2
    toks = [1, 5, 2, 8, 13, 3]
    lg = om.Decoder(s_g, w).forward_block(toks, om.Decoder(s_g, w).new_cache())
    lm = om.Decoder(s_m, wm).forward_block(toks, om.Decoder(s_m, wm).new_cache())
    assert np.max(np.abs(lg - lm)) < 1e-12


def test_moe_single_expert_is_dense_and_full_topk_is_softmax_mixture():
    s_d = tiny_shape()
    w = ai.make_weights(s_d, seed=8)
    s_1 = tiny_shape(n_experts=1, experts_per_tok=1, d_expert_ffn=s_d.d_ffn, d_ffn=0)
    w1 = {k: v for k, v in w.items() if not k.startswith(("w_gate", "w_up", "w_down"))}
    for l in range(s_d.n_layers):
        w1[f"router.{l}"] = np.random.default_rng(l).standard_normal((1, s_d.d_model)).astype(np.float32)
        w1[f"e_gate.{l}"] = w[f"w_gate.{l}"][None]
        w1[f"e_up.{l}"] = w[f"w_up.{l}"][None]
        w1[f"e_down.{l}"] = w[f"w_down.{l}"][None]
    toks = [4, 9, 0, 17]
    a = om.Decoder(s_d, w).forward_block(toks, om.Decoder(s_d, w).new_cache())
    b = om.Decoder(s_1, w1).forward_block(toks, om.Decoder(s_1, w1).new_cache())
    assert np.max(np.abs(a - b)) < 1e-12
    # top_k == n_experts: renormalised weights are the full softmax
    rng = np.random.default_rng(9)
    E, d, F = 5, 8, 6
    h = rng.standard_normal(d)
    R, G, U, D = (rng.standard_normal(sh) for sh in ((E, d), (E, F, d), (E, F, d), (E, d, F)))
    r = np.exp(R @ h) / np.exp(R @ h).sum()
    want = sum(r[e] * om.swiglu(h, G[e], U[e], D[e]) for e in range(E))
    assert np.allclose(om.moe_mlp(h, R, G, U, D, E), want, atol=1e-13)
    # top-2: only the two largest r, renormalised
    top = np.argsort(-r)[:2]
    want2 = sum(r[e] / r[top].sum() * om.swiglu(h, G[e], U[e], D[e]) for e in top)
    assert np.allclose(om.moe_mlp(h, R, G, U, D, 2), want2, atol=1e-13)


def test_moe_equal_router_rows_keep_the_lower_expert_index():
    """Tie rule of the routing: experts 1 and 3 have the same router row, so their
    probabilities are equal bit for bit; with room for only one of them the lower index is
    kept.  Closed form: the mixture over the kept experts with renormalised weights."""
    rng = np.random.default_rng(12)
    E, d, F = 4, 8, 6
    h = rng.standard_normal(d)
    R = rng.standard_normal((E, d))
    R[3] = R[1]
    # make the tied pair the second-largest probability: scale the others
    logits = R @ h
    R[0] = R[0] * 0 + h * (logits[1] + 2.0) / (h @ h)        # expert 0: strictly larger logit
    R[2] = R[2] * 0 + h * (logits[1] - 2.0) / (h @ h)        # expert 2: strictly smaller
    G, U, D = (rng.standard_normal(sh) for sh in ((E, F, d), (E, F, d), (E, d, F)))
    r = np.exp(R @ h) / np.exp(R @ h).sum()
    assert r[1] == r[3] and r[0] > r[1] > r[2]
    want = sum(r[e] / (r[0] + r[1]) * om.swiglu(h, G[e], U[e], D[e]) for e in (0, 1))
    assert np.allclose(om.moe_mlp(h, R, G, U, D, 2), want, atol=1e-13)
    wrong = sum(r[e] / (r[0] + r[3]) * om.swiglu(h, G[e], U[e], D[e]) for e in (0, 3))
    assert not np.allclose(wrong, want, atol=1e-6)
    # with room for both, both are kept
    want3 = sum(r[e] / (r[0] + r[1] + r[3]) * om.swiglu(h, G[e], U[e], D[e]) for e in (0, 1, 3))
    assert np.allclose(om.moe_mlp(h, R, G, U, D, 3), want3, atol=1e-13)


def test_silu_and_swiglu_values():
    assert om.silu(0.0) == 0.0
    assert math.isclose(om.silu(1.0), 1.0 / (1.0 + math.exp(-1.0)))
    # 1x1 matrices: (silu(2*3) * (5*3)) * 7
    got = om.swiglu(np.array([3.0]), np.array([[2.0]]), np.array([[5.0]]), np.array([[7.0]]))
    assert math.isclose(got[0], 6.0 / (1.0 + math.exp(-6.0)) * 15.0 * 7.0)


# ---------------------------------------------------------------------------
# independent rebuild from torch CPU library ops (complex-number rotary,
# scaled_dot_product_attention, rms_norm, silu)
# ---------------------------------------------------------------------------
def test_against_torch_library_ops():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    s = tiny_shape(n_layers=3, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=40, vocab=50)
    w = ai.make_weights(s, seed=10)
    toks = np.random.default_rng(2).integers(0, s.vocab, size=13)
    want = om.Decoder(s, w).forward_block(toks, om.Decoder(s, w).new_cache())

    tw = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    T = len(toks)
    x = tw["tok_emb"][torch.from_numpy(toks.astype(np.int64))]
    half = s.head_dim // 2
    inv = s.rope_theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / s.head_dim)
    phase = torch.polar(torch.ones(T, half, dtype=torch.float64),
                        torch.arange(T, dtype=torch.float64)[:, None] * inv)      # e^{i p w}

    def rot(t):                                   # t [T, H, dh]; pair (i, i+half) is one complex number
        z = torch.complex(t[..., :half], t[..., half:]) * phase[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(s.n_layers):
        h = F.rms_norm(x, (s.d_model,), tw[f"attn_norm.{l}"], s.rms_eps)
        q = rot(F.linear(h, tw[f"wq.{l}"]).view(T, s.n_q_heads, s.head_dim)).transpose(0, 1)
        k = rot(F.linear(h, tw[f"wk.{l}"]).view(T, s.n_kv_heads, s.head_dim)).transpose(0, 1)
        v = F.linear(h, tw[f"wv.{l}"]).view(T, s.n_kv_heads, s.head_dim).transpose(0, 1)
        rep = s.n_q_heads // s.n_kv_heads
        o = F.scaled_dot_product_attention(q[None], k.repeat_interleave(rep, 0)[None],
                                           v.repeat_interleave(rep, 0)[None], is_causal=True)[0]
        x = x + F.linear(o.transpose(0, 1).reshape(T, -1), tw[f"wo.{l}"])
        h = F.rms_norm(x, (s.d_model,), tw[f"mlp_norm.{l}"], s.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, tw[f"w_gate.{l}"])) * F.linear(h, tw[f"w_up.{l}"]),
                         tw[f"w_down.{l}"])
    got = F.linear(F.rms_norm(x, (s.d_model,), tw["final_norm"], s.rms_eps), tw["lm_head"]).numpy()
    assert np.max(np.abs(got - want)) < 1e-10
