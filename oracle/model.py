"""Plain CPU decoder-only transformer (oracle side), numpy, float64.

TEST INFRASTRUCTURE ONLY: nothing under oracle/ is part of the product path,
and nothing here shares code with the HIP path.

What it computes.  The paper's rollout phase is "the inference engine
generates rollouts auto-regressively" (Section 1; Eq. 1, the a ~ pi(theta_k)
term); the paper fixes no architecture beyond naming Qwen3 dense decoders
(Section 3.1), so the network is the textbook pre-norm decoder those models
belong to, in the reading the build documents: RMSNorm -> q/k/v projections
(no bias) -> rotary embedding on q and k (rotate-half pairing) -> causal
softmax attention with grouped KV heads -> output projection + residual ->
RMSNorm -> SwiGLU MLP (or top-k routed mixture of SwiGLU experts) + residual;
final RMSNorm; untied LM head.

All matrices are [out_features, in_features]: y = W @ x.

Pins (tests/test_oracle_model.py): token-by-token KV-cached decode equals a
scalar-loop full recompute written separately; block prefill equals
token-by-token decode; closed forms (equal keys => mean of V, position 0 =>
rotary is identity, rotary keeps norms and makes q.k depend on the position
difference only, constant input => RMSNorm gives g*sign); MoE with one expert
equals the dense MLP; an independent re-build from torch CPU library ops.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def rmsnorm(x, g, eps):
    """y_i = x_i * g_i / sqrt(mean_j x_j^2 + eps) over the last axis."""
    x = np.asarray(x, dtype=F64)
    return x * g / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope(v, pos, theta):
    """Rotary embedding of v[..., head_dim] at integer position `pos` (scalar or an
    array broadcastable to v[..., 0]).  Pair (i, i + head_dim/2) is rotated by the
    angle pos * theta**(-2i/head_dim)."""
    v = np.asarray(v, dtype=F64)
    dh = v.shape[-1]
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=F64) / dh)
    ang = np.asarray(pos, dtype=F64)[..., None] * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax(s):
    s = np.asarray(s, dtype=F64)
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(x):
    return x / (1.0 + np.exp(-x))


def swiglu(h, w_gate, w_up, w_down):
    """(silu(W_g h) * (W_u h)) through W_d, for h [..., d]."""
    return (silu(h @ w_gate.T) * (h @ w_up.T)) @ w_down.T


def moe_mlp(h, router, e_gate, e_up, e_down, top_k, margins=None):
    """Routed mixture for ONE token h [d]: r = softmax over all experts of the
    router logits; the top_k largest r (ties: lower expert index) are kept and
    renormalised to sum 1; output = sum of weight * expert SwiGLU.
    margins (optional list): receives the relative gap between the last kept and the
    first dropped router probability (how robust the routing decision is)."""
    r = softmax(router @ h)
    ranked = sorted(range(r.shape[0]), key=lambda e: (-r[e], e))
    order = ranked[:top_k]
    if margins is not None:
        margins.append((r[ranked[top_k - 1]] - r[ranked[top_k]]) / r[ranked[top_k - 1]]
                       if top_k < r.shape[0] else 1.0)
    z = sum(r[e] for e in order)
    out = np.zeros_like(h)
    for e in order:
        out = out + (r[e] / z) * swiglu(h, e_gate[e], e_up[e], e_down[e])
    return out


class KVCache:
    """Per-sequence cache of rotated keys and values: k[l], v[l] are [len, H_kv, d_h]."""

    def __init__(self, n_layers, n_kv_heads, head_dim, capacity=0):
        self.k = [np.zeros((capacity, n_kv_heads, head_dim), F64) for _ in range(n_layers)]
        self.v = [np.zeros((capacity, n_kv_heads, head_dim), F64) for _ in range(n_layers)]
        self.len = 0

    def ensure(self, need):
        cap = self.k[0].shape[0]
        if need <= cap:
            return
        new_cap = max(need, 2 * cap, 64)
        for arrs in (self.k, self.v):
            for l in range(len(arrs)):
                a = np.zeros((new_cap,) + arrs[l].shape[1:], F64)
                a[:cap] = arrs[l]
                arrs[l] = a


class Decoder:
    def __init__(self, shape, weights):
        """shape: object with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn,
        vocab, n_experts, experts_per_tok, rope_theta, rms_eps.  weights: name -> array."""
        self.s = shape
        self.w = {k: np.asarray(v, dtype=F64) for k, v in weights.items()}
        self.route_margins = None     # set to a list to collect (position, layer, margin) of routed layers

    def new_cache(self, capacity=0):
        s = self.s
        return KVCache(s.n_layers, s.n_kv_heads, s.head_dim, capacity)

    def forward_block(self, tokens, cache):
        """Feed `tokens` (T >= 1 ints) at positions cache.len .. cache.len+T-1, append
        their keys/values to the cache, and return the logits [T, vocab] of every fed
        position (row t predicts the token after tokens[t])."""
        s, w = self.s, self.w
        tokens = np.asarray(tokens, dtype=np.int64)
        T = tokens.shape[0]
        p0 = cache.len
        cache.ensure(p0 + T)
        pos = np.arange(p0, p0 + T)
        group = s.n_q_heads // s.n_kv_heads
        x = w["tok_emb"][tokens]                                   # [T, d]
        for l in range(s.n_layers):
            h = rmsnorm(x, w[f"attn_norm.{l}"], s.rms_eps)
            q = (h @ w[f"wq.{l}"].T).reshape(T, s.n_q_heads, s.head_dim)
            k = (h @ w[f"wk.{l}"].T).reshape(T, s.n_kv_heads, s.head_dim)
            v = (h @ w[f"wv.{l}"].T).reshape(T, s.n_kv_heads, s.head_dim)
            q = rope(q, pos[:, None], s.rope_theta)
            k = rope(k, pos[:, None], s.rope_theta)
            cache.k[l][p0:p0 + T] = k
            cache.v[l][p0:p0 + T] = v
            K = cache.k[l][:p0 + T]                                # [C, H_kv, d_h]
            V = cache.v[l][:p0 + T]
            # key j is visible to the query at position p iff j <= p
            visible = np.arange(p0 + T)[None, :] <= pos[:, None]   # [T, C]
            o = np.zeros((T, s.n_q_heads, s.head_dim), F64)
            for a in range(s.n_q_heads):
                kvh = a // group
                sc = (q[:, a, :] @ K[:, kvh, :].T) / np.sqrt(float(s.head_dim))
                sc = np.where(visible, sc, -np.inf)
                o[:, a, :] = softmax(sc) @ V[:, kvh, :]
            x = x + o.reshape(T, -1) @ w[f"wo.{l}"].T
            h = rmsnorm(x, w[f"mlp_norm.{l}"], s.rms_eps)
            if s.n_experts > 0:
                ys = []
                for t in range(T):
                    mg = [] if self.route_margins is not None else None
                    ys.append(moe_mlp(h[t], w[f"router.{l}"], w[f"e_gate.{l}"], w[f"e_up.{l}"],
                                      w[f"e_down.{l}"], s.experts_per_tok, mg))
                    if mg is not None:
                        self.route_margins.append((int(pos[t]), l, float(mg[0])))
                y = np.stack(ys)
            else:
                y = swiglu(h, w[f"w_gate.{l}"], w[f"w_up.{l}"], w[f"w_down.{l}"])
            x = x + y
        cache.len = p0 + T
        return rmsnorm(x, w["final_norm"], s.rms_eps) @ w["lm_head"].T

    def decode_step(self, token, cache):
        """One token in, logits [vocab] of the next token out."""
        return self.forward_block([token], cache)[0]
