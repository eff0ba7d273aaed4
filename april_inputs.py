"""Seeded synthetic inputs for the APRIL rollout path: model shapes, random-init
weights, prompt pools, forced response lengths, request streams.

This module is shared by the CPU oracle's tests and by the GPU path's tests and
benchmark.  It holds NO arithmetic of the method itself: only shapes, seeded
random draws and the (lossless to describe) rounding of weights to bf16 values.

The workloads stand in for the paper's math-reasoning rollouts (Section 3.2,
long-tail length histogram): response lengths are drawn from a clipped
lognormal so that more than half of the responses finish early while a tail
reaches the length cap.  Termination is *forced* at the drawn length, so the
scheduling is independent of the model's logits.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, replace
from typing import Dict, Iterator, List, Optional, Tuple

import numpy as np

DTYPE_FP32 = 0
DTYPE_BF16 = 1

SAMPLER_GREEDY = 0
SAMPLER_TOPK = 1
SAMPLER_CATEGORICAL = 2


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_experts: int = 0
    experts_per_tok: int = 0
    d_expert_ffn: int = 0
    dtype: int = DTYPE_BF16
    rope_theta: float = 10000.0
    rms_eps: float = 1e-6

    @property
    def is_moe(self) -> bool:
        return self.n_experts > 0


@dataclass(frozen=True)
class Workload:
    """One of the benchmark configurations: model + request stream + APRIL sizes."""
    name: str
    shape: ModelShape
    n_prompts: int            # size of the prompt pool
    prompt_len: int
    n_target: int             # N
    n_overprovision: int      # N'
    max_new: int
    len_mu: float
    len_sigma: float
    len_lo: int
    len_hi: int
    sampler: int
    top_k: int
    steps: int
    seed: int
    kv_block_tokens: int = 16


WORKLOADS: Dict[str, Workload] = {
    "cfg1_tiny_fp32": Workload(
        "cfg1_tiny_fp32",
        ModelShape(2, 128, 4, 4, 32, 512, 512, dtype=DTYPE_FP32),
        16, 32, 16, 24, 256, 4.0, 0.8, 8, 256, SAMPLER_GREEDY, 0, 3, 0),
    "cfg2_small_bf16": Workload(
        "cfg2_small_bf16",
        ModelShape(24, 896, 14, 2, 64, 4864, 151936),
        64, 256, 64, 96, 2048, 6.0, 1.0, 32, 2048, SAMPLER_TOPK, 50, 5, 1),
    "cfg3_mid_bf16": Workload(
        "cfg3_mid_bf16",
        ModelShape(36, 2560, 32, 8, 128, 9728, 151936),
        128, 512, 128, 192, 4096, 6.8, 1.1, 64, 4096, SAMPLER_GREEDY, 0, 5, 2),
    "cfg4_8b_bf16": Workload(
        "cfg4_8b_bf16",
        ModelShape(32, 4096, 32, 8, 128, 14336, 128256),
        256, 512, 256, 384, 8192, 7.2, 1.2, 128, 8192, SAMPLER_GREEDY, 0, 8, 3),
    "cfg5_moe_bf16": Workload(
        "cfg5_moe_bf16",
        ModelShape(48, 2048, 32, 4, 128, 0, 151936, n_experts=128,
                   experts_per_tok=8, d_expert_ffn=768),
        256, 1024, 256, 384, 8192, 7.2, 1.2, 128, 8192, SAMPLER_GREEDY, 0, 8, 4),
}


def reduced(w: Workload, **shape_overrides) -> Workload:
    """Same workload with some model-shape fields overridden (e.g. fewer layers)."""
    return replace(w, shape=replace(w.shape, **shape_overrides))


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit conversion (round to nearest even), used only to produce
# weight VALUES that are exactly representable in bf16.
# ----------------------------------------------------------------------------
def fp32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_fp32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------
def weight_specs(s: ModelShape) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) for every tensor; matrices are [out_features, in_features]
    (y = W x); kind is 'emb', 'gain' or 'linear'."""
    qd, kvd = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    specs: List[Tuple[str, Tuple[int, ...], str]] = [("tok_emb", (s.vocab, s.d_model), "emb")]
    for l in range(s.n_layers):
        specs += [
            (f"attn_norm.{l}", (s.d_model,), "gain"),
            (f"wq.{l}", (qd, s.d_model), "linear"),
            (f"wk.{l}", (kvd, s.d_model), "linear"),
            (f"wv.{l}", (kvd, s.d_model), "linear"),
            (f"wo.{l}", (s.d_model, qd), "linear"),
            (f"mlp_norm.{l}", (s.d_model,), "gain"),
        ]
        if s.is_moe:
            specs += [
                (f"router.{l}", (s.n_experts, s.d_model), "linear"),
                (f"e_gate.{l}", (s.n_experts, s.d_expert_ffn, s.d_model), "linear"),
                (f"e_up.{l}", (s.n_experts, s.d_expert_ffn, s.d_model), "linear"),
                (f"e_down.{l}", (s.n_experts, s.d_model, s.d_expert_ffn), "linear"),
            ]
        else:
            specs += [
                (f"w_gate.{l}", (s.d_ffn, s.d_model), "linear"),
                (f"w_up.{l}", (s.d_ffn, s.d_model), "linear"),
                (f"w_down.{l}", (s.d_model, s.d_ffn), "linear"),
            ]
    specs += [("final_norm", (s.d_model,), "gain"), ("lm_head", (s.vocab, s.d_model), "linear")]
    return specs


def _tensor_rng(seed: int, name: str) -> np.random.Generator:
    h = hashlib.sha256(f"{seed}/{name}".encode()).digest()
    return np.random.default_rng(int.from_bytes(h[:16], "little"))


def weight_tensor(s: ModelShape, name: str, shape: Tuple[int, ...], kind: str, seed: int) -> np.ndarray:
    """One random-init tensor as fp32 values (already bf16-representable when the
    model dtype is bf16).  Linear ~ N(0, 1/fan_in), embedding ~ N(0, 1),
    gains ~ 1 + 0.1 N(0, 1) (non-trivial on purpose, so a misplaced gain shows)."""
    rng = _tensor_rng(seed, name)
    if kind == "emb":
        a = rng.standard_normal(shape, dtype=np.float32)
    elif kind == "gain":
        a = (1.0 + 0.1 * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
    else:
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= np.float32(1.0 / np.sqrt(shape[-1]))
    if s.dtype == DTYPE_BF16:
        a = bf16_bits_to_fp32(fp32_to_bf16_bits(a)).reshape(shape)
    return a


def iter_weights(s: ModelShape, seed: int) -> Iterator[Tuple[str, np.ndarray]]:
    for name, shape, kind in weight_specs(s):
        yield name, weight_tensor(s, name, shape, kind, seed)


def make_weights(s: ModelShape, seed: int) -> Dict[str, np.ndarray]:
    return dict(iter_weights(s, seed))


def n_params(s: ModelShape) -> int:
    return int(sum(int(np.prod(shape)) for _, shape, _ in weight_specs(s)))


# ----------------------------------------------------------------------------
# prompts, lengths, requests
# ----------------------------------------------------------------------------
def make_prompts(n_prompts: int, prompt_len: int, vocab: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 101])
    return rng.integers(0, vocab, size=(n_prompts, prompt_len), dtype=np.int32)


def make_forced_lengths(n: int, mu: float, sigma: float, lo: int, hi: int, seed: int) -> np.ndarray:
    """clip(rint(exp(mu + sigma z)), lo, hi), z standard normal; drawn once here and
    handed as integers to both sides."""
    rng = np.random.default_rng([seed, 202])
    z = rng.standard_normal(n)
    return np.clip(np.rint(np.exp(mu + sigma * z)), lo, hi).astype(np.int32)


@dataclass
class Request:
    request_id: int
    tokens: np.ndarray        # prompt, int32
    forced_len: int           # finish exactly at this many generated tokens


def make_requests(w: Workload, n_requests: int) -> List[Request]:
    """Request r (global, monotone id) uses prompt r mod pool size and its own length."""
    prompts = make_prompts(w.n_prompts, w.prompt_len, w.shape.vocab, w.seed)
    lens = make_forced_lengths(n_requests, w.len_mu, w.len_sigma, w.len_lo, w.len_hi, w.seed)
    return [Request(r, prompts[r % w.n_prompts].copy(), int(lens[r])) for r in range(n_requests)]


def requests_needed(w: Workload, steps: Optional[int] = None, n_over: Optional[int] = None) -> int:
    """Upper bound on how many requests `steps` steps can admit."""
    steps = w.steps if steps is None else steps
    n_over = w.n_overprovision if n_over is None else n_over
    return n_over + steps * max(w.n_target, n_over)
