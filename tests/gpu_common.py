"""Helpers shared by the GPU parity tests: run the same seeded workload through the
HIP library (C ABI via the ctypes binding) and through the CPU oracle."""
import numpy as np

import april_inputs as ai
import paper_2509_18521_amd as ap
from oracle.model import Decoder
from oracle.rollout import OracleRollouts


def have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def sampler_name(w):
    return "greedy" if w.sampler == ai.SAMPLER_GREEDY else "topk"


def make_engine(w, weights, *, debug=False, max_inflight=None, max_ctx=None, temperature=1.0, eos=-1,
                kv_pool_bytes=0, top_p=0.0, logprobs=False, sampler=None, group_size=0, pausable=False):
    s = w.shape
    cfg = ap.make_cfg(s, max_inflight=max_inflight or (w.n_overprovision + 8),
                      max_ctx=max_ctx or (w.prompt_len + w.max_new + 16),
                      sampler=w.sampler if sampler is None else sampler, top_k=max(w.top_k, 1),
                      temperature=temperature, seed=w.seed, eos_token=eos, debug_logits=debug,
                      kv_pool_bytes=kv_pool_bytes, top_p=top_p, logprobs=logprobs,
                      n_samples_per_prompt=group_size, pausable=pausable)
    return ap.april_init(cfg, ap.pack_weights(s, weights))


def req_dicts(reqs, forced=None, group_size=0):
    out = []
    for r in reqs:
        d = dict(request_id=r.request_id, tokens=r.tokens, forced_len=r.forced_len)
        if group_size > 1:
            d["group_id"] = r.request_id // group_size
        if forced is not None and r.request_id in forced:
            d["forced_tokens"] = np.asarray(forced[r.request_id], dtype=np.int32)
        out.append(d)
    return out


def run_gpu(ctx, reqs, n_target, n_over, max_new, steps, *, forced=None, between=None, allow_short=False,
            group_size=0):
    """-> list of per-step dicts (ids, tokens, stats, buffer view).  `between(ctx, buffer)`
    may act on the buffer (e.g. drop its KV) before it is resumed; it returns the
    buffer handle to resume."""
    nxt, out = 0, []
    for _ in range(steps):
        res = ap.april_rollout_step(ctx, req_dicts(reqs[nxt:], forced, group_size), n_target, n_over, max_new)
        nxt += res.n_new_consumed
        view = ap.april_buffer_export(ctx, res.buffer)
        out.append(dict(ids=res.request_id, tokens=[t.tolist() for t in res.tokens], n_resumes=res.n_resumes,
                        consumed=res.n_new_consumed, iters=res.decode_iters, generated=res.tokens_generated,
                        buffer=[(p["request_id"], len(p["generated"]), p["done"]) for p in view],
                        buffer_tokens={p["request_id"]: p["generated"].tolist() for p in view},
                        sum_live=res.sum_live, res=res, n_preempted=res.n_preempted, groups=res.group_id,
                        logprobs=None if res.logprobs is None else [l.tolist() for l in res.logprobs],
                        buffer_logprobs={p["request_id"]: p["logprobs"] for p in view},
                        kv_resident={p["request_id"]: p["kv_resident"] for p in view}))
        buf = res.buffer
        if between is not None:
            buf = between(ctx, buf)
        ap.april_resume(ctx, buf)
    return out


def run_oracle(w, weights, reqs, n_target, n_over, max_new, steps, *, keep_logits=False, temperature=1.0,
               eos=-1, drop_kv=False, pool=None, top_p=1.0, sampler=None):
    eng = OracleRollouts(Decoder(w.shape, weights), sampler or sampler_name(w), top_k=max(w.top_k, 1),
                         temperature=temperature, seed=w.seed, eos_token=eos, keep_logits=keep_logits, top_p=top_p)
    rolls = [eng.make_rollout(r.request_id, r.tokens, r.forced_len) for r in reqs]
    nxt, out = 0, []
    for _ in range(steps):
        if drop_kv:
            eng.drop_kv()
        o = eng.step(rolls[nxt:], n_target, n_over, max_new, pool=pool)
        nxt += o.n_new_consumed
        out.append(dict(ids=[r.request_id for r in o.completed], tokens=[list(r.tokens) for r in o.completed],
                        n_resumes=[r.n_resumes for r in o.completed], consumed=o.n_new_consumed,
                        iters=o.decode_iters, generated=o.tokens_generated,
                        buffer=[(r.request_id, r.gen, int(r.done)) for r in o.buffer],
                        buffer_tokens={r.request_id: list(r.tokens) for r in o.buffer},
                        logprobs=[list(r.user.get("logprobs", [])) for r in o.completed],
                        sum_live=sum(o.live_per_iter), n_preempted=len(o.preempted),
                        kv_resident={r.request_id: int(r.kv > 0) for r in o.buffer}))
    return out, eng


def assert_schedule_equal(got, want):
    """Scheduling outputs are integers: bit-exact."""
    assert len(got) == len(want)
    for k, (g, o) in enumerate(zip(got, want)):
        for key in ("ids", "consumed", "iters", "generated", "buffer", "n_resumes"):
            assert g[key] == o[key], (k, key, g[key], o[key])
        assert [len(t) for t in g["tokens"]] == [len(t) for t in o["tokens"]]


def top2_margin(logits):
    p = np.partition(np.asarray(logits, dtype=np.float64), -2)
    return float(p[-1] - p[-2])


# ---------------------------------------------------------------------------
# Teacher forcing with tokens of the test's own choosing.  The schedule does not depend on
# the token values, and logits parity holds for any fed sequence, so wide models with
# hundreds of rollouts in flight can be compared without the oracle generating token by
# token: request r uses prompt r mod P and is forced the tokens of "class" r mod P, so the
# oracle needs one block forward per class (row P_len - 1 + i predicts generated token i).
# ---------------------------------------------------------------------------
def class_forced_tokens(w, n_classes, seed_tag=303):
    rng = np.random.default_rng([w.seed, seed_tag])
    return rng.integers(0, w.shape.vocab, size=(n_classes, w.max_new), dtype=np.int32)


def run_oracle_schedule(reqs, forced, n_target, n_over, max_new, steps, pool=None):
    """Scheduling half of the oracle alone (integers), fed the forced tokens."""
    from oracle.scheduler import Rollout, rollout_step
    rolls = [Rollout(request_id=r.request_id, prompt_len=len(r.tokens), forced_len=r.forced_len) for r in reqs]
    buf, nxt, out = [], 0, []
    for _ in range(steps):
        o = rollout_step(buf, rolls[nxt:], n_target, n_over, max_new,
                         next_token=lambda r: int(forced[r.request_id][r.gen]), pool=pool)
        buf = o.buffer
        nxt += o.n_new_consumed
        out.append(dict(ids=[r.request_id for r in o.completed], tokens=[list(r.tokens) for r in o.completed],
                        n_resumes=[r.n_resumes for r in o.completed], consumed=o.n_new_consumed,
                        iters=o.decode_iters, generated=o.tokens_generated,
                        buffer=[(r.request_id, r.gen, int(r.done)) for r in o.buffer],
                        buffer_tokens={r.request_id: list(r.tokens) for r in o.buffer},
                        sum_live=sum(o.live_per_iter), n_preempted=len(o.preempted),
                        kv_resident={r.request_id: int(r.kv > 0) for r in o.buffer}))
    return out


def class_reference_logits(dec, prompts, class_tokens, n_gen):
    """Oracle logits of every class: ref[c][i] = logits that predict generated token i."""
    ref = []
    for c in range(len(prompts)):
        feed = np.concatenate([prompts[c], class_tokens[c][:n_gen - 1]])
        rows = dec.forward_block(feed, dec.new_cache())
        ref.append(rows[len(prompts[c]) - 1:])
    return ref
