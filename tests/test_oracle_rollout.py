"""APRIL invariants on the oracle's full path (model + sampler + scheduler), tiny model."""
import numpy as np
import pytest

import april_inputs as ai
from oracle.model import Decoder
from oracle.rollout import OracleRollouts


def tiny_workload(sampler):
    shape = ai.ModelShape(2, 32, 4, 2, 8, 48, 64, dtype=ai.DTYPE_FP32)
    return ai.Workload("tiny", shape, 6, 5, 4, 7, 24, 2.0, 0.7, 2, 24, sampler, 8, 4, 11)


def run(w, n_over, steps, drop_kv=False):
    dec = Decoder(w.shape, ai.make_weights(w.shape, w.seed))
    eng = OracleRollouts(dec, "greedy" if w.sampler == ai.SAMPLER_GREEDY else "topk",
                         top_k=w.top_k, temperature=1.0, seed=w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w, steps, n_over))
    rolls = [eng.make_rollout(r.request_id, r.tokens, r.forced_len) for r in reqs]
    nxt, done = 0, {}
    for _ in range(steps):
        if drop_kv:
            eng.drop_kv()
        out = eng.step(rolls[nxt:], w.n_target, n_over, w.max_new)
        nxt += out.n_new_consumed
        for r in out.completed:
            done[r.request_id] = list(r.tokens)
    return reqs, done, dec


@pytest.mark.parametrize("sampler", [ai.SAMPLER_GREEDY, ai.SAMPLER_TOPK])
def test_resumed_equals_uninterrupted_and_equals_reprefill(sampler):
    w = tiny_workload(sampler)
    reqs, april, dec = run(w, w.n_overprovision, w.steps)
    _, waitall, _ = run(w, w.n_target, w.steps)
    _, reprefill, _ = run(w, w.n_overprovision, w.steps, drop_kv=True)
    assert any(True for _ in april)
    # every rollout, however it was scheduled, equals the rollout generated alone
    eng = OracleRollouts(dec, "greedy" if sampler == ai.SAMPLER_GREEDY else "topk",
                         top_k=w.top_k, temperature=1.0, seed=w.seed)
    for rid, toks in april.items():
        solo = eng.make_rollout(rid, reqs[rid].tokens, reqs[rid].forced_len)
        eng.buffer = []
        out = eng.step([solo], 1, 1, w.max_new)
        assert out.completed[0].tokens == toks
        assert len(toks) == min(reqs[rid].forced_len, w.max_new)
    for rid in set(april) & set(waitall):
        assert april[rid] == waitall[rid]
    assert set(reprefill) == set(april)
    for rid in april:
        assert april[rid] == reprefill[rid]


def test_cfg1_lengths_follow_forced_lengths():
    w = ai.WORKLOADS["cfg1_tiny_fp32"]
    lens = ai.make_forced_lengths(100, w.len_mu, w.len_sigma, w.len_lo, w.len_hi, w.seed)
    assert lens.min() >= w.len_lo and lens.max() <= w.len_hi
    assert 30 < np.median(lens) < 90          # lognormal(mu=4): median ~ e^4 = 55
