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


# ---- policy update between steps (Eq. 1; Section 2.2, mixed-policy trajectories) -----------
def run_with_update(w, weights_by_step, keep_kv, steps=4):
    """weights_by_step[k] = weights in force during step k.  Returns per request: final tokens,
    and how many tokens it had when each update happened."""
    decs = {id(x): Decoder(w.shape, x) for x in weights_by_step}
    eng = OracleRollouts(decs[id(weights_by_step[0])], "greedy", seed=w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w, steps))
    rolls = [eng.make_rollout(r.request_id, r.tokens, r.forced_len) for r in reqs]
    nxt, done, had = 0, {}, {}
    for k in range(steps):
        if k > 0 and weights_by_step[k] is not weights_by_step[k - 1]:
            eng.update_weights(decs[id(weights_by_step[k])], keep_kv=keep_kv)
            for r in eng.buffer:
                had.setdefault(r.request_id, []).append((k, r.gen))
        out = eng.step(rolls[nxt:], w.n_target, w.n_overprovision, w.max_new)
        nxt += out.n_new_consumed
        for r in out.completed:
            done[r.request_id] = list(r.tokens)
    return reqs, done, had, decs


def greedy_continue(dec, prefix, n):
    """n greedy tokens after `prefix` by full recompute of the whole sequence for every token."""
    seq, out = list(prefix), []
    for _ in range(n):
        tok = int(np.argmax(dec.forward_block(seq, dec.new_cache())[-1]))
        out.append(tok)
        seq.append(tok)
    return out


def test_update_with_the_same_weights_changes_nothing():
    w = tiny_workload(ai.SAMPLER_GREEDY)
    wa = ai.make_weights(w.shape, w.seed)
    wa2 = {k: v.copy() for k, v in wa.items()}
    _, plain, _ = run(w, w.n_overprovision, 4)
    for keep in (False, True):
        _, upd, had, _ = run_with_update(w, [wa, wa2, wa, wa2], keep)
        assert had and upd == plain


def test_after_an_update_rollouts_continue_under_the_new_weights():
    """Weights change once, before step 3.  A rollout that was parked then has tokens from the
    old policy followed by tokens from the new one: the latter equal what the new decoder
    generates from the token prefix by full recompute (nothing of the old cache survives)."""
    w = tiny_workload(ai.SAMPLER_GREEDY)
    wa, wb = ai.make_weights(w.shape, w.seed), ai.make_weights(w.shape, w.seed + 100)
    reqs, done, had, decs = run_with_update(w, [wa, wa, wb, wb], keep_kv=False)
    checked = 0
    for rid, marks in had.items():
        if rid not in done:
            continue
        (k, n_before), = marks
        assert k == 2
        toks = done[rid]
        prefix = list(reqs[rid].tokens) + toks[:n_before]
        want = greedy_continue(decs[id(wb)], prefix, len(toks) - n_before)
        assert toks[n_before:] == want, rid
        # and the part before the update is the old policy's
        assert toks[:n_before] == greedy_continue(decs[id(wa)], list(reqs[rid].tokens), n_before)
        checked += len(want)
    assert checked > 10
    # requests admitted after the update are the new policy's from the first token
    new_ids = [rid for rid in done if rid not in had and rid >= max(had)]
    rid = new_ids[-1]
    assert done[rid] == greedy_continue(decs[id(wb)], list(reqs[rid].tokens), len(done[rid]))


def test_stale_kv_variant_keeps_the_old_cache():
    """keep_kv = True: positions cached before the update keep the old policy's keys / values; new
    positions use the new weights.  Replayed by hand for one rollout: old decoder builds the
    cache over the prefix, new decoder decodes on top of it."""
    w = tiny_workload(ai.SAMPLER_GREEDY)
    wa, wb = ai.make_weights(w.shape, w.seed), ai.make_weights(w.shape, w.seed + 100)
    reqs, stale, had, decs = run_with_update(w, [wa, wa, wb, wb], keep_kv=True)
    _, fresh, _, _ = run_with_update(w, [wa, wa, wb, wb], keep_kv=False)
    assert any(stale[r] != fresh[r] for r in had if r in stale and r in fresh)
    rid = next(r for r in had if r in stale and len(stale[r]) - had[r][0][1] >= 3)
    n_before = had[rid][0][1]
    old, new = decs[id(wa)], decs[id(wb)]
    cache = old.new_cache()
    prefix = list(reqs[rid].tokens) + stale[rid][:n_before]
    old.forward_block(prefix[:-1], cache)                 # K/V of every position but the last fed token
    tok_in, out = prefix[-1], []
    for _ in range(len(stale[rid]) - n_before):
        tok_in = int(np.argmax(new.decode_step(tok_in, cache)))
        out.append(tok_in)
    assert stale[rid][n_before:] == out
