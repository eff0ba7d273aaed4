"""GPU parity: the HIP rollout path (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

import april_inputs as ai
from gpu_common import (assert_schedule_equal, have_gpu, make_engine, req_dicts, run_gpu, run_oracle,
                        top2_margin)

pytestmark = pytest.mark.gpu

FP32_LOGIT_TOL = 1e-4          # max-abs, fp32 configuration (the benchmark spec)
BF16_LOGIT_TOL = 2e-2          # max-abs relative to logit scale max(1, max|l_ref|)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not have_gpu():
        pytest.skip("no GPU")


def ap():
    import paper_2509_18521_amd
    return paper_2509_18521_amd


def compare_free_running_tokens(got_steps, want_steps, oracle_eng, tol):
    """Greedy tokens must be identical wherever the oracle's top-2 margin exceeds tol;
    after the first sub-tolerance position of a rollout the two may legitimately part."""
    checked = 0
    for g, o in zip(got_steps, want_steps):
        for rid, gt, ot in zip(g["ids"], g["tokens"], o["tokens"]):
            for i, (a, b) in enumerate(zip(gt, ot)):
                lg = oracle_eng.logits.get((rid, i))
                if lg is not None and top2_margin(lg) <= tol:
                    break
                assert a == b, (rid, i, a, b)
                checked += 1
    return checked


def test_cfg1_full_scenario_fp32():
    """Config 1 end to end: 3 APRIL steps, scheduling bit-exact, greedy tokens identical,
    logits of watched rollouts within 1e-4."""
    w = ai.WORKLOADS["cfg1_tiny_fp32"]
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    want, eng = run_oracle(w, weights, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps, keep_logits=True)
    ctx = make_engine(w, weights, debug=True)
    try:
        watched = [0, 3, 7, 17, 23, 30]
        for rid in watched:
            ap().april_debug_watch(ctx, rid, 0, 256)
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)
        assert_schedule_equal(got, want)
        n = compare_free_running_tokens(got, want, eng, FP32_LOGIT_TOL)
        assert n > 1000
        worst, rows = 0.0, 0
        final = {}
        for g in got:
            final.update(dict(zip(g["ids"], g["tokens"])))
        final.update(got[-1]["buffer_tokens"])
        oracle_tokens = {}
        for o in want:
            oracle_tokens.update(dict(zip(o["ids"], o["tokens"])))
        oracle_tokens.update(want[-1]["buffer_tokens"])
        for rid in watched:
            if rid not in final:
                continue
            for i in range(len(final[rid])):
                if final[rid][:i] != oracle_tokens[rid][:i]:
                    break                                   # prefixes differ: logits are not comparable
                lg, sampled = ap().april_debug_logits(ctx, rid, i, w.shape.vocab)
                ref = eng.logits[(rid, i)]
                worst = max(worst, float(np.max(np.abs(lg - ref))))
                rows += 1
                if top2_margin(ref) > FP32_LOGIT_TOL:
                    assert sampled == int(np.argmax(ref))
        assert rows > 100
        assert worst <= FP32_LOGIT_TOL, worst
    finally:
        ap().april_destroy(ctx)


def small_fp32_workload(sampler=ai.SAMPLER_GREEDY, top_k=0):
    shape = ai.ModelShape(2, 64, 4, 2, 32, 96, 200, dtype=ai.DTYPE_FP32)
    return ai.Workload("small", shape, 8, 21, 6, 10, 40, 2.6, 0.7, 2, 40, sampler, top_k, 4, 21)


@pytest.mark.parametrize("sampler,top_k", [(ai.SAMPLER_GREEDY, 0), (ai.SAMPLER_TOPK, 8)])
def test_resumed_equals_uninterrupted_and_wait_all(sampler, top_k):
    """APRIL invariant: a rollout's tokens do not depend on how it was scheduled (N' > N
    with carry-over, N' = N wait-for-all, or alone)."""
    w = small_fp32_workload(sampler, top_k)
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    ctx = make_engine(w, weights)
    ctx2 = make_engine(w, weights)
    ctx3 = make_engine(w, weights)
    try:
        april = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)
        waitall = run_gpu(ctx2, reqs, w.n_target, w.n_target, w.max_new, w.steps)
        a = {rid: t for g in april for rid, t in zip(g["ids"], g["tokens"])}
        b = {rid: t for g in waitall for rid, t in zip(g["ids"], g["tokens"])}
        assert all(g["buffer"] == [] for g in waitall)
        assert any(r > 0 for g in april for r in g["n_resumes"])
        common = set(a) & set(b)
        assert len(common) >= w.n_target
        for rid in common:
            assert a[rid] == b[rid], rid
        for rid in sorted(a)[:5]:                      # alone
            solo = run_gpu(ctx3, [reqs[rid]], 1, 1, w.max_new, 1)
            assert solo[0]["tokens"][0] == a[rid]
        # and against the oracle (scheduling bit-exact; tokens where the margin allows)
        want, eng = run_oracle(w, weights, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps,
                               keep_logits=True)
        assert_schedule_equal(april, want)
        if sampler == ai.SAMPLER_GREEDY:
            assert compare_free_running_tokens(april, want, eng, FP32_LOGIT_TOL) > 100
    finally:
        for c in (ctx, ctx2, ctx3):
            ap().april_destroy(c)


def test_reprefill_fallback_and_export_import():
    """Dropping the KV of the buffer (re-prefill on resume) and a token-level
    export/import round trip both reproduce the KV-resident run."""
    w = small_fp32_workload()
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    ctxs = [make_engine(w, weights) for _ in range(3)]
    try:
        base = run_gpu(ctxs[0], reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)

        def drop(ctx, buf):
            ap().april_buffer_drop_kv(ctx, buf)
            assert all(p["kv_resident"] == 0 for p in ap().april_buffer_export(ctx, buf))
            return buf

        def roundtrip(ctx, buf):
            view = ap().april_buffer_export(ctx, buf)
            ap().april_buffer_free(ctx, buf)
            return ap().april_buffer_import(ctx, view)

        dropped = run_gpu(ctxs[1], reqs, w.n_target, w.n_overprovision, w.max_new, w.steps, between=drop)
        imported = run_gpu(ctxs[2], reqs, w.n_target, w.n_overprovision, w.max_new, w.steps, between=roundtrip)
        assert sum(g["res"].reprefill_tokens for g in base) == 0
        assert sum(g["res"].reprefill_tokens for g in dropped) > 0
        for other in (dropped, imported):
            assert_schedule_equal(other, base)
            for g, o in zip(other, base):
                assert g["tokens"] == o["tokens"]
                assert g["buffer_tokens"] == o["buffer_tokens"]
        info = ap().april_get_info(ctxs[2])
        held = sum(-(-(w.prompt_len + n - 1) // 16) for _, n, d in imported[-1]["buffer"] if not d)
        # pages: free + owned by the parked rollouts == pool (imported ones hold none until resumed)
        assert info["kv_blocks_free"] <= info["kv_blocks_total"]
        info0 = ap().april_get_info(ctxs[0])
        assert info0["kv_blocks_free"] + held == info0["kv_blocks_total"]
    finally:
        for c in ctxs:
            ap().april_destroy(c)


@pytest.mark.parametrize("sampler,top_k,top_p", [("greedy", 0, 0.0), ("topk", 8, 0.7), ("categorical", 0, 0.0)])
def test_paper_sampling_settings_and_returned_logprobs(sampler, top_k, top_p):
    """The paper's rollout settings (appendix: temperature 0.8; evaluation top_p 0.7) through
    the whole path, with the per-token log-probabilities a trainer needs returned next to the
    tokens: scheduling bit-exact, tokens equal to the oracle's up to the first position where the
    oracle's own decision is within tolerance of flipping, log-probabilities within 5e-4 there.
    A token-level export / import round trip between steps must carry the log-probabilities."""
    kinds = {"greedy": ai.SAMPLER_GREEDY, "topk": ai.SAMPLER_TOPK, "categorical": ai.SAMPLER_CATEGORICAL}
    w = small_fp32_workload(kinds[sampler] if sampler != "categorical" else ai.SAMPLER_GREEDY, top_k)
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    T = float(np.float32(0.8))
    want, eng = run_oracle(w, weights, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps, keep_logits=True,
                           temperature=T, top_p=float(np.float32(top_p)) if top_p else 1.0, sampler=sampler)
    ctx = make_engine(w, weights, temperature=0.8, top_p=top_p, logprobs=True, sampler=kinds[sampler])

    def roundtrip(c, buf):
        view = ap().april_buffer_export(c, buf)
        assert all(p["logprobs"] is not None and len(p["logprobs"]) == len(p["generated"])
                   for p in view if len(p["generated"]))
        ap().april_buffer_free(c, buf)
        return ap().april_buffer_import(c, view)
    try:
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps, between=roundtrip)
        assert_schedule_equal(got, want)
        compared, same_rollouts = 0, 0
        for g, o in zip(got, want):
            assert g["logprobs"] is not None
            for rid, gt, ot, glp, olp in zip(g["ids"], g["tokens"], o["tokens"], g["logprobs"], o["logprobs"]):
                assert len(glp) == len(gt) == len(olp)
                for i, (a, b) in enumerate(zip(gt, ot)):
                    if a != b:
                        break                       # sampling near a boundary: the two runs part here
                    assert abs(glp[i] - olp[i]) < 5e-4, (rid, i, glp[i], olp[i])
                    assert glp[i] <= 1e-6
                    compared += 1
                same_rollouts += gt == ot
        assert compared > 300 and same_rollouts >= len(got) * w.n_target // 2
    finally:
        ap().april_destroy(ctx)


@pytest.mark.parametrize("keep_kv", [False, True])
def test_weight_update_between_steps(keep_kv):
    """The policy changes after the second step (Eq. 1; Section 2.2: parked rollouts finish under
    a newer policy).  keep_kv = False: every parked rollout is re-prefilled under the new weights;
    keep_kv = True: its stale K/V stays.  Both against the oracle doing the same: schedule
    bit-exact, greedy tokens identical wherever the oracle's top-2 margin exceeds the tolerance."""
    from oracle.model import Decoder
    from oracle.rollout import OracleRollouts
    w = small_fp32_workload()
    wa, wb = ai.make_weights(w.shape, w.seed), ai.make_weights(w.shape, w.seed + 100)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    eng = OracleRollouts(Decoder(w.shape, wa), "greedy", seed=w.seed, keep_logits=True)
    rolls = [eng.make_rollout(r.request_id, r.tokens, r.forced_len) for r in reqs]
    want, nxt = [], 0
    for k in range(4):
        if k == 2:
            eng.update_weights(Decoder(w.shape, wb), keep_kv=keep_kv)
        o = eng.step(rolls[nxt:], w.n_target, w.n_overprovision, w.max_new)
        nxt += o.n_new_consumed
        want.append(dict(ids=[r.request_id for r in o.completed], tokens=[list(r.tokens) for r in o.completed],
                         n_resumes=[r.n_resumes for r in o.completed], consumed=o.n_new_consumed,
                         iters=o.decode_iters, generated=o.tokens_generated,
                         buffer=[(r.request_id, r.gen, int(r.done)) for r in o.buffer]))
    A = ap()
    ctx = make_engine(w, wa)
    try:
        got, nxt = [], 0
        for k in range(4):
            if k == 2:
                A.april_update_weights(ctx, A.pack_weights(w.shape, wb), keep_kv=keep_kv)
            res = A.april_rollout_step(ctx, req_dicts(reqs[nxt:]), w.n_target, w.n_overprovision, w.max_new)
            nxt += res.n_new_consumed
            view = A.april_buffer_export(ctx, res.buffer)
            got.append(dict(ids=res.request_id, tokens=[t.tolist() for t in res.tokens], n_resumes=res.n_resumes,
                            consumed=res.n_new_consumed, iters=res.decode_iters, generated=res.tokens_generated,
                            buffer=[(p["request_id"], len(p["generated"]), p["done"]) for p in view]))
            if k == 2:
                assert (res.reprefill_tokens > 0) == (not keep_kv)
            A.april_resume(ctx, res.buffer)
        assert_schedule_equal(got, want)
        assert compare_free_running_tokens(got, want, eng, FP32_LOGIT_TOL) > 150
        # the update really changed the policy: rollouts admitted after it differ from the old policy's
        old_ctx = make_engine(w, wa)
        try:
            old = run_gpu(old_ctx, reqs, w.n_target, w.n_overprovision, w.max_new, 4)
        finally:
            A.april_destroy(old_ctx)
        assert got[3]["tokens"] != old[3]["tokens"] and got[1]["tokens"] == old[1]["tokens"]
    finally:
        A.april_destroy(ctx)


@pytest.mark.parametrize("G,n_target,n_over", [(4, 8, 16), (2, 6, 10), (8, 8, 8)])
def test_instance_level_group_completion(G, n_target, n_over):
    """n_samples_per_prompt = G (Section 3.2.3; Section 3.1): a step stops once N / G groups have
    every member complete and returns those groups whole; complete members of an unfinished group
    wait in the buffer.  Against the oracle: schedule bit-exact (ids in delivery order, buffer
    with its done flags, iterations, tokens), greedy tokens equal where the margin allows, and a
    rollout's tokens do not depend on the grouping (same request alone)."""
    from oracle.model import Decoder
    from oracle.rollout import OracleRollouts
    shape = ai.ModelShape(2, 64, 4, 2, 32, 96, 200, dtype=ai.DTYPE_FP32)
    w = ai.Workload("groups", shape, 8, 21, n_target, n_over, 40, 2.4, 0.8, 2, 40, ai.SAMPLER_GREEDY, 0, 4, 21)
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, n_over + 4 * max(n_target, n_over))
    eng = OracleRollouts(Decoder(w.shape, weights), "greedy", seed=w.seed, keep_logits=True)
    rolls = [eng.make_rollout(r.request_id, r.tokens, r.forced_len, group=r.request_id // G) for r in reqs]
    want, nxt = [], 0
    for _ in range(w.steps):
        o = eng.step(rolls[nxt:], n_target, n_over, w.max_new, group_size=G)
        nxt += o.n_new_consumed
        want.append(dict(ids=[r.request_id for r in o.completed], tokens=[list(r.tokens) for r in o.completed],
                         n_resumes=[r.n_resumes for r in o.completed], consumed=o.n_new_consumed,
                         iters=o.decode_iters, generated=o.tokens_generated,
                         buffer=[(r.request_id, r.gen, int(r.done)) for r in o.buffer]))
    ctx = make_engine(w, weights, group_size=G, max_inflight=n_over + 8)
    solo_ctx = make_engine(w, weights)
    try:
        got = run_gpu(ctx, reqs, n_target, n_over, w.max_new, w.steps, group_size=G)
        assert_schedule_equal(got, want)
        assert compare_free_running_tokens(got, want, eng, FP32_LOGIT_TOL) > 100
        waited = 0
        for g in got:
            assert g["groups"] == [rid // G for rid in g["ids"]]
            for k in range(0, len(g["ids"]), G):                     # whole groups, members in id order
                assert g["ids"][k:k + G] == list(range(g["ids"][k], g["ids"][k] + G)) and g["ids"][k] % G == 0
            waited += sum(d for _, _, d in g["buffer"])
        assert waited > 0 or n_over == n_target
        rid = got[-1]["ids"][0]
        solo = run_gpu(solo_ctx, [reqs[rid]], 1, 1, w.max_new, 1)
        assert solo[0]["tokens"][0] == got[-1]["tokens"][0]
    finally:
        ap().april_destroy(ctx)
        ap().april_destroy(solo_ctx)


@pytest.mark.parametrize("dtype,pool_mib", [(ai.DTYPE_FP32, 256), (ai.DTYPE_BF16, 256), (ai.DTYPE_BF16, 2296)])
def test_memory_pause_and_resume_by_remapping(dtype, pool_mib):
    """cfg.pausable: between two steps the physical memory behind the KV pool and the weights is
    released (the free device memory grows by about their size) and mapped again at the same
    addresses; the weights are pushed again, the parked rollouts are re-prefilled, and the run goes
    on - replaying the iteration graphs captured before the pause - exactly like a run whose buffer
    dropped its KV at the same point (same kernels, same order: identical tokens).  The 2296 MiB
    pool is mapped in three pieces, the last one smaller than the others (the pool of the
    benchmark's default workload is 143 pieces of that kind)."""
    A = ap()
    shape = ai.ModelShape(2, 128, 4, 2, 32, 256, 512, dtype=dtype)
    w = ai.Workload("pause", shape, 8, 21, 6, 10, 40, 2.6, 0.7, 2, 40, ai.SAMPLER_GREEDY, 0, 4, 21)
    weights = ai.make_weights(shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    ref_ctx = make_engine(w, weights)
    try:
        def drop_after_second(state={"k": 0}):
            def f(c, buf):
                state["k"] += 1
                if state["k"] == 2:
                    A.april_buffer_drop_kv(c, buf)
                return buf
            return f
        want = run_gpu(ref_ctx, reqs, w.n_target, w.n_overprovision, w.max_new, 4, between=drop_after_second())
    finally:
        A.april_destroy(ref_ctx)
    ctx = make_engine(w, weights, pausable=True, kv_pool_bytes=pool_mib << 20)
    try:
        got, nxt = [], 0
        for k in range(4):
            res = A.april_rollout_step(ctx, req_dicts(reqs[nxt:]), w.n_target, w.n_overprovision, w.max_new)
            nxt += res.n_new_consumed
            view = A.april_buffer_export(ctx, res.buffer)
            got.append(dict(ids=res.request_id, tokens=[t.tolist() for t in res.tokens], n_resumes=res.n_resumes,
                            consumed=res.n_new_consumed, iters=res.decode_iters, generated=res.tokens_generated,
                            buffer=[(p["request_id"], len(p["generated"]), p["done"]) for p in view],
                            reprefill=res.reprefill_tokens))
            A.april_resume(ctx, res.buffer)
            if k == 1:
                before = A.april_get_info(ctx)
                A.april_memory_pause(ctx, A.APRIL_MEM_KV | A.APRIL_MEM_WEIGHTS)
                paused = A.april_get_info(ctx)
                released = paused["hbm_free"] - before["hbm_free"]
                assert released >= 0.9 * (before["kv_pool_bytes"] + before["weight_bytes"]), (released, before)
                with pytest.raises(A.AprilError):                      # nothing runs while paused
                    A.april_rollout_step(ctx, req_dicts(reqs[nxt:]), w.n_target, w.n_overprovision, w.max_new)
                A.april_memory_resume(ctx, A.APRIL_MEM_KV | A.APRIL_MEM_WEIGHTS)
                with pytest.raises(A.AprilError):                      # the weights' memory came back empty
                    A.april_rollout_step(ctx, req_dicts(reqs[nxt:]), w.n_target, w.n_overprovision, w.max_new)
                A.april_update_weights(ctx, A.pack_weights(shape, weights))
                after = A.april_get_info(ctx)
                assert after["kv_blocks_free"] == after["kv_blocks_total"]
                assert abs(after["hbm_free"] - before["hbm_free"]) < 64 << 20
        assert got[2]["reprefill"] > 0
        assert_schedule_equal(got, want)
        for g, o in zip(got, want):
            assert g["tokens"] == o["tokens"]
    finally:
        A.april_destroy(ctx)


@pytest.mark.parametrize("name", list(ai.WORKLOADS))
def test_scheduling_bit_exact_at_all_five_configs(name):
    """Scheduling depends only on the forced lengths, so each configuration's N, N',
    max_new and length stream is run at full size on a one-layer toy model."""
    full = ai.WORKLOADS[name]
    # long contexts: the bf16 path (MFMA attention) for the big configurations, fp32 for the rest
    dtype = ai.DTYPE_FP32 if full.max_new <= 2048 else ai.DTYPE_BF16
    shape = ai.ModelShape(1, 32, 1, 1, 32, 32, 64, dtype=dtype)
    w = ai.Workload(full.name, shape, 4, 4, full.n_target, full.n_overprovision, full.max_new, full.len_mu,
                    full.len_sigma, full.len_lo, full.len_hi, ai.SAMPLER_GREEDY, 0, full.steps, full.seed)
    weights = ai.make_weights(shape, 0)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    from oracle.scheduler import Rollout, rollout_step
    rolls = [Rollout(request_id=r.request_id, prompt_len=len(r.tokens), forced_len=r.forced_len) for r in reqs]
    ctx = make_engine(w, weights)
    try:
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)
        buf, nxt = [], 0
        for g in got:
            o = rollout_step(buf, rolls[nxt:], w.n_target, w.n_overprovision, w.max_new)
            nxt += o.n_new_consumed
            buf = o.buffer
            assert g["ids"] == [r.request_id for r in o.completed]
            assert g["iters"] == o.decode_iters and g["generated"] == o.tokens_generated
            assert g["consumed"] == o.n_new_consumed
            assert g["buffer"] == [(r.request_id, r.gen, int(r.done)) for r in o.buffer]
            assert [len(t) for t in g["tokens"]] == [r.gen for r in o.completed]
            # the device counter covers the rows of the decode kernels: every in-flight
            # rollout in every iteration, minus the newly admitted ones in iteration 1
            # (those rows go through prefill)
            assert g["sum_live"] == sum(o.live_per_iter) - o.n_new_consumed
    finally:
        ap().april_destroy(ctx)


def test_eos_token_ends_rollouts_on_device():
    """Natural EOS: completion is decided by the sampled token, so the stop iteration is
    only known on the device; compare with the oracle running the same rule."""
    w = small_fp32_workload()
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    # pick as EOS a token the oracle actually emits a few times
    base, eng0 = run_oracle(w, weights, reqs, w.n_target, w.n_overprovision, w.max_new, 1)
    toks = [t for o in base for ts in o["tokens"] for t in ts]
    eos = int(np.bincount(toks).argmax())
    want, eng = run_oracle(w, weights, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps, eos=eos,
                           keep_logits=True)
    ctx = make_engine(w, weights, eos=eos)
    try:
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)
        assert_schedule_equal(got, want)
        assert any(len(t) < reqs[rid].forced_len for g in got for rid, t in zip(g["ids"], g["tokens"]))
        assert compare_free_running_tokens(got, want, eng, FP32_LOGIT_TOL) > 50
    finally:
        ap().april_destroy(ctx)


def test_error_paths():
    w = small_fp32_workload()
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, 40)
    A = ap()
    ctx = make_engine(w, weights, max_inflight=12, max_ctx=80)
    try:
        with pytest.raises(A.AprilError) as e:
            A.april_rollout_step(ctx, req_dicts(reqs[:3]), 6, 10, 40)
        assert e.value.code == A.APRIL_ESTARVED
        with pytest.raises(A.AprilError) as e:
            A.april_rollout_step(ctx, req_dicts(reqs), 6, 4, 40)            # N' < N
        assert e.value.code == A.APRIL_EINVAL
        with pytest.raises(A.AprilError) as e:
            unlimited = [dict(d, forced_len=0) for d in req_dicts(reqs)]
            A.april_rollout_step(ctx, unlimited, 6, 10, 400)                # prompt + limit > max_ctx
        assert e.value.code == A.APRIL_EINVAL
        with pytest.raises(A.AprilError) as e:
            A.april_rollout_step(ctx, req_dicts(reqs), 13, 16, 40)          # more slots than max_inflight
        assert e.value.code == A.APRIL_ENOMEM
        res = A.april_rollout_step(ctx, req_dicts(reqs), 6, 10, 40)         # the context still works
        assert len(res.request_id) == 6
        A.april_resume(ctx, res.buffer)
        with pytest.raises(A.AprilError) as e:
            A.april_resume(ctx, res.buffer)                                 # stale handle
        assert e.value.code == A.APRIL_EHANDLE
        bad = dict(w.shape.__dict__)
        with pytest.raises(A.AprilError):
            A.april_init(A.make_cfg(ai.ModelShape(**{**bad, "head_dim": 48}), max_inflight=4, max_ctx=64),
                         A.pack_weights(w.shape, weights))
        with pytest.raises(A.AprilError):
            missing = {k: v for k, v in weights.items() if k != "wo.1"}
            A.april_init(A.make_cfg(w.shape, max_inflight=4, max_ctx=64), A.pack_weights(w.shape, missing))
        tiny_pool = make_engine(w, weights, kv_pool_bytes=1 * 16 * 2 * 2 * 64 * 4)   # 1 page < one prompt
        with pytest.raises(A.AprilError) as e:
            A.april_rollout_step(tiny_pool, req_dicts(reqs), 6, 10, 40)
        assert e.value.code == A.APRIL_ENOMEM
        A.april_destroy(tiny_pool)
    finally:
        A.april_destroy(ctx)


def test_failed_step_loses_no_rollout(monkeypatch):
    """A step that fails after admission (here: the device-side bounds check of the scheduler,
    forced from the host in the second step's sixth iteration - every kernel still exits normally)
    must not lose a rollout: the ones that were resumed go back to the pending set with the tokens
    they have (their KV is dropped), the new requests are not consumed, and repeating the call
    goes on from there.  Every request is delivered exactly once, with the tokens an undisturbed
    run gives it (fp32 path: re-prefilled and resident agree bit for bit)."""
    w = small_fp32_workload()
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    A = ap()
    ref_ctx = make_engine(w, weights)
    try:
        want = run_gpu(ref_ctx, reqs, w.n_target, w.n_overprovision, w.max_new, 4)
    finally:
        A.april_destroy(ref_ctx)
    want_tokens = {rid: t for g in want for rid, t in zip(g["ids"], g["tokens"])}
    monkeypatch.setenv("APRIL_DEBUG_FAIL_AT", "2:6")
    ctx = make_engine(w, weights)
    monkeypatch.delenv("APRIL_DEBUG_FAIL_AT")
    try:
        nxt, steps, failed, delivered, last_buffer = 0, 0, 0, {}, []
        pages_total = A.april_get_info(ctx)["kv_blocks_total"]
        while steps < 4:
            try:
                res = A.april_rollout_step(ctx, req_dicts(reqs[nxt:]), w.n_target, w.n_overprovision, w.max_new)
            except A.AprilError as e:
                assert e.code == A.APRIL_EDEVICE and failed == 0 and steps == 1
                failed += 1
                continue                       # the same call again: nothing new was consumed
            steps += 1
            nxt += res.n_new_consumed
            for rid, t in zip(res.request_id, res.tokens):
                assert rid not in delivered
                delivered[rid] = t.tolist()
            last_buffer = [p["request_id"] for p in A.april_buffer_export(ctx, res.buffer)]
            if steps == 2:
                assert res.reprefill_tokens > 0          # the resumed rollouts came back without KV
            A.april_resume(ctx, res.buffer)
        assert failed == 1
        assert len(delivered) == 4 * w.n_target
        # nobody lost: every admitted request is delivered or still buffered
        assert sorted(list(delivered) + last_buffer) == list(range(nxt))
        common = set(delivered) & set(want_tokens)
        assert len(common) >= 3 * w.n_target
        for rid in common:
            assert delivered[rid] == want_tokens[rid], rid
    finally:
        A.april_destroy(ctx)


def test_failed_step_loses_no_rollout_with_groups(monkeypatch):
    """The same forced failure with instance-level completion (groups of 4): the members of
    resumed groups, complete or not, go back to the pending set, the new groups are not consumed,
    and the repeated call goes on.  Every group is delivered whole and exactly once, every request
    with the tokens it gets in an undisturbed run."""
    G, n_target, n_over = 4, 8, 16
    shape = ai.ModelShape(2, 64, 4, 2, 32, 96, 200, dtype=ai.DTYPE_FP32)
    w = ai.Workload("groups_fail", shape, 8, 21, n_target, n_over, 40, 2.4, 0.8, 2, 40, ai.SAMPLER_GREEDY, 0, 4, 21)
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, n_over + 5 * n_over)
    A = ap()
    ref_ctx = make_engine(w, weights, group_size=G, max_inflight=n_over + 8)
    try:
        want = run_gpu(ref_ctx, reqs, n_target, n_over, w.max_new, 4, group_size=G)
    finally:
        A.april_destroy(ref_ctx)
    want_tokens = {rid: t for g in want for rid, t in zip(g["ids"], g["tokens"])}
    monkeypatch.setenv("APRIL_DEBUG_FAIL_AT", "2:4")
    ctx = make_engine(w, weights, group_size=G, max_inflight=n_over + 8)
    monkeypatch.delenv("APRIL_DEBUG_FAIL_AT")
    try:
        nxt, steps, failed, delivered, last_buffer = 0, 0, 0, {}, []
        while steps < 4:
            try:
                res = A.april_rollout_step(ctx, req_dicts(reqs[nxt:], group_size=G), n_target, n_over, w.max_new)
            except A.AprilError as e:
                assert e.code == A.APRIL_EDEVICE and failed == 0 and steps == 1
                failed += 1
                continue
            steps += 1
            nxt += res.n_new_consumed
            assert res.n_new_consumed % G == 0
            ids = list(res.request_id)
            assert len(ids) == n_target
            for k in range(0, len(ids), G):                         # whole groups, members in id order
                assert ids[k] % G == 0 and ids[k:k + G] == list(range(ids[k], ids[k] + G))
            for rid, t in zip(ids, res.tokens):
                assert rid not in delivered
                delivered[rid] = t.tolist()
            last_buffer = [p["request_id"] for p in A.april_buffer_export(ctx, res.buffer)]
            A.april_resume(ctx, res.buffer)
        assert failed == 1
        assert sorted(list(delivered) + last_buffer) == list(range(nxt))      # nobody lost, nobody twice
        common = set(delivered) & set(want_tokens)
        assert len(common) >= 2 * n_target
        for rid in common:
            assert delivered[rid] == want_tokens[rid], rid
    finally:
        A.april_destroy(ctx)


def test_kv_pool_exhaustion_preempts_youngest_and_reprefills():
    """A KV pool far smaller than the worst case of the step: admission stops when prompt
    pages do not fit, the youngest decoding rollouts are preempted on the device, come back
    token-only and are re-prefilled.  Scheduling (ids, iteration counts, who was preempted,
    who holds KV) is bit-exact against the oracle's page arithmetic; tokens are unchanged."""
    from oracle.scheduler import PagePool
    w = small_fp32_workload()
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w, 8))
    s = w.shape
    n_pages = 19                                   # 10 rollouts in flight would need up to 40
    page_bytes = 16 * 2 * s.n_layers * s.n_kv_heads * s.head_dim * 4
    steps = 8
    want, eng = run_oracle(w, weights, reqs, w.n_target, w.n_overprovision, w.max_new, steps, keep_logits=True,
                           pool=PagePool(total=n_pages, page_tokens=16))
    assert sum(o["n_preempted"] for o in want) > 0
    ctx = make_engine(w, weights, kv_pool_bytes=n_pages * page_bytes)
    ample = make_engine(w, weights)
    try:
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, steps)
        assert_schedule_equal(got, want)
        for g, o in zip(got, want):
            assert g["n_preempted"] == o["n_preempted"]
            assert g["kv_resident"] == o["kv_resident"]
        assert sum(g["res"].reprefill_tokens for g in got) > 0
        assert compare_free_running_tokens(got, want, eng, FP32_LOGIT_TOL) > 100
        # same rollouts as with an ample pool, token for token
        base = run_gpu(ample, reqs, w.n_target, w.n_overprovision, w.max_new, steps)
        a = {rid: t for g in got for rid, t in zip(g["ids"], g["tokens"])}
        b = {rid: t for g in base for rid, t in zip(g["ids"], g["tokens"])}
        assert sum(g["n_preempted"] for g in base) == 0
        for rid in set(a) & set(b):
            assert a[rid] == b[rid], rid
        info = ap().april_get_info(ctx)
        assert info["kv_blocks_total"] == n_pages
    finally:
        ap().april_destroy(ctx)
        ap().april_destroy(ample)
