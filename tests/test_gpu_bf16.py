"""GPU parity for the bf16 path (MFMA GEMMs, bf16 KV cache) at the real layer shapes of
the benchmark configurations, teacher-forced with the oracle's tokens."""
import numpy as np
import pytest

import april_inputs as ai
from gpu_common import assert_schedule_equal, have_gpu, make_engine, run_gpu, run_oracle
from oracle import sampler as osampler
from oracle.philox import uniform_for

pytestmark = pytest.mark.gpu

BF16_LOGIT_TOL = 2e-2          # max-abs relative to the logit scale max(1, max|l_ref|)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not have_gpu():
        pytest.skip("no GPU")


def ap():
    import paper_2509_18521_amd
    return paper_2509_18521_amd


def teacher_forced_parity(w, steps, n_requests, min_rows=20):
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, n_requests)
    want, eng = run_oracle(w, weights, reqs, w.n_target, w.n_overprovision, w.max_new, steps, keep_logits=True)
    ref_tokens = {}
    for o in want:
        ref_tokens.update(dict(zip(o["ids"], o["tokens"])))
    ref_tokens.update(want[-1]["buffer_tokens"])
    ctx = make_engine(w, weights, debug=True)
    try:
        for rid in ref_tokens:
            ap().april_debug_watch(ctx, rid, 0, w.max_new)
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, steps, forced=ref_tokens)
        assert_schedule_equal(got, want)
        for g, o in zip(got, want):
            assert g["tokens"] == o["tokens"]            # forced tokens went through
        worst, rows, sampler_rows = 0.0, 0, 0
        for rid, toks in ref_tokens.items():
            for i in range(len(toks)):
                lg, sampled = ap().april_debug_logits(ctx, rid, i, w.shape.vocab)
                ref = eng.logits[(rid, i)]
                scale = max(1.0, float(np.max(np.abs(ref))))
                worst = max(worst, float(np.max(np.abs(lg - ref))) / scale)
                rows += 1
                # the device sampler on the device's own fp32 logits == oracle sampler on them
                if w.sampler == ai.SAMPLER_GREEDY:
                    assert sampled == osampler.greedy(lg)
                else:
                    u = uniform_for(w.seed, rid, i)
                    idx, p = osampler.top_k_probs(lg, w.top_k, 1.0)
                    cdf = np.cumsum(p)
                    if np.min(np.abs(cdf - u)) > 1e-9:
                        assert sampled == osampler.top_k_sample(lg, w.top_k, 1.0, u)
                        sampler_rows += 1
        assert rows >= min_rows
        assert worst <= BF16_LOGIT_TOL, worst
        return worst, rows
    finally:
        ap().april_destroy(ctx)


def test_cfg2_shape_two_layers_topk_teacher_forced():
    base = ai.WORKLOADS["cfg2_small_bf16"]
    w = ai.Workload("cfg2_L2", ai.reduced(base, n_layers=2).shape, 8, 256, 3, 5, 16, 2.2, 0.5, 4, 16,
                    ai.SAMPLER_TOPK, 50, 2, base.seed)
    teacher_forced_parity(w, 2, 12)


def test_down_projection_folding_the_next_norm(monkeypatch):
    """The optional folding of a layer's first RMSNorm into the previous down projection
    (off by default, APRIL_FUSE_DOWN=1) computes the same thing."""
    monkeypatch.setenv("APRIL_FUSE_DOWN", "1")
    base = ai.WORKLOADS["cfg2_small_bf16"]
    w = ai.Workload("cfg2_L3", ai.reduced(base, n_layers=3, vocab=4096).shape, 6, 64, 3, 5, 8, 1.8, 0.4, 3, 8,
                    ai.SAMPLER_GREEDY, 0, 2, base.seed)
    teacher_forced_parity(w, 2, 10)


def test_cfg2_full_depth_sampled_positions():
    """All 24 layers of configuration 2 on a few rollouts and positions."""
    base = ai.WORKLOADS["cfg2_small_bf16"]
    w = ai.Workload("cfg2_full", base.shape, 4, 256, 2, 3, 6, 1.5, 0.3, 3, 6, ai.SAMPLER_TOPK, 50, 1, base.seed)
    teacher_forced_parity(w, 1, 4, min_rows=10)


@pytest.mark.parametrize("name", ["cfg3_mid_bf16", "cfg4_8b_bf16"])
def test_wide_shapes_head_dim_128_gqa4(name):
    """Layer shapes of configurations 3 and 4 (head_dim 128, 4 query heads per KV head),
    one layer, reduced vocabulary, greedy, ragged prompt lengths via re-prefill."""
    base = ai.WORKLOADS[name]
    shape = ai.reduced(base, n_layers=1, vocab=8192).shape
    w = ai.Workload(name + "_L1", shape, 4, 70, 2, 4, 12, 2.0, 0.5, 3, 12, ai.SAMPLER_GREEDY, 0, 2, base.seed)
    teacher_forced_parity(w, 2, 8)


@pytest.mark.parametrize("head_dim", [64, 128])
def test_long_context_spans_several_kv_splits(head_dim):
    """Contexts beyond a KV split (1024 tokens for head_dim 64, 4096 for 128): the decode attention
    cuts them into splits whose partial results a second kernel merges.  2100-token prompts
    (three splits) and 4150-token prompts (two), then a resumed step on resident KV."""
    shape = ai.ModelShape(1, 256, 256 // head_dim, 2, head_dim, 256, 512)
    prompt_len = 2100 if head_dim == 64 else 4150
    w = ai.Workload("long_ctx", shape, 3, prompt_len, 2, 3, 8, 1.6, 0.4, 3, 8, ai.SAMPLER_GREEDY, 0, 2, 77)
    teacher_forced_parity(w, 2, 5, min_rows=12)


@pytest.mark.parametrize("n_target,n_over,d_model", [(100, 160, 128), (200, 300, 128), (100, 160, 192)])
def test_more_than_128_rows_in_flight(n_target, n_over, d_model):
    """160 / 300 rollouts in flight: several m-groups in every decode GEMM, the LM head through
    the tall-batch kernel (its sampling rows exceed 128) in prefill and in decode, the gate/up GEMM
    through the LDS-tiled kernel (160 rows), or not: beyond 256 rows with a narrow MLP, and with a
    d_model that is not a multiple of 128, it stays on the skinny kernel."""
    shape = ai.ModelShape(2, d_model, d_model // 32, 2, 32, 256, 512)
    w = ai.Workload("many_rows", shape, 40, 6, n_target, n_over, 5, 1.2, 0.4, 2, 5, ai.SAMPLER_GREEDY, 0, 1, 5)
    teacher_forced_parity(w, 1, n_over, min_rows=2 * n_over - 20)


def test_bf16_scheduling_invariance():
    """On the bf16 path a rollout's tokens do not depend on how it was scheduled: carried over
    with resident KV or run with N' = N, token for token.  A rollout whose KV was dropped is
    re-prefilled by the tall-batch GEMM, whose k order differs from the decode GEMM's in the
    last fp32 bit: the schedule (integers) must still match exactly, and so must every token
    generated before the rollout was first parked."""
    shape = ai.ModelShape(3, 128, 4, 2, 64, 256, 1024)
    w = ai.Workload("bf16_small", shape, 8, 37, 5, 9, 60, 3.0, 0.6, 3, 60, ai.SAMPLER_GREEDY, 0, 4, 31)
    weights = ai.make_weights(shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    ctxs = [make_engine(w, weights) for _ in range(3)]
    try:
        def drop(ctx, buf):
            ap().april_buffer_drop_kv(ctx, buf)
            return buf
        a = run_gpu(ctxs[0], reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)
        b = run_gpu(ctxs[1], reqs, w.n_target, w.n_overprovision, w.max_new, w.steps, between=drop)
        c = run_gpu(ctxs[2], reqs, w.n_target, w.n_target, w.max_new, w.steps)
        assert sum(g["res"].reprefill_tokens for g in b) > 0
        assert_schedule_equal(b, a)
        first_park = {}                      # request id -> tokens it held when first parked
        final_a, final_b = {}, {}
        for g, o in zip(b, a):
            for rid, toks in o["buffer_tokens"].items():
                first_park.setdefault(rid, len(toks))
            final_a.update({rid: t for rid, t in zip(o["ids"], o["tokens"])})
            final_b.update({rid: t for rid, t in zip(g["ids"], g["tokens"])})
        assert final_a.keys() == final_b.keys() and len(first_park) > 0
        n_same = 0
        for rid, ta in final_a.items():
            keep = first_park.get(rid, len(ta))          # never parked: the whole rollout
            assert final_b[rid][:keep] == ta[:keep], rid
            n_same += final_b[rid] == ta
        assert n_same >= len(final_a) // 2               # and most re-prefilled ones agree to the end
        tc = {rid: t for g in c for rid, t in zip(g["ids"], g["tokens"])}
        for rid in set(final_a) & set(tc):
            assert final_a[rid] == tc[rid], rid
    finally:
        for x in ctxs:
            ap().april_destroy(x)


def test_cfg2_bench_launch_configuration_sampled_outputs():
    """Configuration 2 at full size, launched as the benchmark launches it (24 layers, N = 64,
    N' = 96, max_new = 2048, top-k sampling, graph replay, the GPU's own sampled tokens): the
    step's invariants, and for two rollouts the logits at sampled positions against the oracle
    fed with the same prefix (one full recompute per rollout gives every position's logits)."""
    from oracle.model import Decoder
    w = ai.WORKLOADS["cfg2_small_bf16"]
    weights = ai.make_weights(w.shape, w.seed)
    reqs = ai.make_requests(w, w.n_overprovision)
    lens = {r.request_id: r.forced_len for r in reqs}
    short = next(r for r in reqs if 40 <= r.forced_len <= 150)        # completes in the first step
    long_ = next(r for r in reqs if r.forced_len >= 1200)             # still running when it ends
    n_watch = 260
    ctx = make_engine(w, weights, debug=True)
    try:
        ap().april_debug_watch(ctx, short.request_id, 0, short.forced_len)
        ap().april_debug_watch(ctx, long_.request_id, 0, n_watch)
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, 1)[0]
        # APRIL's invariants at the real sizes
        assert len(got["ids"]) == w.n_target and len(set(got["ids"])) == w.n_target
        assert all(len(t) == lens[rid] for rid, t in zip(got["ids"], got["tokens"]))
        assert len(got["buffer"]) == w.n_overprovision - w.n_target
        assert set(got["ids"]) | {b[0] for b in got["buffer"]} == set(lens)          # nobody lost
        assert got["generated"] == sum(len(t) for t in got["tokens"]) + sum(b[1] for b in got["buffer"])
        assert short.request_id in got["ids"] and long_.request_id in got["buffer_tokens"]
        dec = Decoder(w.shape, weights)
        worst = 0.0
        for r, toks in ((short, got["tokens"][got["ids"].index(short.request_id)]),
                        (long_, got["buffer_tokens"][long_.request_id][:n_watch])):
            n = len(toks)
            positions = sorted({0, 1, n // 3, n // 2, n - 2, n - 1})
            feed = np.concatenate([r.tokens, np.asarray(toks[:n - 1], dtype=np.int32)])
            ref_all = dec.forward_block(feed, dec.new_cache())          # row P-1+i predicts generated token i
            for i in positions:
                lg, sampled = ap().april_debug_logits(ctx, r.request_id, i, w.shape.vocab)
                ref = ref_all[w.prompt_len - 1 + i]
                worst = max(worst, float(np.max(np.abs(lg - ref))) / max(1.0, float(np.max(np.abs(ref)))))
                assert sampled == toks[i]
                u = uniform_for(w.seed, r.request_id, i)
                idx, p = osampler.top_k_probs(lg, w.top_k, 1.0)
                if np.min(np.abs(np.cumsum(p) - u)) > 1e-9:
                    assert sampled == osampler.top_k_sample(lg, w.top_k, 1.0, u)
        assert worst <= BF16_LOGIT_TOL, worst
    finally:
        ap().april_destroy(ctx)


def test_bf16_kv_pool_exhaustion_schedule_is_bit_exact():
    """A KV pool of 40 pages under ten bf16 rollouts with 40-token prompts and up to 60 generated
    tokens: admission stops when prompt pages do not fit, the scheduler kernel preempts the
    youngest decoding rollouts, and the rows it then lists for the MFMA attention (its work list
    is rebuilt after the preemption pass) are the survivors.  Tokens are teacher-forced, so the
    whole schedule - ids, iteration counts, who was preempted, who still holds K/V - is compared
    bit for bit with the oracle's page arithmetic, and the delivered tokens are the forced ones."""
    from oracle.scheduler import PagePool
    from gpu_common import run_oracle_schedule
    shape = ai.ModelShape(2, 128, 4, 2, 32, 256, 512)
    w = ai.Workload("pool_bf16", shape, 8, 40, 6, 10, 60, 3.2, 0.6, 4, 60, ai.SAMPLER_GREEDY, 0, 6, 31)
    weights = ai.make_weights(shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w, 6))
    rng = np.random.default_rng(4)
    forced = {r.request_id: rng.integers(0, shape.vocab, size=w.max_new, dtype=np.int32)[:min(r.forced_len, w.max_new)]
              for r in reqs}
    n_pages = 40
    page_bytes = 16 * 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2
    want = run_oracle_schedule(reqs, forced, w.n_target, w.n_overprovision, w.max_new, 6,
                               pool=PagePool(total=n_pages, page_tokens=16))
    assert sum(o["n_preempted"] for o in want) > 0
    ctx = make_engine(w, weights, kv_pool_bytes=n_pages * page_bytes, debug=True)     # teacher forcing needs parity mode
    try:
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, 6, forced=forced)
        assert_schedule_equal(got, want)
        for g, o in zip(got, want):
            assert g["n_preempted"] == o["n_preempted"]
            assert g["kv_resident"] == o["kv_resident"]
            assert g["tokens"] == o["tokens"]
        assert sum(g["res"].reprefill_tokens for g in got) > 0
        assert ap().april_get_info(ctx)["kv_blocks_total"] == n_pages
    finally:
        ap().april_destroy(ctx)


def test_cfg3_bench_launch_configuration_sampled_outputs():
    """Configuration 3 (the benchmark's default workload) at full size, launched as the benchmark
    launches it: 36 layers, 152 k vocabulary, N = 128, N' = 192, max_new = 4096, greedy sampling
    from the LM head's (maximum, column) records with no logits written, graph replay, the
    GPU's own tokens.  One step: APRIL's invariants; then the same step on an engine in parity
    mode (logits written and kept for two rollouts) must give every rollout the same tokens, and
    the kept logits at sampled positions are compared with the oracle fed with the same prefix."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle.model import Decoder
    w = ai.WORKLOADS["cfg3_mid_bf16"]
    s = w.shape
    specs = ai.weight_specs(s)

    def one(spec):
        name, shape, kind = spec
        a = ai.weight_tensor(s, name, shape, kind, w.seed)
        return name, a, ap().pack_weights(s, {name: a})[name]
    weights, packed = {}, {}
    with ThreadPoolExecutor(max_workers=16) as ex:
        for name, a, pk in ex.map(one, specs):
            weights[name], packed[name] = a, pk
    reqs = ai.make_requests(w, w.n_overprovision)
    lens = {r.request_id: min(r.forced_len, w.max_new) for r in reqs}
    short = next(r for r in reqs if 40 <= r.forced_len <= 120)        # completes in the first step
    long_ = next(r for r in reqs if r.forced_len >= 2500)             # still running when it ends
    n_watch = 96
    runs = []
    kept = {}
    for debug in (False, True):
        cfg = ap().make_cfg(s, max_inflight=w.n_overprovision + 8, max_ctx=w.prompt_len + w.max_new + 16,
                            sampler=w.sampler, top_k=max(w.top_k, 1), temperature=1.0, seed=w.seed,
                            debug_logits=debug)
        ctx = ap().april_init(cfg, packed)
        try:
            if debug:
                ap().april_debug_watch(ctx, short.request_id, 0, short.forced_len)
                ap().april_debug_watch(ctx, long_.request_id, 0, n_watch)
            got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, 1)[0]
            runs.append(got)
            if debug:
                for r, n in ((short, short.forced_len), (long_, n_watch)):
                    for i in sorted({0, 1, n // 3, n // 2, n - 2, n - 1}):
                        kept[(r.request_id, i)] = ap().april_debug_logits(ctx, r.request_id, i, s.vocab)
        finally:
            ap().april_destroy(ctx)
    got, ref_run = runs
    assert len(got["ids"]) == w.n_target and len(set(got["ids"])) == w.n_target
    assert all(len(t) == lens[rid] for rid, t in zip(got["ids"], got["tokens"]))
    assert len(got["buffer"]) == w.n_overprovision - w.n_target
    assert set(got["ids"]) | {b[0] for b in got["buffer"]} == set(lens)          # nobody lost
    assert got["generated"] == sum(len(t) for t in got["tokens"]) + sum(b[1] for b in got["buffer"])
    assert short.request_id in got["ids"] and long_.request_id in got["buffer_tokens"]
    assert_schedule_equal([got], [ref_run])
    assert got["tokens"] == ref_run["tokens"] and got["buffer_tokens"] == ref_run["buffer_tokens"]
    dec = Decoder(s, weights)
    worst = 0.0
    for r, toks, n in ((short, got["tokens"][got["ids"].index(short.request_id)], short.forced_len),
                       (long_, got["buffer_tokens"][long_.request_id][:n_watch], n_watch)):
        feed = np.concatenate([r.tokens, np.asarray(toks[:n - 1], dtype=np.int32)])
        ref_all = dec.forward_block(feed, dec.new_cache())          # row P-1+i predicts generated token i
        for (rid, i), (lg, sampled) in kept.items():
            if rid != r.request_id:
                continue
            ref = ref_all[w.prompt_len - 1 + i]
            worst = max(worst, float(np.max(np.abs(lg - ref))) / max(1.0, float(np.max(np.abs(ref)))))
            assert sampled == toks[i] == int(np.argmax(lg))
            top2 = np.sort(ref)[-2:]
            if top2[1] - top2[0] > 2 * BF16_LOGIT_TOL * max(1.0, float(np.max(np.abs(ref)))):
                assert sampled == int(np.argmax(ref))
    assert worst <= BF16_LOGIT_TOL, worst


@pytest.mark.parametrize("n_target,n_over", [(30, 40), (100, 150), (150, 230)])      # 128-, 192- and 256-row tile
def test_tiled_decode_gate_up_gives_the_skinny_kernels_bits(monkeypatch, n_target, n_over):
    """With many rows in flight the decode gate/up GEMM runs in the LDS-tiled kernel, which
    closes its accumulator chain at the skinny kernel's quarter boundaries and folds the same
    RMSNorm: forcing either kernel for every iteration must change no bit of any logit."""
    shape = ai.ModelShape(2, 256, 4, 2, 64, 512, 1024)
    w = ai.Workload("tile_decode", shape, 8, 21, n_target, n_over, 9, 1.7, 0.4, 3, 9, ai.SAMPLER_GREEDY, 0, 2, 11)
    weights = ai.make_weights(shape, w.seed)
    reqs = ai.make_requests(w, ai.requests_needed(w))
    runs = []
    for threshold in ("0", "1"):                 # never / always the tiled kernel
        monkeypatch.setenv("APRIL_TILE_DECODE_ROWS", threshold)
        ctx = make_engine(w, weights, debug=True)
        try:
            for r in reqs:
                ap().april_debug_watch(ctx, r.request_id, 0, w.max_new)
            got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)
            logits = {}
            for g in got:
                for rid, toks in list(zip(g["ids"], g["tokens"])) + list(g["buffer_tokens"].items()):
                    for i in range(len(toks)):
                        logits[(rid, i)] = ap().april_debug_logits(ctx, rid, i, shape.vocab)[0]
            runs.append((got, logits))
        finally:
            ap().april_destroy(ctx)
    (a, la), (b, lb) = runs
    assert_schedule_equal(b, a)
    assert [g["tokens"] for g in a] == [g["tokens"] for g in b]
    assert la.keys() == lb.keys() and len(la) > 200
    assert all(np.array_equal(la[k], lb[k]) for k in la)


@pytest.mark.parametrize("head_dim", [64, 128])
def test_attention_work_list_gives_the_grid_launch_bits(monkeypatch, head_dim):
    """Decode attention takes its (row, KV split) items from the list the scheduler kernel sorts
    by length every iteration; APRIL_ATTN_LIST=0 launches one workgroup per (row, head, split)
    of a grid instead.  Prompts that end 24-60 tokens short of a split boundary (1024 and 2048
    tokens for head_dim 64, 4096 for 128) put rows with different split counts and last-split
    lengths into the same iteration; no bit of any logit may depend on which launch ran, nor any
    token or scheduling decision."""
    shape = ai.ModelShape(1, 256, 256 // head_dim, 2, head_dim, 256, 512)
    runs = []
    for flag in ("0", "1"):
        monkeypatch.setenv("APRIL_ATTN_LIST", flag)
        per_prompt = []
        for prompt_len in ((1000, 2030) if head_dim == 64 else (1000, 4060)):
            w = ai.Workload("att_list", shape, 6, prompt_len, 10, 16, 70, 3.3, 0.8, 3, 70, ai.SAMPLER_GREEDY, 0, 2, 21)
            weights = ai.make_weights(shape, w.seed)
            reqs = ai.make_requests(w, ai.requests_needed(w))
            ctx = make_engine(w, weights, debug=True)
            try:
                for r in reqs:
                    ap().april_debug_watch(ctx, r.request_id, 0, w.max_new)
                got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps)
                logits = {}
                for g in got:
                    for rid, toks in list(zip(g["ids"], g["tokens"])) + list(g["buffer_tokens"].items()):
                        for i in range(len(toks)):
                            logits[(rid, i)] = ap().april_debug_logits(ctx, rid, i, shape.vocab)[0]
                per_prompt.append((got, logits))
            finally:
                ap().april_destroy(ctx)
        runs.append(per_prompt)
    for (a, la), (b, lb) in zip(*runs):
        assert_schedule_equal(b, a)
        assert [g["tokens"] for g in a] == [g["tokens"] for g in b]
        assert la.keys() == lb.keys() and len(la) > 300
        assert all(np.array_equal(la[k], lb[k]) for k in la)


@pytest.mark.parametrize("n_target,n_over", [(30, 40), (100, 150)])      # skinny LM head; tall-batch LM head
def test_greedy_sampling_without_logits_equals_sampling_from_logits(monkeypatch, n_target, n_over):
    """Greedy, not in parity mode: the LM head writes no logits, only the maximum of every 64
    columns and the column holding it, and the sampler works from those.  Same tokens as with
    the logits written and searched (APRIL_WRITE_LOGITS=1), also where maxima tie exactly: the LM
    head rows are equal in blocks of 8 here, so every maximum is an 8-way tie across both lane
    halves of the accumulator tile, and the lowest index must win (a multiple of 8)."""
    shape = ai.ModelShape(2, 128, 4, 2, 32, 256, 1024)
    w = ai.Workload("nologits", shape, 8, 9, n_target, n_over, 7, 1.6, 0.3, 3, 7, ai.SAMPLER_GREEDY, 0, 2, 13)
    weights = ai.make_weights(shape, w.seed)
    head = weights["lm_head"].copy()
    head[:] = head[(np.arange(shape.vocab) // 8) * 8]
    weights["lm_head"] = head
    reqs = ai.make_requests(w, ai.requests_needed(w))
    runs = []
    for flag in ("1", "0"):
        monkeypatch.setenv("APRIL_WRITE_LOGITS", flag)
        ctx = make_engine(w, weights)
        try:
            runs.append(run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, w.steps))
        finally:
            ap().april_destroy(ctx)
    a, b = runs
    assert_schedule_equal(b, a)
    assert [g["tokens"] for g in a] == [g["tokens"] for g in b]
    assert [g["buffer_tokens"] for g in a] == [g["buffer_tokens"] for g in b]
    toks = [t for g in b for seq in g["tokens"] for t in seq]
    assert len(toks) > 200 and all(t % 8 == 0 for t in toks)
