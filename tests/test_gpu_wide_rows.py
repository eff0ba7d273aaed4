"""GPU parity at the layer widths of the large configurations WITH hundreds of rollouts in
flight: the decode GEMM variants that only such batches launch (several m-groups, two n-tiles
per workgroup, the residual-epilogue kernel with four m-tiles, the LDS-tiled gate/up kernel at
the real widths, expert GEMMs with several row groups per expert) compared with the oracle.

One layer, reduced vocabulary, short prompts.  Tokens are teacher-forced per prompt class
(request r: prompt and forced tokens of class r mod P, P prime so that rows a multiple of 32
apart never share a class), which makes the oracle's share one block forward per class.
"""
import numpy as np
import pytest

import april_inputs as ai
from gpu_common import (assert_schedule_equal, class_forced_tokens, class_reference_logits, have_gpu, make_engine,
                        run_gpu, run_oracle_schedule)
from oracle import sampler as osampler
from oracle.model import Decoder

pytestmark = pytest.mark.gpu

BF16_LOGIT_TOL = 2e-2          # max-abs relative to the logit scale max(1, max|l_ref|)
ROUTE_MARGIN = 3e-2


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not have_gpu():
        pytest.skip("no GPU")


def ap():
    import paper_2509_18521_amd
    return paper_2509_18521_amd


_weights_cache = {}


def _weights(shape, seed):
    key = (shape, seed)
    if key not in _weights_cache:
        _weights_cache.clear()                       # one wide model at a time on the host
        _weights_cache[key] = ai.make_weights(shape, seed)
    return _weights_cache[key]


def class_parity(w, steps, min_rows, skip_positions=None):
    """Runs `steps` rollout steps of workload w on the GPU with class-forced tokens and compares
    the schedule (bit-exact) and every generated position's logits with the oracle."""
    P = w.n_prompts
    weights = _weights(w.shape, w.seed)
    n_req = w.n_overprovision + steps * w.n_target
    reqs = ai.make_requests(w, n_req)
    ctoks = class_forced_tokens(w, P)
    forced = {r.request_id: ctoks[r.request_id % P][:min(r.forced_len, w.max_new)] for r in reqs}
    want = run_oracle_schedule(reqs, forced, w.n_target, w.n_overprovision, w.max_new, steps)
    dec = Decoder(w.shape, weights)
    if skip_positions is not None:
        dec.route_margins = []
    prompts = [reqs[c].tokens for c in range(P)]
    ref = []
    bad = [set() for _ in range(P)]
    for c in range(P):
        if skip_positions is not None:
            dec.route_margins = []
        ref.append(class_reference_logits(dec, [prompts[c]], [ctoks[c]], w.max_new)[0])
        if skip_positions is not None:
            PL = len(prompts[c])
            bad[c] = {p - (PL - 1) for p, l, m in dec.route_margins if m < ROUTE_MARGIN and p >= PL - 1}
    seen = {}
    for o in want:
        seen.update(dict(zip(o["ids"], o["tokens"])))
    seen.update(want[-1]["buffer_tokens"])
    ctx = make_engine(w, weights, debug=True, max_inflight=w.n_overprovision + 8)
    try:
        for rid in seen:
            ap().april_debug_watch(ctx, rid, 0, w.max_new)
        got = run_gpu(ctx, reqs, w.n_target, w.n_overprovision, w.max_new, steps, forced=forced)
        assert_schedule_equal(got, want)
        for g, o in zip(got, want):
            assert g["tokens"] == o["tokens"]
            assert g["buffer_tokens"] == o["buffer_tokens"]
        worst, rows, skipped, worst_at = 0.0, 0, 0, None
        for rid, toks in seen.items():
            c = rid % P
            for i in range(len(toks)):
                if i in bad[c]:
                    skipped += 1
                    continue
                lg, sampled = ap().april_debug_logits(ctx, rid, i, w.shape.vocab)
                r = ref[c][i]
                err = float(np.max(np.abs(lg - r))) / max(1.0, float(np.max(np.abs(r))))
                if err > worst:
                    worst, worst_at = err, (rid, i)
                rows += 1
                assert sampled == osampler.greedy(lg)
        print(f"{w.name}: rows={rows} skipped={skipped} worst={worst:.4g} at {worst_at}")
        share = f"skipped {skipped} of {rows + skipped} positions ({skipped / max(rows + skipped, 1):.0%})"
        assert rows >= min_rows, f"compared only {rows} rows; {share}"
        assert worst <= BF16_LOGIT_TOL, f"worst {worst:.4g} at {worst_at}; {share}"
        return got
    finally:
        ap().april_destroy(ctx)


@pytest.mark.parametrize("name,n_target,n_over", [
    ("cfg3_mid_bf16", 128, 192), ("cfg3_mid_bf16", 200, 300),
    ("cfg4_8b_bf16", 128, 192), ("cfg4_8b_bf16", 200, 300),
])
def test_dense_wide_layer_many_rows(name, n_target, n_over):
    """One layer of configuration 3 (d 2560, F 9728) / 4 (d 4096, F 14336), 192 or 300 rollouts
    in flight, two steps (the second decodes resumed rollouts next to a fresh prefill).
    Decode launches reached (rocprofv3 kernel trace of this test): qkv and down through
    gemm_mfma_kernel<2,4,EPI_F32,true> with 2-3 m-groups; the output projection through
    gemm_mfma_kernel<1,4,EPI_RESID,true>; gate/up through gemm_tile_chain_kernel<2,2,3,2,2,3>
    (192 rows) and <4,2,2,2,2,3> (300 rows of configuration 4: two row groups) or, for 300 rows of configuration
    3, gemm_mfma_kernel<2,4,EPI_SWIGLU,true> with three m-groups; the LM head through the
    tall-batch kernel."""
    base = ai.WORKLOADS[name]
    shape = ai.reduced(base, n_layers=1, vocab=8192).shape
    w = ai.Workload(f"{name}_L1_{n_over}", shape, 37, 7, n_target, n_over, 5, 1.45, 0.2, 3, 5,
                    ai.SAMPLER_GREEDY, 0, 2, base.seed)
    got = class_parity(w, 2, min_rows=4 * n_over)
    # the decode iterations really had that many rows in flight
    assert got[0]["sum_live"] >= n_over * 2


@pytest.mark.parametrize("name,n_over", [("cfg3_mid_bf16", 150), ("cfg3_mid_bf16", 230), ("cfg3_mid_bf16", 300),
                                         ("cfg4_8b_bf16", 230), ("cfg4_8b_bf16", 300)])
def test_wide_layer_batch_size_changes_no_bit(name, n_over):
    """At the widths of configurations 3 and 4 the row count picks the kernels: qkv and down on the
    skinny kernel with one or several m-groups, except the down projection of configuration 4,
    which above 128 rows runs on the LDS-tiled kernel with the same summation chains (long k
    slices that fall on stage boundaries); the output projection with
    one or four m-tiles per workgroup; gate/up on the skinny kernel (4 rows, and 300 of
    configuration 3), the 192-row LDS tile (150) or the 256-row one (230, and 300 of
    configuration 4); the LM head skinny or tall.  Each choice keeps every output element's
    summation chain, so the first four requests must get bit-identical logits whether they run
    alone or among n_over rollouts (teacher-forced tokens: both runs feed the same sequences)."""
    base = ai.WORKLOADS[name]
    shape = ai.reduced(base, n_layers=1, vocab=8192).shape
    runs = []
    for n_flight in (4, n_over):
        w = ai.Workload(f"{name}_L1_bits_{n_flight}", shape, 37, 7, n_flight, n_flight, 5, 1.45, 0.2, 5, 5,
                        ai.SAMPLER_GREEDY, 0, 1, base.seed)
        weights = _weights(w.shape, w.seed)
        reqs = ai.make_requests(w, n_flight)
        ctoks = class_forced_tokens(w, w.n_prompts)
        forced = {r.request_id: ctoks[r.request_id % w.n_prompts][:w.max_new] for r in reqs}
        ctx = make_engine(w, weights, debug=True, max_inflight=n_flight + 8)
        try:
            for rid in range(4):
                ap().april_debug_watch(ctx, rid, 0, w.max_new)
            got = run_gpu(ctx, reqs, n_flight, n_flight, w.max_new, 1, forced=forced)[0]
            assert sorted(got["ids"]) == list(range(n_flight))
            runs.append({(rid, i): ap().april_debug_logits(ctx, rid, i, shape.vocab)[0]
                         for rid in range(4) for i in range(w.max_new)})
        finally:
            ap().april_destroy(ctx)
    alone, crowd = runs
    assert alone.keys() == crowd.keys() and len(alone) == 20
    assert all(np.array_equal(alone[k], crowd[k]) for k in alone)


def test_moe_cfg5_layer_many_rows():
    """One layer of configuration 5 (128 experts, 8 per token, expert ffn 768, d 2048), 384
    rollouts in flight over 5 prompt classes: a class's rows take the same experts, so in decode
    an expert gets about 77 rows (two row groups of 64) and in prefill (384 x 12 tokens)
    several hundred (row groups of 128).  Positions whose routing decision in the oracle is
    within ROUTE_MARGIN of a tie are not compared; the skipped share is reported."""
    base = ai.WORKLOADS["cfg5_moe_bf16"]
    shape = ai.reduced(base, n_layers=1, vocab=4096).shape
    w = ai.Workload("cfg5_L1_384", shape, 5, 12, 256, 384, 5, 1.45, 0.2, 3, 5, ai.SAMPLER_GREEDY, 0, 2, base.seed)
    got = class_parity(w, 2, min_rows=1000, skip_positions=True)
    assert got[0]["sum_live"] >= 384 * 2
