#!/usr/bin/env python3
"""Benchmark of the APRIL rollout hot path on one MI355X.

A "step" is one rollout step (admission, prefill, decode loop with early termination,
parking) of the configured workload.  The metric is the paper's rollout throughput
(Section 3.2.1: tokens generated divided by the wall-clock time of the rollout
iterations), reported for APRIL (N' > N) with the wait-for-all baseline (N' = N) on
the same request stream beside it.  Inputs are synthetic and already resident in HBM
(weights, KV pool); prompts are a few KB per step.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BF16_PEAK_TFLOPS = 2500.0      # dense bf16 MFMA, published


VERBOSE = False


def note(msg):
    """Progress line on stderr (stdout carries only the JSON line): a step of the larger
    configurations takes 10-25 s, and a run that prints nothing for minutes looks hung."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def run_arm(ap, ctx, reqs, n_target, n_over, max_new, steps, profile_every=0, between=None, group_size=0):
    """Run `steps` rollout steps from a clean context state; returns per-step results.
    between(ctx): called after every step but the last (e.g. a weight update).
    group_size G > 1: request r belongs to group r // G (instance-level completion)."""
    ap.april_profile_enable(ctx, profile_every)
    nxt, results = 0, []
    t0 = time.perf_counter()
    for k in range(steps):
        new = [dict(request_id=r.request_id, tokens=r.tokens, forced_len=r.forced_len) for r in reqs[nxt:nxt + n_over]]
        if group_size > 1:
            for d in new:
                d["group_id"] = d["request_id"] // group_size
        res = ap.april_rollout_step(ctx, new, n_target, n_over, max_new)
        nxt += res.n_new_consumed
        results.append(res)
        note(f"step {len(results)}/{steps}: {res.tokens_generated} tokens in {res.t_total_s:.2f} s, {res.decode_iters} iterations")
        ap.april_resume(ctx, res.buffer)
        if between is not None and k + 1 < steps:
            between(ctx)
    import torch
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return results, wall


def cpu_baseline(w, weights, reqs, budget_s=10.0):
    """The oracle as it stands, timed on the host cores for a bounded slice of the
    workload: whole rollouts (prefill of the prompt, then decode) one after another
    until the time budget is used."""
    import numpy as np
    from oracle.model import Decoder
    from oracle.rollout import OracleRollouts
    import threadpoolctl
    eng = OracleRollouts(Decoder(w.shape, weights), "topk" if w.sampler else "greedy", top_k=max(w.top_k, 1),
                         seed=w.seed)
    t0 = time.perf_counter()
    tokens = 0
    n_roll = 0
    per_roll = 8
    while time.perf_counter() - t0 < budget_s and n_roll < len(reqs):
        r = reqs[n_roll]
        roll = eng.make_rollout(r.request_id, r.tokens, per_roll)
        eng.buffer = []
        out = eng.step([roll], 1, 1, per_roll)
        tokens += out.tokens_generated
        n_roll += 1
    dt = time.perf_counter() - t0
    threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    return dict(value=tokens / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"{n_roll} rollouts of the workload, each: prefill of its {w.prompt_len}-token prompt + "
                       f"{per_roll} generated tokens, one rollout at a time ({dt:.1f} s)")


def generate_weights(ai, ap, s, seed, keep_fp32, threads=16):
    """Random-init tensors of the model, drawn tensor by tensor on a thread pool (every tensor has
    its own seeded stream, so the order does not matter); returns (packed for the library, fp32
    values for the oracle leg or {})."""
    from concurrent.futures import ThreadPoolExecutor
    specs = ai.weight_specs(s)

    def one(spec):
        name, shape, kind = spec
        a = ai.weight_tensor(s, name, shape, kind, seed)
        return name, a, ap.pack_weights(s, {name: a})[name]
    packed, weights = {}, {}
    with ThreadPoolExecutor(max_workers=threads) as ex:
        for name, a, pk in ex.map(one, specs):
            packed[name] = pk
            if keep_fp32:
                weights[name] = a
    return packed, weights


def measured_traffic(workload, kernel_class, key="traffic_bytes_per_launch"):
    """HBM bytes per launch of a kernel class (fetch + write), from the committed summary of
    the two rocprofv3 --pmc runs over this benchmark's command (already scaled by the copy
    calibration recorded in the same file); None when no summary covers the class.
    key = "algorithmic_bytes_per_launch_same_run": the algorithmic bytes per launch of the
    counter run itself (one layer, one step: shorter contexts than a long run sees)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == key and parts[1] == kernel_class:
                    return float(parts[2])
    except OSError:
        pass
    return None


def copy_calibration(n_bytes=1 << 30, reps=3):
    """A plain device copy of known size, so that a --pmc run of this command also holds
    the counter reading for known traffic (n_bytes read + n_bytes written per launch)."""
    import torch
    src = torch.empty(n_bytes, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=5)
    p.add_argument("--warmup", type=int, default=1)
    p.add_argument("--workload", default="cfg3_mid_bf16",
                   help="the largest configuration whose --steps 20 --warmup 5 run fits a 10-minute limit on one GPU")
    p.add_argument("--wait-all-steps", type=int, default=2,
                   help="steps of the wait-for-all arm (same request stream; each of its steps runs to the length cap)")
    p.add_argument("--layers", type=int, default=0, help="override the layer count (debug only; invalidates the number)")
    p.add_argument("--max-new", type=int, default=0, help="cap the generated length (debug only; invalidates the number)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-wait-all", action="store_true")
    p.add_argument("--profile-every", type=int, default=128,
                   help="every n-th decode iteration runs eagerly with an event pair around each launch (0 = never)")
    p.add_argument("--verbose", action="store_true", help="progress lines on stderr")
    p.add_argument("--update-weights", type=int, default=0, metavar="STEPS",
                   help="extra APRIL arm of STEPS steps with a policy update (april_update_weights, device-resident "
                        "source) after every step: once re-prefilling the parked rollouts, once keeping their stale KV")
    p.add_argument("--next-rows", type=int, default=0, metavar="STEPS",
                   help="also measure, over STEPS steps each on a fresh engine: the paper's rollout sampling "
                        "(temperature 0.8 over the whole vocabulary, log-probabilities returned) and its evaluation "
                        "sampling (top-p 0.7), instance-level completion in groups of 8, and releasing / re-mapping "
                        "the KV pool and the weights")
    p.add_argument("--kv-pool-gib", type=float, default=0.0, help="KV pool size (0 = the library's default)")
    p.add_argument("--copy-calibration", action="store_true",
                   help="also run three 1 GiB device copies first (reference dispatches for --pmc counter runs)")
    args = p.parse_args()
    global VERBOSE
    VERBOSE = args.verbose
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import april_inputs as ai
    import paper_2509_18521_amd as ap

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if args.copy_calibration:
        copy_calibration()
    w = ai.WORKLOADS[args.workload]
    if args.layers:
        w = ai.reduced(w, n_layers=args.layers)
    if args.max_new:
        import dataclasses
        w = dataclasses.replace(w, max_new=args.max_new)
    s = w.shape
    t_setup = time.perf_counter()
    # the library's element types, tensor by tensor; the fp32 values are kept only for the
    # oracle leg (the large configurations would not fit the host twice)
    packed, weights = generate_weights(ai, ap, s, w.seed, keep_fp32=not args.no_cpu_baseline)
    note(f"weights generated ({ai.n_params(s) / 1e9:.2f} B parameters, {time.perf_counter() - t_setup:.1f} s)")
    total_steps = args.steps
    reqs = ai.make_requests(w, ai.requests_needed(w, max(total_steps, args.warmup)))
    cfg = ap.make_cfg(s, max_inflight=w.n_overprovision + 32, max_ctx=w.prompt_len + w.max_new + 16,
                      sampler=w.sampler, top_k=max(w.top_k, 1), temperature=1.0, seed=w.seed,
                      kv_pool_bytes=int(args.kv_pool_gib * (1 << 30)),
                      stream=torch.cuda.current_stream().cuda_stream or None)
    ctx = ap.april_init(cfg, packed)
    info = ap.april_get_info(ctx)
    setup_s = time.perf_counter() - t_setup
    note(f"engine ready: KV pool {info['kv_pool_bytes'] / 2**30:.1f} GiB, weights {info['weight_bytes'] / 2**30:.1f} GiB")

    def fresh_arm(n_over, steps, profile_every):
        """Run an arm on the current engine (created fresh for each arm by reset_engine)."""
        results, wall = run_arm(ap, ctx, reqs, w.n_target, n_over, w.max_new, steps, profile_every)
        ap.april_profile_enable(ctx, 0)
        return results, wall

    def reset_engine():
        nonlocal ctx
        ap.april_destroy(ctx)
        ctx = ap.april_init(cfg, packed)

    # warm-up (untimed), then a fresh engine for the timed region
    if args.warmup > 0:
        fresh_arm(w.n_overprovision, args.warmup, 0)
        reset_engine()
    torch.cuda.synchronize()
    ap.april_profile_reset(ctx)
    res_april, wall_april = fresh_arm(w.n_overprovision, total_steps, args.profile_every)
    stats = ap.april_profile_get(ctx)
    torch.cuda.synchronize()

    tok_april = sum(r.tokens_generated for r in res_april)
    delivered_april = sum(len(t) for r in res_april for t in r.tokens)
    step_time = sum(r.t_total_s for r in res_april)
    decode_time = sum(r.t_decode_s for r in res_april)
    iters = sum(r.decode_iters for r in res_april)
    value = tok_april / step_time
    # Algorithmic bytes of the decode iterations that t_decode_s covers (iterations 2.. of
    # every step): all decode weights once per iteration, the KV of every live context
    # read once, one KV row written per live rollout, the fp32 residual stream around each
    # sub-block, token in / token out.
    sum_live = sum(r.dec_sum_live for r in res_april)
    sum_ctx = sum(r.dec_sum_ctx for r in res_april)
    kv_tok = info["kv_bytes_per_token"]
    dec_bytes = (sum(max(r.decode_iters - 1, 0) for r in res_april) * info["decode_weight_bytes"]
                 + sum(r.dec_sum_experts for r in res_april) * info["expert_bytes"]
                 + sum_ctx * kv_tok + sum_live * kv_tok
                 + sum_live * s.d_model * 4 * 2 * (2 * s.n_layers + 1) + sum_live * 8)
    decode_gbs = dec_bytes / decode_time / 1e9 if decode_time > 0 else 0.0

    out = {
        "metric": "rollout tokens/s on 1 MI355X (APRIL vs wait-all); decode HBM GB/s % of peak",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": total_steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * step_time / total_steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if s.dtype == ai.DTYPE_BF16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "n_layers": s.n_layers, "d_model": s.d_model, "vocab": s.vocab,
                   "n_target": w.n_target, "n_overprovision": w.n_overprovision, "max_new": w.max_new,
                   "prompt_len": w.prompt_len, "sampler": "top-k" if w.sampler else "greedy", "top_k": w.top_k,
                   "forced_len": f"lognormal(mu={w.len_mu}, sigma={w.len_sigma}) clipped to [{w.len_lo},{w.len_hi}]"},
        "april": {"tokens_generated": tok_april, "tokens_delivered": delivered_april, "decode_iters": iters,
                  "step_time_s": step_time, "decode_time_s": decode_time,
                  "prefill_time_s": sum(r.t_prefill_s for r in res_april), "wall_s": wall_april,
                  "delivered_tokens_per_s": delivered_april / step_time},
        "decode": {"algorithmic_bytes": dec_bytes, "GBps": decode_gbs, "frac_of_hbm_peak": decode_gbs / HBM_PEAK_GBS,
                   "sum_live": sum_live, "sum_ctx": sum_ctx},
        "setup_s": setup_s,
    }

    # roofline of the dominant kernel (largest share of the timed decode launches).
    # A pair of event records around one eager launch also reads the cost of the pair itself;
    # the engine times a pair with nothing between the records, and that reading is subtracted
    # from every class's average (the raw average stays beside it).
    def pair_us(name):
        k = [k for k in stats if k["name"] == name and k["launches"] > 0]
        return 1e3 * k[0]["total_ms"] / k[0]["launches"] if k else None
    pair_none_us, pair_empty_us = pair_us("event_pair_no_kernel"), pair_us("event_pair_empty_kernel")
    timed = [k for k in stats if k["launches"] > 0 and not k["name"].startswith("event_pair") and k["name"] != "sched"]

    def launch_us(k):
        raw = 1e3 * k["total_ms"] / k["launches"]
        return max(raw - (pair_none_us or 0.0), 0.1 * raw)
    if timed:
        dom = max(timed, key=lambda k: k["total_ms"])
        ach = dom["alg_bytes"] / dom["launches"] / (launch_us(dom) * 1e-6) / 1e9
        out["roofline"] = {"kernel": dom["name"], "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(w.name, dom["name"]),
                           "traffic_source": f"profiles/hbm_traffic_{w.name}.txt (committed rocprofv3 --pmc reading of this "
                                             "command with --layers 1 --steps 1, not a measurement of this run: compare it with "
                                             "traffic_run_alg_bytes_per_launch, the algorithmic bytes per launch of that counter run)",
                           "traffic_run_alg_bytes_per_launch": measured_traffic(w.name, dom["name"], "algorithmic_bytes_per_launch_same_run"),
                           "alg_bytes_per_launch": dom["alg_bytes"] / dom["launches"],
                           "avg_launch_us": launch_us(dom),
                           "avg_event_pair_us": 1e3 * dom["total_ms"] / dom["launches"],
                           "launches_timed": dom["launches"],
                           "event_pair_no_kernel_us": pair_none_us, "event_pair_empty_kernel_us": pair_empty_us}
        tot = sum(k["total_ms"] for k in timed)
        out["kernels"] = [{"name": k["name"], "launches": k["launches"], "avg_us": launch_us(k),
                           "avg_event_pair_us": 1e3 * k["total_ms"] / k["launches"],
                           "share": k["total_ms"] / tot,
                           "GBps": k["alg_bytes"] / k["launches"] / (launch_us(k) * 1e-6) / 1e9,
                           "TFLOPs": k["alg_flops"] / k["launches"] / (launch_us(k) * 1e-6) / 1e12} for k in timed]

    if not args.no_wait_all:
        reset_engine()
        wait_steps = max(1, min(total_steps, args.wait_all_steps))
        res_wait, wall_wait = fresh_arm(w.n_target, wait_steps, 0)
        tok_wait = sum(r.tokens_generated for r in res_wait)
        t_wait = sum(r.t_total_s for r in res_wait)
        out["wait_all"] = {"steps": wait_steps, "tokens_generated": tok_wait, "decode_iters": sum(r.decode_iters for r in res_wait),
                           "step_time_s": t_wait, "tokens_per_s": tok_wait / t_wait, "wall_s": wall_wait}
        out["april_speedup_vs_wait_all"] = value / (tok_wait / t_wait)
    if args.update_weights > 0:
        # the trainer's new weights would already be on this GPU: keep a device copy as the source
        dev_w = {k: torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda() for k, v in packed.items()}
        out["weight_update"] = {"steps": args.update_weights}
        for label, keep in (("reprefill", False), ("stale_kv", True)):
            reset_engine()
            t_upd = []

            def upd(c, keep=keep):
                t0 = time.perf_counter()
                ap.april_update_weights(c, dev_w, keep_kv=keep)
                torch.cuda.synchronize()
                t_upd.append(time.perf_counter() - t0)
            res_u, _ = run_arm(ap, ctx, reqs, w.n_target, w.n_overprovision, w.max_new, args.update_weights, 0, between=upd)
            tok_u, t_u = sum(r.tokens_generated for r in res_u), sum(r.t_total_s for r in res_u)
            out["weight_update"][label] = {
                "tokens_per_s": tok_u / t_u, "tokens_per_s_including_update_calls": tok_u / (t_u + sum(t_upd)),
                "update_call_s": sum(t_upd) / max(len(t_upd), 1), "reprefill_tokens": sum(r.reprefill_tokens for r in res_u),
                "prefill_time_s": sum(r.t_prefill_s for r in res_u), "step_time_s": t_u, "tokens_generated": tok_u}
        # the KV-resident number over the same steps of the main arm
        t_same = sum(r.t_total_s for r in res_april[:args.update_weights])
        out["weight_update"]["kv_resident_tokens_per_s_same_steps"] = (
            sum(r.tokens_generated for r in res_april[:args.update_weights]) / t_same if t_same > 0 else None)
        del dev_w
    ap.april_destroy(ctx)

    if args.next_rows > 0:
        nx = {"steps": args.next_rows}
        base_kw = dict(max_inflight=w.n_overprovision + 32, max_ctx=w.prompt_len + w.max_new + 16, seed=w.seed,
                       kv_pool_bytes=int(args.kv_pool_gib * (1 << 30)),
                       stream=torch.cuda.current_stream().cuda_stream or None)

        def arm(label, group_size=0, **kw):
            c = ap.april_init(ap.make_cfg(s, **base_kw, **kw), packed)
            try:
                res, _ = run_arm(ap, c, reqs, w.n_target, w.n_overprovision, w.max_new, args.next_rows, 0,
                                 group_size=group_size)
            finally:
                ap.april_destroy(c)
            tok, t = sum(r.tokens_generated for r in res), sum(r.t_total_s for r in res)
            nx[label] = {"tokens_per_s": tok / t, "tokens_generated": tok, "step_time_s": t,
                         "decode_iters": sum(r.decode_iters for r in res)}
        # same steps of the main arm (greedy, rollout-level completion), for comparison
        t_same = sum(r.t_total_s for r in res_april[:args.next_rows])
        nx["main_arm_same_steps_tokens_per_s"] = sum(r.tokens_generated for r in res_april[:args.next_rows]) / t_same
        arm("rollout_sampling_T0.8_full_vocab_logprobs", sampler=ap.APRIL_SAMPLER_CATEGORICAL, temperature=0.8, logprobs=True)
        arm("eval_sampling_top_k64_top_p0.7_T0.8", sampler=ap.APRIL_SAMPLER_TOPK, top_k=64, top_p=0.7, temperature=0.8)
        if w.n_target % 8 == 0 and w.n_overprovision % 8 == 0:
            arm("groups_of_8_instance_level", group_size=8, sampler=w.sampler, top_k=max(w.top_k, 1),
                n_samples_per_prompt=8)
        # releasing and re-mapping the physical memory of the KV pool and of the weights
        c = ap.april_init(ap.make_cfg(s, **base_kw, sampler=w.sampler, top_k=max(w.top_k, 1), pausable=True), packed)
        try:
            inf = ap.april_get_info(c)
            res0, _ = run_arm(ap, c, reqs, w.n_target, w.n_overprovision, w.max_new, 1, 0)
            dev_w = {k: torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda() for k, v in packed.items()}
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ap.april_memory_pause(c, ap.APRIL_MEM_KV | ap.APRIL_MEM_WEIGHTS)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            ap.april_memory_resume(c, ap.APRIL_MEM_KV | ap.APRIL_MEM_WEIGHTS)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            ap.april_update_weights(c, dev_w, keep_kv=False)
            torch.cuda.synchronize()
            t3 = time.perf_counter()
            res1 = ap.april_rollout_step(c, [dict(request_id=r.request_id, tokens=r.tokens, forced_len=r.forced_len)
                                             for r in reqs[res0[0].n_new_consumed:][:w.n_overprovision]],
                                         w.n_target, w.n_overprovision, w.max_new)
            nx["memory_pause_resume"] = {
                "bytes_released": inf["kv_pool_bytes"] + inf["weight_bytes"], "pause_s": t1 - t0, "resume_s": t2 - t1,
                "weights_reload_device_to_device_s": t3 - t2, "step_after_resume_tokens_per_s": res1.tokens_generated / res1.t_total_s,
                "step_before_pause_tokens_per_s": res0[0].tokens_generated / res0[0].t_total_s}
            del dev_w
        finally:
            ap.april_destroy(c)
        out["next_rows"] = nx

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, weights, reqs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
