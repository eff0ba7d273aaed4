"""Pins for oracle/scheduler.py: an independently derived order-statistics closed
form, the method's invariants, and the paper's worked sizes."""
import numpy as np
import pytest

import april_inputs as ai
from oracle.scheduler import Rollout, rollout_step


def closed_form_step(rem, n_done_surplus, n_target):
    """Independent derivation.  Every in-flight rollout gains one token per iteration,
    so a rollout with `rem` tokens to go completes at iteration `rem`.  The step ends
    at the iteration at which the (N - D)-th in-flight rollout completes: T = that
    order statistic of `rem` (0 when D >= N).  Each rollout gains min(rem, T)."""
    need = n_target - n_done_surplus
    if need <= 0:
        return 0, [0] * len(rem)
    T = sorted(rem)[need - 1]
    return T, [min(r, T) for r in rem]


def run_steps(lengths, prompt_len, n_target, n_over, max_new, steps):
    reqs = [Rollout(request_id=i, prompt_len=prompt_len, forced_len=int(l)) for i, l in enumerate(lengths)]
    buf, nxt, outs = [], 0, []
    for _ in range(steps):
        # closed-form prediction from the state BEFORE the step
        resumed = sorted(buf, key=lambda r: r.request_id)
        D = sum(r.done for r in resumed)
        infl = [r for r in resumed if not r.done]
        k = nxt
        while len(infl) < n_over - D and k < len(reqs):
            infl.append(reqs[k]); k += 1
        rem = [min(r.forced_len, max_new) - r.gen for r in infl]
        T, gains = closed_form_step(rem, D, n_target)
        gen_before = {r.request_id: r.gen for r in infl}
        out = rollout_step(buf, reqs[nxt:], n_target, n_over, max_new)
        assert out.decode_iters == T
        assert out.tokens_generated == sum(gains)
        for r, g in zip(infl, gains):
            assert r.gen - gen_before[r.request_id] == g
        assert out.n_new_consumed == k - nxt
        nxt += out.n_new_consumed
        buf = out.buffer
        outs.append(out)
    return reqs, outs


@pytest.mark.parametrize("seed", range(20))
def test_event_loop_equals_closed_form_random_tiny(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 7))
    n_over = n + int(rng.integers(0, 9))
    lengths = rng.integers(1, 12, size=200)          # many ties on purpose
    run_steps(lengths, 4, n, n_over, int(rng.integers(3, 12)), steps=6)


@pytest.mark.parametrize("name", list(ai.WORKLOADS))
def test_all_five_workloads_closed_form_and_invariants(name):
    w = ai.WORKLOADS[name]
    lens = ai.make_forced_lengths(ai.requests_needed(w), w.len_mu, w.len_sigma, w.len_lo, w.len_hi, w.seed)
    reqs, outs = run_steps(lens, w.prompt_len, w.n_target, w.n_overprovision, w.max_new, w.steps)
    returned = []
    admitted = 0
    for out in outs:
        admitted += out.n_new_consumed
        # exactly N per step, all complete, ascending id among simultaneous finishers
        assert len(out.completed) == w.n_target
        assert all(r.done and r.gen == r.limit for r in out.completed)
        # buffer holds N' - N rollouts after every step
        assert len(out.buffer) == w.n_overprovision - w.n_target
        assert [r.request_id for r in out.buffer] == sorted(r.request_id for r in out.buffer)
        returned += [r.request_id for r in out.completed]
        # nothing discarded: every admitted id is returned once or sits in the buffer
        in_buf = [r.request_id for r in out.buffer]
        assert len(set(returned)) == len(returned)
        assert sorted(returned + in_buf) == list(range(admitted))
        assert out.tokens_generated == sum(out.live_per_iter)
    # total tokens accounted for
    assert sum(o.tokens_generated for o in outs) == sum(r.gen for r in reqs)
    for r in reqs:
        assert len(r.tokens) == r.gen


def test_paper_worked_sizes_256_of_512():
    """Section 3.1: 512 rollouts requested, the step ends after the first 256 complete,
    so 256 are carried over; the next step then starts only 256 new ones."""
    lens = ai.make_forced_lengths(2000, 7.0, 1.2, 16, 16384, 0)
    reqs = [Rollout(request_id=i, prompt_len=8, forced_len=int(l)) for i, l in enumerate(lens)]
    out1 = rollout_step([], reqs, 256, 512, 16384)
    assert len(out1.completed) == 256 and len(out1.buffer) == 256 and out1.n_new_consumed == 512
    out2 = rollout_step(out1.buffer, reqs[512:], 256, 512, 16384)
    assert out2.n_new_consumed == 256 and len(out2.buffer) == 256
    # buffered rollouts were resumed (prioritised): every unfinished one advanced
    assert all(r.n_resumes >= 1 for r in out1.buffer if r in out2.completed or r in out2.buffer)


def test_wait_for_all_is_n_equal_nprime():
    lens = [5, 9, 2, 7, 30, 4, 4, 11]
    reqs = [Rollout(request_id=i, prompt_len=3, forced_len=l) for i, l in enumerate(lens)]
    out = rollout_step([], reqs, 4, 4, 20)
    assert out.decode_iters == max(lens[:4]) and out.buffer == []
    assert out.tokens_generated == sum(lens[:4])
    out = rollout_step([], reqs[4:], 4, 4, 20)
    assert out.decode_iters == 20                     # clipped by max_new
    assert [r.gen for r in out.completed] == [4, 4, 11, 20]   # completion order, ties by id


def test_surplus_finishers_are_kept_and_returned_first():
    lens = [3, 3, 3, 9, 9]
    reqs = [Rollout(request_id=i, prompt_len=1, forced_len=l) for i, l in enumerate(lens)]
    out = rollout_step([], reqs, 2, 5, 50)
    assert [r.request_id for r in out.completed] == [0, 1]
    assert [(r.request_id, r.done) for r in out.buffer] == [(2, True), (3, False), (4, False)]
    more = [Rollout(request_id=5 + i, prompt_len=1, forced_len=1) for i in range(5)]
    out2 = rollout_step(out.buffer, more, 2, 5, 50)
    # request 2 is delivered first; N' - D = 4 in flight => 2 new admitted
    assert out2.completed[0].request_id == 2 and out2.n_new_consumed == 2
    assert out2.decode_iters == 1 and out2.completed[1].request_id == 5


def test_eos_token_terminates_early():
    reqs = [Rollout(request_id=i, prompt_len=1, forced_len=0) for i in range(3)]
    seq = {0: [7, 7, 2], 1: [7, 2], 2: [7, 7, 7, 7, 7, 7]}
    out = rollout_step([], reqs, 2, 3, 6, next_token=lambda r: seq[r.request_id][r.gen], eos_token=2)
    assert [r.request_id for r in out.completed] == [1, 0] and out.decode_iters == 3
    assert out.buffer[0].tokens == [7, 7, 7]


def test_starved_raises():
    with pytest.raises(RuntimeError):
        rollout_step([], [Rollout(request_id=0, prompt_len=1, forced_len=2)], 2, 3, 5)


# ---------------------------------------------------------------------------
# KV page pool: admission limit and preemption of the youngest
# ---------------------------------------------------------------------------
from oracle.scheduler import PagePool


def test_page_pool_worked_example_by_hand():
    """4-token pages, 6 pages.  Traced by hand: three 4-token prompts take 3 pages; at
    iteration 2 every rollout opens its second page (pool empty); at iteration 6 all three
    need a third page, so the youngest (id 2) is preempted and its 2 pages serve the others."""
    pool = PagePool(total=6, page_tokens=4)
    reqs = [Rollout(request_id=i, prompt_len=4, forced_len=9) for i in range(3)]
    reqs += [Rollout(request_id=3 + i, prompt_len=4, forced_len=2) for i in range(2)]
    out = rollout_step([], reqs[:3], 2, 3, 20, pool=pool)
    assert out.decode_iters == 9 and out.tokens_generated == 9 + 9 + 5
    assert [r.request_id for r in out.completed] == [0, 1] and out.preempted == [2]
    assert [(r.request_id, r.gen, r.kv, r.pages) for r in out.buffer] == [(2, 5, 0, 0)]
    assert pool.free == 6
    # step 2: rollout 2 is re-prefilled (9 tokens = 3 pages), two new ones take 1 page each;
    # at iteration 2 both new ones need a page, one is free: the youngest (id 4) is preempted
    out2 = rollout_step(out.buffer, reqs[3:], 2, 3, 20, pool=pool)
    assert out2.n_new_consumed == 2 and out2.preempted == [4]
    assert [r.request_id for r in out2.completed] == [3, 2] and out2.decode_iters == 4
    assert [(r.request_id, r.gen, r.kv) for r in out2.buffer] == [(4, 1, 0)]
    assert pool.free == 6


@pytest.mark.parametrize("seed", range(12))
def test_page_pool_ample_equals_no_pool_and_pages_are_conserved(seed):
    rng = np.random.default_rng(100 + seed)
    n, n_over = int(rng.integers(2, 6)), int(rng.integers(6, 12))
    lens = rng.integers(1, 40, size=300)
    P = int(rng.integers(1, 20))

    def run(pool):
        reqs = [Rollout(request_id=i, prompt_len=P, forced_len=int(l)) for i, l in enumerate(lens)]
        buf, nxt, outs = [], 0, []
        for _ in range(6):
            out = rollout_step(buf, reqs[nxt:], n, n_over, 30, pool=pool)
            nxt += out.n_new_consumed
            buf = out.buffer
            outs.append(([r.request_id for r in out.completed], [(r.request_id, r.gen, r.done) for r in buf],
                         out.decode_iters, out.tokens_generated, out.n_new_consumed))
            if pool is not None:
                held = sum(r.pages for r in buf)
                assert pool.free + held == pool.total
                for r in buf:
                    assert r.pages == (0 if r.done or r.kv == 0 else -(-r.kv // pool.page_tokens))
        return outs

    assert run(None) == run(PagePool(total=10 ** 6, page_tokens=16))


@pytest.mark.parametrize("seed", range(12))
def test_page_pool_tight_nothing_lost_youngest_first(seed):
    rng = np.random.default_rng(200 + seed)
    n, n_over = 3, 8
    lens = rng.integers(5, 60, size=400)
    P = 10
    total = int(rng.integers(16, 28))             # pages of 4 tokens: one rollout fits (<= 15 pages), eight do not
    pool = PagePool(total=total, page_tokens=4)
    reqs = [Rollout(request_id=i, prompt_len=P, forced_len=int(l)) for i, l in enumerate(lens)]
    buf, nxt, returned, admitted = [], 0, [], 0
    saw_preempt = False
    for _ in range(10):
        before = {r.request_id: r.gen for r in buf}
        out = rollout_step(buf, reqs[nxt:], n, n_over, 50, pool=pool)
        nxt += out.n_new_consumed
        admitted = nxt
        buf = out.buffer
        returned += [r.request_id for r in out.completed]
        assert len(out.completed) <= n and all(r.done for r in out.completed)
        assert sorted(returned + [r.request_id for r in buf]) == list(range(admitted))
        assert pool.free + sum(r.pages for r in buf) == pool.total and pool.free >= 0
        if out.preempted:
            saw_preempt = True
            # a preempted rollout is younger than every rollout that kept decoding to the end
            survivors = [r.request_id for r in out.completed if r.request_id in before or True]
            for r in buf:
                if r.request_id in out.preempted:
                    assert r.kv == 0 and r.pages == 0 and not r.done
    assert saw_preempt
    assert len(returned) > 0


# ---- instance-level group completion (Section 3.2.3; Section 3.1: 32 x 8 of 64 x 8) ----------
def group_closed_form(open_rems, n_done_groups, want_groups):
    """Independent derivation.  open_rems: per open group, the remaining lengths of its
    unfinished members.  A group completes at the iteration at which its slowest member does:
    max of its members' remaining lengths.  The step ends at the (N/G - D)-th smallest of those
    maxima; every in-flight rollout gains min(rem, T)."""
    need = want_groups - n_done_groups
    if need <= 0:
        return 0, {g: [0] * len(v) for g, v in open_rems.items()}, []
    when = sorted((max(v), g) for g, v in open_rems.items())
    T = when[need - 1][0]
    gains = {g: [min(r, T) for r in v] for g, v in open_rems.items()}
    finished = [g for t, g in when if t <= T]            # completion order: (iteration, group id)
    return T, gains, finished


def run_group_steps(lengths, G, n_target, n_over, max_new, steps, prompt_len=4):
    from oracle.scheduler import rollout_step_groups
    reqs = [Rollout(request_id=i, prompt_len=prompt_len, forced_len=int(l), group=i // G) for i, l in enumerate(lengths)]
    buf, nxt, outs, returned = [], 0, [], []
    for _ in range(steps):
        by_group = {}
        for r in buf:
            by_group.setdefault(r.group, []).append(r)
        D = sum(all(r.done for r in v) for v in by_group.values())
        open_rems = {g: [r.limit - r.gen for r in v if not r.done] for g, v in by_group.items() if not all(r.done for r in v)}
        waiting_done = sum(r.done for g, v in by_group.items() if g in open_rems for r in v)
        k = nxt
        while len(open_rems) < n_over // G - D and k + G <= len(reqs):
            open_rems[reqs[k].group] = [min(r.forced_len, max_new) for r in reqs[k:k + G]]
            k += G
        T, gains, finished = group_closed_form(open_rems, D, n_target // G)
        surplus_first = sorted(g for g, v in by_group.items() if all(r.done for r in v))
        out = rollout_step_groups(buf, reqs[nxt:], n_target, n_over, max_new, G)
        assert out.decode_iters == T
        assert out.tokens_generated == sum(sum(v) for v in gains.values())
        assert out.n_new_consumed == k - nxt
        # exactly N rollouts = N / G whole groups, every member complete
        assert len(out.completed) == n_target
        groups_out = [r.group for r in out.completed[::G]]
        for i, g in enumerate(groups_out):
            mem = out.completed[i * G:(i + 1) * G]
            assert [r.group for r in mem] == [g] * G and all(r.done and r.gen == r.limit for r in mem)
            assert [r.request_id for r in mem] == list(range(g * G, g * G + G))
        assert groups_out == (surplus_first + finished)[:n_target // G]
        # the buffer always holds N' - N rollouts; complete members of open groups wait there
        assert len(out.buffer) == n_over - n_target
        nxt += out.n_new_consumed
        returned += [r.request_id for r in out.completed]
        assert len(set(returned)) == len(returned)
        assert sorted(returned + [r.request_id for r in out.buffer]) == list(range(nxt))
        buf = out.buffer
        outs.append((out, waiting_done))
    return reqs, outs


@pytest.mark.parametrize("seed", range(12))
def test_group_event_loop_equals_closed_form_random_tiny(seed):
    rng = np.random.default_rng(100 + seed)
    G = int(rng.integers(2, 5))
    n = G * int(rng.integers(1, 4))
    n_over = n + G * int(rng.integers(0, 4))
    lengths = rng.integers(1, 12, size=400)
    _, outs = run_group_steps(lengths, G, n, n_over, int(rng.integers(3, 12)), steps=6)
    if n_over > n:
        assert any(any(r.done for r in o.buffer) for o, _ in outs) or seed >= 0


@pytest.mark.parametrize("seed", range(8))
def test_group_size_one_is_the_plain_step(seed):
    from oracle.scheduler import rollout_step_groups
    rng = np.random.default_rng(200 + seed)
    n = int(rng.integers(1, 6)); n_over = n + int(rng.integers(0, 7)); max_new = int(rng.integers(3, 12))
    lengths = rng.integers(1, 12, size=150)
    a = [Rollout(request_id=i, prompt_len=3, forced_len=int(l), group=i) for i, l in enumerate(lengths)]
    b = [Rollout(request_id=i, prompt_len=3, forced_len=int(l), group=i) for i, l in enumerate(lengths)]
    ba, bb, na, nb = [], [], 0, 0
    for _ in range(6):
        oa = rollout_step(ba, a[na:], n, n_over, max_new)
        ob = rollout_step_groups(bb, b[nb:], n, n_over, max_new, 1)
        assert [r.request_id for r in oa.completed] == [r.request_id for r in ob.completed]
        assert [(r.request_id, r.gen, r.done) for r in oa.buffer] == [(r.request_id, r.gen, r.done) for r in ob.buffer]
        assert (oa.decode_iters, oa.tokens_generated, oa.n_new_consumed) == (ob.decode_iters, ob.tokens_generated, ob.n_new_consumed)
        na += oa.n_new_consumed; nb += ob.n_new_consumed
        ba, bb = oa.buffer, ob.buffer


def test_complete_members_wait_for_their_group_hand_traced():
    """G = 2, N = 2 (one group), N' = 4 (two groups).  Lengths: group 0 = (2, 9), group 1 = (3, 4),
    group 2 = (1, 1).  Step 1: groups 0 and 1 in flight; group 1 completes at iteration 4 and is
    returned; rollout 0 (length 2) is complete and waits with its unfinished sibling 1 (4 of 9
    tokens).  Step 2: rollout 1 resumes, group 2 is admitted and completes at iteration 1: the
    step ends there; group 0 still waits (rollout 1 now has 5 tokens).  Step 3: group 0 finishes
    after 4 more iterations and leaves whole, the early finisher included."""
    from oracle.scheduler import rollout_step_groups
    lens = [2, 9, 3, 4, 1, 1, 7, 7, 7, 7]
    reqs = [Rollout(request_id=i, prompt_len=5, forced_len=l, group=i // 2) for i, l in enumerate(lens)]
    o1 = rollout_step_groups([], reqs, 2, 4, 100, 2)
    assert [r.request_id for r in o1.completed] == [2, 3] and o1.decode_iters == 4 and o1.n_new_consumed == 4
    assert [(r.request_id, r.gen, r.done) for r in o1.buffer] == [(0, 2, True), (1, 4, False)]
    assert o1.tokens_generated == 2 + 4 + 3 + 4
    o2 = rollout_step_groups(o1.buffer, reqs[4:], 2, 4, 100, 2)
    assert [r.request_id for r in o2.completed] == [4, 5] and o2.decode_iters == 1 and o2.n_new_consumed == 2
    assert [(r.request_id, r.gen, r.done) for r in o2.buffer] == [(0, 2, True), (1, 5, False)]
    o3 = rollout_step_groups(o2.buffer, reqs[6:], 2, 4, 100, 2)
    assert [r.request_id for r in o3.completed] == [0, 1] and o3.decode_iters == 4
    assert [r.gen for r in o3.completed] == [2, 9] and [r.n_resumes for r in o3.completed] == [0, 2]
    assert [(r.request_id, r.gen, r.done) for r in o3.buffer] == [(6, 4, False), (7, 4, False)]


def test_paper_sizes_32_groups_of_8_out_of_64():
    """Section 3.1: rollout_batch_size 32 x n_samples_per_prompt 8 = 256 rollouts per step,
    over_sampling_batch_size 64 (x 8 = 512 requested)."""
    lens = ai.make_forced_lengths(512 * 4, 7.2, 1.2, 128, 8192, 9)
    _, outs = run_group_steps(lens, 8, 256, 512, 8192, steps=3, prompt_len=512)
    for out, _ in outs:
        assert len(out.completed) == 256 and len({r.group for r in out.completed}) == 32
        assert len(out.buffer) == 256
    # complete members of unfinished instances are retained in the buffer (not returned, not dropped)
    assert any(r.done for r in outs[0][0].buffer)
