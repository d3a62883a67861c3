"""Pins of the scheduler oracle (oracle/sched_oracle.py) to what the paper and arithmetic fix:
the chunking rule on hand-worked numbers, the stated KVC-demand rule, Eq. 6, the remaining-time formula on
hand-computed numbers, the nearest-demand choice of Alg. 2 against a brute-force search, and the
invariants any correct schedule has, over simulated traces.  CPU only."""
import math
import os

import numpy as np
import pytest

import workloads as W
from oracle import sched_oracle as SO

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_block_and_chunk_arithmetic.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            vals = [float(x) if "." in x else int(x) for x in v.split()]
            out[k.strip()] = vals[0] if len(vals) == 1 else vals
    return out


def make(b=16, nb=4096, s_pf=768, t_pf=0.1, t_max=0.1, gamma=0.75, max_tokens=8192, order=None):
    return SO.Scheduler(b, nb, s_pf, t_pf, t_max, gamma, max_tokens, order)


def test_dynamic_chunking_rule_on_hand_worked_numbers():
    """Sec. 4.2 gives the rule (tokens in queue order until S_f = S_b or the KVC ends); the numbers
    are worked by hand from it in the golden file."""
    g = golden()
    picks = SO.sequential_chunks(g["dyn_chunk_example_lengths"], g["dyn_chunk_example_budgets"], g["dyn_chunk_example_kvc"])
    assert picks[0] == [(0, g["dyn_chunk_example_first_iteration"][0]), (1, g["dyn_chunk_example_first_iteration"][1])]
    assert [t for it in picks for (i, t) in it if i == 1] == g["dyn_chunk_example_chunks_of_prompt2"]


def test_scheduler_cuts_a_prompt_where_budget_or_kvc_ends():
    """The same rule inside the scheduler: a 5000-token prompt alone with a budget of 250; before
    the third iteration the rest of the pool is taken away except for 96 tokens."""
    s = make(b=4, nb=3000, s_pf=250, t_pf=0.1, t_max=0.1)
    s.add_request(2, 5000, 1, 0.1, 0.1, 0.0)     # SLO == T_pf: S_b == S_pf
    got = []
    for it in range(3):
        if it == 2:
            del s.free[: len(s.free) - 96 // 4]
        batch = s.next_batch(0.1 * it)
        got.append([(e.req.id, e.tokens) for e in batch])
        s.complete(0.1 * (it + 1))
    assert got == [[(2, 250)], [(2, 250)], [(2, 96)]] and len(s.free) == 0
    assert s.next_batch(0.3) == []               # nothing fits any more


def test_kvc_demand_rule():
    g = golden()
    s = make(b=16)
    r = SO.Request(1, 101, 5, 1.0, 1.0, 0.0)
    assert s.new_blocks(r, 37) == 3
    r.blocks, r.processed = [0, 1, 2], 37
    assert s.new_blocks(r, 64) == g["new_blocks_b16_prior37_chunk64"]
    s128 = make(b=128)
    tot = sum(s128.new_blocks(SO.Request(i, n, 1, 1.0, 1.0, 0.0), n) * 128 for i, n in enumerate([1, 128, 129, 300]))
    assert tot == g["alloc_b128_lens_1_128_129_300"]
    # a generation task: no demand while its last block has room, one block when it is full
    t = SO.Request(2, 31, 9, 1.0, 1.0, 0.0, processed=31, generated=1, state=SO.RETURNED, blocks=[5, 6])
    assert s.new_blocks(t, 1) == 0       # context 31 -> 32 fits two blocks of 16
    t.generated = 2
    assert s.new_blocks(t, 1) == 1       # context 32 -> 33 opens a third


def test_token_budget_eq6():
    g = golden()
    for s_pf in (g["pivot_forward_size_opt13b"], g["pivot_forward_size_opt175b"]):
        s = make(s_pf=s_pf, t_pf=0.125, t_max=0.125, max_tokens=100000)
        s.add_request(1, 50000, 4, 0.125, 0.125, 0.0)
        s.next_batch(0.0)
        assert s.token_budget == s_pf                       # SLO_min == T_pf
        s = make(s_pf=s_pf, t_pf=0.125, t_max=0.125, max_tokens=100000)
        s.add_request(1, 50000, 4, g["reading_speed_slo"], 0.125, 0.0)
        s.next_batch(0.0)
        assert s.token_budget == s_pf * 3 // 2              # 0.1875 / 0.125
        s = make(s_pf=s_pf, t_pf=0.125, t_max=0.125, max_tokens=1000)
        s.add_request(1, 50000, 4, 10.0, 0.125, 0.0)
        s.next_batch(0.0)
        assert s.token_budget == 1000                        # capped


def test_remaining_time_formula():
    s = make(s_pf=768, t_max=0.2)
    r = SO.Request(1, 1000, 5, 1.5, 0.1875, 10.0)
    # waited 0.4 s, 1000 tokens left, L_c = 768 before any chunk: 2 chunks of 0.2 s
    assert s.remaining_time(r, 10.4) == pytest.approx(1.5 - 0.4 - 0.4, abs=1e-12)
    s.chunk_tokens, s.chunks = 1000, 4        # L_c = 250 -> 4 chunks
    assert s.remaining_time(r, 10.4) == pytest.approx(1.5 - 0.4 - 0.8, abs=1e-12)
    r.processed = 900                          # 100 left -> 1 chunk
    assert s.remaining_time(r, 10.4) == pytest.approx(1.5 - 0.4 - 0.2, abs=1e-12)
    t = SO.Request(2, 10, 5, 1.5, 0.1875, 3.0, processed=10, generated=2, state=SO.RETURNED)
    assert s.remaining_time(t, 99.0) == pytest.approx(0.1875 - 0.2, abs=1e-12)   # no waiting time
    t.state = SO.PREEMPTED
    assert s.remaining_time(t, 3.05) == pytest.approx(0.1875 - 0.05 - 0.2, abs=1e-12)


def test_queue_order_and_urgency():
    s = make(s_pf=64, t_pf=0.125, t_max=0.125, gamma=0.0, max_tokens=1000)
    # three short prompts with SLOs 0.5, 0.1875 (urgent: 0.1875 - 0 - 0.125 <= 0.125), 0.3125
    s.add_request(1, 10, 1, 0.5, 0.5, 0.0)
    s.add_request(2, 10, 1, 0.1875, 0.5, 0.0)
    s.add_request(3, 10, 1, 0.3125, 0.5, 0.0)
    batch = s.next_batch(0.0)
    # urgent 2 first; gamma 0 admits only the head of the rest (3)
    assert [e.req.id for e in batch] == [2, 3]
    assert s.token_budget == 96                  # 64 * 0.1875 / 0.125, the head's SLO


def test_token_budget_takes_the_tightest_slo_of_the_certain_members():
    """Eq. 6 uses SLO_min, "the minimum SLO of the requests in a batch" (Sec. 4.2).  The queue is
    ordered by remaining time, so its head can be a prompt with a loose SLO that has waited long
    while a generation task with a much tighter SLO is back from the last iteration: the budget
    must follow the task's 0.05 s, not the head's 1.0 s."""
    s = make(s_pf=768, t_pf=0.1, t_max=0.01, gamma=0.75, max_tokens=100000)
    s.add_request(1, 5000, 4, 1.0, 1.0, 0.0)                  # waits 0.91 s: T_r = 1.0 - 0.91 - 7 * 0.01 = 0.02
    t = SO.Request(2, 10, 50, 1.0, 0.05, 0.0, processed=10, generated=1, state=SO.RETURNED, blocks=[s.free.pop()])
    s.reqs[2] = t                                             # T_r = 0.05 - 0.01 = 0.04
    batch = s.next_batch(0.91)
    assert s.t_max < s.reqs[1].t_r < t.t_r                    # the prompt is the head and not urgent
    assert s.token_budget == math.floor(768 * 0.05 / 0.1) == 384
    assert [(e.req.id, e.tokens) for e in batch] == [(2, 1), (1, 383)]


def _generation_task(s, rid, slo_token, context, state=SO.RETURNED, t_enter=0.0):
    """A generation task whose cached context is `context` tokens, holding exactly the blocks for it."""
    nblk = -(-context // s.b)
    r = SO.Request(rid, context, 100, 9.0, slo_token, t_enter, processed=context, generated=1, state=state,
                   blocks=[s.free.pop() for _ in range(nblk)])
    s.reqs[rid] = r
    return r


def test_algorithm1_preempts_the_largest_remaining_time_when_blocks_run_out():
    """Alg. 1, the preemption loop (Sec. 4.4): while a resource is over-committed the request of the batch
    with the largest T_r gives way.  Hand-built: block size 16, a pool of 8 blocks; three generation
    tasks back from the last iteration, each with a full last block (context 32: the next token
    needs a new block), T_r = slo_token - T_max = 0.2, 0.4, 0.3 for ids 10, 11, 12; an urgent prompt
    of 16 tokens arrives (T_r = 0.15 - 0.1 = 0.05 <= T_max).  Held 6 blocks, free 2, demand 3 + 1:
    over-committed.  The victim must be id 11 (T_r 0.4); giving its two blocks back makes 4 free for
    a demand of 3, so nobody else goes.  A smallest-T_r rule would drop the urgent prompt (id 20), a
    first-come rule id 10: both leave a different batch."""
    s = make(b=16, nb=8, s_pf=64, t_pf=0.1, t_max=0.1, gamma=0.0, max_tokens=64)
    for rid, slo in ((10, 0.3), (11, 0.5), (12, 0.4)):
        _generation_task(s, rid, slo, 32)
    s.add_request(20, 16, 2, 0.15, 0.3, 0.0)
    assert len(s.free) == 2
    batch = s.next_batch(0.0)
    assert [round(s.reqs[i].t_r, 12) for i in (10, 11, 12, 20)] == [0.2, 0.4, 0.3, 0.05]
    assert s.preempted_now == [11]
    assert sorted(e.req.id for e in batch) == [10, 12, 20]
    # the victim was preempted for KVC: its blocks are back and it re-enters as a prompt over all its tokens
    v = s.reqs[11]
    assert v.blocks == [] and v.state == SO.WAITING and v.prompt_len == 33 and v.processed == 0
    assert len(s.free) == 4 - 3       # 2 free + 2 returned - 3 handed out


def test_algorithm1_preempts_the_largest_remaining_time_when_tokens_run_out():
    """The same rule with the token budget over-committed (all numbers exact in binary): T_pf 0.125,
    T_max 0.0625, S_pf 6; three returned generation tasks with SLOs 0.0625, 0.3125, 0.1875 (T_r 0,
    0.25, 0.125 for ids 1, 2, 3) and a fourth that was set aside earlier and has become urgent (id 4:
    SLO 0.125, waited 0.125 s, T_r = -0.0625).  S_b = floor(6 * 0.0625 / 0.125) = 3 tokens for four
    tasks: id 2 gives way.  It keeps its blocks (the KVC is not short)."""
    s = make(b=16, nb=64, s_pf=6, t_pf=0.125, t_max=0.0625, gamma=0.0, max_tokens=64)
    for rid, slo in ((1, 0.0625), (2, 0.3125), (3, 0.1875)):
        _generation_task(s, rid, slo, 20)
    _generation_task(s, 4, 0.125, 20, state=SO.PREEMPTED, t_enter=0.875)
    batch = s.next_batch(1.0)
    assert [s.reqs[i].t_r for i in (1, 2, 3, 4)] == [0.0, 0.25, 0.125, -0.0625]
    assert s.token_budget == 3
    assert s.preempted_now == [2] and sorted(e.req.id for e in batch) == [1, 3, 4]
    assert s.reqs[2].state == SO.PREEMPTED and len(s.reqs[2].blocks) == 2


def brute_force_pick(a_c, a_m, b, demands):
    best, arg = None, None
    for i, (d_c, d_m) in enumerate(demands):
        if d_c <= a_c and d_m <= a_m:
            d = math.hypot(a_c - d_c, a_m - d_m)
            if best is None or d < best - 1e-9:
                best, arg = d, i
    return arg


@pytest.mark.parametrize("seed", range(6))
def test_select_requests_takes_the_nearest_demand_first(seed):
    """First pick of Alg. 2 against a brute-force search over (D_c, D_m) with real square roots."""
    rng = np.random.default_rng(seed)
    b, nb = 16, 200
    s = make(b=b, nb=nb, s_pf=512, t_pf=0.1, t_max=0.1, gamma=100.0, max_tokens=512)
    lens = rng.integers(1, 700, size=8)
    for i, n in enumerate(lens):
        s.add_request(i, int(n), 2, 5.0 + 0.001 * i, 5.0, 0.0)   # nobody urgent, all within gamma
    batch = s.next_batch(0.0)
    a_c, a_m = 512, nb * b
    demands = []
    for n in lens:
        d_c = min(int(n), a_c, a_m)
        demands.append((d_c, -(-d_c // b) * b))
    first = brute_force_pick(a_c, a_m, b, demands)
    assert batch[0].req.id == first
    assert sum(e.tokens for e in batch) <= 512


def brute_force_selection(a_c, a_m, b, cands):
    """Alg. 2's greedy selection loop written out on plain numbers: cands = [(id, tokens left, is_long)]; every
    round re-derives each remaining candidate's chunk (all its tokens, or what the tokens / the
    KVC left allow), its KVC demand in tokens (whole blocks), and takes the smallest real Euclidean
    distance to (A_c, A_m); only one long prompt may be under way."""
    picked, left, long_taken = [], list(cands), False
    while True:
        best = None
        for rid, n, is_long in left:
            if is_long and long_taken:
                continue
            d_c = min(n, a_c, a_m)
            if d_c < 1:
                continue
            d_m = -(-d_c // b) * b
            if d_m > a_m:
                continue
            d = math.hypot(a_c - d_c, a_m - d_m)
            if best is None or d < best[0] - 1e-9:
                best = (d, rid, n, is_long, d_c, d_m)
        if best is None:
            return picked
        _, rid, n, is_long, d_c, d_m = best
        picked.append((rid, d_c))
        left = [c for c in left if c[0] != rid]
        long_taken = long_taken or is_long
        a_c, a_m = a_c - d_c, a_m - d_m


@pytest.mark.parametrize("seed", range(8))
def test_select_requests_whole_sequence_inside_the_gamma_window(seed):
    """Alg. 2 from its first line to its last: only requests whose T_r lies within gamma of the
    first one are candidates (0 < gamma < the spread of the queue, so the window cuts it), and
    the whole order of picks and chunk lengths equals the brute-force selection."""
    rng = np.random.default_rng(100 + seed)
    b, nb, s_pf = 16, int(rng.integers(12, 60)), 512     # free blocks: sometimes the KVC binds, sometimes the budget
    s = make(b=b, nb=64, s_pf=s_pf, t_pf=0.1, t_max=0.1, gamma=1.0, max_tokens=512)
    del s.free[: 64 - nb]
    lens = rng.integers(1, 700, size=10)
    slos = 5.0 + 0.3 * np.arange(10) + 0.1 * (lens > s_pf) * np.ceil(lens / s_pf - 1)   # T_r = 4.9 + 0.3 i exactly enough apart
    for i, n in enumerate(lens):
        s.add_request(i, int(n), 2, float(slos[i]), 5.0, 0.0)
    batch = s.next_batch(0.0)
    t_r = [s.reqs[i].t_r for i in range(10)]
    window = [i for i in range(10) if t_r[i] <= min(t_r) + 1.0]
    assert 1 < len(window) < 10                       # the window really cuts the queue
    cands = [(i, int(lens[i]), bool(lens[i] > s_pf)) for i in sorted(window, key=lambda i: (t_r[i], i))]
    want = brute_force_selection(512, nb * b, b, cands)
    assert [(e.req.id, e.tokens) for e in batch] == want
    assert all(e.req.id in window for e in batch)


def simulate(s, trace, n_iter, iter_time, on_batch=None):
    """Feeds a trace to a scheduler; the iteration time follows the forward size."""
    now, nxt, done = 0.0, 0, []
    n = len(trace["arrival"])
    for it in range(n_iter):
        while nxt < n and trace["arrival"][nxt] <= now:
            s.add_request(nxt, int(trace["prompt_len"][nxt]), int(trace["max_new"][nxt]),
                          float(trace["slo_first"][nxt]), float(trace["slo_token"][nxt]), float(trace["arrival"][nxt]))
            nxt += 1
        batch = s.next_batch(now)
        if on_batch:
            on_batch(s, batch, now)
        now += iter_time(sum(e.tokens for e in batch))
        done += s.complete(now)
    return done


@pytest.mark.parametrize("seed,nb", [(1, 4096), (2, 1500), (3, 600)])
def test_schedule_invariants_over_a_trace(seed, nb):
    """Whatever the decisions: the budget is never exceeded, no block is ever shared or lost, every
    request's tokens run exactly once and in order, returned generation tasks stay unless
    preempted, and at most one new long prompt starts while another is in progress (urgent ones
    aside).  The small pools force preemptions and recomputation."""
    b = 16
    trace = W.poisson_trace(150, seed, rate=8.0, max_prompt=3000, max_new=64)
    s = make(b=b, nb=nb, s_pf=768, t_pf=0.05, t_max=0.05, gamma=0.75, max_tokens=2048)
    seen = {}
    state = {"batches": 0, "tokens": 0, "preempted": 0}

    def check(s, batch, now):
        assert sum(e.tokens for e in batch) <= s.token_budget
        ids = [e.req.id for e in batch]
        assert len(set(ids)) == len(ids)
        held = [blk for r in s.reqs.values() for blk in r.blocks]
        assert len(set(held)) == len(held) and not (set(held) & set(s.free))
        assert len(held) + len(s.free) == nb
        _, cs, ctx, slots, tables = s.batch_arrays()
        assert len(set(slots)) == len(slots)
        for e, c, tab in zip(batch, ctx, tables):
            r = e.req
            assert len(tab) == -(-c // b) == len(r.blocks)
            prior = c - e.tokens
            hist = seen.setdefault(r.id, [0, 0])     # [tokens in cache, recomputations]
            if prior == 0 and hist[0] != 0:
                hist[0] = 0                           # recomputation restarts the sequence
                hist[1] += 1
            assert prior == hist[0]
            hist[0] = c
        state["batches"] += 1
        state["tokens"] += sum(e.tokens for e in batch)
        state["preempted"] += len(s.preempted_now)

    done = simulate(s, trace, 1500, lambda sf: 0.05 * max(sf, 64) / 768, check)
    assert len(done) == len(set(done)) and len(done) > (50 if nb >= 1500 else 10)
    assert state["tokens"] > 0
    if nb <= 600:
        assert state["preempted"] > 0
    for rid in done:
        # a finished request was fed its prompt and all generated tokens but the last
        assert seen[rid][0] >= int(trace["prompt_len"][rid])


def test_offline_allowance_and_its_propagation():
    """Sec. 4.3, SLOs of offline applications, on hand-computed numbers: L_c = 768, a 2000-token
    prompt (3 chunks), 100 predicted tokens, T_max 0.1 s, P_max 2 s, P 0.05:
    T_e = 3 * 0.1 + 100 * (0.1 + 0.1) = 20.3 s; with a JCT SLO of 61.5 s each of the 103 iterations
    may wait (61.5 - 20.3) / 103 = 0.4 s.  Waiting 0.25 s leaves 0.15 s for the next iteration
    (allowance + d); waiting 0.7 s of the 0.55 s then allowed takes 0.15 s from the one after
    (allowance - d)."""
    s = SO.Scheduler(16, 4096, 768, 0.1, 0.1, 0.75, 768, None, preempt_max_time=2.0, preempt_probability=0.05)
    s.add_offline_request(1, 2000, 50, 100, 61.5, 10.0)
    r = s.reqs[1]
    assert r.allowance == pytest.approx(0.4, abs=1e-12)
    assert s.remaining_time(r, 10.1) == pytest.approx(0.3, abs=1e-12)
    batch = s.next_batch(10.25)                      # scheduled after waiting 0.25 s
    assert [e.req.id for e in batch] == [1]
    assert r.carry == pytest.approx(0.15, abs=1e-12)
    s.complete(10.35)                                # its next chunk waits from here
    assert s.remaining_time(r, 10.35) == pytest.approx(0.55, abs=1e-12)
    s.next_batch(10.35 + 0.7)
    assert r.carry == pytest.approx(-0.15, abs=1e-12)
    s.complete(11.15)
    assert s.remaining_time(r, 11.15) == pytest.approx(0.25, abs=1e-12)
    # Eq. 6 sees the allowance plus one batch execution as this request's iteration SLO
    assert s.slo_of(r) == pytest.approx(0.5, abs=1e-12)
    # once it generates, a task that returns and runs at once has waited 0 s: the whole allowance moves on
    s.next_batch(11.15)
    s.complete(11.25)
    assert r.state == SO.RETURNED and r.carry == pytest.approx(0.25, abs=1e-12)
    s.next_batch(11.25)
    assert r.carry == pytest.approx(0.65, abs=1e-12)


@pytest.mark.parametrize("seed,nb,swap", [(3, 600, 400), (2, 500, 64), (5, 700, 30000)])
def test_swap_pool_keeps_preempted_tasks_whole(seed, nb, swap):
    """With a swap pool a generation task preempted for KVC keeps its tokens: its blocks are copied
    out (pairs reported), freed here, and copied back into fresh blocks when it runs again, its
    context continuing where it stopped.  Both pools conserve their blocks; every copy's source is
    owned by the victim at that moment and every destination is free; when the swap pool is too
    small the task is recomputed instead."""
    b = 16
    trace = W.poisson_trace(150, seed, rate=8.0, max_prompt=3000, max_new=64)
    s = SO.Scheduler(b, nb, 768, 0.05, 0.05, 0.75, 2048, None, swap_blocks=swap)
    seen, stats = {}, {"out": 0, "in": 0, "recomputed": 0}
    owner_before = {}

    def check(s, batch, now):
        out_pairs, in_pairs = s.batch_swaps()
        held = [blk for r in s.reqs.values() for blk in r.blocks]
        swapped = [blk for r in s.reqs.values() for blk in r.swap]
        assert len(set(held)) == len(held) and len(held) + len(s.free) == nb
        assert len(set(swapped)) == len(swapped) and len(swapped) + len(s.swap_free) == swap
        assert len({d for _, d in out_pairs}) == len(out_pairs) and len({d for _, d in in_pairs}) == len(in_pairs)
        for src, dst in out_pairs:
            assert owner_before.get(src) is not None, "a block copied out belonged to somebody before this decision"
        for src, dst in in_pairs:
            assert dst in held
        stats["out"] += len(out_pairs)
        stats["in"] += len(in_pairs)
        _, cs, ctx, slots, tables = s.batch_arrays()
        for e, c in zip(batch, ctx):
            prior = c - e.tokens
            hist = seen.setdefault(e.req.id, [0])
            if prior == 0 and hist[0] != 0:
                stats["recomputed"] += 1
                hist[0] = 0
            assert prior == hist[0]
            hist[0] = c
        owner_before.clear()
        owner_before.update({blk: r.id for r in s.reqs.values() for blk in r.blocks})

    done = simulate(s, trace, 1500, lambda sf: 0.05 * max(sf, 64) / 768, check)
    assert stats["out"] > 0 and stats["in"] > 0 and len(done) > 10
    if swap >= 30000:
        assert stats["recomputed"] == 0
    if swap <= 64:
        assert stats["recomputed"] > 0
