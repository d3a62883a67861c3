"""The scheduler of libmpa.so (include/mpa_sched.h) against the Python oracle: the same trace,
the same clock, every iteration's batch compared array by array (ids, chunk_starts, context_lens,
slot_map, block table, budget, preemptions, finished requests) -- integer work, bit-exact.
Host only: runs without a GPU."""
import numpy as np
import pytest

import paper_2503_13737_amd as mpa
import workloads as W
from oracle import sched_oracle as SO


def run_both(trace, n_iter, b, nb, s_pf, t_pf, t_max, gamma, max_tokens, order, iter_time, offline_every=0, swap=0):
    """offline_every = k > 0: every k-th request is an offline one with a JCT SLO of 40 times its
    first-token SLO and a predicted length of half its real one."""
    o = SO.Scheduler(b, nb, s_pf, t_pf, t_max, gamma, max_tokens, order, 1.5, 0.1, swap)
    c = mpa.Scheduler(b, nb, s_pf, t_pf, t_max, gamma, max_tokens, order, 1.5, 0.1, swap)
    now, nxt, n = 0.0, 0, len(trace["arrival"])
    stats = {"batches": 0, "tokens": 0, "preempted": 0, "finished": 0, "chunks": 0, "swapped": 0}
    for it in range(n_iter):
        while nxt < n and trace["arrival"][nxt] <= now:
            args = (nxt, int(trace["prompt_len"][nxt]), int(trace["max_new"][nxt]), float(trace["slo_first"][nxt]),
                    float(trace["slo_token"][nxt]), float(trace["arrival"][nxt]))
            if offline_every and nxt % offline_every == 0:
                off = (nxt, args[1], args[2], max(1, args[2] // 2), 40.0 * args[3], args[5])
                o.add_offline_request(*off)
                c.add_offline_request(*off)
            else:
                o.add_request(*args)
                c.add_request(*args)
            nxt += 1
        ob = o.next_batch(now)
        info = c.next_batch(now)
        ids, cs, ctx, slots, tables = o.batch_arrays()
        what = f"iteration {it}"
        assert info.num_seqs == len(ob), what
        assert info.token_budget == o.token_budget and info.num_preempted == len(o.preempted_now), what
        assert info.free_blocks == len(o.free), what
        assert info.num_prompt_chunks == sum(1 for e in ob if e.req.is_prompt), what
        g_ids, g_cs, g_ctx, g_slots, g_tab = c.batch_arrays()
        assert g_ids.tolist() == ids and g_cs.tolist() == cs and g_ctx.tolist() == ctx and g_slots.tolist() == slots, what
        o_out, o_in = o.batch_swaps()
        c_out, c_in = c.batch_swaps()
        assert c_out.tolist() == [list(x) for x in o_out] and c_in.tolist() == [list(x) for x in o_in], what
        stats["swapped"] += len(o_out)
        for row, ref in zip(g_tab, tables):
            assert row[: len(ref)].tolist() == ref and (row[len(ref):] == -1).all(), what
        now += iter_time(info.num_tokens)
        assert sorted(c.complete(now).tolist()) == sorted(o.complete(now)), what
        assert c.live_requests == len(o.reqs)
        stats["batches"] += 1 if info.num_seqs else 0
        stats["tokens"] += info.num_tokens
        stats["preempted"] += info.num_preempted
        stats["chunks"] += info.num_prompt_chunks
    return stats


@pytest.mark.parametrize("seed,b,nb,rate", [(1, 16, 4096, 8.0), (2, 16, 1500, 8.0), (3, 16, 600, 8.0),
                                            (4, 32, 400, 12.0), (5, 128, 96, 6.0), (6, 1, 20000, 10.0)])
def test_same_batches_as_the_oracle_over_a_trace(seed, b, nb, rate):
    trace = W.poisson_trace(160, seed, rate=rate, max_prompt=3000, max_new=64)
    order = W.permutation(nb, 77 + seed)
    st = run_both(trace, 1200, b, nb, 768, 0.05, 0.05, 0.75, 2048, order,
                  lambda sf: 0.05 * max(sf, 64) / 768)
    assert st["batches"] > 300 and st["chunks"] > 50
    if nb * b <= 12800:
        assert st["preempted"] > 0     # the small pools exercise preemption and recomputation


@pytest.mark.parametrize("seed,nb,every", [(11, 4096, 2), (12, 700, 3), (13, 1500, 1)])
def test_same_batches_with_offline_requests_in_the_mix(seed, nb, every):
    trace = W.poisson_trace(140, seed, rate=8.0, max_prompt=3000, max_new=64)
    st = run_both(trace, 1200, 16, nb, 768, 0.05, 0.05, 0.75, 2048, W.permutation(nb, seed),
                  lambda sf: 0.05 * max(sf, 64) / 768, offline_every=every)
    assert st["batches"] > 300 and st["chunks"] > 50


@pytest.mark.parametrize("seed,b,nb,swap", [(3, 16, 600, 400), (2, 16, 500, 64), (4, 32, 300, 1000), (7, 16, 600, 5)])
def test_same_batches_with_a_swap_pool(seed, b, nb, swap):
    """Preemption by swapping: the same block pairs out and in, the same fall-back to recomputation
    when the swap pool is full."""
    trace = W.poisson_trace(150, seed, rate=8.0, max_prompt=3000, max_new=64)
    st = run_both(trace, 1200, b, nb, 768, 0.05, 0.05, 0.75, 2048, W.permutation(nb, seed + 40),
                  lambda sf: 0.05 * max(sf, 64) / 768, offline_every=5, swap=swap)
    assert st["preempted"] > 0 and st["swapped"] > 0


def test_same_batches_with_tight_slos_and_a_small_budget():
    """Budget below the pivot (SLO_min < T_pf), many urgent requests, gamma 0."""
    trace = W.poisson_trace(120, 9, rate=20.0, max_prompt=1500, max_new=32, base_token_slo=0.03, base_first_slo=0.2)
    st = run_both(trace, 1000, 16, 2048, 512, 0.04, 0.06, 0.0, 1024, None, lambda sf: 0.04 * max(sf, 32) / 512)
    assert st["tokens"] > 10000


def test_scheduler_argument_checks():
    with pytest.raises(mpa.MpaError):
        mpa.Scheduler(16, 8, 768, 0.05, 0.05, 0.75, 2048, block_order=[0, 1, 2, 3, 4, 5, 6, 6])
    with pytest.raises(mpa.MpaError):
        mpa.Scheduler(0, 8, 768, 0.05, 0.05, 0.75, 2048)
    s = mpa.Scheduler(16, 8, 768, 0.05, 0.05, 0.75, 2048)
    s.add_request(1, 100, 4, 1.0, 1.0, 0.0)
    with pytest.raises(mpa.MpaError):
        s.add_request(1, 10, 4, 1.0, 1.0, 0.0)          # duplicate id
    with pytest.raises(mpa.MpaError):
        s.add_request(2, 128, 2, 1.0, 1.0, 0.0)         # 129 tokens do not fit 8 blocks of 16
    with pytest.raises(mpa.MpaError):
        s.add_request(3, 0, 2, 1.0, 1.0, 0.0)
    with pytest.raises(mpa.MpaError):
        s.add_offline_request(4, 10, 2, 0, 100.0, 0.0)   # no predicted length
    info = s.next_batch(0.0)
    assert (info.num_seqs, info.num_tokens, info.num_prompt_chunks) == (1, 100, 1)
    ids, cs, ctx, slots, tab = s.batch_arrays(stride=9)
    assert tab.shape == (1, 9) and (tab[0, 7:] == -1).all() and cs.tolist() == [0, 100] and ctx.tolist() == [100]
    assert s.complete(0.05).tolist() == [] and s.live_requests == 1
    lib = mpa.load()
    assert lib.mpa_sched_next_batch(None, 0.0, None) == mpa.MPA_ERR_INVALID_ARG
    assert lib.mpa_sched_destroy(None) == mpa.MPA_OK
