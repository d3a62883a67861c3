"""GPU: kv_append + mixed_paged_attention (or the one call with the append inside the attention launch) on the batches the scheduler forms, iteration after
iteration over one persistent paged cache (blocks handed out, freed and reused by the scheduler's
pool, prompts cut wherever the budget ends, generation tasks growing by a token, preemption with
recomputation in the small pool), against the oracle run on a numpy copy of the same cache."""
import numpy as np
import pytest

import workloads as W
from harness import assert_close, to_dev, to_host_u16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("H,HK,D,bs,nb,dtype,swap,inside", [
    (4, 4, 128, 16, 1024, "bf16", 0, 0), (8, 2, 64, 32, 60, "fp16", 0, 0), (4, 2, 128, 32, 60, "bf16", 80, 0),
    # the same with the append inside the attention launch (one call per iteration)
    (4, 4, 128, 16, 1024, "bf16", 0, 1), (8, 2, 64, 32, 60, "fp16", 0, 1), (4, 2, 128, 32, 60, "bf16", 80, 1)])
def test_scheduler_batches_through_the_kernels(H, HK, D, bs, nb, dtype, swap, inside):
    import oracle
    import paper_2503_13737_amd as mpa
    import torch
    trace = W.poisson_trace(40, 5, rate=30.0, max_prompt=700, max_new=10)
    sched = mpa.Scheduler(bs, nb, 256, 0.02, 0.02, 0.75, 512, block_order=W.permutation(nb, 5), swap_blocks=swap)
    # the swap pool: a second pair of caches, on the device here as well
    sk = np.full((max(swap, 1), HK, bs, D), W.POISON, dtype=np.uint16)
    sv = sk.copy()
    d_sk, d_sv = to_dev(sk), to_dev(sv)
    swapped = 0
    ctx = mpa.Context(H, D, block_size=bs, num_kv_heads=HK, dtype=mpa.MPA_FP16 if dtype == "fp16" else mpa.MPA_BF16)
    ctx.set_option(mpa.MPA_OPT_FUSE_APPEND, inside)
    kc = np.full((nb, HK, bs, D), W.POISON, dtype=np.uint16)
    vc = kc.copy()
    d_kc, d_vc = to_dev(kc), to_dev(vc)
    ws = torch.empty(ctx.workspace_bytes(64, 512, nb * bs), dtype=torch.uint8, device="cuda")
    now, nxt, iters, preempted, chunks, finished = 0.0, 0, 0, 0, 0, 0
    scale = 1.0 / np.sqrt(D)
    while iters < 160 and (nxt < 40 or sched.live_requests):
        while nxt < 40 and trace["arrival"][nxt] <= now:
            sched.add_request(nxt, int(trace["prompt_len"][nxt]), int(trace["max_new"][nxt]),
                              float(trace["slo_first"][nxt]), float(trace["slo_token"][nxt]), float(trace["arrival"][nxt]))
            nxt += 1
        info = sched.next_batch(now)
        iters += 1
        preempted += info.num_preempted
        chunks += info.num_prompt_chunks
        now += 0.02 * max(info.num_tokens, 16) / 256
        # preempted tasks leave for the swap pool and return from it before anything else touches the blocks
        out_pairs, in_pairs = sched.batch_swaps()
        swapped += len(out_pairs)
        if len(out_pairs):
            ctx.copy_blocks(d_kc, d_vc, d_sk, d_sv, to_dev(out_pairs))
            oracle.copy_blocks(kc, vc, sk, sv, out_pairs)
            kc[out_pairs[:, 0]], vc[out_pairs[:, 0]] = W.POISON, W.POISON      # given up: nobody may read them
            d_kc[torch.from_numpy(out_pairs[:, 0]).cuda()] = 0x7FFF
            d_vc[torch.from_numpy(out_pairs[:, 0]).cuda()] = 0x7FFF
        if len(in_pairs):
            ctx.copy_blocks(d_sk, d_sv, d_kc, d_vc, to_dev(in_pairs))
            oracle.copy_blocks(sk, sv, kc, vc, in_pairs)
        if info.num_seqs == 0:
            sched.complete(now)
            continue
        ids, cs, ctxl, slots, table = sched.batch_arrays()
        q_len = np.diff(cs)
        rid = np.repeat(ids, q_len)
        pos = np.concatenate([np.arange(c - n, c) for c, n in zip(ctxl, q_len)])
        q = W.token_rows(rid, pos, H * D, 11, dtype).reshape(-1, H, D)
        kn = W.token_rows(rid, pos, HK * D, 12, dtype).reshape(-1, HK, D)
        vn = W.token_rows(rid, pos, HK * D, 13, dtype).reshape(-1, HK, D)
        what = f"iteration {iters}: {info.num_seqs} seqs, {info.num_tokens} tokens"
        print(what, flush=True)
        # GPU
        out = torch.full((info.num_tokens, H, D), 0x7FFF, dtype=torch.int16, device="cuda")
        ws.fill_(0xFF)
        if inside:
            ctx.append_and_attend(to_dev(kn), to_dev(vn), to_dev(slots), to_dev(q), d_kc, d_vc,
                                  to_dev(np.ascontiguousarray(table)), cs, ctxl, out, ws, scale=scale)
        else:
            ctx.kv_append(to_dev(kn), to_dev(vn), to_dev(slots), d_kc, d_vc)
            ctx.mixed_paged_attention(to_dev(q), d_kc, d_vc, to_dev(np.ascontiguousarray(table)), cs, ctxl, out, ws, scale=scale)
        torch.cuda.synchronize()
        # oracle
        oracle.kv_append(kn, vn, slots, kc, vc)
        ref = oracle.attention(q, kc, vc, table, cs, ctxl, scale, dtype=dtype)
        assert_close(to_host_u16(out), ref, what, dtype=dtype)
        finished += len(sched.complete(now))
    assert np.array_equal(to_host_u16(d_kc), kc) and np.array_equal(to_host_u16(d_vc), vc)
    assert chunks > 20 and finished > 5
    if nb * bs < 8000:
        assert preempted > 0
    if swap:
        assert swapped > 0
