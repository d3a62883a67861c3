"""GPU tests of the runtime behaviour of the library: streams, repeated and interleaved calls,
run-to-run determinism, staging-buffer reuse."""
import numpy as np
import pytest

import workloads as W
from harness import DeviceBatch, assert_close, oracle_run, to_host_u16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mpa():
    import paper_2503_13737_amd as m
    m.load()
    return m


def run_on(ctx, db, b, ws, stream=None):
    ctx.kv_append(db.k_new, db.v_new, db.slot_map, db.k_cache, db.v_cache, stream=stream)
    ctx.mixed_paged_attention(db.q, db.k_cache, db.v_cache, db.block_table, b.chunk_starts, b.context_lens,
                              db.out, ws, scale=b.scale, stream=stream)


def test_side_stream_and_many_calls_in_flight(mpa):
    """40 calls enqueued without waiting (more than the staging ring holds) on a side stream."""
    import torch
    b = W.config1()
    ref, _, _ = oracle_run(b)
    ctx = mpa.Context(b.H, b.D)
    s = torch.cuda.Stream()
    dbs = [DeviceBatch(b, "prior") for _ in range(4)]
    wss = [torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8,
                       device="cuda") for _ in range(4)]
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        for i in range(40):
            run_on(ctx, dbs[i % 4], b, wss[i % 4], stream=s)
    s.synchronize()
    outs = [to_host_u16(d.out) for d in dbs]
    for o in outs:
        assert_close(o, ref, "side stream")
        assert np.array_equal(o, outs[0])  # same work decomposition -> bit-identical


def test_one_context_alternating_batches(mpa):
    import torch
    b1 = W.random_ragged(9001, H=4, D=128, n_pp=2, n_tg=3, max_q=300, max_prior=500, max_ctx=900)
    b2 = W.random_ragged(9002, H=4, D=128, n_pp=1, n_tg=6, max_q=150, max_prior=100, max_ctx=2000)
    ctx = mpa.Context(4, 128)
    refs = [oracle_run(b)[0] for b in (b1, b2)]
    for rep in range(3):
        for b, ref in ((b1, refs[0]), (b2, refs[1])):
            db = DeviceBatch(b, "prior")
            ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8,
                             device="cuda")
            ws.fill_(0xFF)
            run_on(ctx, db, b, ws)
            torch.cuda.synchronize()
            assert_close(to_host_u16(db.out), ref, f"{b.name} rep {rep}")


def test_reused_work_list_same_batch_then_same_sizes_other_lengths(mpa):
    """A call with the previous call's chunk_starts / context_lens reuses its work list (fresh
    workspace, poisoned, each time); a batch of the same sizes but other context lengths, and an
    option change, must not."""
    import torch
    ql = [200, 1, 1, 1]
    ctx_a, ctx_b = [700, 300, 64, 1500], [700, 301, 64, 900]
    ba = W.make_batch("reuse-a", 41, 4, 128, 16, 200, ql, ctx_a)
    bb = W.make_batch("reuse-b", 42, 4, 128, 16, 200, ql, ctx_b)
    ctx = mpa.Context(4, 128)
    refs = {id(b): oracle_run(b)[0] for b in (ba, bb)}
    for step, b in enumerate((ba, ba, bb, bb, ba)):
        if step == 3:
            ctx.set_option(mpa.MPA_OPT_TG_SPLIT_BLOCKS, 2)
        db = DeviceBatch(b, "prior")
        ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        run_on(ctx, db, b, ws)
        torch.cuda.synchronize()
        assert_close(to_host_u16(db.out), refs[id(b)], f"{b.name} call {step}")


def test_run_to_run_bit_identical_on_split_heavy_batch(mpa):
    import torch
    b = W.random_ragged(9100, H=5, D=128, n_pp=2, n_tg=4, max_q=400, max_prior=3000, max_ctx=4000)
    ctx = mpa.Context(5, 128)
    ctx.set_option(mpa.MPA_OPT_TG_SPLIT_BLOCKS, 4)
    ctx.set_option(mpa.MPA_OPT_PP_SPLIT_TOKENS, 256)
    ref = oracle_run(b)[0]
    first = None
    for rep in range(5):
        db = DeviceBatch(b, "prior")
        ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF if rep % 2 else 0x00)
        run_on(ctx, db, b, ws)
        torch.cuda.synchronize()
        out = to_host_u16(db.out)
        if first is None:
            first = out
            assert_close(out, ref, b.name)
        assert np.array_equal(out, first)


def test_workspace_too_small_is_rejected_before_launch(mpa):
    import torch
    b = W.config1()
    ctx = mpa.Context(b.H, b.D)
    db = DeviceBatch(b, "ctx")
    need = ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    with pytest.raises(mpa.MpaError) as e:
        ctx.mixed_paged_attention(db.q, db.k_cache, db.v_cache, db.block_table, b.chunk_starts, b.context_lens,
                                  db.out, ws, scale=b.scale, workspace_bytes=need - 1)
    assert e.value.status == mpa.MPA_ERR_WORKSPACE
    assert ctx.last_hip_error() == 0
