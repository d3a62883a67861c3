"""The entry point that allocates nothing (mpa_mixed_paged_attention_static) against the entry
point it is a variant of, through the C ABI: two calls in a row on the same GPU, the second with a
smaller batch, so that what the first left in the library's device array must not matter.  Both
forms run the same kernels over the same plan, so their outputs are compared bit for bit (and the
workspace form against the CPU oracle, to the usual bars)."""
import ctypes

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


def both_forms(mpa, ctx, b):
    """out of the workspace form and of the static form, on the same cache (the append done once)."""
    import torch
    db = DeviceBatch(b, "prior")
    ctx.kv_append(db.k_new, db.v_new, db.slot_map, db.k_cache, db.v_cache)
    ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    ctx.mixed_paged_attention(db.q, db.k_cache, db.v_cache, db.block_table, b.chunk_starts, b.context_lens, db.out, ws,
                              scale=b.scale)
    out_static = torch.full_like(db.out, 0x7FFF)
    ctx.mixed_paged_attention_static(db.q, db.k_cache, db.v_cache, db.block_table, b.chunk_starts, b.context_lens,
                                     out_static, scale=b.scale)
    torch.cuda.synchronize()
    return to_host_u16(db.out), to_host_u16(out_static)


def test_static_form_equals_workspace_form_on_two_calls_in_a_row(mpa):
    # first call: prompt chunks and generation rows with every key range forced short, so that the
    # array holds a long work list and many partial results
    ql, ctx = [300, 150, 1, 1, 1, 1], [1400, 150, 900, 64, 2100, 17]
    big = W.make_batch("static-big", 321, 8, 128, 16, sum((c + 15) // 16 for c in ctx) + 5, ql, ctx)
    c1 = mpa.Context(big.H, big.D, block_size=big.bs, num_kv_heads=big.HK)
    c1.set_option(mpa.MPA_OPT_PP_SPLIT_TOKENS, 128)
    c1.set_option(mpa.MPA_OPT_TG_SPLIT_BLOCKS, 4)
    items, counts = c1.plan_describe(big.chunk_starts, big.context_lens)
    assert counts[3] > 0 and len(items) * 32 + counts[2] * 16 > 2 * 3584     # several list chunks, partials in use
    out_ws, out_st = both_forms(mpa, c1, big)
    ref, _, _ = oracle_run(big)
    assert_close(out_ws, ref, "workspace form, first batch")
    assert np.array_equal(out_st, out_ws), "static form differs from the workspace form (first call)"

    # second call, right behind it: a smaller batch of another shape on another context
    small = W.config1()
    c2 = mpa.Context(small.H, small.D, block_size=small.bs, num_kv_heads=small.HK)
    out_ws, out_st = both_forms(mpa, c2, small)
    ref, _, _ = oracle_run(small)
    assert_close(out_ws, ref, "workspace form, second batch")
    assert np.array_equal(out_st, out_ws), "static form differs from the workspace form (second, smaller call)"

    # and the first shape again without forced splits (its own automatic plan)
    c3 = mpa.Context(big.H, big.D, block_size=big.bs, num_kv_heads=big.HK)
    out_ws, out_st = both_forms(mpa, c3, big)
    assert np.array_equal(out_st, out_ws)


def test_static_form_refuses_a_batch_that_does_not_fit(mpa):
    """Config 5's 25th iteration needs about 130 MiB of partial results: refused with
    MPA_ERR_WORKSPACE before anything is launched (the pointers are never dereferenced)."""
    b = W.config5(24)
    c = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK)
    assert c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens) > mpa.MPA_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    rc = mpa.load().mpa_mixed_paged_attention_static(c._h, fake, fake, fake, fake, 8192, mpa._ptr(b.chunk_starts),
                                                     mpa._ptr(b.context_lens), b.S, b.T, 0.0, fake, None)
    assert rc == mpa.MPA_ERR_WORKSPACE


def test_static_form_replays_from_a_hip_graph(mpa):
    """The entry point that allocates nothing reads no host memory after it returns (its work list travels as
    kernel arguments) and records no memset, so a serving loop can capture it into a HIP graph for a fixed
    batch shape.  Captured once, replayed four times with eager calls on another batch (which overwrite the
    library's device array) and fresh query values in between; every replay must equal the eager call on the
    same inputs bit for bit."""
    import torch
    b = W.make_batch("graph-decode", 77, 8, 128, 16, 400, [1, 1, 1, 1, 40], [900, 64, 2100, 17, 300])
    other = W.config1()
    ctx = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK)
    ctx2 = mpa.Context(other.H, other.D, block_size=other.bs, num_kv_heads=other.HK)
    db, db2 = DeviceBatch(b, "prior"), DeviceBatch(other, "prior")
    ctx.kv_append(db.k_new, db.v_new, db.slot_map, db.k_cache, db.v_cache)
    ctx2.kv_append(db2.k_new, db2.v_new, db2.slot_map, db2.k_cache, db2.v_cache)

    def eager(out):
        ctx.mixed_paged_attention_static(db.q, db.k_cache, db.v_cache, db.block_table, b.chunk_starts, b.context_lens, out,
                                         scale=b.scale)

    def eager_other():
        ctx2.mixed_paged_attention_static(db2.q, db2.k_cache, db2.v_cache, db2.block_table, other.chunk_starts,
                                          other.context_lens, db2.out, scale=other.scale)

    want = torch.full_like(db.out, 0x7FFF)
    eager(want)                       # also the first use of the device array on this GPU: its address is looked up here
    eager_other()
    torch.cuda.synchronize()
    ref = oracle_run(b)[0]
    assert_close(to_host_u16(want), ref, "eager static call")

    got = torch.full_like(db.out, 0x7FFF)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):      # the binding launches on torch's current stream: the capturing one
        eager(got)
    q0 = db.q.clone()
    for rep in range(4):
        if rep:                        # new query values in the same buffer: rows rotated by `rep`
            db.q.copy_(torch.roll(q0, rep, dims=2))
            eager(want)
        eager_other()                  # overwrites the work list and the partial results in the device array
        torch.cuda.synchronize()
        got.fill_(0x7FFF)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"replay {rep} differs from the eager call"
    assert not torch.equal(got, torch.full_like(got, 0x7FFF))
