"""GPU tests of the runtime behaviour of the library: streams, repeated and interleaved calls,
run-to-run determinism, staging-buffer reuse."""
import numpy as np
import pytest

import workloads as W
from harness import DeviceBatch, assert_close, oracle_run, to_dev, to_host_u16

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


def test_work_list_left_in_the_workspace_is_reused(mpa):
    """Plan cache level 2: same batch, same workspace, same stream -> no upload; the inputs change
    from call to call (as from layer to layer) and every result is checked.  Another workspace,
    another batch and a return to the first batch each upload again.  Includes a prompt-heavy
    batch with few resident work-groups, whose progress words must be back at their start value."""
    import torch
    ql, ctxl = [600, 300, 1, 1, 1], [1500, 300, 700, 64, 2000]
    batches = [W.make_batch(f"keep-{seed}", seed, 4, 128, 16, sum((c + 15) // 16 for c in ctxl) + 3, ql, ctxl) for seed in (51, 52, 53)]
    other = W.make_batch("keep-other", 54, 4, 128, 16, 200, [100, 1], [400, 900])
    ctx = mpa.Context(4, 128)
    ctx.set_option(mpa.MPA_OPT_PLAN_CACHE, 2)
    ctx.set_option(mpa.MPA_OPT_PP_RESIDENT_WGS, 3)
    ctx.set_option(mpa.MPA_OPT_PP_TEAM_MIN_STEPS, 1)
    need = max(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens) for b in batches + [other])
    ws1 = torch.empty(need, dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(need, dtype=torch.uint8, device="cuda")
    ws1.fill_(0xFF)
    ws2.fill_(0xFF)
    for step, (b, ws) in enumerate([(batches[0], ws1), (batches[1], ws1), (batches[2], ws1), (batches[0], ws2),
                                    (batches[1], ws2), (other, ws2), (batches[2], ws2), (batches[0], ws2)]):
        db = DeviceBatch(b, "prior")
        run_on(ctx, db, b, ws)
        torch.cuda.synchronize()
        assert_close(to_host_u16(db.out), oracle_run(b)[0], f"{b.name} call {step}")
    with pytest.raises(mpa.MpaError):
        ctx.set_option(mpa.MPA_OPT_PLAN_CACHE, 3)


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


@pytest.mark.parametrize("H,HK,D,bs", [(4, 4, 64, 16), (8, 2, 128, 32), (5, 5, 128, 128)])
def test_copy_blocks_swaps_a_sequence_out_and_back_in(mpa, H, HK, D, bs):
    """Blocks of two sequences go to a second pool and come back into other blocks: bit-exact
    against the oracle's copies on both pools (untouched blocks included, a negative pair is
    skipped), and attention through the re-mapped table is bit-identical to before."""
    import oracle
    import torch
    ql, ctx = [70, 1, 1, 33], [200, 300, 17, 33 + 3 * bs]
    b = W.make_batch("swap", 404, H, D, bs, sum((c + bs - 1) // bs for c in ctx) + 40, ql, ctx, Hkv=HK)
    c = mpa.Context(H, D, block_size=bs, num_kv_heads=HK)
    kc, vc = b.full_cache("ctx")
    d_kc, d_vc = to_dev(kc), to_dev(vc)
    ws = torch.empty(c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")

    def attend(table):
        out = torch.full((b.T, H, D), 0x7FFF, dtype=torch.int16, device="cuda")
        c.mixed_paged_attention(to_dev(b.q), d_kc, d_vc, to_dev(np.ascontiguousarray(table)), b.chunk_starts, b.context_lens,
                                out, ws, scale=b.scale)
        torch.cuda.synchronize()
        return to_host_u16(out)

    before = attend(b.block_table)
    nbl = b.n_blocks()
    held = np.concatenate([b.block_table[i, : nbl[i]] for i in (0, 3)]).astype(np.int64)
    n = held.size
    host_k = np.full((n + 3,) + kc.shape[1:], 0x4321, dtype=np.uint16)
    host_v = host_k.copy()
    d_hk, d_hv = to_dev(host_k), to_dev(host_v)
    out_pairs = np.stack([held, W.permutation(n, 9)], axis=1)
    out_pairs = np.concatenate([out_pairs, [[-1, n + 1], [held[0], -1]]]).astype(np.int64)   # skipped
    c.copy_blocks(d_kc, d_vc, d_hk, d_hv, to_dev(out_pairs))
    oracle.copy_blocks(kc, vc, host_k, host_v, out_pairs[:n])
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(d_hk), host_k) and np.array_equal(to_host_u16(d_hv), host_v)
    # the old blocks are given up (poisoned here), the sequence returns into unreferenced blocks
    free = np.setdiff1d(np.arange(b.NB), b.referenced_blocks())[:n].astype(np.int64)
    kc[held], vc[held] = W.POISON, W.POISON
    d_kc[torch.from_numpy(held).cuda()] = 0x7FFF
    d_vc[torch.from_numpy(held).cuda()] = 0x7FFF
    in_pairs = np.stack([out_pairs[:n, 1], free], axis=1)
    c.copy_blocks(d_hk, d_hv, d_kc, d_vc, to_dev(in_pairs))
    oracle.copy_blocks(host_k, host_v, kc, vc, in_pairs)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(d_kc), kc) and np.array_equal(to_host_u16(d_vc), vc)
    table = b.block_table.copy()
    remap = dict(zip(held.tolist(), free.tolist()))
    for i in (0, 3):
        table[i, : nbl[i]] = [remap[int(x)] for x in table[i, : nbl[i]]]
    assert np.array_equal(attend(table), before)
    # inside one pool (migration), and the empty call
    moved = np.stack([free[:2], held[:2]], axis=1)
    c.copy_blocks(d_kc, d_vc, d_kc, d_vc, to_dev(moved))
    oracle.copy_blocks(kc.copy(), vc.copy(), kc, vc, moved)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(d_kc), kc)
    assert mpa.load().mpa_copy_blocks(c._h, None, None, None, None, None, 0, None) == 0


@pytest.mark.parametrize("make", [
    lambda: W.config1(),
    lambda: W.config1(dtype="fp16"),
    lambda: W.random_ragged(7100, H=8, D=128, bs=32, n_pp=3, n_tg=5, max_q=300, max_prior=900, max_ctx=1500, Hkv=2),
    lambda: W.make_batch("fused-mixed", 61, 4, 128, 16, 400, [600, 300, 1, 1, 1], [1500, 300, 700, 64, 2000]),
], ids=["cfg1", "cfg1-fp16", "ragged-gqa-bs32", "prompt-heavy"])
def test_append_and_attend_equals_the_two_calls(mpa, make):
    """The one-call form (append sharing a launch with the work-list upload) against kv_append
    followed by mixed_paged_attention: caches and outputs bit for bit, first with a fresh work
    list, then with the list left in the workspace (plan cache level 2), and against the oracle."""
    import torch
    b = make()
    dt = mpa.MPA_FP16 if b.dtype == "fp16" else mpa.MPA_BF16
    ref = oracle_run(b)[0]
    outs = []
    for fused in (False, True):
        ctx = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK, dtype=dt)
        ctx.set_option(mpa.MPA_OPT_PLAN_CACHE, 2)
        ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        for call in range(2):
            db = DeviceBatch(b, "prior")
            if fused:
                ctx.append_and_attend(db.k_new, db.v_new, db.slot_map, db.q, db.k_cache, db.v_cache, db.block_table,
                                      b.chunk_starts, b.context_lens, db.out, ws, scale=b.scale)
            else:
                run_on(ctx, db, b, ws)
            torch.cuda.synchronize()
            outs.append((to_host_u16(db.out), to_host_u16(db.k_cache), to_host_u16(db.v_cache)))
    for o in outs[1:]:
        for got, want in zip(o, outs[0]):
            assert np.array_equal(got, want)
    assert_close(outs[0][0], ref, b.name, dtype=b.dtype)
    kc, vc = oracle_run(b)[1:]
    assert np.array_equal(outs[2][1], kc) and np.array_equal(outs[2][2], vc)


INSIDE_CASES = {
    # chunks that start inside a page / on a page / at position 0, chunks shorter than a page, generation
    # rows whose own token is first / last / in the middle of its page
    "cfg1": lambda: W.config1(),
    "cfg1-fp16": lambda: W.config1(dtype="fp16"),
    "ragged-pages": lambda: W.make_batch("inside-ragged", 71, 4, 128, 16, 700,
                                         [600, 300, 5, 130, 64, 1, 1, 1, 1, 1], [1500, 300, 21, 130 + 47, 64 + 1024, 1, 16, 17, 700, 2000]),
    "ragged-gqa-bs32": lambda: W.random_ragged(7100, H=8, D=128, bs=32, n_pp=3, n_tg=5, max_q=300, max_prior=900, max_ctx=1500, Hkv=2),
    "group-items-bs128": lambda: W.make_batch("inside-groups", 72, 16, 128, 128, 40, [1, 1, 1, 200], [1, 129, 1000, 333], Hkv=2),
    "d64": lambda: W.make_batch("inside-d64", 73, 4, 64, 16, 300, [257, 1, 1, 33], [257 + 30, 100, 1, 33 + 640]),
}


@pytest.mark.parametrize("case", sorted(INSIDE_CASES))
@pytest.mark.parametrize("opts", [{}, {"MPA_OPT_TILE_MODE": 2}, {"MPA_OPT_PP_SPLIT_TOKENS": 128, "MPA_OPT_TG_SPLIT_BLOCKS": 2}],
                         ids=["auto", "wide", "split"])
def test_append_inside_the_attention_launch(mpa, case, opts):
    """MPA_OPT_FUSE_APPEND: the iteration's K/V stored by work-groups of the attention launch itself while
    every row reads its own sequence's new keys from k_new / v_new.  The cache slots of the new tokens hold
    NaN patterns when the launch starts, so a row that read them instead would show.  Outputs and caches
    bit for bit equal to kv_append followed by mixed_paged_attention, with a fresh work list and with the
    list left in the workspace (then the call is the attention launch and the merge alone)."""
    import torch
    b = INSIDE_CASES[case]()
    dt = mpa.MPA_FP16 if b.dtype == "fp16" else mpa.MPA_BF16
    outs = []
    for inside in (False, True):
        ctx = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK, dtype=dt)
        ctx.set_option(mpa.MPA_OPT_PLAN_CACHE, 2)
        ctx.set_option(mpa.MPA_OPT_FUSE_APPEND, 1 if inside else 0)
        for k, v in opts.items():
            ctx.set_option(getattr(mpa, k), v)
        ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        for call in range(2):
            db = DeviceBatch(b, "prior")
            if inside:
                ctx.append_and_attend(db.k_new, db.v_new, db.slot_map, db.q, db.k_cache, db.v_cache, db.block_table,
                                      b.chunk_starts, b.context_lens, db.out, ws, scale=b.scale)
            else:
                run_on(ctx, db, b, ws)
            torch.cuda.synchronize()
            outs.append((to_host_u16(db.out), to_host_u16(db.k_cache), to_host_u16(db.v_cache)))
    for o in outs[1:]:
        for got, want in zip(o, outs[0]):
            assert np.array_equal(got, want)
    ref, kc, vc = oracle_run(b)
    assert_close(outs[0][0], ref, b.name, dtype=b.dtype)
    assert np.array_equal(outs[3][1], kc) and np.array_equal(outs[3][2], vc)


def test_append_inside_the_launch_falls_back_for_streamed_prompt_rows(mpa):
    """With prompt rows on the row-streaming body (a test option) a row would need several new keys: the
    call then appends before the attention launch as usual, with the same results."""
    import torch
    b = W.config1()
    ref = oracle_run(b)[0]
    ctx = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK)
    ctx.set_option(mpa.MPA_OPT_FUSE_APPEND, 1)
    ctx.set_option(mpa.MPA_OPT_PP_ROWSTREAM, 1)
    ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
    db = DeviceBatch(b, "prior")
    ctx.append_and_attend(db.k_new, db.v_new, db.slot_map, db.q, db.k_cache, db.v_cache, db.block_table,
                          b.chunk_starts, b.context_lens, db.out, ws, scale=b.scale)
    torch.cuda.synchronize()
    assert_close(to_host_u16(db.out), ref, b.name)


def test_two_threads_two_contexts_two_streams(mpa):
    """Two host threads, each with its own context, workspace and stream, issue forty calls at the same time
    (the binding releases the interpreter lock inside a call): every output equals the single-threaded one."""
    import threading
    import torch
    batches = [W.config1(), W.make_batch("thread-b", 91, 8, 128, 16, 300, [130, 1, 1, 1], [700, 900, 33, 1500])]
    want, jobs = [], []
    for b in batches:
        ctx = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK)
        db = DeviceBatch(b, "prior")
        ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
        run_on(ctx, db, b, ws)
        torch.cuda.synchronize()
        want.append(to_host_u16(db.out))
        jobs.append((ctx, db, b, ws, torch.cuda.Stream()))
    errors_seen = []

    def worker(k):
        ctx, db, b, ws, stream = jobs[k]
        try:
            for _ in range(40):
                db.out.fill_(0x7FFF)          # on torch's default stream: ordered before the side stream below by the wait
                stream.wait_stream(torch.cuda.current_stream())
                run_on(ctx, db, b, ws, stream=stream)
                stream.synchronize()
                if not np.array_equal(to_host_u16(db.out), want[k]):
                    errors_seen.append(f"thread {k}: output differs")
                    return
        except Exception as e:   # noqa: BLE001
            errors_seen.append(f"thread {k}: {e!r}")

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors_seen, errors_seen
