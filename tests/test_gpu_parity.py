"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

import workloads as W
from harness import DeviceBatch, assert_close, errors, gpu_run, oracle_run, to_dev, to_host_u16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mpa():
    import paper_2503_13737_amd as m
    m.load()
    return m


def ctx_for(mpa, b, **opts):
    c = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK, dtype=mpa.MPA_FP16 if b.dtype == "fp16" else mpa.MPA_BF16)
    for k, v in opts.items():
        c.set_option(getattr(mpa, k), v)
    return c


def test_config1_append_bit_exact_and_attention(mpa):
    b = W.config1()
    out, kc, vc = gpu_run(ctx_for(mpa, b), b)
    ref, okc, ovc = oracle_run(b)
    assert np.array_equal(kc, okc) and np.array_equal(vc, ovc)
    ma, rl = assert_close(out, ref, b.name)
    print(f"cfg1 max-abs {ma:.2e} rel-L2 {rl:.2e}")
    # per sequence worst case
    for i in range(b.S):
        r0, r1 = b.chunk_starts[i], b.chunk_starts[i + 1]
        assert_close(out[r0:r1], ref[r0:r1], f"{b.name} seq {i}")


def test_kv_append_skips_negative_slots_and_leaves_rest(mpa):
    import oracle
    import torch
    b = W.config1()
    db = DeviceBatch(b, "prior")
    sm = b.slot_map.copy()
    sm[1::2] = -1
    ctx_for(mpa, b).kv_append(db.k_new, db.v_new, to_dev(sm), db.k_cache, db.v_cache)
    torch.cuda.synchronize()
    kc, vc = b.full_cache("prior")
    kn, vn = b.new_kv()
    oracle.kv_append(kn, vn, sm, kc, vc)
    assert np.array_equal(to_host_u16(db.k_cache), kc) and np.array_equal(to_host_u16(db.v_cache), vc)


@pytest.mark.parametrize("tg_split", [1, 2, 3, 7, 1000])
def test_forced_row_splits_agree(mpa, tg_split):
    b = W.config1()
    ref, _, _ = oracle_run(b)
    out, _, _ = gpu_run(ctx_for(mpa, b, MPA_OPT_TG_SPLIT_BLOCKS=tg_split), b)
    assert_close(out, ref, f"tg_split={tg_split}")


@pytest.mark.parametrize("pp_split", [64, 128, 192, 100000])
def test_forced_tile_splits_agree(mpa, pp_split):
    b = W.config1()
    ref, _, _ = oracle_run(b)
    out, _, _ = gpu_run(ctx_for(mpa, b, MPA_OPT_PP_SPLIT_TOKENS=pp_split), b)
    assert_close(out, ref, f"pp_split={pp_split}")


@pytest.mark.parametrize("resident", [1, 3, 7])
@pytest.mark.parametrize("team_min_steps", [0, 1])
def test_few_resident_tile_work_groups_and_pacing(mpa, resident, team_min_steps):
    """A handful of work-groups walk all prompt-tile units one after the other (the launch mode of
    prompt-heavy mixed batches), with and without the q-tiles of a range keeping pace with each
    other: same results as one work-group per unit."""
    ql, ctx = [600, 300, 1, 1, 1], [1500, 300, 700, 64, 2000]
    b = W.make_batch("resident", 123, 4, 128, 16, sum((c + 15) // 16 for c in ctx) + 3, ql, ctx)
    ref, _, _ = oracle_run(b)
    for split in (0, 256):
        out, _, _ = gpu_run(ctx_for(mpa, b, MPA_OPT_PP_RESIDENT_WGS=resident, MPA_OPT_PP_TEAM_MIN_STEPS=team_min_steps,
                                    MPA_OPT_PP_SPLIT_TOKENS=split), b)
        assert_close(out, ref, f"{b.name} resident={resident} pacing={team_min_steps} split={split}")


def test_rowstream_body_on_prompt_rows(mpa):
    b = W.config1()
    ref, _, _ = oracle_run(b)
    out, _, _ = gpu_run(ctx_for(mpa, b, MPA_OPT_PP_ROWSTREAM=1), b)
    assert_close(out, ref, "rowstream")


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("D,H", [(64, 2), (128, 3), (128, 5)])
def test_random_ragged_batches(mpa, seed, D, H):
    b = W.random_ragged(1000 + seed, H=H, D=D, n_pp=2 + seed % 2, n_tg=3, max_q=200, max_prior=300, max_ctx=400)
    ref, okc, ovc = oracle_run(b)
    out, kc, vc = gpu_run(ctx_for(mpa, b), b)
    assert np.array_equal(kc, okc) and np.array_equal(vc, ovc)
    assert_close(out, ref, b.name)


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("D,H,HK", [(64, 8, 2), (128, 8, 1), (128, 12, 4), (128, 16, 2)])
def test_grouped_kv_heads(mpa, seed, D, H, HK):
    """Query heads sharing K/V heads (h reads K/V head h / (H/HK)): append and attention."""
    b = W.random_ragged(3000 + seed, H=H, D=D, n_pp=2, n_tg=4, max_q=260, max_prior=400, max_ctx=700, Hkv=HK)
    ref, okc, ovc = oracle_run(b)
    for opts in ({}, {"MPA_OPT_PP_SPLIT_TOKENS": 128, "MPA_OPT_TG_SPLIT_BLOCKS": 3}):
        out, kc, vc = gpu_run(ctx_for(mpa, b, **opts), b)
        assert kc.shape[1] == HK
        assert np.array_equal(kc, okc) and np.array_equal(vc, ovc)
        assert_close(out, ref, f"{b.name} H={H} HK={HK} {opts}")


@pytest.mark.parametrize("H,HK,D", [(8, 2, 128), (32, 1, 64), (40, 8, 128), (16, 4, 64), (128, 1, 64), (192, 1, 64)])
def test_generation_rows_of_grouped_heads_on_the_matrix_core_body(mpa, H, HK, D):
    """Group sizes 4, 5, 32, 128 (a full tile) and 192 (more than a tile: back on the streaming body): a generation row runs as one tile per K/V head whose rows are the
    group's query heads.  Contexts of one key, block and step boundaries, long ones with forced
    short ranges (several partials per row), next to a prompt chunk."""
    ql = [1, 1, 1, 1, 1, 1, 1, 150]
    ctx = [1, 16, 64, 65, 129, 1000, 2500, 400]
    b = W.make_batch(f"gqa-rows-{H}-{HK}", 321, H, D, 16, sum((c + 15) // 16 for c in ctx) + 3, ql, ctx, Hkv=HK)
    ref, _, _ = oracle_run(b)
    for opts in ({}, {"MPA_OPT_TG_SPLIT_BLOCKS": 4}, {"MPA_OPT_TG_SPLIT_BLOCKS": 9, "MPA_OPT_PP_RESIDENT_WGS": 5}):
        out, _, _ = gpu_run(ctx_for(mpa, b, **opts), b)
        assert_close(out, ref, f"{b.name} {opts}")
        for i in range(b.S):
            r0, r1 = b.chunk_starts[i], b.chunk_starts[i + 1]
            assert_close(out[r0:r1], ref[r0:r1], f"{b.name} {opts} seq {i}")


@pytest.mark.parametrize("bs", [32, 64, 128])
@pytest.mark.parametrize("D,H,HK", [(128, 4, 4), (64, 8, 2)])
def test_block_sizes(mpa, bs, D, H, HK):
    """KV blocks of 32, 64 and 128 tokens (2, 4, 8 pages of 16): append bit-exact, attention over
    prompt chunks that start inside a block, generation rows ending on every kind of boundary,
    forced short ranges; with grouped heads the generation rows take the matrix-core body."""
    ql = [300, 77, 1, 1, 1, 1, 1, 1]
    ctx = [700, 77 + 3 * bs + 5, 1, bs, bs + 1, 5 * bs - 1, 2000, 16]
    b = W.make_batch(f"bs{bs}", 555 + bs, H, D, bs, sum((c + bs - 1) // bs for c in ctx) + 3, ql, ctx, Hkv=HK)
    ref, okc, ovc = oracle_run(b)
    for opts in ({}, {"MPA_OPT_PP_SPLIT_TOKENS": 128, "MPA_OPT_TG_SPLIT_BLOCKS": 1}, {"MPA_OPT_TG_SPLIT_BLOCKS": 3}):
        out, kc, vc = gpu_run(ctx_for(mpa, b, **opts), b)
        assert np.array_equal(kc, okc) and np.array_equal(vc, ovc)
        assert_close(out, ref, f"{b.name} {opts}")
        for i in range(b.S):
            r0, r1 = b.chunk_starts[i], b.chunk_starts[i + 1]
            assert_close(out[r0:r1], ref[r0:r1], f"{b.name} {opts} seq {i}")


@pytest.mark.parametrize("ql,ctx", [
    ([1], [1]),                      # single key
    ([1], [16]), ([1], [17]),        # block boundary
    ([2], [2]), ([16], [16]), ([17], [33]),
    ([128], [128]), ([129], [129]), ([127], [200]),   # tile boundary
    ([64], [64 + 48]), ([37], [37]),
    ([300], [300]), ([130, 1, 1], [700, 65, 1]),
])
def test_edge_shapes(mpa, ql, ctx):
    b = W.make_batch(f"edge-{ql}-{ctx}", 77, 4, 128, 16, sum((c + 15) // 16 for c in ctx) + 2, ql, ctx)
    ref, okc, ovc = oracle_run(b)
    for opts in ({}, {"MPA_OPT_PP_SPLIT_TOKENS": 64, "MPA_OPT_TG_SPLIT_BLOCKS": 1}):
        out, kc, vc = gpu_run(ctx_for(mpa, b, **opts), b)
        assert np.array_equal(kc, okc) and np.array_equal(vc, ovc)
        assert_close(out, ref, f"{b.name} {opts}")


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("scale", [1.0, 4.0, 16.0])
def test_steep_softmax(mpa, scale, D):
    """Scores spread over hundreds of powers of two (the scale is far above 1/sqrt(D)): a row's
    largest score keeps growing as more keys are seen, so the tile body's softmax reference has
    to be reset several times per row, also from weights that overflowed, and stale contributions
    have to vanish.  Prompt tiles (split and unsplit) and generation rows.  A peaked softmax
    returns single V rows, values up to about 4.5 where one bf16 step is 0.03: the absolute
    bound scales with the largest expected output, the relative one stays as it is."""
    ql, ctx = [700, 300, 1, 1, 130], [900, 300, 500, 64, 2000]
    b = W.make_batch(f"steep-{scale}-{D}", 91, 4, D, 16, sum((c + 15) // 16 for c in ctx) + 3, ql, ctx)
    ref, _, _ = oracle_run(b, scale=scale)
    for opts in ({}, {"MPA_OPT_PP_SPLIT_TOKENS": 256, "MPA_OPT_TG_SPLIT_BLOCKS": 4}):
        out, _, _ = gpu_run(ctx_for(mpa, b, **opts), b, scale=scale)
        assert_close(out, ref, f"{b.name} {opts}", abs_scale=max(1.0, float(np.abs(ref).max())))


def test_empty_batch_is_a_noop(mpa):
    c = mpa.Context(4, 64)
    lib = mpa.load()
    assert lib.mpa_mixed_paged_attention(c._h, None, None, None, None, 0, None, None, 0, 0, 0.0, None, None, 0, None) == 0
    assert lib.mpa_kv_append(c._h, None, None, None, 0, None, None, None) == 0


def test_I3_block_permutation_is_bit_identical(mpa):
    import torch
    b = W.config1()
    c = ctx_for(mpa, b)
    base, _, _ = gpu_run(c, b, append=False)
    kc, vc = b.full_cache("ctx")
    perm = W.permutation(b.NB, 4242)
    kc2, vc2 = np.empty_like(kc), np.empty_like(vc)
    kc2[perm], vc2[perm] = kc, vc
    tab2 = np.where(b.block_table >= 0, perm[np.maximum(b.block_table, 0)], -1).astype(np.int32)
    db = DeviceBatch(b, "ctx")
    db.k_cache, db.v_cache, db.block_table = to_dev(kc2), to_dev(vc2), to_dev(tab2)
    ws = torch.empty(c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
    c.mixed_paged_attention(db.q, db.k_cache, db.v_cache, db.block_table, b.chunk_starts, b.context_lens, db.out, ws, scale=b.scale)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(db.out), base)


def test_I1_I2_chunked_and_generation_rows_match_one_shot(mpa):
    L, H, D = 150, 4, 128
    one = W.make_batch("one", 31, H, D, 16, 12, [L], [L])
    ids = one.block_table[0, : (L + 15) // 16]
    ref, _, _ = oracle_run(one)
    full, _, _ = gpu_run(ctx_for(mpa, one), one)
    assert_close(full, ref, "one-shot")
    p = 0
    for n in (37, 64, 1, 47, 1):
        part = W.make_batch("part", 31, H, D, 16, 12, [n], [p + n], block_ids=ids)
        part.q = one.q[p:p + n].copy()
        got, _, _ = gpu_run(ctx_for(mpa, part), part, append=False)
        assert_close(got, ref[p:p + n], f"chunk at {p}+{n}")
        # against the one-shot GPU result: same math up to re-association
        d = np.abs(W.bf16_to_f64(got) - W.bf16_to_f64(full[p:p + n])).max()
        assert d <= 2e-2
        p += n
    assert p == L


def test_I4_batch_order_independence(mpa):
    b = W.config1()
    base, _, _ = gpu_run(ctx_for(mpa, b), b, append=False)
    sub = b.compact([6, 1, 3])
    import torch
    kc, vc = sub.compact_cache(b)
    c = ctx_for(mpa, sub)
    out = torch.zeros((sub.T, sub.H, sub.D), dtype=torch.int16, device="cuda")
    ws = torch.empty(c.workspace_bytes_for_batch(sub.chunk_starts, sub.context_lens), dtype=torch.uint8, device="cuda")
    c.mixed_paged_attention(to_dev(sub.q), to_dev(kc), to_dev(vc), to_dev(sub.block_table), sub.chunk_starts,
                            sub.context_lens, out, ws, scale=sub.scale)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(out), base[sub.rows_src])


# ------------------------------------------------------------------------------------------------
# fp16 storage (the precision of the paper's experiments): same cases, IEEE-half patterns in
# q / K / V / out, against the oracle decoding the same patterns.  The bars are four times
# tighter than the bf16 ones (see harness.TOL).
# ------------------------------------------------------------------------------------------------
def fp16_check(mpa, b, opts_list=({},), scale=None, abs_scale=None, append=True):
    assert b.dtype == "fp16"
    ref, okc, ovc = oracle_run(b, scale=scale)
    for opts in opts_list:
        out, kc, vc = gpu_run(ctx_for(mpa, b, **opts), b, scale=scale)
        assert np.array_equal(kc, okc) and np.array_equal(vc, ovc)
        k = 1.0 if abs_scale is None else abs_scale(ref)
        assert_close(out, ref, f"{b.name} {opts}", abs_scale=k, dtype="fp16")
        for i in range(b.S):
            r0, r1 = b.chunk_starts[i], b.chunk_starts[i + 1]
            assert_close(out[r0:r1], ref[r0:r1], f"{b.name} {opts} seq {i}", abs_scale=k, dtype="fp16")
    return ref


def test_fp16_config1_all_bodies_and_splits(mpa):
    b = W.config1(dtype="fp16")
    fp16_check(mpa, b, [{}, {"MPA_OPT_TG_SPLIT_BLOCKS": 1}, {"MPA_OPT_TG_SPLIT_BLOCKS": 3},
                        {"MPA_OPT_PP_SPLIT_TOKENS": 64}, {"MPA_OPT_PP_SPLIT_TOKENS": 128, "MPA_OPT_TG_SPLIT_BLOCKS": 2},
                        {"MPA_OPT_PP_ROWSTREAM": 1}, {"MPA_OPT_PP_RESIDENT_WGS": 2, "MPA_OPT_PP_TEAM_MIN_STEPS": 1}])


def test_fp16_and_bf16_contexts_read_the_same_bits_differently(mpa):
    """The same bit patterns through a bf16 context give other numbers: the dtype reaches the kernels."""
    b = W.config1(dtype="fp16")
    ref, _, _ = oracle_run(b)
    as_bf16 = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK)
    out, _, _ = gpu_run(as_bf16, b)
    ma, _ = errors(out, ref, "fp16")
    assert not (ma <= 0.1)


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("D,H,HK", [(64, 2, 2), (128, 3, 3), (128, 5, 5), (64, 8, 2), (128, 12, 4), (128, 16, 2)])
def test_fp16_random_ragged_batches(mpa, seed, D, H, HK):
    b = W.random_ragged(5000 + seed, H=H, D=D, n_pp=2 + seed % 2, n_tg=4, max_q=260, max_prior=400, max_ctx=700,
                        Hkv=HK, dtype="fp16")
    fp16_check(mpa, b, [{}, {"MPA_OPT_PP_SPLIT_TOKENS": 128, "MPA_OPT_TG_SPLIT_BLOCKS": 3}])


@pytest.mark.parametrize("bs", [16, 32, 128])
@pytest.mark.parametrize("D,H,HK", [(128, 4, 4), (64, 8, 2)])
def test_fp16_block_sizes_and_boundaries(mpa, bs, D, H, HK):
    ql = [300, 77, 129, 1, 1, 1, 1, 1, 1]
    ctx = [700, 77 + 3 * bs + 5, 129, 1, bs, bs + 1, 5 * bs - 1, 2000, 16]
    b = W.make_batch(f"fp16-bs{bs}", 655 + bs, H, D, bs, sum((c + bs - 1) // bs for c in ctx) + 3, ql, ctx, Hkv=HK,
                     dtype="fp16")
    fp16_check(mpa, b, [{}, {"MPA_OPT_PP_SPLIT_TOKENS": 128, "MPA_OPT_TG_SPLIT_BLOCKS": 1}, {"MPA_OPT_TG_SPLIT_BLOCKS": 3}])


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("scale", [1.0, 4.0, 16.0])
def test_fp16_steep_softmax(mpa, scale, D):
    """As test_steep_softmax.  With fp16 weights the range above the reference is 2^16, not 2^128:
    weights that saturate the format must send the row through the re-referencing path, and the
    reference shift must reach the partial results' merge unchanged."""
    ql, ctx = [700, 300, 1, 1, 130], [900, 300, 500, 64, 2000]
    b = W.make_batch(f"fp16-steep-{scale}-{D}", 91, 4, D, 16, sum((c + 15) // 16 for c in ctx) + 3, ql, ctx, dtype="fp16")
    fp16_check(mpa, b, [{}, {"MPA_OPT_PP_SPLIT_TOKENS": 256, "MPA_OPT_TG_SPLIT_BLOCKS": 4}], scale=scale,
               abs_scale=lambda ref: max(1.0, float(np.abs(ref).max())))


def test_fp16_flat_softmax_over_a_long_context(mpa):
    """A tiny scale makes all weights nearly equal: thousands of weights near the reference, row
    sums far above the fp16 range (they are kept in fp32)."""
    ql, ctx = [200, 1, 1], [6000, 9000, 3000]
    b = W.make_batch("fp16-flat", 17, 4, 128, 16, sum((c + 15) // 16 for c in ctx) + 3, ql, ctx, dtype="fp16")
    fp16_check(mpa, b, [{}, {"MPA_OPT_PP_SPLIT_TOKENS": 1024}], scale=1e-3)


def test_random_combinations_of_geometry_dtype_and_options(mpa):
    """Thirty seeded draws over head layout, head_dim, block size, storage type, batch mix and
    planner options at once (the dedicated tests vary these one or two at a time), each through the
    one-call form -- with the append before or inside the attention launch -- and checked against the
    oracle, caches included."""
    import torch
    draws = W.bits(30 * 12, 4711).reshape(30, 12)
    for n, u in enumerate(draws):
        u = [int(x) for x in u]
        D = (64, 128)[u[0] % 2]
        HK = (1, 2, 3, 4)[u[1] % 4]
        group = (1, 1, 2, 4, 8)[u[2] % 5]
        H = HK * group
        bs = (16, 32, 64, 128)[u[3] % 4]
        dtype = ("bf16", "fp16")[u[4] % 2]
        n_pp, n_tg = u[5] % 3, 1 + u[6] % 5
        b = W.random_ragged(8000 + n, H=H, D=D, bs=bs, n_pp=n_pp, n_tg=n_tg, max_q=40 + u[7] % 400,
                            max_prior=u[8] % 1500, max_ctx=1 + u[9] % 2500, Hkv=HK, dtype=dtype)
        opts = {}
        if u[10] % 3 == 1:
            opts = {"MPA_OPT_TG_SPLIT_BLOCKS": 1 + u[11] % 7, "MPA_OPT_PP_SPLIT_TOKENS": 64 * (1 + u[11] % 5)}
        elif u[10] % 3 == 2:
            opts = {"MPA_OPT_PP_RESIDENT_WGS": 1 + u[11] % 9, "MPA_OPT_PP_TEAM_MIN_STEPS": 1 + u[11] % 3}
        inside = (u[11] // 16) % 2     # every other draw or so: the append inside the attention launch
        what = f"draw {n}: H={H} HK={HK} D={D} bs={bs} {dtype} pp={n_pp} tg={n_tg} T={b.T} {opts} append inside {inside}"
        print(what, flush=True)
        ctx = ctx_for(mpa, b, **opts)
        ctx.set_option(mpa.MPA_OPT_FUSE_APPEND, inside)
        db = DeviceBatch(b, "prior")
        ws = torch.empty(ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        ctx.append_and_attend(db.k_new, db.v_new, db.slot_map, db.q, db.k_cache, db.v_cache, db.block_table,
                              b.chunk_starts, b.context_lens, db.out, ws, scale=b.scale)
        torch.cuda.synchronize()
        ref, okc, ovc = oracle_run(b)
        assert np.array_equal(to_host_u16(db.k_cache), okc) and np.array_equal(to_host_u16(db.v_cache), ovc), what
        assert_close(to_host_u16(db.out), ref, what, dtype=dtype)


# ---- the wide work-group shape (MPA_OPT_TILE_MODE 2): eight wavefronts, 256-row tiles, ring of K/V tiles

WIDE = {"MPA_OPT_TILE_MODE": 2}


@pytest.mark.parametrize("opts", [{}, {"MPA_OPT_PP_SPLIT_TOKENS": 64}, {"MPA_OPT_PP_SPLIT_TOKENS": 192, "MPA_OPT_TG_SPLIT_BLOCKS": 2},
                                  {"MPA_OPT_PP_RESIDENT_WGS": 1}])
def test_wide_shape_config1(mpa, opts):
    b = W.config1()
    ref, _, _ = oracle_run(b)
    out, _, _ = gpu_run(ctx_for(mpa, b, **WIDE, **opts), b)
    assert_close(out, ref, f"wide {opts}")


@pytest.mark.parametrize("resident", [1, 3, 0])
@pytest.mark.parametrize("split", [0, 64, 320, 1024])
def test_wide_shape_chunks_of_several_tiles_and_every_ring_phase(mpa, resident, split):
    """Chunks of 600, 300 and 257 rows (256-row tiles and their remainders: one full wavefront, a
    wavefront of one row), contexts that make ranges of 1 to 40 steps (shorter than the ring's look-ahead,
    ending on every phase of the barrier interval, partial last tiles), next to generation rows;
    few work-groups walking all units, and one per unit."""
    ql, ctx = [600, 300, 257, 1, 1, 1, 40], [1500, 300, 2560, 700, 64, 2000, 103]
    b = W.make_batch("wide-multi", 123, 4, 128, 16, sum((c + 15) // 16 for c in ctx) + 3, ql, ctx)
    ref, _, _ = oracle_run(b)
    out, _, _ = gpu_run(ctx_for(mpa, b, **WIDE, MPA_OPT_PP_RESIDENT_WGS=resident, MPA_OPT_PP_SPLIT_TOKENS=split), b)
    assert_close(out, ref, f"wide resident={resident} split={split}")
    for i in range(b.S):
        r0, r1 = b.chunk_starts[i], b.chunk_starts[i + 1]
        assert_close(out[r0:r1], ref[r0:r1], f"wide resident={resident} split={split} seq {i}")


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("D,H,HK,dtype,bs", [(64, 2, 2, "bf16", 16), (128, 5, 5, "bf16", 32), (128, 12, 4, "bf16", 16),
                                             (64, 8, 2, "fp16", 16), (128, 16, 2, "fp16", 128), (128, 9, 9, "fp16", 16)])
def test_wide_shape_random_ragged_batches(mpa, seed, D, H, HK, dtype, bs):
    """Both element types, both head dimensions, grouped K/V heads (group items on the wide tile
    body), larger blocks; automatic ranges and forced short ones."""
    b = W.random_ragged(5000 + seed, H=H, D=D, n_pp=2 + seed % 2, n_tg=3, max_q=520, max_prior=700, max_ctx=1200, Hkv=HK,
                        dtype=dtype, bs=bs)
    ref, okc, ovc = oracle_run(b)
    for opts in ({}, {"MPA_OPT_PP_SPLIT_TOKENS": 128, "MPA_OPT_TG_SPLIT_BLOCKS": 3}):
        out, kc, vc = gpu_run(ctx_for(mpa, b, **WIDE, **opts), b)
        assert np.array_equal(kc, okc) and np.array_equal(vc, ovc)
        assert_close(out, ref, f"wide {b.name} {opts}", dtype=dtype)


def test_wide_shape_equals_the_narrow_one_on_unsplit_rows(mpa):
    """A row's arithmetic does not depend on the work-group shape: same tile steps, same order of keys.
    With every range unsplit the two shapes give the same bits."""
    ql, ctx = [300, 129, 1, 1], [900, 129, 500, 31]
    b = W.make_batch("wide-vs-narrow", 77, 4, 128, 16, sum((c + 15) // 16 for c in ctx) + 3, ql, ctx)
    big = {"MPA_OPT_PP_SPLIT_TOKENS": 1 << 20, "MPA_OPT_TG_SPLIT_BLOCKS": 1 << 16}
    out_n, _, _ = gpu_run(ctx_for(mpa, b, MPA_OPT_TILE_MODE=1, **big), b)
    out_w, _, _ = gpu_run(ctx_for(mpa, b, **WIDE, **big), b)
    assert np.array_equal(out_n, out_w)


def test_wide_shape_steep_softmax(mpa):
    b = W.random_ragged(4242, H=3, D=128, n_pp=2, n_tg=2, max_q=300, max_prior=500, max_ctx=900)
    ref, _, _ = oracle_run(b, scale=4.0)
    out, _, _ = gpu_run(ctx_for(mpa, b, **WIDE), b, scale=4.0)
    assert_close(out, ref, "wide steep", abs_scale=max(1.0, float(np.abs(ref).max())))
