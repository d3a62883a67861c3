"""Host-only property tests of the planner through the C ABI (no GPU): for random ragged batches
every (row, key) pair is covered exactly once, ranges are whole blocks / 64-key steps, partial
rows are consistent, and the documented workspace upper bound holds."""
import numpy as np
import pytest

import paper_2503_13737_amd as mpa
import workloads as W
from test_abi_host import check_plan_covers


@pytest.mark.parametrize("wide", [False, True], ids=["narrow", "wide"])
@pytest.mark.parametrize("seed", range(12))
def test_random_batches_plan_invariants(seed, wide):
    H = [1, 4, 12, 40][seed % 4]
    b = W.random_ragged(500 + seed, H=H, D=128, n_pp=1 + seed % 3, n_tg=seed % 5, max_q=700, max_prior=3000,
                        max_ctx=5000)
    c = mpa.Context(H, 128)
    c.set_option(mpa.MPA_OPT_TILE_MODE, 2 if wide else 1)
    tile_rows = 256 if wide else 128
    if seed % 3 == 1:
        c.set_option(mpa.MPA_OPT_TG_SPLIT_BLOCKS, 1 + seed)
        c.set_option(mpa.MPA_OPT_PP_SPLIT_TOKENS, 64 * (1 + seed % 4))
    items, counts = c.plan_describe(b.chunk_starts, b.context_lens)
    n_tile, n_row, n_merge, n_part = (int(x) for x in counts)
    assert n_tile + n_row == len(items)
    assert ((items[:n_tile, 7] & 0xFF) == 1).all() and (items[n_tile:, 7] == 0).all()
    # bit 8 of a tile's kind: no other tile starts at the same key of the same sequence
    tiles = items[:n_tile]
    for it in tiles:
        alone = ((tiles[:, 0] == it[0]) & (tiles[:, 4] == it[4])).sum() == 1
        assert ((it[7] >> 8) & 1) == int(alone)
        # above it: the tile's first row counted from its chunk's first row (q_pos0 minus it = the first
        # position of the sequence whose K/V arrives with this iteration)
        seq = int(it[0])
        assert (it[7] >> 9) == int(it[1]) - int(b.chunk_starts[seq])
        assert int(it[3]) - (it[7] >> 9) == int(b.context_lens[seq]) - int(b.q_lens[seq])
    assert (items[:, 4] % 16 == 0).all() and (items[:n_tile, 4] % 64 == 0).all()
    assert (items[:, 5] > items[:, 4]).all()
    assert (items[n_tile:, 2] == 1).all() and (items[:n_tile, 2] <= tile_rows).all() and (items[:, 2] >= 1).all()
    if wide and n_tile:   # the chunks longer than a narrow tile really are cut into 256-row tiles
        assert items[:n_tile, 2].max() == min(int(b.q_lens.max()), 256)
    check_plan_covers(b, items, counts, H)
    # partial rows: disjoint ranges [part_row, part_row + q_rows) inside [0, n_part)
    parts = sorted((int(it[6]), int(it[6]) + int(it[2])) for it in items if it[6] >= 0)
    for (a0, a1), (b0, b1) in zip(parts, parts[1:]):
        assert a1 <= b0
    assert not parts or (parts[0][0] >= 0 and parts[-1][1] <= n_part)
    need = c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
    assert need >= 256
    assert c.workspace_bytes(b.S, b.T, int(b.context_lens.max())) >= need


def test_tiles_of_a_chunk_cut_their_keys_at_common_positions():
    """All q-tiles of a chunk use the same range boundaries (multiples of one length), so the tiles
    over one range start at the same key and can share its K/V; a tile has fewer ranges when its
    rows end earlier."""
    c = mpa.Context(8, 128)
    for split in (0, 256, 1024):
        c.set_option(mpa.MPA_OPT_PP_SPLIT_TOKENS, split)
        cs, cl = np.array([0, 1000, 1300], dtype=np.int32), np.array([9000, 5000], dtype=np.int32)
        items, counts = c.plan_describe(cs, cl)
        tiles = items[: counts[0]]
        for seq in (0, 1):
            t = tiles[tiles[:, 0] == seq]
            begins = np.unique(t[:, 4])
            if len(begins) > 1:
                step = begins[1] - begins[0]
                assert step % 64 == 0 and (begins % step == 0).all()
                full = t[t[:, 5] - t[:, 4] == step]
                assert len(full) > 0 and ((t[:, 5] - t[:, 4]) <= step).all()
            # every tile starts its first range at key 0 and its ranges are contiguous
            for row0 in np.unique(t[:, 1]):
                r = t[t[:, 1] == row0]
                r = r[np.argsort(r[:, 4])]
                assert r[0, 4] == 0 and (r[1:, 4] == r[:-1, 5]).all()


def test_resident_and_pacing_options_do_not_change_the_work_list():
    b = W.random_ragged(77, H=12, D=128, n_pp=2, n_tg=4, max_q=600, max_prior=4000, max_ctx=3000)
    c = mpa.Context(12, 128)
    base, counts0 = c.plan_describe(b.chunk_starts, b.context_lens)
    for opt, val in ((mpa.MPA_OPT_PP_RESIDENT_WGS, 5), (mpa.MPA_OPT_PP_TEAM_MIN_STEPS, 1)):
        c.set_option(opt, val)
        items, counts = c.plan_describe(b.chunk_starts, b.context_lens)
        assert np.array_equal(items, base) and np.array_equal(counts, counts0)
        need = c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
        assert c.workspace_bytes(b.S, b.T, int(b.context_lens.max())) >= need
    with pytest.raises(mpa.MpaError):
        c.set_option(mpa.MPA_OPT_PP_RESIDENT_WGS, -1)


@pytest.mark.parametrize("H,HK", [(8, 2), (16, 2), (8, 1), (12, 4), (8, 4), (128, 1), (256, 1), (384, 2)])
def test_grouped_heads_plan(H, HK):
    """From group size 4 on generation rows become matrix-core items, one per K/V head and key
    range (kind 2); below it, and for groups larger than one tile's 128 rows, they stay row items.  Coverage, partial rows and bounds as usual."""
    b = W.random_ragged(900 + H + HK, H=H, D=128, n_pp=1, n_tg=5, max_q=300, max_prior=1500, max_ctx=4000, Hkv=HK)
    c = mpa.Context(H, 128, num_kv_heads=HK)
    for split in (0, 3):
        c.set_option(mpa.MPA_OPT_TG_SPLIT_BLOCKS, split)
        items, counts = c.plan_describe(b.chunk_starts, b.context_lens)
        kinds = items[:, 7] & 0xFF
        assert counts[0] + counts[1] == len(items)
        if H != HK:   # shared K/V heads: no tile is marked as the only reader of its keys
            assert (((items[kinds == 1][:, 7] >> 8) & 1) == 0).all()
        if 4 <= H // HK <= 128:
            assert counts[1] == 0 and (kinds == 2).sum() > 0 and (items[kinds == 2][:, 4] % 64 == 0).all()
            # group items sit between the prompt tiles and the (absent) row items
            first = int(np.argmax(kinds == 2))
            assert (kinds[:first] == 1).all() and (kinds[first:] == 2).all()
        else:
            assert (kinds != 2).all() and counts[1] > 0
        check_plan_covers(b, items, counts, H, HK)
        need = c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
        assert c.workspace_bytes(b.S, b.T, int(b.context_lens.max())) >= need


@pytest.mark.parametrize("bs", [32, 64, 128])
def test_block_sizes_plan(bs):
    """Row items cover whole KV blocks of the configured size; tiles and group items whole
    64-key steps; coverage and bounds as usual."""
    for H, HK in ((4, 4), (8, 2)):
        b = W.random_ragged(1200 + bs + H, H=H, D=128, bs=bs, n_pp=2, n_tg=5, max_q=300, max_prior=2000, max_ctx=5000,
                            Hkv=HK)
        c = mpa.Context(H, 128, block_size=bs, num_kv_heads=HK)
        for split in (0, 1, 3):
            c.set_option(mpa.MPA_OPT_TG_SPLIT_BLOCKS, split)
            items, counts = c.plan_describe(b.chunk_starts, b.context_lens)
            kinds = items[:, 7] & 0xFF
            assert (items[kinds == 0][:, 4] % bs == 0).all() and (items[kinds != 0][:, 4] % 64 == 0).all()
            if split and (kinds == 0).any():
                assert ((items[kinds == 0][:, 5] - items[kinds == 0][:, 4]) <= split * bs).all()
            check_plan_covers(b, items, counts, H, HK)
            need = c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
            assert c.workspace_bytes(b.S, b.T, int(b.context_lens.max())) >= need


def test_workspace_bound_is_monotone():
    c = mpa.Context(40, 128)
    a = c.workspace_bytes(64, 64, 2048)
    assert c.workspace_bytes(128, 128, 2048) >= a and c.workspace_bytes(64, 64, 4096) >= a
    assert c.workspace_bytes(0, 0, 0) >= 0


def test_range_lengths_of_generation_only_batches_fill_rounds_of_resident_work_groups():
    """Batches of generation rows alone, few rounds: the range length is the one near the target
    whose work-groups fill whole rounds of the 512 resident slots best -- for row items (a
    work-group covers 4 heads of an item) and for group items (one work-group each)."""
    z = W.uniform_ints(256, 2048, 8192, 77)
    cs = np.arange(257, dtype=np.int32)
    cl = z.astype(np.int32)
    for H, HK in ((8, 1), (8, 8)):
        c = mpa.Context(H, 128, num_kv_heads=HK)
        items, counts = c.plan_describe(cs, cl)
        kinds = items[:, 7] & 0xFF
        wgs = int((kinds == 2).sum()) if HK == 1 else int((kinds == 0).sum()) * (H // 4)
        assert wgs > 0
        fill = wgs / (-(-wgs // 512) * 512)
        assert fill >= 0.93, (H, HK, wgs, fill)
        # and the plan is a function of the batch alone
        items2, _ = c.plan_describe(cs, cl)
        assert np.array_equal(items, items2)
