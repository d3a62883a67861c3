"""Host-only property tests of the planner through the C ABI (no GPU): for random ragged batches
every (row, key) pair is covered exactly once, ranges are whole blocks / 64-key steps, partial
rows are consistent, and the documented workspace upper bound holds."""
import numpy as np
import pytest

import paper_2503_13737_amd as mpa
import workloads as W
from test_abi_host import check_plan_covers


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_plan_invariants(seed):
    H = [1, 4, 12, 40][seed % 4]
    b = W.random_ragged(500 + seed, H=H, D=128, n_pp=1 + seed % 3, n_tg=seed % 5, max_q=700, max_prior=3000,
                        max_ctx=5000)
    c = mpa.Context(H, 128)
    if seed % 3 == 1:
        c.set_option(mpa.MPA_OPT_TG_SPLIT_BLOCKS, 1 + seed)
        c.set_option(mpa.MPA_OPT_PP_SPLIT_TOKENS, 64 * (1 + seed % 4))
    items, counts = c.plan_describe(b.chunk_starts, b.context_lens)
    n_tile, n_row, n_merge, n_part = (int(x) for x in counts)
    assert n_tile + n_row == len(items)
    assert (items[:n_tile, 7] == 1).all() and (items[n_tile:, 7] == 0).all()
    assert (items[:, 4] % 16 == 0).all() and (items[:n_tile, 4] % 64 == 0).all()
    assert (items[:, 5] > items[:, 4]).all()
    assert (items[n_tile:, 2] == 1).all() and (items[:n_tile, 2] <= 128).all() and (items[:, 2] >= 1).all()
    check_plan_covers(b, items, counts, H)
    # partial rows: disjoint ranges [part_row, part_row + q_rows) inside [0, n_part)
    parts = sorted((int(it[6]), int(it[6]) + int(it[2])) for it in items if it[6] >= 0)
    for (a0, a1), (b0, b1) in zip(parts, parts[1:]):
        assert a1 <= b0
    assert not parts or (parts[0][0] >= 0 and parts[-1][1] <= n_part)
    need = c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
    assert need >= 256
    assert c.workspace_bytes(b.S, b.T, int(b.context_lens.max())) >= need


def test_workspace_bound_is_monotone():
    c = mpa.Context(40, 128)
    a = c.workspace_bytes(64, 64, 2048)
    assert c.workspace_bytes(128, 128, 2048) >= a and c.workspace_bytes(64, 64, 4096) >= a
    assert c.workspace_bytes(0, 0, 0) >= 0
