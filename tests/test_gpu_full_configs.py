"""GPU parity at the full benchmark sizes (configs 2-5), in the launch configuration bench.py
times: kv_append + mixed_paged_attention on the whole batch, compared with the oracle on outputs it
can compute one by one -- every row and every head on configs 2 and 3; on configs 4 and 5 every
generation row and, of the prompt rows, the first, the last, every 61st and those straddling 16-
and 128-row boundaries, all heads each -- plus bit-exact kv_append on the blocks the new tokens
land in.  The whole output is NaN-poisoned first and checked for rows left unwritten.  Most configs then run
once more with the append inside the attention launch and must reproduce output and caches bit for bit."""
import os
import sys

import numpy as np
import pytest

import workloads as W
from harness import TOL, errors, to_host_u16

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

pytestmark = pytest.mark.gpu


def sample_rows(b, all_prompt_rows):
    rows, heads = [], []
    for i in range(b.S):
        r0, n = int(b.chunk_starts[i]), int(b.q_lens[i])
        if n == 1 or all_prompt_rows:
            js = range(n)
        else:
            js = {0, n - 1} | set(range(0, n, 61))
            for edge in list(range(16, n, 16))[:3] + list(range(128, n, 128)):
                js |= {edge - 1, edge}
            js = sorted(j for j in js if 0 <= j < n)
        for j in js:
            for h in range(b.H):
                rows.append(r0 + j)
                heads.append(h)
    return np.asarray(rows, dtype=np.int32), np.asarray(heads, dtype=np.int32)


def check_append_inside_the_launch(b, dw):
    """The same step with the append inside the attention launch (MPA_OPT_FUSE_APPEND) on a fresh copy of
    the workload, whose new tokens' cache slots hold NaN patterns when the launch starts: output and the
    blocks the new tokens land in bit for bit equal to the step just checked."""
    import torch
    import bench
    import paper_2503_13737_amd as mpa
    dw2 = bench.DeviceWorkload(b, mpa)
    dw2.ctx.set_option(mpa.MPA_OPT_FUSE_APPEND, 1)
    dw2.out.fill_(0x7FFF)
    dw2.ws.fill_(0xFF)
    dw2.step()
    torch.cuda.synchronize()
    assert torch.equal(dw2.out, dw.out), f"{b.name}: output differs with the append inside the launch"
    touched = torch.from_numpy(np.unique(b.slot_map // b.bs)).cuda()
    assert torch.equal(dw2.k_cache[touched], dw.k_cache[touched]) and torch.equal(dw2.v_cache[touched], dw.v_cache[touched])
    del dw2
    torch.cuda.empty_cache()
    print(f"[{b.name}] append inside the launch: identical", flush=True)


def check_config(b, all_prompt_rows=False, also_fused=False):
    import torch
    import bench
    import oracle
    import paper_2503_13737_amd as mpa
    print(f"[{b.name}] T={b.T} S={b.S} blocks={b.referenced_blocks().size}", flush=True)
    dw = bench.DeviceWorkload(b, mpa)
    dw.out.fill_(0x7FFF)
    dw.ws.fill_(0xFF)
    dw.step()
    torch.cuda.synchronize()
    out = to_host_u16(dw.out)
    assert not np.isnan(W.to_f64(out, b.dtype)).any(), "NaN (or unwritten rows) in the output"

    # kv_append: the blocks holding the new tokens must equal the oracle's append, bit for bit
    touched = np.unique(b.slot_map // b.bs)
    kn, vn = b.new_kv()
    for which, cache, new in (("k", dw.k_cache, kn), ("v", dw.v_cache, vn)):
        exp = b.blocks_state(which, touched, "prior")
        # oracle append into a pool holding only the touched blocks
        remap = {int(x): i for i, x in enumerate(touched)}
        sm = np.array([remap[int(s // b.bs)] * b.bs + int(s % b.bs) for s in b.slot_map], dtype=np.int64)
        other = exp.copy()
        if which == "k":
            oracle.kv_append(new, new, sm, exp, other)
        else:
            oracle.kv_append(new, new, sm, other, exp)
        got = to_host_u16(cache[torch.from_numpy(touched).cuda()])
        assert np.array_equal(got, exp), f"{b.name}: kv_append({which}) differs"

    rows, heads = sample_rows(b, all_prompt_rows)
    sub = b.compact(range(b.S))
    kc, vc = sub.compact_cache(b, "ctx")
    ref = oracle.attention_rows(sub.q, kc, vc, sub.block_table, sub.chunk_starts, sub.context_lens, b.scale, rows, heads,
                                dtype=b.dtype)
    got = out[rows, heads]
    ma, rl = errors(got, ref, b.dtype)
    abs_tol, rel_tol = TOL[b.dtype]
    print(f"[{b.name}] {rows.size} of {b.T * b.H} (row, head) outputs: max-abs {ma:.3e} rel-L2 {rl:.3e}", flush=True)
    assert ma <= abs_tol and rl <= rel_tol
    # per-row worst case stays within the absolute bound too
    per_row = np.abs(W.to_f64(got, b.dtype) - ref).max(axis=1)
    assert per_row.max() <= abs_tol
    if also_fused:
        check_append_inside_the_launch(b, dw)
    del dw
    torch.cuda.empty_cache()


def test_config2_13b_generation_only():
    check_config(W.config2(), all_prompt_rows=True)


def test_config3_13b_mixed():
    check_config(W.config3(), all_prompt_rows=True, also_fused=True)


@pytest.mark.parametrize("prior", [0, 2048, 4096])
def test_config3_prior_extremes(prior):
    check_config(W.config3(prior=prior), all_prompt_rows=True)


def test_config4_175b_slice():
    check_config(W.config4(), also_fused=True)


def test_grouped_kv_layer():
    check_config(W.config_gqa(), also_fused=True)


def test_grouped_kv_decode_of_a_whole_layer():
    """64 query / 8 K/V heads, 64 generation rows at 4-12 K: every row runs as group items over
    several key ranges (streamed K/V, partials, merge)."""
    check_config(W.config_gqa_decode(), also_fused=True)


@pytest.mark.parametrize("iteration", [0, 12, 24, 36, 47, 48])
def test_config5_long_prompt(iteration):
    check_config(W.config5(iteration), also_fused=iteration in (24, 48))


@pytest.mark.parametrize("make", [W.config2, W.config3, W.config4, lambda dtype: W.config5(47, dtype=dtype)],
                         ids=["cfg2", "cfg3", "cfg4", "cfg5:47"])
def test_fp16_storage_at_full_size(make):
    check_config(make(dtype="fp16"), also_fused=True)


def test_million_token_contexts():
    """The largest shape tried: a generation row and a 64-row prompt chunk, each over a context of 2^20
    tokens (65,536 blocks per sequence; the tile body walks 16,384 steps, the table words of a range are
    re-read every 64 pages), plus a short sequence beside them."""
    n = 1 << 20
    b = W.make_batch("million", 99, 2, 128, 16, 2 * (n // 16) + 16, [1, 64, 1], [n, n, 100])
    check_config(b, also_fused=True)
