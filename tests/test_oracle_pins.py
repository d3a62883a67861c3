"""Pins of the CPU oracle against things other than itself (CPU only).

The paper prints no numeric attention example, so the oracle's values are pinned by
  P1  a structurally different dense brute force (explicit masked L x L score matrix),
  P2  closed forms,
  P3  a library causal scaled-dot-product attention in fp64,
  I1-I5 the invariants of paging / chunking / mixing,
and the block / chunk arithmetic the paper does state is pinned from tests/golden/.
"""
import math
import os

import numpy as np
import pytest

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_block_and_chunk_arithmetic.txt")


def read_golden():
    vals = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            if len(v.split()) == 1 and "." not in v:     # the scheduler's entries (lists, seconds) are read by its own pins
                vals[k.strip()] = int(v)
    return vals


def rand_seq(L, H, D, seed):
    return W.normal_bf16((L, H, D), seed), W.normal_bf16((L, H, D), seed + 1)


def dense_causal(qf, kf, vf, scale, prior):
    """Brute force: qf [n,H,D] are rows prior..prior+n-1 of a sequence whose keys/values are
    kf, vf [L,H,D] (L = prior+n).  Explicit score matrix with -inf above the diagonal."""
    n, H, D = qf.shape
    L = kf.shape[0]
    out = np.zeros((n, H, D))
    for h in range(H):
        s = (qf[:, h, :] @ kf[:, h, :].T) * scale  # [n, L]
        col = np.arange(L)[None, :]
        row = prior + np.arange(n)[:, None]
        s = np.where(col <= row, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        w = np.exp(s)
        w = w / w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ vf[:, h, :]
    return out


def run_single(q, k, v, prior, bs=16, seed=7, scale=None, NB=None):
    """One sequence: q [n,H,D] rows at positions prior.., k/v [L,H,D]."""
    L = k.shape[0]
    n = q.shape[0]
    assert L == prior + n
    NB = NB or ((L + bs - 1) // bs + 3)
    kc, vc, tab = W.paginate([(k, v)], bs, NB, seed)
    scale = scale if scale is not None else 1.0 / math.sqrt(q.shape[2])
    return oracle.attention(q, kc, vc, tab, np.array([0, n]), np.array([L]), scale)


# ---------------------------------------------------------------- golden (paper's own values)
def test_golden_block_arithmetic():
    g = read_golden()
    blocks = lambda L, b: (L + b - 1) // b
    assert blocks(128, 128) == g["b128_blocks_for_128_tokens"]
    assert blocks(129, 128) == g["b128_blocks_for_129_tokens"]
    assert sum(blocks(L, 128) * 128 for L in (1, 128, 129, 300)) == g["alloc_b128_lens_1_128_129_300"]
    assert 8192 // 512 == g["chunks_8192_by_512"]
    assert 2 * 2 * 5120 == g["kv_bytes_per_token_one_layer_H5120"]
    # the generator's block counts follow the same rule
    b = W.make_batch("g", 3, 1, 64, 128, 16, [1, 1, 1, 1], [1, 128, 129, 300])
    assert int((b.n_blocks() * 128).sum()) == g["alloc_b128_lens_1_128_129_300"]
    # forward size = rows in the batch
    b = W.make_batch("g", 3, 1, 64, 16, 2000, [512] + [1] * 31, [512] + [20] * 31)
    assert b.T == g["forward_size_512_plus_31"]


def test_golden_non_first_chunk_fills_previous_block():
    g = read_golden()
    # chunk of 64 rows after 37 prior tokens, b = 16
    b = W.make_batch("g", 5, 1, 64, 16, 16, [64], [37 + 64])
    slots = b.slot_map
    blocks_touched = np.unique(slots // 16)
    prior_blocks = set(b.block_table[0, : (37 + 15) // 16].tolist())
    new_blocks = [x for x in blocks_touched if x not in prior_blocks]
    assert len(new_blocks) == g["new_blocks_b16_prior37_chunk64"]
    # first new token continues in the previous chunk's last block at offset 37 % 16
    assert slots[0] == b.block_table[0, 2] * 16 + 37 % 16
    assert len(set(slots.tolist())) == 64


def test_config1_uses_48_of_64_blocks():
    b = W.config1()
    assert b.T == 107 and b.S == 8
    assert b.referenced_blocks().size == 3 + 7 + (1 + 3 + 4 + 7 + 10 + 13)
    assert len(set(b.referenced_blocks().tolist())) == 48


# ---------------------------------------------------------------- P1 brute force
@pytest.mark.parametrize("L,prior,H,D,bs", [(1, 0, 1, 8, 16), (5, 0, 2, 16, 4), (37, 0, 2, 64, 16),
                                             (100, 63, 3, 64, 16), (50, 49, 2, 32, 16), (70, 16, 1, 128, 32)])
def test_brute_force_dense(L, prior, H, D, bs):
    k, v = rand_seq(L, H, D, 100 + L)
    n = L - prior
    q = W.normal_bf16((n, H, D), 200 + L)
    got = run_single(q, k, v, prior, bs=bs)
    ref = dense_causal(W.bf16_to_f64(q), W.bf16_to_f64(k), W.bf16_to_f64(v), 1 / math.sqrt(D), prior)
    assert np.abs(got - ref).max() < 1e-12


def test_brute_force_whole_config1():
    b = W.config1()
    kc, vc = b.full_cache("ctx")
    got = oracle.attention(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    assert not np.isnan(got).any()
    for i in range(b.S):
        L, n, prior = int(b.context_lens[i]), int(b.q_lens[i]), int(b.priors[i])
        pos = np.arange(L)
        k = kc[b.block_table[i, pos // 16], :, pos % 16, :]
        v = vc[b.block_table[i, pos // 16], :, pos % 16, :]
        r0 = b.chunk_starts[i]
        ref = dense_causal(W.bf16_to_f64(b.q[r0:r0 + n]), W.bf16_to_f64(k), W.bf16_to_f64(v), b.scale, prior)
        assert np.abs(got[r0:r0 + n] - ref).max() < 1e-12


def test_rows_entry_point_matches_full():
    b = W.config1()
    kc, vc = b.full_cache("ctx")
    full = oracle.attention(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    rows = np.array([0, 36, 37, 100, 101, 106, 50])
    heads = np.array([0, 3, 1, 2, 0, 3, 1])
    sel = oracle.attention_rows(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale, rows, heads)
    assert np.array_equal(sel, full[rows, heads])


# ---------------------------------------------------------------- P2 closed forms
def test_single_key_returns_its_value():
    k, v = rand_seq(1, 2, 64, 11)
    q = W.normal_bf16((1, 2, 64), 12)
    got = run_single(q, k, v, 0)
    assert np.array_equal(got[0], W.bf16_to_f64(v)[0])


def test_zero_query_gives_running_mean_of_values():
    L, H, D = 45, 2, 64
    k, v = rand_seq(L, H, D, 21)
    q = np.zeros((L, H, D), dtype=np.uint16)
    got = run_single(q, k, v, 0)
    vf = W.bf16_to_f64(v)
    ref = np.cumsum(vf, axis=0) / np.arange(1, L + 1)[:, None, None]
    assert np.abs(got - ref).max() < 1e-13


def test_equal_keys_give_mean_even_with_nonzero_query():
    L, H, D = 33, 1, 64
    k1 = W.normal_bf16((1, H, D), 31)
    k = np.repeat(k1, L, axis=0)
    v = W.normal_bf16((L, H, D), 32)
    q = W.normal_bf16((1, H, D), 33)
    got = run_single(q, k, v, L - 1)
    assert np.abs(got[0] - W.bf16_to_f64(v).mean(axis=0)).max() < 1e-13


def test_constant_values_come_back():
    L, H, D = 40, 2, 64
    k, _ = rand_seq(L, H, D, 41)
    v = np.repeat(W.normal_bf16((1, H, D), 42), L, axis=0)
    q = W.normal_bf16((L, H, D), 43)
    got = run_single(q, k, v, 0)
    assert np.abs(got - W.bf16_to_f64(v)).max() < 1e-13


def test_one_hot_values_give_probabilities():
    L, H, D = 64, 1, 64
    k, _ = rand_seq(L, H, D, 51)
    v = W.f32_to_bf16(np.eye(L, D, dtype=np.float32)).reshape(L, 1, D)
    q = W.normal_bf16((1, H, D), 53)
    got = run_single(q, k, v, L - 1)[0, 0]
    assert (got >= 0).all() and abs(got.sum() - 1.0) < 1e-13
    # and they are the softmax weights themselves
    s = (W.bf16_to_f64(k)[:, 0, :] @ W.bf16_to_f64(q)[0, 0]) / math.sqrt(D)
    w = np.exp(s - s.max())
    assert np.abs(got - w / w.sum()).max() < 1e-13


def test_dominant_key_selects_its_value():
    L, H, D = 30, 1, 64
    k = np.zeros((L, H, D), dtype=np.float32)
    q = np.zeros((1, H, D), dtype=np.float32)
    q[0, 0, 0] = 16.0
    k[17, 0, 0] = 32.0  # score 16*32/8 = 64 above the others (all 0)
    v = W.normal_bf16((L, H, D), 61)
    got = run_single(W.f32_to_bf16(q), W.f32_to_bf16(k), v, L - 1)
    assert np.abs(got[0, 0] - W.bf16_to_f64(v)[17, 0]).max() < 1e-12


def test_scale_is_applied_to_scores_not_values():
    # doubling q with half the scale leaves the result unchanged (powers of two are exact)
    L, H, D = 20, 1, 64
    k, v = rand_seq(L, H, D, 71)
    q = W.normal_bf16((L, H, D), 73)
    q2 = W.f32_to_bf16(W.bf16_to_f64(q).astype(np.float32) * 2)
    a = run_single(q, k, v, 0, scale=0.125)
    b = run_single(q2, k, v, 0, scale=0.0625)
    assert np.abs(a - b).max() < 1e-13


# ---------------------------------------------------------------- P3 library special case
def test_against_library_causal_sdpa_fp64():
    torch = pytest.importorskip("torch")
    L, H, D = 96, 3, 64
    k, v = rand_seq(L, H, D, 81)
    q = W.normal_bf16((L, H, D), 83)
    got = run_single(q, k, v, 0)
    tq, tk, tv = (torch.from_numpy(W.bf16_to_f64(x)).permute(1, 0, 2)[None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.abs(got - ref).max() < 1e-12


# ---------------------------------------------------------------- invariants
def test_I1_chunked_prefill_equals_one_shot():
    L, H, D = 112, 2, 64
    k, v = rand_seq(L, H, D, 91)
    q = W.normal_bf16((L, H, D), 93)
    one = run_single(q, k, v, 0)
    for cuts in ([37, 64, 11], [1] * 8 + [104], [16, 16, 80], [111, 1]):
        p = 0
        for n in cuts:
            part = run_single(q[p:p + n], k[:p + n], v[:p + n], p)
            assert np.array_equal(part, one[p:p + n]), (cuts, p)
            p += n
        assert p == L


def test_I2_generation_row_equals_last_prompt_row():
    L, H, D = 77, 2, 64
    k, v = rand_seq(L, H, D, 101)
    q = W.normal_bf16((L, H, D), 103)
    pp = run_single(q, k, v, 0)
    tg = run_single(q[L - 1:], k, v, L - 1)
    assert np.array_equal(tg[0], pp[L - 1])


def test_I3_physical_block_permutation():
    b = W.config1()
    kc, vc = b.full_cache("ctx")
    base = oracle.attention(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    perm = W.permutation(b.NB, 999)  # new id of old block x is perm[x]
    kc2, vc2 = np.empty_like(kc), np.empty_like(vc)
    kc2[perm], vc2[perm] = kc, vc
    tab2 = np.where(b.block_table >= 0, perm[np.maximum(b.block_table, 0)], -1).astype(np.int32)
    moved = oracle.attention(b.q, kc2, vc2, tab2, b.chunk_starts, b.context_lens, b.scale)
    assert np.array_equal(base, moved)


def test_I4_batch_independence_and_order():
    b = W.config1()
    kc, vc = b.full_cache("ctx")
    base = oracle.attention(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    order = [5, 1, 7, 0]
    sub = b.compact(order)
    kc2, vc2 = sub.compact_cache(b)
    got = oracle.attention(sub.q, kc2, vc2, sub.block_table, sub.chunk_starts, sub.context_lens, sub.scale)
    assert np.array_equal(got, base[sub.rows_src])


def test_I5_poisoned_unused_slots_do_not_matter():
    b = W.config1()
    kc, vc = b.full_cache("ctx")
    assert (kc == W.POISON).any()
    base = oracle.attention(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    assert not np.isnan(base).any()
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[kc == W.POISON] = 0x3F80
    vc2[vc == W.POISON] = 0xC000
    again = oracle.attention(b.q, kc2, vc2, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    assert np.array_equal(base, again)


# ---------------------------------------------------------------- kv_append
def test_kv_append_oracle_bytes():
    b = W.config1()
    kc, vc = b.full_cache("prior")
    kn, vn = b.new_kv()
    before_k = kc.copy()
    oracle.kv_append(kn, vn, b.slot_map, kc, vc)
    # independent check: python loop over the definition cache[slot//bs, h, slot%bs, :]
    exp_k, exp_v = before_k.copy(), b.full_cache("prior")[1]
    for t, s in enumerate(b.slot_map):
        exp_k[s // 16, :, s % 16, :] = kn[t]
        exp_v[s // 16, :, s % 16, :] = vn[t]
    assert np.array_equal(kc, exp_k) and np.array_equal(vc, exp_v)
    # and the appended state equals the generator's "after" state, untouched slots still poison
    k2, v2 = b.full_cache("ctx")
    assert np.array_equal(kc, k2) and np.array_equal(vc, v2)
    assert (kc != before_k).any()


def test_kv_append_skips_negative_slots():
    b = W.config1()
    kc, vc = b.full_cache("prior")
    kn, vn = b.new_kv()
    sm = b.slot_map.copy()
    sm[::3] = -1
    k0 = kc.copy()
    oracle.kv_append(kn, vn, sm, kc, vc)
    for t, s in enumerate(b.slot_map):
        if sm[t] < 0:
            assert np.array_equal(kc[s // 16, :, s % 16, :], k0[s // 16, :, s % 16, :])
        else:
            assert np.array_equal(kc[s // 16, :, s % 16, :], kn[t])


# ---------------------------------------------------------------- planted mistakes are caught
def test_pins_catch_planted_mistakes():
    """Variants of the definition with one plausible mistake each must fail the pins above
    (here: disagree with the oracle, which those pins hold in place)."""
    L, H, D = 40, 1, 64
    k, v = rand_seq(L, H, D, 111)
    q = W.normal_bf16((L, H, D), 113)
    good = run_single(q, k, v, 0)
    qf, kf, vf = (W.bf16_to_f64(x)[:, 0, :] for x in (q, k, v))
    sc = 1 / math.sqrt(D)

    def variant(mask_strict=False, no_scale=False, no_max_shift_sign=False, swap_kv=False):
        kk, vv = (vf, kf) if swap_kv else (kf, vf)
        s = qf @ kk.T * (1.0 if no_scale else sc)
        r, c = np.arange(L)[:, None], np.arange(L)[None, :]
        keep = (c < r) | ((c == r) & (r == 0)) if mask_strict else (c <= r)
        s = np.where(keep, s, -np.inf)
        w = np.exp(-(s - s.max(1, keepdims=True))) if no_max_shift_sign else np.exp(s - s.max(1, keepdims=True))
        w = np.where(keep, w, 0)
        return (w / w.sum(1, keepdims=True)) @ vv

    assert np.abs(variant() - good[:, 0]).max() < 1e-12
    for kw in (dict(mask_strict=True), dict(no_scale=True), dict(no_max_shift_sign=True), dict(swap_kv=True)):
        assert np.abs(variant(**kw) - good[:, 0]).max() > 1e-3, kw


# ---------------------------------------------------------------- grouped K/V heads
def test_grouped_kv_heads_equal_repeated_heads():
    """Query heads sharing K/V heads in groups == ordinary attention over caches in which each
    K/V head is repeated for every query head of its group (bit-exact on the oracle), and both
    agree with the dense brute force."""
    H, HK, D = 8, 2, 64
    b = W.random_ragged(4321, H=H, D=D, n_pp=2, n_tg=3, max_q=40, max_prior=50, max_ctx=60, Hkv=HK)
    kc, vc = b.full_cache("ctx")
    assert kc.shape[1] == HK
    got = oracle.attention(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    kc_rep, vc_rep = np.repeat(kc, H // HK, axis=1), np.repeat(vc, H // HK, axis=1)
    ref = oracle.attention(b.q, kc_rep, vc_rep, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    assert np.array_equal(got, ref)
    # a wrong head map (h % HK instead of h / group) must differ
    kc_bad, vc_bad = np.tile(kc, (1, H // HK, 1, 1)), np.tile(vc, (1, H // HK, 1, 1))
    bad = oracle.attention(b.q, kc_bad, vc_bad, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    assert np.abs(bad - got).max() > 1e-3
    for i in range(b.S):
        L, n, prior = int(b.context_lens[i]), int(b.q_lens[i]), int(b.priors[i])
        pos = np.arange(L)
        k = kc_rep[b.block_table[i, pos // 16], :, pos % 16, :]
        v = vc_rep[b.block_table[i, pos // 16], :, pos % 16, :]
        r0 = b.chunk_starts[i]
        dense = dense_causal(W.bf16_to_f64(b.q[r0:r0 + n]), W.bf16_to_f64(k), W.bf16_to_f64(v), b.scale, prior)
        assert np.abs(got[r0:r0 + n] - dense).max() < 1e-12


def test_grouped_kv_append_writes_kv_heads_only():
    H, HK, D = 8, 2, 64
    b = W.random_ragged(77, H=H, D=D, n_pp=1, n_tg=2, max_q=20, max_prior=20, max_ctx=30, Hkv=HK)
    kc, vc = b.full_cache("prior")
    kn, vn = b.new_kv()
    assert kn.shape == (b.T, HK, D)
    oracle.kv_append(kn, vn, b.slot_map, kc, vc)
    k2, v2 = b.full_cache("ctx")
    assert np.array_equal(kc, k2) and np.array_equal(vc, v2)


# ---------------------------------------------------------------- fp16 storage (the paper's precision)
def test_fp16_decode_matches_the_library_for_every_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    got, ref = oracle.widen(bits, "fp16"), bits.view(np.float16).astype(np.float64)
    ok = ~np.isnan(ref)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(got[ok], ref[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(ref[ok]))
    # and bf16 against the upper half of a single
    ref_bf = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    got_bf = oracle.widen(bits, "bf16")
    ok = ~np.isnan(ref_bf)
    assert np.array_equal(got_bf[ok], ref_bf[ok])


def test_generator_fp16_rounding_matches_the_library():
    rng = np.random.default_rng(11)
    x = (rng.standard_normal(100000) * 10.0 ** rng.integers(-9, 5, 100000)).astype(np.float32)
    edge = np.array([0.0, -0.0, 65504, 65519.9, 65520, 1e-8, 5.96e-8, 2.98e-8, 2.99e-8, 6.1e-5, 6.0e-5,
                     1.0009765625, 1.00048828125, 1.00146484375], dtype=np.float32)
    x = np.concatenate([x, edge, -edge])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(W.round_16(x, "fp16"), ref)
    b = W.make_batch("fp16-gen", 5, 8, 128, 16, 40, [60, 1], [80, 33], dtype="fp16")
    vals = W.to_f64(b.q, "fp16")
    assert vals.size > 50000 and abs(vals.std() - 1.0) < 0.02 and abs(vals.mean()) < 0.02


@pytest.mark.parametrize("L,prior,H,D,bs", [(5, 0, 2, 16, 4), (100, 63, 3, 64, 16), (70, 16, 1, 128, 32)])
def test_brute_force_dense_fp16(L, prior, H, D, bs):
    k = W.normal_bf16((L, H, D), 300 + L, dtype="fp16")
    v = W.normal_bf16((L, H, D), 301 + L, dtype="fp16")
    n = L - prior
    q = W.normal_bf16((n, H, D), 400 + L, dtype="fp16")
    NB = (L + bs - 1) // bs + 3
    kc, vc, tab = W.paginate([(k, v)], bs, NB, 7)
    got = oracle.attention(q, kc, vc, tab, np.array([0, n]), np.array([L]), 1 / math.sqrt(D), dtype="fp16")
    ref = dense_causal(W.to_f64(q, "fp16"), W.to_f64(k, "fp16"), W.to_f64(v, "fp16"), 1 / math.sqrt(D), prior)
    assert np.abs(got - ref).max() < 1e-12
    # the same bits read as bf16 are other numbers: the format switch is not a no-op
    other = oracle.attention(q, kc, vc, tab, np.array([0, n]), np.array([L]), 1 / math.sqrt(D), dtype="bf16")
    assert np.abs(other - ref).max() > 1e-3


# ---------------------------------------------------------------- block copies (swap out / in)
def test_copy_blocks_round_trip_and_untouched_blocks():
    """Out to a second pool and back in to other blocks: the moved blocks arrive bit for bit, every
    other block of both pools keeps its content, and attention through the re-mapped table gives
    the identical result (blocks are position-independent)."""
    b = W.config1()
    kc, vc = b.full_cache("ctx")
    seq = 7
    nblk = int(b.n_blocks()[seq])
    held = b.block_table[seq, :nblk].astype(np.int64)
    host_k = np.full((nblk + 2,) + kc.shape[1:], 0x1234, dtype=np.uint16)
    host_v = host_k.copy()
    out_pairs = np.stack([held, np.arange(nblk)[::-1]], axis=1)
    oracle.copy_blocks(kc, vc, host_k, host_v, out_pairs)
    for s, d in out_pairs:
        for byte_for_byte in (np.array_equal(host_k[d], kc[s]), np.array_equal(host_v[d], vc[s])):
            assert byte_for_byte
    assert (host_k[nblk:] == 0x1234).all() and (host_v[nblk:] == 0x1234).all()
    # back in, to blocks nobody references
    free = np.setdiff1d(np.arange(b.NB), b.referenced_blocks())[:nblk].astype(np.int64)
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[held], vc2[held] = W.POISON, W.POISON
    oracle.copy_blocks(host_k, host_v, kc2, vc2, np.stack([np.arange(nblk)[::-1], free], axis=1))
    assert np.array_equal(kc2[free], kc[held]) and np.array_equal(vc2[free], vc[held])
    others = np.setdiff1d(np.arange(b.NB), np.concatenate([held, free]))
    assert np.array_equal(kc2[others], kc[others])
    tab2 = b.block_table.copy()
    tab2[seq, :nblk] = free
    ref = oracle.attention(b.q, kc, vc, b.block_table, b.chunk_starts, b.context_lens, b.scale)
    got = oracle.attention(b.q, kc2, vc2, tab2, b.chunk_starts, b.context_lens, b.scale)
    assert np.array_equal(got, ref)
