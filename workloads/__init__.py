"""Seeded synthetic mixed batches (prompt-chunk + generation tasks over a paged KV cache).

This module only *describes inputs*: sequence lengths, block tables, slot maps and N(0,1) tensor
contents rounded to bf16.  It contains none of the attention arithmetic and is the only code the
CPU oracle's tests and the GPU path's tests have in common.

All randomness is counter based (value = f(seed, index), see gen.c), so any part of a large
tensor can be produced alone and both sides see bit-identical arrays.

Layouts (bf16 stored as uint16 bit patterns):
    q               : [T, H, D]     T = total query rows of the batch (ragged concatenation)
    k_cache, v_cache: [NB, HK, bs, D] one (block, kv head) tile is bs*D contiguous elements; HK = H
                      unless query heads share K/V heads in groups of H/HK consecutive heads
    k_new, v_new    : [T, HK, D]
    block_table     : [S, MB] int32, -1 padded, logical block j of sequence i -> physical block
    chunk_starts    : [S+1] int32 row offsets of each sequence's rows in q/out
    context_lens    : [S] int32 KV length of each sequence *including* this iteration's rows
    slot_map        : [T] int64 physical slot (block*bs + offset) each new token's K/V goes to

The cache content is a function of the physical position alone: element (b, h, o, d) of the K
(or V) pool is N(0,1) at counter ((b*H + h)*bs + o)*D + d under the K (or V) seed.  The new
tokens' k_new/v_new are defined as the values their destination slots hold, so the cache state
after the append is "generated content for every token below context_len", and the state before
it is the same with the new tokens' slots poisoned.  Slots past a sequence's length and blocks no
sequence references always hold the poison pattern (a bf16 NaN), so reading them shows up.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmpagen.so")
_lib = None

POISON = np.uint16(0x7FFF)  # bf16 quiet NaN
BASE_SEED = 20250313


def build(force: bool = False) -> str:
    """Compile gen.c with gcc (host only)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", src, "-o", _LIB_PATH, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        u64, p = ctypes.c_uint64, ctypes.c_void_p
        lib.mpagen_fill_normal_16.argtypes = [p, u64, u64, u64, ctypes.c_int]
        lib.mpagen_fill_normal_16.restype = None
        lib.mpagen_fill_normal_16_segments.argtypes = [p, u64, u64, u64, p, ctypes.c_int]
        lib.mpagen_fill_normal_16_segments.restype = None
        lib.mpagen_round_16.argtypes = [p, p, u64, ctypes.c_int]
        lib.mpagen_round_16.restype = None
        lib.mpagen_fill_bits.argtypes = [p, u64, u64, u64]
        lib.mpagen_fill_bits.restype = None
        _lib = lib
    return _lib


DTYPES = {"bf16": 1, "fp16": 2}   # 16-bit storage formats of q, K, V and the output


def normal_bf16(shape, seed: int, offset: int = 0, dtype: str = "bf16") -> np.ndarray:
    """16-bit patterns (bf16 unless dtype says fp16) of N(0,1) draws at counters offset .. offset+prod(shape)."""
    out = np.empty(shape, dtype=np.uint16)
    _load().mpagen_fill_normal_16(out.ctypes.data, out.size, seed, offset, DTYPES[dtype])
    return out


def normal_bf16_segments(offsets: np.ndarray, seglen: int, seed: int, dtype: str = "bf16") -> np.ndarray:
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    out = np.empty((offsets.size, seglen), dtype=np.uint16)
    _load().mpagen_fill_normal_16_segments(out.ctypes.data, offsets.size, seglen, seed, offsets.ctypes.data,
                                           DTYPES[dtype])
    return out


def round_16(a, dtype: str) -> np.ndarray:
    """The generator's float32 -> 16-bit rounding on its own (for tests)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    _load().mpagen_round_16(a.ctypes.data, out.ctypes.data, a.size, DTYPES[dtype])
    return out


def bits(n: int, seed: int, offset: int = 0) -> np.ndarray:
    out = np.empty(n, dtype=np.uint64)
    _load().mpagen_fill_bits(out.ctypes.data, n, seed, offset)
    return out


def uniform_ints(n: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """n integers uniform on [lo, hi], both ends included."""
    return (lo + (bits(n, seed) % np.uint64(hi - lo + 1)).astype(np.int64)).astype(np.int64)


def standard_normals(n: int, seed: int) -> np.ndarray:
    """float64 N(0,1) draws for *length* distributions (Box-Muller on the seeded bits)."""
    z = bits(n, seed)
    u1 = ((z >> np.uint64(40)).astype(np.float64) + 0.5) / 16777216.0
    u2 = (((z >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) + 0.5) / 16777216.0
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)


def permutation(n: int, seed: int) -> np.ndarray:
    return np.argsort(bits(n, seed), kind="stable").astype(np.int64)


def bf16_to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (test utility, no rounding involved)."""
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def to_f64(a: np.ndarray, dtype: str = "bf16") -> np.ndarray:
    """Exact widening of 16-bit patterns of the given format (library conversion for fp16)."""
    if dtype == "fp16":
        return np.ascontiguousarray(a, dtype=np.uint16).view(np.float16).astype(np.float64)
    return bf16_to_f64(a)


@dataclass
class Batch:
    name: str
    seed: int
    H: int
    D: int
    bs: int
    NB: int
    chunk_starts: np.ndarray
    context_lens: np.ndarray
    block_table: np.ndarray
    slot_map: np.ndarray = field(default=None)
    q: np.ndarray = field(default=None)
    content_seed: int = field(default=None)  # seed of the cache content (defaults to `seed`)
    Hkv: int = field(default=None)           # K/V heads (query heads share them in groups); None = H
    dtype: str = "bf16"                      # storage format of q, K, V, out: "bf16" or "fp16"

    # ---- derived metadata -------------------------------------------------------------
    @property
    def S(self) -> int:
        return int(self.context_lens.size)

    @property
    def HK(self) -> int:
        return self.H if self.Hkv is None else self.Hkv

    @property
    def T(self) -> int:
        return int(self.chunk_starts[-1])

    @property
    def q_lens(self) -> np.ndarray:
        return np.diff(self.chunk_starts).astype(np.int64)

    @property
    def priors(self) -> np.ndarray:
        return self.context_lens.astype(np.int64) - self.q_lens

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def seed_k(self) -> int:
        return (self.seed if self.content_seed is None else self.content_seed) * 4 + 1

    @property
    def seed_v(self) -> int:
        return (self.seed if self.content_seed is None else self.content_seed) * 4 + 2

    @property
    def seed_q(self) -> int:
        return self.seed * 4 + 3

    def n_blocks(self) -> np.ndarray:
        return (self.context_lens.astype(np.int64) + self.bs - 1) // self.bs

    def referenced_blocks(self) -> np.ndarray:
        nb = self.n_blocks()
        return np.concatenate([self.block_table[i, : nb[i]] for i in range(self.S)]).astype(np.int64)

    def tg_kv_tokens(self) -> int:
        ql = self.q_lens
        return int(self.context_lens[ql == 1].sum())

    def pp_pairs(self) -> int:
        """(query, key) pairs of the multi-row tasks under the inclusive causal mask."""
        ql, pr = self.q_lens, self.priors
        m = ql > 1
        return int((ql[m] * pr[m] + ql[m] * (ql[m] + 1) // 2).sum())

    # ---- tensor contents --------------------------------------------------------------
    def _finish(self):
        """Fill slot_map and q from the metadata."""
        T, bs = self.T, self.bs
        sm = np.empty(T, dtype=np.int64)
        for i in range(self.S):
            r0, n = int(self.chunk_starts[i]), int(self.q_lens[i])
            pos = int(self.priors[i]) + np.arange(n)
            sm[r0 : r0 + n] = self.block_table[i, pos // bs].astype(np.int64) * bs + pos % bs
        self.slot_map = sm
        self.q = normal_bf16((T, self.H, self.D), self.seed_q, dtype=self.dtype)
        return self

    def block_contents(self, which: str, ids: np.ndarray) -> np.ndarray:
        """Generated content of physical blocks `ids`: [n, HK, bs, D] bf16 bits, no poison."""
        seed = self.seed_k if which == "k" else self.seed_v
        per = self.HK * self.bs * self.D
        offs = np.asarray(ids, dtype=np.uint64) * np.uint64(per)
        return normal_bf16_segments(offs, per, seed, self.dtype).reshape(len(ids), self.HK, self.bs, self.D)

    def new_kv(self):
        """k_new, v_new [T,HK,D]: the values the destination slots are defined to hold."""
        blk = self.slot_map // self.bs
        off = self.slot_map % self.bs
        outs = []
        for which in ("k", "v"):
            seed = self.seed_k if which == "k" else self.seed_v
            # one segment of D values per (token, head)
            base = (blk[:, None] * self.HK + np.arange(self.HK)[None, :]) * self.bs + off[:, None]
            offs = (base.astype(np.uint64) * np.uint64(self.D)).reshape(-1)
            outs.append(normal_bf16_segments(offs, self.D, seed, self.dtype).reshape(self.T, self.HK, self.D))
        return outs[0], outs[1]

    def poison_mask(self, ids: np.ndarray, limit: str) -> np.ndarray:
        """[n, bs] bool: True where slot (ids[n], o) holds no token below `limit`
        ('prior' = state before the append, 'ctx' = state after it)."""
        lim = self.priors if limit == "prior" else self.context_lens.astype(np.int64)
        valid = np.zeros(self.NB, dtype=np.int64)  # valid tokens per physical block
        nb = self.n_blocks()
        for i in range(self.S):
            j = np.arange(nb[i])
            valid[self.block_table[i, : nb[i]]] = np.clip(lim[i] - j * self.bs, 0, self.bs)
        v = valid[np.asarray(ids, dtype=np.int64)]
        return np.arange(self.bs)[None, :] >= v[:, None]

    def blocks_state(self, which: str, ids: np.ndarray, limit: str = "prior") -> np.ndarray:
        """Content of physical blocks `ids` with the poison applied."""
        c = self.block_contents(which, ids)
        m = self.poison_mask(ids, limit)
        c[np.broadcast_to(m[:, None, :, None], c.shape)] = POISON
        return c

    def full_cache(self, limit: str = "prior"):
        """(k_cache, v_cache) [NB,H,bs,D] — small pools only."""
        ids = np.arange(self.NB)
        return self.blocks_state("k", ids, limit), self.blocks_state("v", ids, limit)

    def compact(self, seq_ids) -> "Batch":
        """A batch holding only sequences `seq_ids`, its blocks renumbered 0..n-1 in a small pool.
        `self.compact_src` on the result maps new block id -> old block id.  (Relies on the
        result not depending on which physical block holds what; the oracle tests pin that.)"""
        seq_ids = list(seq_ids)
        nb = self.n_blocks()
        old = np.concatenate([self.block_table[i, : nb[i]] for i in seq_ids]).astype(np.int64)
        newtab = np.full((len(seq_ids), max(1, int(nb[seq_ids].max()))), -1, dtype=np.int32)
        p = 0
        for r, i in enumerate(seq_ids):
            newtab[r, : nb[i]] = np.arange(p, p + nb[i])
            p += int(nb[i])
        ql = self.q_lens[seq_ids]
        cs = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
        rows = np.concatenate([np.arange(self.chunk_starts[i], self.chunk_starts[i + 1]) for i in seq_ids])
        b = Batch(self.name + "/compact", self.seed, self.H, self.D, self.bs, max(1, len(old)), cs,
                  self.context_lens[seq_ids].copy(), newtab, content_seed=self.content_seed, Hkv=self.Hkv,
                  dtype=self.dtype)
        b.compact_src = old
        b.rows_src = rows
        b.q = self.q[rows]
        sm = np.empty(b.T, dtype=np.int64)
        for r in range(b.S):
            pos = int(b.priors[r]) + np.arange(int(b.q_lens[r]))
            sm[cs[r] : cs[r + 1]] = newtab[r, pos // b.bs].astype(np.int64) * b.bs + pos % b.bs
        b.slot_map = sm
        return b

    def compact_cache(self, parent: "Batch", limit: str = "ctx"):
        """Caches for a batch made by parent.compact(): parent's content moved with the blocks."""
        return (parent.blocks_state("k", self.compact_src, limit),
                parent.blocks_state("v", self.compact_src, limit))


def make_batch(name, seed, H, D, bs, NB, q_lens, context_lens, block_ids=None, Hkv=None, dtype="bf16") -> Batch:
    """Build a batch from per-sequence (q_len, context_len); block ids are drawn without
    replacement from the pool unless given."""
    q_lens = np.asarray(q_lens, dtype=np.int64)
    ctx = np.asarray(context_lens, dtype=np.int64)
    assert np.all(q_lens >= 1) and np.all(ctx >= q_lens)
    nb = (ctx + bs - 1) // bs
    need = int(nb.sum())
    assert need <= NB, f"{name}: needs {need} blocks, pool has {NB}"
    if block_ids is None:
        block_ids = permutation(NB, seed * 4)[:need]
    MB = int(nb.max())
    tab = np.full((len(ctx), MB), -1, dtype=np.int32)
    p = 0
    for i in range(len(ctx)):
        tab[i, : nb[i]] = block_ids[p : p + nb[i]]
        p += int(nb[i])
    cs = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    return Batch(name, seed, H, D, bs, NB, cs, ctx.astype(np.int32), tab, Hkv=Hkv, dtype=dtype)._finish()


def _sfx(dtype: str) -> str:
    return "" if dtype == "bf16" else "-" + dtype


def config_seed(index: int) -> int:
    return BASE_SEED * 10 + index


def config1(dtype: str = "bf16") -> Batch:
    """Tiny mixed batch: 4 heads, head_dim 64; chunks 37@0 and 64@48; six generation rows."""
    ql = [37, 64, 1, 1, 1, 1, 1, 1]
    ctx = [37, 48 + 64, 10, 33, 64, 100, 150, 200]
    return make_batch("cfg1-tiny-mixed" + _sfx(dtype), config_seed(1), 4, 64, 16, 64, ql, ctx, dtype=dtype)


def config2(bs: int = 16, dtype: str = "bf16") -> Batch:
    """13B-shaped layer, generation only: 64 sequences, contexts uniform on [256, 2048].
    bs: tokens per KV block (the pool keeps its size in tokens)."""
    s = config_seed(2)
    ctx = uniform_ints(64, 256, 2048, s * 4 + 3)
    return make_batch("cfg2-13b-tg" + (f"-bs{bs}" if bs != 16 else "") + _sfx(dtype), s, 40, 128, bs, 32768 * 16 // bs,
                      np.ones(64, dtype=np.int64), ctx, dtype=dtype)


def config3(prior: int | None = None, bs: int = 16, dtype: str = "bf16") -> Batch:
    """13B-shaped layer, mixed: one 512-token chunk at prior context uniform on [0, 4096] plus
    48 generation rows with contexts uniform on [512, 4096].  bs: tokens per KV block."""
    s = config_seed(3)
    if prior is None:
        prior = int(uniform_ints(1, 0, 4096, s * 4 + 3)[0])
    ctx_tg = uniform_ints(48, 512, 4096, s * 4 + 2)
    ql = np.concatenate([[512], np.ones(48, dtype=np.int64)])
    ctx = np.concatenate([[prior + 512], ctx_tg])
    return make_batch("cfg3-13b-mixed" + (f"-bs{bs}" if bs != 16 else "") + _sfx(dtype), s, 40, 128, bs, 32768 * 16 // bs,
                      ql, ctx, dtype=dtype)


def config4(dtype: str = "bf16") -> Batch:
    """12-head slice of a 96-head layer: four 512-token chunks at prior contexts uniform on
    [0, 32768]; 128 generation rows with lognormal contexts (median 1024, sigma 1, cap 8192)."""
    s = config_seed(4)
    priors = uniform_ints(4, 0, 32768, s * 4 + 3)
    z = standard_normals(128, s * 4 + 2)
    ctx_tg = np.clip(np.rint(np.exp(math.log(1024.0) + 1.0 * z)), 1, 8192).astype(np.int64)
    ql = np.concatenate([np.full(4, 512), np.ones(128, dtype=np.int64)])
    ctx = np.concatenate([priors + 512, ctx_tg])
    return make_batch("cfg4-175b-slice" + _sfx(dtype), s, 12, 128, 16, 32768, ql, ctx, dtype=dtype)


def config_gqa() -> Batch:
    """Grouped-query layer (not one of the benchmark's five configs): a 4-way tensor-parallel
    share of a 64-query-head / 8-KV-head layer (the head layout of the Llama-3-70B model the paper
    also serves): 16 query heads over 2 K/V heads, head_dim 128.  Same sequence mix as config 3:
    one 512-row chunk at prior context uniform on [0, 4096], 48 generation rows with contexts
    uniform on [512, 4096]."""
    s = config_seed(6)
    prior = int(uniform_ints(1, 0, 4096, s * 4 + 3)[0])
    ctx_tg = uniform_ints(48, 512, 4096, s * 4 + 2)
    ql = np.concatenate([[512], np.ones(48, dtype=np.int64)])
    ctx = np.concatenate([[prior + 512], ctx_tg])
    return make_batch("gqa-16q-2kv-mixed", s, 16, 128, 16, 32768, ql, ctx, Hkv=2)


def config_gqa_decode() -> Batch:
    """Decode batch of a whole grouped-query layer (not one of the benchmark's five configs): 64 query
    heads over 8 K/V heads, head_dim 128 (the head layout of the Llama-3-70B model the paper also
    serves), 64 generation rows with contexts uniform on [4096, 12288]: 2 GB of K/V per step."""
    s = config_seed(7)
    ctx = uniform_ints(64, 4096, 12288, s * 4 + 2)
    nb = int(sum((int(c) + 15) // 16 for c in ctx)) + 8
    return make_batch("gqa-64q-8kv-decode", s, 64, 128, 16, nb, np.ones(64, dtype=np.int64), ctx, Hkv=8)


HELD_OUT = ("fwd768-13b", "fwd1280-13b", "fwd1280-12h", "fwd768-24h", "small-chunks-13b", "two-long-13b")


def held_out(name: str) -> Batch:
    """Scheduler-shaped batches that no planner constant was fitted on (not among the benchmark's
    five configs): forward sizes of the paper's two pivot values, 768 and 1280 tokens (Sec. 3.1),
    made of several dynamic chunks of unequal lengths that start anywhere in their prompts
    (Sec. 4.2) next to generation rows; 13B-shaped layers (40 heads) and 12- and 24-head shares of a
    96-head layer."""
    i = HELD_OUT.index(name)
    s = config_seed(20 + i)
    if name == "fwd768-13b":        # 650 prompt tokens in three chunks + 118 generation rows
        H, chunks = 40, [(300, 1000), (200, 0), (150, 3500)]
        ctx_tg = uniform_ints(118, 256, 4096, s * 4 + 2)
    elif name == "fwd1280-13b":     # one long prompt under way, three short ones, 50 generation rows
        H, chunks = 40, [(1000, 6000), (100, 0), (90, 700), (40, 40)]
        ctx_tg = uniform_ints(50, 128, 8192, s * 4 + 2)
    elif name == "fwd1280-12h":     # a 12-head share: long priors, lognormal generation contexts
        H, chunks = 12, [(640, 9000), (400, 0), (200, 20000)]
        z = standard_normals(40, s * 4 + 2)
        ctx_tg = np.clip(np.rint(np.exp(math.log(2048.0) + 1.0 * z)), 1, 16384).astype(np.int64)
    elif name == "fwd768-24h":      # a 24-head share: eight chunks of about 90 tokens
        H = 24
        lens = uniform_ints(8, 60, 120, s * 4 + 1)
        chunks = list(zip(lens.tolist(), uniform_ints(8, 0, 8000, s * 4 + 3).tolist()))
        ctx_tg = uniform_ints(768 - int(lens.sum()), 512, 4096, s * 4 + 2)
    elif name == "small-chunks-13b":   # prompts only: sixteen chunks of 20-200 tokens
        H = 40
        lens = uniform_ints(16, 20, 200, s * 4 + 1)
        chunks = list(zip(lens.tolist(), uniform_ints(16, 0, 6000, s * 4 + 3).tolist()))
        ctx_tg = np.zeros(0, dtype=np.int64)
    else:                           # two long prompts' chunks in one batch (urgent ones are not held back)
        H, chunks = 40, [(768, 12000), (512, 30000)]
        ctx_tg = uniform_ints(64, 1024, 6000, s * 4 + 2)
    ql = np.concatenate([[c[0] for c in chunks], np.ones(ctx_tg.size, dtype=np.int64)]).astype(np.int64)
    ctx = np.concatenate([[c[0] + c[1] for c in chunks], ctx_tg]).astype(np.int64)
    nb = int(((ctx + 15) // 16).sum()) + 64
    return make_batch("held-" + name, s, H, 128, 16, nb, ql, ctx)


CFG5_PROMPT = 100_000
CFG5_CHUNK = 2048
CFG5_ITERS = (CFG5_PROMPT + CFG5_CHUNK - 1) // CFG5_CHUNK  # 49


def config5(iteration: int, dtype: str = "bf16") -> Batch:
    """Long prompt: iteration k processes prompt tokens [2048k, min(2048(k+1), 100000)) against
    all earlier ones, batched with 64 generation rows whose contexts start uniform on
    [1024, 16384] and grow by one per iteration.  Block tables are drawn once for all
    iterations (each sequence's blocks up to its final length)."""
    assert 0 <= iteration < CFG5_ITERS
    s = config_seed(5)
    H, D, bs, NB = 40, 128, 16, 65536
    ctx0 = uniform_ints(64, 1024, 16384, s * 4 + 2)
    final = np.concatenate([[CFG5_PROMPT], ctx0 + (CFG5_ITERS - 1)])
    nb_final = (final + bs - 1) // bs
    assert int(nb_final.sum()) <= NB
    ids = permutation(NB, s * 4)[: int(nb_final.sum())]
    prior = CFG5_CHUNK * iteration
    qn = min(CFG5_CHUNK, CFG5_PROMPT - prior)
    ql = np.concatenate([[qn], np.ones(64, dtype=np.int64)])
    ctx = np.concatenate([[prior + qn], ctx0 + iteration])
    # per-sequence block lists are prefixes of the final allocation
    nb = (ctx + bs - 1) // bs
    MB = int(nb.max())
    tab = np.full((65, MB), -1, dtype=np.int32)
    p = 0
    for i in range(65):
        tab[i, : nb[i]] = ids[p : p + nb[i]]
        p += int(nb_final[i])
    cs = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
    # the cache content seed stays the config's, so the prompt's K/V is the same in every
    # iteration; only q is redrawn per iteration
    b = Batch(f"cfg5-long-prompt-it{iteration}" + _sfx(dtype), s * 100 + iteration, H, D, bs, NB, cs,
              ctx.astype(np.int32), tab, content_seed=s, dtype=dtype)
    return b._finish()


def random_ragged(seed: int, H: int = 2, D: int = 64, bs: int = 16, n_pp: int = 2, n_tg: int = 3,
                  max_q: int = 70, max_prior: int = 90, max_ctx: int = 120, NB: int | None = None,
                  Hkv: int | None = None, dtype: str = "bf16") -> Batch:
    """Small random mixed batch for property-style tests (sizes are arbitrary integers)."""
    ql_pp = uniform_ints(n_pp, 2, max_q, seed * 8 + 1) if n_pp else np.zeros(0, dtype=np.int64)
    pr_pp = uniform_ints(n_pp, 0, max_prior, seed * 8 + 2) if n_pp else np.zeros(0, dtype=np.int64)
    ctx_tg = uniform_ints(n_tg, 1, max_ctx, seed * 8 + 3) if n_tg else np.zeros(0, dtype=np.int64)
    ql = np.concatenate([ql_pp, np.ones(n_tg, dtype=np.int64)])
    ctx = np.concatenate([ql_pp + pr_pp, ctx_tg])
    order = permutation(len(ql), seed * 8 + 4)
    ql, ctx = ql[order], ctx[order]
    need = int(((ctx + bs - 1) // bs).sum())
    return make_batch(f"ragged-{seed}" + _sfx(dtype), seed, H, D, bs, NB or (need + 5), ql, ctx, Hkv=Hkv, dtype=dtype)


def f32_to_bf16(a) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (input preparation utility)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    return r


def paginate(kv_per_seq, bs: int, NB: int, seed: int):
    """Scatter logical per-sequence tensors into a paged pool.

    kv_per_seq: list of (k [L,H,D] uint16, v [L,H,D] uint16).  Returns (k_cache, v_cache,
    block_table) with blocks drawn without replacement from a pool of NB blocks; every slot not
    holding a token is poisoned."""
    H, D = kv_per_seq[0][0].shape[1:]
    nb = [(k.shape[0] + bs - 1) // bs for k, _ in kv_per_seq]
    ids = permutation(NB, seed)[: sum(nb)]
    kc = np.full((NB, H, bs, D), POISON, dtype=np.uint16)
    vc = np.full((NB, H, bs, D), POISON, dtype=np.uint16)
    tab = np.full((len(nb), max(max(nb), 1)), -1, dtype=np.int32)
    p = 0
    for i, (k, v) in enumerate(kv_per_seq):
        tab[i, : nb[i]] = ids[p : p + nb[i]]
        p += nb[i]
        for t in range(k.shape[0]):
            b, o = tab[i, t // bs], t % bs
            kc[b, :, o, :] = k[t]
            vc[b, :, o, :] = v[t]
    return kc, vc, tab


# ------------------------------------------------------------------------------------------------
# Request traces for the scheduler (inputs only: arrival times, lengths, SLOs).
# ------------------------------------------------------------------------------------------------
def _uniform01(n: int, seed: int) -> np.ndarray:
    return ((bits(n, seed) >> np.uint64(11)).astype(np.float64) + 0.5) / 9007199254740992.0


def _log_uniform_ints(u: np.ndarray, lo: int, hi: int) -> np.ndarray:
    return np.clip(np.floor(np.exp(math.log(lo) + u * (math.log(hi + 1) - math.log(lo)))), lo, hi).astype(np.int64)


def poisson_trace(n: int, seed: int, rate: float = 8.0, max_prompt: int = 100_000, max_new: int = 2048,
                  base_token_slo: float = 0.1875, base_first_slo: float = 1.5):
    """n requests shaped like the paper's mixed trace (Sec. 3 setup and request features): Poisson
    arrivals at `rate` per second; prompt lengths 34 % in [10, 512], 52 % in [512, 4096], 14 %
    above (to max_prompt), outputs 51 % / 36 % / 13 % over the same ranges and cut at max_new
    (log-uniform inside a range); heterogeneous SLOs: the per-token SLO is 1, 2 or 4 times the
    reading speed of 0.1875 s/token, the first-token SLO the same multiple of base_first_slo.
    Returns a dict of arrays: arrival (s), prompt_len, max_new, slo_first, slo_token."""
    gaps = -np.log(_uniform01(n, seed * 16 + 1)) / rate
    arrival = np.cumsum(gaps)

    def lengths(cls_u, in_u, shares, cap):
        out = np.empty(n, dtype=np.int64)
        c0, c1 = shares
        small, mid = cls_u < c0, (cls_u >= c0) & (cls_u < c0 + c1)
        big = ~(small | mid)
        out[small] = _log_uniform_ints(in_u[small], 10, 512)
        out[mid] = _log_uniform_ints(in_u[mid], 512, 4096)
        out[big] = _log_uniform_ints(in_u[big], 4096, max(cap, 4097))
        return np.minimum(out, cap)

    prompt = lengths(_uniform01(n, seed * 16 + 2), _uniform01(n, seed * 16 + 3), (0.34, 0.52), max_prompt)
    new = lengths(_uniform01(n, seed * 16 + 4), _uniform01(n, seed * 16 + 5), (0.51, 0.36), max_new)
    mult = np.array([1.0, 2.0, 4.0])[(bits(n, seed * 16 + 6) % np.uint64(3)).astype(np.int64)]
    return {"arrival": arrival, "prompt_len": prompt, "max_new": new,
            "slo_first": base_first_slo * mult, "slo_token": base_token_slo * mult}


def token_rows(request_ids, positions, width: int, seed: int, dtype: str = "bf16") -> np.ndarray:
    """One row of `width` N(0,1) draws per (request, position) pair, a function of the pair alone:
    the content of a token of a scheduled request, whichever iteration or block it lands in."""
    rid = np.asarray(request_ids, dtype=np.uint64)
    pos = np.asarray(positions, dtype=np.uint64)
    offs = (rid * np.uint64(1 << 20) + pos) * np.uint64(width)
    return normal_bf16_segments(offs, width, seed, dtype)
