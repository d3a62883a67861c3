"""Thin Python binding of libmpa.so (argument marshalling only; all compute is in the HIP library).

Device tensors are anything with a ``data_ptr()`` (torch tensors on the GPU); the host-side batch
description (chunk_starts, context_lens) is a numpy int32 array or a sequence of ints.  There is
no CPU fallback: if the library is missing, importing names from here raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmpa.so")

MPA_OK = 0
MPA_ERR_INVALID_ARG = -1
MPA_ERR_UNSUPPORTED = -2
MPA_ERR_WORKSPACE = -3
MPA_ERR_BAD_BATCH = -4
MPA_ERR_HIP = -5
MPA_ERR_NO_MEMORY = -6
MPA_BF16 = 1
MPA_FP16 = 2
MPA_OPT_TG_SPLIT_BLOCKS = 1
MPA_OPT_PP_SPLIT_TOKENS = 2
MPA_OPT_PP_ROWSTREAM = 3
MPA_OPT_PP_RESIDENT_WGS = 4
MPA_OPT_PP_TEAM_MIN_STEPS = 5
MPA_OPT_PLAN_CACHE = 6
MPA_OPT_PROFILE_EVERY = 7
MPA_OPT_STAGING_TIMEOUT_MS = 8
MPA_OPT_TEST_STUCK_UPLOAD = 9
MPA_OPT_TILE_MODE = 10
MPA_OPT_PROFILE_REPEAT = 11
MPA_OPT_FUSE_APPEND = 12
MPA_STATIC_SCRATCH_BYTES = 64 << 20
MPA_CEIL_STREAM_READ, MPA_CEIL_RANDOM_4K, MPA_CEIL_RANDOM_16K, MPA_CEIL_MFMA_BF16, MPA_CEIL_MFMA_BF16_NOISY = 1, 2, 3, 4, 5

MPA_ABI_VERSION = 3   # of include/mpa.h as this binding was written for it

EXPORTS = [
    "mpa_abi_version", "mpa_create", "mpa_destroy", "mpa_set_option", "mpa_last_hip_error", "mpa_status_string",
    "mpa_workspace_bytes_for_batch", "mpa_workspace_bytes", "mpa_kv_append", "mpa_copy_blocks", "mpa_append_and_attend",
    "mpa_mixed_paged_attention", "mpa_mixed_paged_attention_static", "mpa_plan_describe", "mpa_profile_enable", "mpa_profile_read", "mpa_ceiling_launch",
    "mpa_sched_create", "mpa_sched_destroy", "mpa_sched_add_request", "mpa_sched_add_offline_request", "mpa_sched_next_batch",
    "mpa_sched_batch_arrays", "mpa_sched_batch_swaps", "mpa_sched_complete", "mpa_sched_live_requests",
]


class MpaConfig(ctypes.Structure):
    _fields_ = [("num_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class SchedConfig(ctypes.Structure):
    _fields_ = [("block_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32),
                ("pivot_forward_size", ctypes.c_int32), ("max_batch_tokens", ctypes.c_int32),
                ("pivot_time", ctypes.c_double), ("max_batch_time", ctypes.c_double), ("gamma", ctypes.c_double),
                ("preempt_max_time", ctypes.c_double), ("preempt_probability", ctypes.c_double),
                ("num_swap_blocks", ctypes.c_int32)]


class SchedBatch(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("num_seqs", "num_tokens", "token_budget", "num_prompt_chunks",
                                              "num_generation", "num_preempted", "max_blocks_per_seq", "free_blocks",
                                              "num_swap_out", "num_swap_in")]


class MpaError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


_lib = None


def load() -> ctypes.CDLL:
    """Load libmpa.so (build it first with paper_2503_13737_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2503_13737_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        try:
            lib.mpa_abi_version.restype = ctypes.c_int
            built = int(lib.mpa_abi_version())
        except AttributeError:
            built = None
        if built != MPA_ABI_VERSION:
            raise ImportError(f"{LIB_PATH} was built from another version of include/mpa.h ({built}, this binding: "
                              f"{MPA_ABI_VERSION}); run `python -m paper_2503_13737_amd.build`")
        lib.mpa_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(MpaConfig)]
        lib.mpa_create.restype = ctypes.c_int
        lib.mpa_destroy.argtypes = [vp]
        lib.mpa_destroy.restype = ctypes.c_int
        lib.mpa_set_option.argtypes = [vp, i32, i64]
        lib.mpa_set_option.restype = ctypes.c_int
        lib.mpa_last_hip_error.argtypes = [vp]
        lib.mpa_last_hip_error.restype = ctypes.c_int
        lib.mpa_status_string.argtypes = [ctypes.c_int]
        lib.mpa_status_string.restype = ctypes.c_char_p
        lib.mpa_workspace_bytes_for_batch.argtypes = [vp, vp, vp, i32]
        lib.mpa_workspace_bytes_for_batch.restype = sz
        lib.mpa_workspace_bytes.argtypes = [vp, i32, i32, i32]
        lib.mpa_workspace_bytes.restype = sz
        lib.mpa_kv_append.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp]
        lib.mpa_kv_append.restype = ctypes.c_int
        lib.mpa_copy_blocks.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp]
        lib.mpa_copy_blocks.restype = ctypes.c_int
        lib.mpa_mixed_paged_attention.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, i32, i32,
                                                  ctypes.c_float, vp, vp, sz, vp]
        lib.mpa_mixed_paged_attention.restype = ctypes.c_int
        lib.mpa_mixed_paged_attention_static.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, i32, i32,
                                                         ctypes.c_float, vp, vp]
        lib.mpa_mixed_paged_attention_static.restype = ctypes.c_int
        lib.mpa_append_and_attend.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i32, i32,
                                              ctypes.c_float, vp, vp, sz, vp]
        lib.mpa_append_and_attend.restype = ctypes.c_int
        lib.mpa_profile_enable.argtypes = [vp, i32]
        lib.mpa_profile_enable.restype = ctypes.c_int
        lib.mpa_profile_read.argtypes = [vp, vp, i32, vp]
        lib.mpa_profile_read.restype = ctypes.c_int
        lib.mpa_ceiling_launch.argtypes = [i32, vp, sz, i32, vp, vp]
        lib.mpa_ceiling_launch.restype = i64
        lib.mpa_plan_describe.argtypes = [vp, vp, vp, i32, vp, i64, vp]
        lib.mpa_plan_describe.restype = i64
        f64 = ctypes.c_double
        lib.mpa_sched_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(SchedConfig), vp]
        lib.mpa_sched_create.restype = ctypes.c_int
        lib.mpa_sched_destroy.argtypes = [vp]
        lib.mpa_sched_destroy.restype = ctypes.c_int
        lib.mpa_sched_add_request.argtypes = [vp, i64, i32, i32, f64, f64, f64]
        lib.mpa_sched_add_request.restype = ctypes.c_int
        lib.mpa_sched_add_offline_request.argtypes = [vp, i64, i32, i32, i32, f64, f64]
        lib.mpa_sched_add_offline_request.restype = ctypes.c_int
        lib.mpa_sched_next_batch.argtypes = [vp, f64, ctypes.POINTER(SchedBatch)]
        lib.mpa_sched_next_batch.restype = ctypes.c_int
        lib.mpa_sched_batch_arrays.argtypes = [vp, vp, vp, vp, vp, vp, i32]
        lib.mpa_sched_batch_arrays.restype = ctypes.c_int
        lib.mpa_sched_batch_swaps.argtypes = [vp, vp, vp]
        lib.mpa_sched_batch_swaps.restype = ctypes.c_int
        lib.mpa_sched_complete.argtypes = [vp, f64, vp, i32, vp]
        lib.mpa_sched_complete.restype = ctypes.c_int
        lib.mpa_sched_live_requests.argtypes = [vp]
        lib.mpa_sched_live_requests.restype = i32
        _lib = lib
    return _lib


def ceiling_launch(kind: int, buf, nbytes: int, iters: int, sink, stream=None) -> int:
    """One launch of a ceiling micro-kernel (see include/mpa.h); returns its bytes or flops."""
    work = load().mpa_ceiling_launch(int(kind), _ptr(buf), int(nbytes), int(iters), _ptr(sink), _stream_ptr(stream))
    if work < 0:
        raise MpaError(int(work), "mpa_ceiling_launch")
    return int(work)


def status_string(status: int) -> str:
    return load().mpa_status_string(int(status)).decode()


def _ptr(t):
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return ctypes.c_void_p(t.data_ptr())
    if isinstance(t, np.ndarray):
        return ctypes.c_void_p(t.ctypes.data)
    return ctypes.c_void_p(int(t))


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


class Context:
    """Owns an mpa_ctx for one cache geometry."""

    def __init__(self, num_heads: int, head_dim: int, block_size: int = 16, num_kv_heads: int | None = None,
                 dtype: int = MPA_BF16):
        cfg = MpaConfig(num_heads, num_heads if num_kv_heads is None else num_kv_heads, head_dim,
                        block_size, dtype)
        h = ctypes.c_void_p()
        rc = load().mpa_create(ctypes.byref(h), ctypes.byref(cfg))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_create")
        self._h = h
        self.num_heads, self.head_dim, self.block_size = num_heads, head_dim, block_size

    def close(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.mpa_destroy(h)

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: module globals may already be gone
            pass

    def set_option(self, option: int, value: int):
        rc = load().mpa_set_option(self._h, option, value)
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_set_option")

    def last_hip_error(self) -> int:
        return load().mpa_last_hip_error(self._h)

    def profile_enable(self, max_calls: int):
        rc = load().mpa_profile_enable(self._h, int(max_calls))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_profile_enable")

    def profile_read(self, cap: int = 4096) -> np.ndarray:
        """Milliseconds the main attention kernel took in each profiled call."""
        ms = np.zeros(cap, dtype=np.float32)
        n = ctypes.c_int32(0)
        rc = load().mpa_profile_read(self._h, _ptr(ms), cap, ctypes.byref(n))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_profile_read")
        return ms[: n.value].copy()

    def workspace_bytes_for_batch(self, chunk_starts, context_lens) -> int:
        cs, cl = _host_i32(chunk_starts), _host_i32(context_lens)
        return int(load().mpa_workspace_bytes_for_batch(self._h, _ptr(cs), _ptr(cl), cl.size))

    def workspace_bytes(self, max_seqs: int, max_tokens: int, max_ctx: int) -> int:
        return int(load().mpa_workspace_bytes(self._h, max_seqs, max_tokens, max_ctx))

    def plan_describe(self, chunk_starts, context_lens):
        """(items [n,8] int32, counts [4] int32) — host-only view of the work list."""
        cs, cl = _host_i32(chunk_starts), _host_i32(context_lens)
        counts = np.zeros(4, dtype=np.int32)
        n = load().mpa_plan_describe(self._h, _ptr(cs), _ptr(cl), cl.size, None, 0, _ptr(counts))
        if n < 0:
            raise MpaError(int(n), "mpa_plan_describe")
        items = np.zeros((max(int(n), 1), 8), dtype=np.int32)
        load().mpa_plan_describe(self._h, _ptr(cs), _ptr(cl), cl.size, _ptr(items), int(n), _ptr(counts))
        return items[: int(n)], counts

    def kv_append(self, k_new, v_new, slot_map, k_cache, v_cache, stream=None, num_tokens=None):
        n = int(k_new.shape[0]) if num_tokens is None else int(num_tokens)
        rc = load().mpa_kv_append(self._h, _ptr(k_new), _ptr(v_new), _ptr(slot_map), n,
                                  _ptr(k_cache), _ptr(v_cache), _stream_ptr(stream))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_kv_append")

    def copy_blocks(self, src_k, src_v, dst_k, dst_v, pairs, stream=None, num_pairs=None):
        n = int(pairs.shape[0]) if num_pairs is None else int(num_pairs)
        rc = load().mpa_copy_blocks(self._h, _ptr(src_k), _ptr(src_v), _ptr(dst_k), _ptr(dst_v), _ptr(pairs), n,
                                    _stream_ptr(stream))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_copy_blocks")

    def mixed_paged_attention(self, q, k_cache, v_cache, block_table, chunk_starts, context_lens, out,
                              workspace, scale: float = 0.0, stream=None, block_table_stride=None,
                              workspace_bytes=None):
        cs, cl = _host_i32(chunk_starts), _host_i32(context_lens)
        stride = int(block_table.shape[1]) if block_table_stride is None else int(block_table_stride)
        wsb = (int(workspace.numel() * workspace.element_size()) if workspace_bytes is None
               else int(workspace_bytes))
        rc = load().mpa_mixed_paged_attention(
            self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table), stride, _ptr(cs), _ptr(cl),
            cl.size, int(q.shape[0]), float(scale), _ptr(out), _ptr(workspace), wsb, _stream_ptr(stream))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_mixed_paged_attention")

    def mixed_paged_attention_static(self, q, k_cache, v_cache, block_table, chunk_starts, context_lens, out,
                                     scale: float = 0.0, stream=None, block_table_stride=None):
        """The form that allocates nothing and takes no workspace (the library's own device array)."""
        cs, cl = _host_i32(chunk_starts), _host_i32(context_lens)
        stride = int(block_table.shape[1]) if block_table_stride is None else int(block_table_stride)
        rc = load().mpa_mixed_paged_attention_static(
            self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table), stride, _ptr(cs), _ptr(cl),
            cl.size, int(q.shape[0]), float(scale), _ptr(out), _stream_ptr(stream))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_mixed_paged_attention_static")

    def append_and_attend(self, k_new, v_new, slot_map, q, k_cache, v_cache, block_table, chunk_starts, context_lens,
                          out, workspace, scale: float = 0.0, stream=None, block_table_stride=None,
                          workspace_bytes=None):
        cs, cl = _host_i32(chunk_starts), _host_i32(context_lens)
        stride = int(block_table.shape[1]) if block_table_stride is None else int(block_table_stride)
        wsb = (int(workspace.numel() * workspace.element_size()) if workspace_bytes is None
               else int(workspace_bytes))
        rc = load().mpa_append_and_attend(
            self._h, _ptr(k_new), _ptr(v_new), _ptr(slot_map), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
            stride, _ptr(cs), _ptr(cl), cl.size, int(q.shape[0]), float(scale), _ptr(out), _ptr(workspace), wsb,
            _stream_ptr(stream))
        if rc != MPA_OK:
            raise MpaError(rc, "mpa_append_and_attend")


def _stream_ptr(stream):
    if stream is None:
        try:
            import torch
            if torch.cuda.is_available():
                return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        except ImportError:
            pass
        return None
    if hasattr(stream, "cuda_stream"):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


# module-level functions with the names of the C entry points
def kv_append(ctx: Context, k_new, v_new, slot_map, k_cache, v_cache, stream=None):
    ctx.kv_append(k_new, v_new, slot_map, k_cache, v_cache, stream)


def mixed_paged_attention(ctx: Context, q, k_cache, v_cache, block_table, chunk_starts, context_lens, out,
                          workspace, scale: float = 0.0, stream=None):
    ctx.mixed_paged_attention(q, k_cache, v_cache, block_table, chunk_starts, context_lens, out, workspace,
                              scale, stream)


class Scheduler:
    """Owns an mpa_sched (include/mpa_sched.h): forms the batch of every iteration and returns the
    arrays mpa_kv_append / mpa_mixed_paged_attention take.  Host only."""

    def __init__(self, block_size: int, num_blocks: int, pivot_forward_size: int, pivot_time: float,
                 max_batch_time: float, gamma: float, max_batch_tokens: int, block_order=None,
                 preempt_max_time: float = 0.0, preempt_probability: float = 0.0, swap_blocks: int = 0):
        self._lib = load()
        self._h = ctypes.c_void_p()
        cfg = SchedConfig(block_size, num_blocks, pivot_forward_size, max_batch_tokens, pivot_time, max_batch_time, gamma,
                          preempt_max_time, preempt_probability, swap_blocks)
        order = None if block_order is None else _host_i32(block_order)
        if order is not None and order.size != num_blocks:
            raise MpaError(MPA_ERR_INVALID_ARG, "mpa_sched_create")
        st = self._lib.mpa_sched_create(ctypes.byref(self._h), ctypes.byref(cfg), _ptr(order))
        if st != MPA_OK:
            raise MpaError(st, "mpa_sched_create")
        self.info = SchedBatch()

    def close(self):
        if self._h:
            self._lib.mpa_sched_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def add_request(self, rid: int, prompt_len: int, max_new_tokens: int, slo_first: float, slo_token: float, now: float):
        st = self._lib.mpa_sched_add_request(self._h, rid, prompt_len, max_new_tokens, slo_first, slo_token, now)
        if st != MPA_OK:
            raise MpaError(st, "mpa_sched_add_request")

    def add_offline_request(self, rid: int, prompt_len: int, max_new_tokens: int, predicted_new_tokens: int,
                            slo_jct: float, now: float):
        st = self._lib.mpa_sched_add_offline_request(self._h, rid, prompt_len, max_new_tokens, predicted_new_tokens,
                                                     slo_jct, now)
        if st != MPA_OK:
            raise MpaError(st, "mpa_sched_add_offline_request")

    def next_batch(self, now: float) -> SchedBatch:
        st = self._lib.mpa_sched_next_batch(self._h, now, ctypes.byref(self.info))
        if st != MPA_OK:
            raise MpaError(st, "mpa_sched_next_batch")
        return self.info

    def batch_arrays(self, stride: int | None = None):
        """(request_ids [S] int64, chunk_starts [S+1] int32, context_lens [S] int32, slot_map [T] int64,
        block_table [S, stride] int32) of the batch formed last."""
        i = self.info
        stride = max(i.max_blocks_per_seq, 1) if stride is None else stride
        ids = np.empty(i.num_seqs, dtype=np.int64)
        cs = np.empty(i.num_seqs + 1, dtype=np.int32)
        ctx = np.empty(i.num_seqs, dtype=np.int32)
        slots = np.empty(i.num_tokens, dtype=np.int64)
        table = np.empty((i.num_seqs, stride), dtype=np.int32)
        st = self._lib.mpa_sched_batch_arrays(self._h, _ptr(ids), _ptr(cs), _ptr(ctx), _ptr(slots), _ptr(table), stride)
        if st != MPA_OK:
            raise MpaError(st, "mpa_sched_batch_arrays")
        return ids, cs, ctx, slots, table

    def batch_swaps(self):
        """(out_pairs [n,2], in_pairs [m,2]) int64 {source, destination} block pairs for mpa_copy_blocks: out of
        the cache pool into the swap pool, and back in; both before the iteration's append, out first."""
        out = np.empty((self.info.num_swap_out, 2), dtype=np.int64)
        inn = np.empty((self.info.num_swap_in, 2), dtype=np.int64)
        st = self._lib.mpa_sched_batch_swaps(self._h, _ptr(out), _ptr(inn))
        if st != MPA_OK:
            raise MpaError(st, "mpa_sched_batch_swaps")
        return out, inn

    def complete(self, now: float) -> np.ndarray:
        cap = max(self.info.num_seqs, 1)
        out = np.empty(cap, dtype=np.int64)
        n = ctypes.c_int32(0)
        st = self._lib.mpa_sched_complete(self._h, now, _ptr(out), cap, ctypes.byref(n))
        if st != MPA_OK:
            raise MpaError(st, "mpa_sched_complete")
        return out[: n.value].copy()

    @property
    def live_requests(self) -> int:
        return int(self._lib.mpa_sched_live_requests(self._h))
