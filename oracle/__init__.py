"""ctypes loader for the fp64 CPU oracle (oracle/mpa_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's cpu_baseline
leg.  The product package never imports this module, and this module never imports the product.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmpa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "mpa_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", src, "-o", _LIB_PATH, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        p, i, d = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        lib.mpa_oracle_threads.restype = i
        lib.mpa_oracle_kv_append.argtypes = [p, p, p, i, i, i, i, p, p]
        lib.mpa_oracle_kv_append.restype = None
        lib.mpa_oracle_attention.argtypes = [p, p, p, p, i, p, p, i, i, i, i, i, d, i, p]
        lib.mpa_oracle_attention.restype = i
        lib.mpa_oracle_attention_rows.argtypes = [p, p, p, p, i, p, p, i, i, i, i, i, d, i, p, p, i, p]
        lib.mpa_oracle_widen.argtypes = [p, ctypes.c_int64, i, p]
        lib.mpa_oracle_widen.restype = None
        lib.mpa_oracle_attention_rows.restype = i
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().mpa_oracle_threads())


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def kv_append(k_new, v_new, slot_map, k_cache, v_cache):
    """In place on k_cache/v_cache ([NB,HK,bs,D] uint16, C-contiguous); k_new/v_new [T,HK,D]."""
    T, H, D = k_new.shape
    bs = k_cache.shape[2]
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    assert k_cache.dtype == np.uint16 and v_cache.dtype == np.uint16
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    slot_map = _c(slot_map, np.int64)
    _load().mpa_oracle_kv_append(k_new.ctypes.data, v_new.ctypes.data, slot_map.ctypes.data,
                                 T, H, D, bs, k_cache.ctypes.data, v_cache.ctypes.data)


def copy_blocks(src_k, src_v, dst_k, dst_v, pairs):
    """Whole-block copies between cache pools ([NB,HK,bs,D] uint16 each), in place on dst_k/dst_v:
    block pairs[i][1] of the destination becomes block pairs[i][0] of the source, K and V, all
    heads.  This is what moving a preempted request's blocks to another pool and back amounts to
    (the engine's handling of KVC overflow, paper Sec. 5).  Written as the definition: one
    assignment per pair, in order."""
    pairs = np.asarray(pairs, dtype=np.int64).reshape(-1, 2)
    assert src_k.shape[1:] == dst_k.shape[1:] and src_v.shape[1:] == dst_v.shape[1:]
    for s, d in pairs:
        dst_k[d] = src_k[s]
        dst_v[d] = src_v[s]


DTYPES = {"bf16": 1, "fp16": 2}


def widen(bits, dtype: str = "bf16") -> np.ndarray:
    """The float64 values of 16-bit patterns as the oracle reads them."""
    bits = _c(bits, np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().mpa_oracle_widen(ctypes.c_void_p(bits.ctypes.data), ctypes.c_int64(bits.size), DTYPES[dtype],
                             ctypes.c_void_p(out.ctypes.data))
    return out


def attention(q, k_cache, v_cache, block_table, chunk_starts, context_lens, scale, dtype: str = "bf16") -> np.ndarray:
    """Returns out [T,H,D] float64."""
    T, H, D = q.shape
    bs = k_cache.shape[2]
    q, k_cache, v_cache = _c(q, np.uint16), _c(k_cache, np.uint16), _c(v_cache, np.uint16)
    block_table = _c(block_table, np.int32)
    chunk_starts, context_lens = _c(chunk_starts, np.int32), _c(context_lens, np.int32)
    S = context_lens.size
    assert chunk_starts.size == S + 1 and int(chunk_starts[-1]) == T
    out = np.empty((T, H, D), dtype=np.float64)
    rc = _load().mpa_oracle_attention(q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data,
                                      block_table.ctypes.data, block_table.shape[1],
                                      chunk_starts.ctypes.data, context_lens.ctypes.data,
                                      S, H, k_cache.shape[1], D, bs, float(scale), DTYPES[dtype], out.ctypes.data)
    if rc != 0:
        raise ValueError("malformed batch")
    return out


def attention_rows(q, k_cache, v_cache, block_table, chunk_starts, context_lens, scale, rows, heads,
                   dtype: str = "bf16") -> np.ndarray:
    """Selected (row, head) pairs only; returns [n, D] float64."""
    T, H, D = q.shape
    bs = k_cache.shape[2]
    q, k_cache, v_cache = _c(q, np.uint16), _c(k_cache, np.uint16), _c(v_cache, np.uint16)
    block_table = _c(block_table, np.int32)
    chunk_starts, context_lens = _c(chunk_starts, np.int32), _c(context_lens, np.int32)
    rows, heads = _c(rows, np.int32), _c(heads, np.int32)
    S = context_lens.size
    out = np.empty((rows.size, D), dtype=np.float64)
    rc = _load().mpa_oracle_attention_rows(q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data,
                                           block_table.ctypes.data, block_table.shape[1],
                                           chunk_starts.ctypes.data, context_lens.ctypes.data,
                                           S, H, k_cache.shape[1], D, bs, float(scale), DTYPES[dtype], rows.ctypes.data,
                                           heads.ctypes.data, rows.size, out.ctypes.data)
    if rc != 0:
        raise ValueError("malformed batch or row list")
    return out
