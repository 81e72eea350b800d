"""CPU oracle (fp64) for the paged-KV decode path.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``kvc_oracle.c`` (plain C, built with gcc).  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the product path never does, and this
package never imports the product.

The definitions (block-structured KV cache: paper Section 1 and 3.3.1; swap as a
move of a request's KV values out and back: Section 2.5 and 3.5) are written
out in ``kvc_oracle.c``; this file only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvc_oracle.c")
# KVC_ORACLE_LIBRARY points at another build of the same source (the sanitizer run of the tests)
_LIB = os.environ.get("KVC_ORACLE_LIBRARY") or os.path.join(_HERE, "libkvc_oracle.so")
_DT = {"f32": 0, "bf16": 1, "f64": 2}
_NP = {"f32": np.float32, "bf16": np.uint16, "f64": np.float64}
_lib = None


def build(force: bool = False, out: Optional[str] = None, extra_flags: Sequence[str] = ()) -> str:
    """Compile the oracle with gcc (about a second) when the library is missing or older than
    its source.  Starts a child process: call it before anything in the process touches the GPU.
    `out` / `extra_flags` build a variant elsewhere (e.g. with sanitizers) and leave _LIB alone."""
    target = out or _LIB
    if out is None and os.environ.get("KVC_ORACLE_LIBRARY"):
        return target                  # a library somebody else built: used as it is
    if force or not os.path.exists(target) or os.path.getmtime(target) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", *extra_flags,
                               "-o", target, _SRC, "-lm"])
    return target


def _load():
    global _lib
    if _lib is None:
        # an existing library is loaded as it is; only a missing one is compiled here
        lib = ctypes.CDLL(_LIB if os.path.exists(_LIB) else build())
        lib.oracle_paged_attention_decode.restype = ctypes.c_int
        lib.oracle_paged_attention_decode.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_double, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int]
        lib.oracle_kv_block_copy.restype = ctypes.c_int
        lib.oracle_kv_block_copy.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_kv_cache_append.restype = ctypes.c_int
        lib.oracle_kv_cache_append.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64]
        lib.oracle_paged_attention_prefill.restype = ctypes.c_int
        lib.oracle_paged_attention_prefill.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_num_threads_available.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads_available() -> int:
    return int(_load().oracle_num_threads_available())


def paged_attention_decode(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                           block_tables: np.ndarray, context_lens: np.ndarray, scale: float,
                           *, dtype: str, rows: Optional[Sequence] = None,
                           num_threads: int = 1) -> np.ndarray:
    """softmax(q K^T scale) V over each sequence's block list, in fp64.

    q [num_seqs][Hq][D]; k_cache, v_cache [NB][Hkv][Bs][D]; block_tables
    [num_seqs][Lmax] int32; context_lens [num_seqs] int32.  ``dtype`` names the
    storage of q/k/v: "f32", "bf16" (uint16 bit patterns) or "f64".
    Returns float64 [num_seqs][Hq][D]; with ``rows`` (pairs (seq, head)) only
    those rows are computed and the rest are NaN.
    """
    lib = _load()
    npdt = _NP[dtype]
    q = np.ascontiguousarray(q, dtype=npdt)
    k_cache = np.ascontiguousarray(k_cache, dtype=npdt)
    v_cache = np.ascontiguousarray(v_cache, dtype=npdt)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    context_lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    nseq, hq, d = q.shape
    nb, hkv, bs, d2 = k_cache.shape
    assert d2 == d and v_cache.shape == k_cache.shape
    assert block_tables.shape[0] == nseq and context_lens.shape == (nseq,)
    lmax = block_tables.shape[1]
    # the oracle trusts its tables only after checking them here
    nblk = (context_lens.astype(np.int64) + bs - 1) // bs
    for n in range(nseq):
        used = block_tables[n, :nblk[n]]
        if used.size and (used.min() < 0 or used.max() >= nb):
            raise ValueError(f"sequence {n}: block id outside the pool")
    out = np.full((nseq, hq, d), np.nan, dtype=np.float64)
    rows_arr = None
    n_rows = 0
    if rows is not None:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 2))
        n_rows = rows_arr.shape[0]
    rc = lib.oracle_paged_attention_decode(
        q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data, block_tables.ctypes.data,
        context_lens.ctypes.data, float(scale), out.ctypes.data, _DT[dtype], nseq, hq, hkv, d,
        bs, lmax, rows_arr.ctypes.data if rows_arr is not None else None, n_rows,
        int(num_threads))
    if rc != 0:
        raise ValueError("oracle_paged_attention_decode rejected its arguments")
    return out


def attention_of_workload(w, *, rows=None, num_threads: int = 1) -> np.ndarray:
    """Convenience: run the oracle on a kvc_workloads.PagedWorkload."""
    return paged_attention_decode(w.q, w.k_cache, w.v_cache, w.block_tables, w.context_lens,
                                  w.scale, dtype=w.dtype, rows=rows, num_threads=num_threads)


def kv_block_copy(src_pool: np.ndarray, dst_pool: np.ndarray, block_mapping: np.ndarray) -> None:
    """dst[plane][d] = src[plane][s] for every (s, d) in block_mapping, bytewise, in place.

    Pools are arrays shaped [num_planes][num_blocks][...] (any dtype); everything
    after the first two axes is one block's payload.
    """
    lib = _load()
    assert src_pool.flags.c_contiguous and dst_pool.flags.c_contiguous
    assert dst_pool.flags.writeable
    planes, sb = src_pool.shape[:2]
    planes2, db = dst_pool.shape[:2]
    assert planes == planes2
    block_bytes = src_pool[0, 0].nbytes
    assert dst_pool[0, 0].nbytes == block_bytes
    mapping = np.ascontiguousarray(block_mapping, dtype=np.int64).reshape(-1, 2)
    rc = lib.oracle_kv_block_copy(src_pool.ctypes.data, dst_pool.ctypes.data, block_bytes, planes,
                                  sb * block_bytes, db * block_bytes, sb, db,
                                  mapping.ctypes.data, mapping.shape[0])
    if rc != 0:
        raise ValueError("block id outside the pool")


def kv_cache_append(k_new: np.ndarray, v_new: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                    block_tables: np.ndarray, positions: np.ndarray) -> None:
    """cache[table[n][pos // Bs]][h][pos % Bs] = new[n][h] for K and V, in place, bytewise.

    k_new, v_new [num_seqs][Hkv][D]; caches [NB][Hkv][Bs][D] (same dtype); positions int32
    [num_seqs], negative = skip.
    """
    lib = _load()
    for a in (k_new, v_new, k_cache, v_cache):
        assert a.flags.c_contiguous
    assert k_cache.flags.writeable and v_cache.flags.writeable
    nseq, hkv, d = k_new.shape
    nb, hkv2, bs, d2 = k_cache.shape
    assert (hkv2, d2) == (hkv, d) and v_new.shape == k_new.shape and v_cache.shape == k_cache.shape
    assert k_new.dtype == k_cache.dtype == v_new.dtype == v_cache.dtype
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    positions = np.ascontiguousarray(positions, dtype=np.int32)
    rc = lib.oracle_kv_cache_append(k_new.ctypes.data, v_new.ctypes.data, k_cache.ctypes.data,
                                    v_cache.ctypes.data, block_tables.ctypes.data,
                                    positions.ctypes.data, nseq, hkv, d * k_new.itemsize, bs,
                                    block_tables.shape[1], nb)
    if rc != 0:
        raise ValueError("position or block id out of range")


def paged_attention_prefill(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                            block_tables: np.ndarray, context_lens: np.ndarray, q_start: np.ndarray,
                            scale: float, *, dtype: str, num_threads: int = 1) -> np.ndarray:
    """Causal attention of the last Qn = q_start[n+1]-q_start[n] positions of every sequence over
    its block list, in fp64.  q [total_q][Hq][D]; returns float64 [total_q][Hq][D]."""
    lib = _load()
    npdt = _NP[dtype]
    q = np.ascontiguousarray(q, dtype=npdt)
    k_cache = np.ascontiguousarray(k_cache, dtype=npdt)
    v_cache = np.ascontiguousarray(v_cache, dtype=npdt)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    context_lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    q_start = np.ascontiguousarray(q_start, dtype=np.int32)
    total_q, hq, d = q.shape
    nb, hkv, bs, d2 = k_cache.shape
    nseq = context_lens.shape[0]
    assert d2 == d and v_cache.shape == k_cache.shape and q_start.shape == (nseq + 1,)
    assert q_start[0] == 0 and q_start[-1] == total_q
    nblk = (context_lens.astype(np.int64) + bs - 1) // bs
    for n in range(nseq):
        used = block_tables[n, :nblk[n]]
        if used.size and (used.min() < 0 or used.max() >= nb):
            raise ValueError(f"sequence {n}: block id outside the pool")
    out = np.zeros((total_q, hq, d), dtype=np.float64)
    rc = lib.oracle_paged_attention_prefill(
        q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data, block_tables.ctypes.data,
        context_lens.ctypes.data, q_start.ctypes.data, float(scale), out.ctypes.data, _DT[dtype],
        nseq, hq, hkv, d, bs, block_tables.shape[1], int(num_threads))
    if rc != 0:
        raise ValueError("oracle_paged_attention_prefill rejected its arguments")
    return out
