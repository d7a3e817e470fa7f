"""CPU oracle of the walk -> RPE -> join path.  TEST INFRASTRUCTURE ONLY.

``surel_oracle.c`` is the oracle; this file compiles it with gcc and exposes it
to NumPy through ctypes.  Only tests, the smoke check and the benchmark's
cpu_baseline leg import this package; the HIP library and its Python binding
never do, and nothing here imports them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "surel_oracle.c")
_LIB = os.path.join(_HERE, "libsurel_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
                        "-o", tmp, _SRC], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        lib.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_sample_walks.argtypes = [i32p, i32p, ctypes.c_int32, i32p, ctypes.c_int64,
                                            ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64,
                                            i32p]
        lib.oracle_sample_walks.restype = ctypes.c_int
        lib.oracle_build_rpe.argtypes = [i32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int64, i64p, i32p, u16p]
        lib.oracle_build_rpe.restype = ctypes.c_int64
        lib.oracle_join_queries.argtypes = [i64p, i32p, u16p, ctypes.c_int64, ctypes.c_int32,
                                            i32p, ctypes.c_int64, ctypes.c_int32,
                                            ctypes.c_int64, i64p, i32p, u16p]
        lib.oracle_join_queries.restype = ctypes.c_int64
        lib.oracle_query_rpe_ids.argtypes = [i32p, i64p, i32p, ctypes.c_int64, ctypes.c_int32,
                                             ctypes.c_int32, i32p, ctypes.c_int64,
                                             ctypes.c_int32, i64p]
        lib.oracle_query_rpe_ids.restype = ctypes.c_int
        lib.oracle_prune_rpe.argtypes = [u16p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64,
                                         u16p, i32p]
        lib.oracle_prune_rpe.restype = ctypes.c_int64
        lib.oracle_bfs_batch.argtypes = [i32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                         i32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         i32p, i32p, i64p]
        lib.oracle_bfs_batch.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a, ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _arr(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def philox4x32_10(ctr, key) -> np.ndarray:
    """Four output words for a counter of four and a key of two uint32 words."""
    c = _arr(ctr, np.uint32)
    k = _arr(key, np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(c, ctypes.c_uint32), _ptr(k, ctypes.c_uint32),
                                 _ptr(out, ctypes.c_uint32))
    return out


def sample_walks(row_ptr, col_idx, seeds, M: int, m: int, rng_seed: int = 0) -> np.ndarray:
    """walks int32[n_seeds][M][m+1]; position 0 of every walk is its seed."""
    row_ptr = _arr(row_ptr, np.int32)
    col_idx = _arr(col_idx, np.int32)
    seeds = _arr(seeds, np.int32)
    n_nodes = row_ptr.size - 1
    walks = np.empty((seeds.size, M, m + 1), dtype=np.int32)
    rc = _load().oracle_sample_walks(_ptr(row_ptr, ctypes.c_int32),
                                     _ptr(col_idx, ctypes.c_int32), n_nodes,
                                     _ptr(seeds, ctypes.c_int32), seeds.size, M, m,
                                     ctypes.c_uint64(rng_seed), _ptr(walks, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_sample_walks failed with {rc}")
    return walks


def build_rpe(walks):
    """(rpe_off int64[n_seeds+1], rpe_ids int32[R], rpe_cnt uint16[R][m+1])."""
    walks = _arr(walks, np.int32)
    n_seeds, M, L = walks.shape
    m = L - 1
    off = np.zeros(n_seeds + 1, dtype=np.int64)
    lib = _load()
    rows = lib.oracle_build_rpe(_ptr(walks, ctypes.c_int32), n_seeds, M, m, 0,
                                _ptr(off, ctypes.c_int64), _ptr(None, ctypes.c_int32),
                                _ptr(None, ctypes.c_uint16))
    if rows < 0:
        raise ValueError(f"oracle_build_rpe failed with {rows}")
    ids = np.empty(rows, dtype=np.int32)
    cnt = np.empty((rows, L), dtype=np.uint16)
    rows2 = lib.oracle_build_rpe(_ptr(walks, ctypes.c_int32), n_seeds, M, m, rows,
                                 _ptr(off, ctypes.c_int64), _ptr(ids, ctypes.c_int32),
                                 _ptr(cnt, ctypes.c_uint16))
    if rows2 != rows:
        raise ValueError(f"oracle_build_rpe failed with {rows2}")
    return off, ids, cnt


def join_queries(rpe_off, rpe_ids, rpe_cnt, queries):
    """(join_off int64[n_q+1], join_ids int32[J], join_cnt uint16[J][k][m+1])."""
    rpe_off = _arr(rpe_off, np.int64)
    rpe_ids = _arr(rpe_ids, np.int32)
    rpe_cnt = _arr(rpe_cnt, np.uint16)
    queries = _arr(queries, np.int32)
    n_q, k = queries.shape
    L = rpe_cnt.shape[1]
    m = L - 1
    n_blocks = rpe_off.size - 1
    off = np.zeros(n_q + 1, dtype=np.int64)
    lib = _load()
    args = (_ptr(rpe_off, ctypes.c_int64), _ptr(rpe_ids, ctypes.c_int32),
            _ptr(rpe_cnt, ctypes.c_uint16), n_blocks, m, _ptr(queries, ctypes.c_int32), n_q, k)
    rows = lib.oracle_join_queries(*args, 0, _ptr(off, ctypes.c_int64),
                                   _ptr(None, ctypes.c_int32), _ptr(None, ctypes.c_uint16))
    if rows < 0:
        raise ValueError(f"oracle_join_queries failed with {rows}")
    ids = np.empty(rows, dtype=np.int32)
    cnt = np.empty((rows, k, L), dtype=np.uint16)
    rows2 = lib.oracle_join_queries(*args, rows, _ptr(off, ctypes.c_int64),
                                    _ptr(ids, ctypes.c_int32), _ptr(cnt, ctypes.c_uint16))
    if rows2 != rows:
        raise ValueError(f"oracle_join_queries failed with {rows2}")
    return off, ids, cnt


def query_rpe_ids(walks, rpe_off, rpe_ids, queries) -> np.ndarray:
    """int64[n_q][k][M][m+1][k]: for every node occurrence in the concatenated walks of a
    query, the table rows of that node in each of the query's blocks (-1 where absent)."""
    walks = _arr(walks, np.int32)
    rpe_off = _arr(rpe_off, np.int64)
    rpe_ids = _arr(rpe_ids, np.int32)
    queries = _arr(queries, np.int32)
    n_blocks, M, L = walks.shape
    assert rpe_off.size == n_blocks + 1
    n_q, k = queries.shape
    out = np.empty((n_q, k, M, L, k), dtype=np.int64)
    rc = _load().oracle_query_rpe_ids(_ptr(walks, ctypes.c_int32), _ptr(rpe_off, ctypes.c_int64),
                                      _ptr(rpe_ids, ctypes.c_int32), n_blocks, M, L - 1,
                                      _ptr(queries, ctypes.c_int32), n_q, k,
                                      _ptr(out, ctypes.c_int64))
    if rc != 0:
        raise ValueError(f"oracle_query_rpe_ids failed with {rc}")
    return out


def prune_rpe(rpe_cnt):
    """(T uint16[n_T][m+1], code int32[R]): the distinct count vectors in ascending order and,
    for every table row, the index of its vector in T."""
    rpe_cnt = _arr(rpe_cnt, np.uint16)
    n_rows, L = rpe_cnt.shape
    lib = _load()
    n_T = lib.oracle_prune_rpe(_ptr(rpe_cnt, ctypes.c_uint16), n_rows, L - 1, 0,
                               _ptr(None, ctypes.c_uint16), _ptr(None, ctypes.c_int32))
    if n_T < 0:
        raise ValueError(f"oracle_prune_rpe failed with {n_T}")
    T = np.empty((n_T, L), dtype=np.uint16)
    code = np.empty(n_rows, dtype=np.int32)
    n2 = lib.oracle_prune_rpe(_ptr(rpe_cnt, ctypes.c_uint16), n_rows, L - 1, n_T,
                              _ptr(T, ctypes.c_uint16), _ptr(code, ctypes.c_int32))
    if n2 != n_T:
        raise ValueError(f"oracle_prune_rpe failed with {n2}")
    return T, code


def bfs_batch(queries, n_nodes: int, start, B1: int, B2: int):
    """(vbar int32[<=B1], batch int32[<=B2]): the node set and the queries that a breadth-first
    search from the seed-set `start` over query-sharing nodes reaches, each in the order reached,
    until the node set has B1 members or the batch B2."""
    queries = _arr(queries, np.int32)
    if queries.ndim != 2:
        raise ValueError("queries must be int32[n_queries][k]")
    start = _arr(start, np.int32).reshape(-1)
    vbar = np.empty(max(B1, 1), dtype=np.int32)
    batch = np.empty(max(B2, 1), dtype=np.int32)
    counts = np.zeros(2, dtype=np.int64)
    rc = _load().oracle_bfs_batch(_ptr(queries, ctypes.c_int32), queries.shape[0],
                                  queries.shape[1], n_nodes, _ptr(start, ctypes.c_int32),
                                  start.shape[0], B1, B2, _ptr(vbar, ctypes.c_int32),
                                  _ptr(batch, ctypes.c_int32), _ptr(counts, ctypes.c_int64))
    if rc != 0:
        raise ValueError(f"oracle_bfs_batch failed with {rc}")
    return vbar[:counts[0]].copy(), batch[:counts[1]].copy()
