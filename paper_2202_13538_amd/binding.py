"""ctypes binding of libsurel's C ABI (see include/surel.h).

Argument marshalling only: tensors are passed as raw device pointers, outputs are allocated
with torch, and every step of the path runs in the library's HIP kernels.  There is no CPU
fallback: if ``libsurel.so`` has not been built, ``load()`` raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libsurel.so")

OK, E_NULL, E_RANGE, E_HIP, E_CAPACITY, E_CTX, E_DEVICE = 0, -1, -2, -3, -4, -5, -6
DEV_BAD_SEED, DEV_BAD_GRAPH, DEV_BAD_WALK, DEV_BAD_QUERY = 0x01, 0x02, 0x04, 0x08
DEV_SET_TOO_LARGE, DEV_CAPACITY, DEV_BAD_TABLE, DEV_BAD_SIZES = 0x10, 0x20, 0x40, 0x80
DEV_STALL = 0x100
MAX_NODES, MAX_STEPS, MAX_WALKS = 268435455, 15, 65535
MAX_WALK_ENTRIES, MAX_SET, MAX_TUPLE = 2048, 2048, 3
MAX_DISTINCT = 1 << 24
MAX_BATCH = 1 << 20
NOALLOC_MAX_QUERIES = 1 << 20

(K_WALK, K_RPE_COUNT, K_RPE_FILL, K_JOIN_COUNT, K_JOIN_FILL, K_SCAN, K_WALK_RPE,
 K_EDGE_RECORDS, K_QUERY_IDS, K_PRUNE, K_BATCH, K_COUNT) = range(12)
KERNEL_NAMES = {K_WALK: "walk", K_RPE_COUNT: "rpe_count", K_RPE_FILL: "rpe_fill",
                K_JOIN_COUNT: "join_count", K_JOIN_FILL: "join_fill", K_SCAN: "scan",
                K_WALK_RPE: "walk_rpe", K_EDGE_RECORDS: "edge_records",
                K_QUERY_IDS: "query_ids", K_PRUNE: "prune", K_BATCH: "batch"}

_vp = ctypes.c_void_p
_i32, _i64, _u64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64

# name -> (restype, argtypes); the order and types of include/surel.h
SIGNATURES = {
    "surel_create": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.c_int, _vp]),
    "surel_destroy": (None, [_vp]),
    "surel_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "surel_rpe_rows_bound": (_i64, [_i64, _i32, _i32]),
    "surel_sample_walks": (ctypes.c_int, [_vp, _vp, _vp, _i32, _i64, _vp, _i64, _i32, _i32,
                                          _u64, _vp, _vp]),
    "surel_build_rpe": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _i64, _vp, _vp,
                                       _vp, ctypes.POINTER(_i64)]),
    "surel_build_rpe_count": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp,
                                             ctypes.POINTER(_i64)]),
    "surel_build_rpe_fill": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _i64, _vp, _vp]),
    "surel_sample_walks_rpe": (ctypes.c_int, [_vp, _vp, _vp, _i32, _i64, _vp, _i64, _i32, _i32,
                                              _u64, _vp, _i64, _vp, _vp, _vp,
                                              ctypes.POINTER(_i64)]),
    "surel_sample_walks_rpe_ids": (ctypes.c_int, [_vp, _vp, _vp, _i32, _i64, _vp, _i64, _i32, _i32,
                                                  _u64, _vp, _i64, _vp, _vp, _vp, _vp, _i64, _vp,
                                                  ctypes.POINTER(_i64), ctypes.POINTER(_i64)]),
    "surel_join_queries": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i64, _i32,
                                          _i64, _vp, _vp, _vp, ctypes.POINTER(_i64)]),
    "surel_join_queries_noalloc": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i64,
                                                  _i32, _i64, _vp, _vp, _vp, ctypes.POINTER(_i64)]),
    "surel_join_count": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i32, _vp, _i64, _i32, _vp,
                                        ctypes.POINTER(_i64)]),
    "surel_join_fill": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i64, _i32, _vp,
                                       _i64, _vp, _vp]),
    "surel_join_query_ids": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i32, _vp, _i64, _i32, _i64,
                                            _vp, _vp, _vp, ctypes.POINTER(_i64)]),
    "surel_query_rpe_ids": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i32, _i32, _i32,
                                           _vp, _i64, _i32, _vp]),
    "surel_prune_rpe": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i64, _vp, _vp,
                                       ctypes.POINTER(_i64)]),
    "surel_query_incidence": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _vp, _vp]),
    "surel_bfs_batches": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _i64, _i32,
                                         _i32, _i32, _vp, _vp, _vp, _vp]),
    "surel_set_spin_limit": (ctypes.c_int, [_vp, ctypes.c_uint32]),
    "surel_check": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_uint32)]),
    "surel_profile_enable": (ctypes.c_int, [_vp, ctypes.c_int]),
    "surel_profile_read": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(_i64)]),
}

_lib = None


class SurelError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load().surel_strerror(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


def load() -> ctypes.CDLL:
    """Load libsurel.so.  Raises if it is missing: there is no other implementation."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is not built; run `python -m paper_2202_13538_amd.build` "
                "(hipcc cross-compiles for gfx950, no GPU needed)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (restype, argtypes) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = restype
            fn.argtypes = argtypes
        _lib = lib
    return _lib


def _ptr(t: torch.Tensor | None, dtype: torch.dtype, what: str) -> int | None:
    if t is None:
        return None
    if t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError(f"{what} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t.data_ptr()


class Context:
    """Owns one ``surel_ctx`` bound to a device and a HIP stream (torch's current one)."""

    def __init__(self, device: int | torch.device | None = None,
                 stream: torch.cuda.Stream | None = None):
        if device is None:
            device = torch.cuda.current_device()
        self.device = torch.device("cuda", device) if isinstance(device, int) else device
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self.stream = stream
        self._h = _vp()
        rc = load().surel_create(ctypes.byref(self._h), self.device.index or 0,
                                 _vp(stream.cuda_stream))
        if rc != OK:
            raise SurelError(rc, "surel_create")

    @property
    def handle(self) -> ctypes.c_void_p:
        return self._h

    def check(self) -> int:
        """Synchronise and return the device error word (also clears it)."""
        flags = ctypes.c_uint32(0)
        rc = load().surel_check(self._h, ctypes.byref(flags))
        if rc not in (OK, E_DEVICE):
            raise SurelError(rc, "surel_check")
        return flags.value

    def set_spin_limit(self, spins: int) -> None:
        rc = load().surel_set_spin_limit(self._h, spins)
        if rc != OK:
            raise SurelError(rc, "surel_set_spin_limit")

    def profile(self, on: bool) -> None:
        rc = load().surel_profile_enable(self._h, 1 if on else 0)
        if rc != OK:
            raise SurelError(rc, "surel_profile_enable")

    def profile_read(self) -> dict:
        """{kernel name: (total ms, launches)} since profiling was switched on."""
        out = {}
        for kid, name in KERNEL_NAMES.items():
            ms = ctypes.c_double(0.0)
            n = _i64(0)
            rc = load().surel_profile_read(self._h, kid, ctypes.byref(ms), ctypes.byref(n))
            if rc != OK:
                raise SurelError(rc, "surel_profile_read")
            out[name] = (ms.value, n.value)
        return out

    def close(self):
        if self._h:
            load().surel_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rpe_rows_bound(n_seeds: int, M: int, m: int) -> int:
    return load().surel_rpe_rows_bound(n_seeds, M, m)


def sample_walks(ctx: Context, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                 seeds: torch.Tensor, M: int, m: int, rng_seed: int = 0,
                 out: torch.Tensor | None = None,
                 set_sizes: torch.Tensor | None = None) -> torch.Tensor:
    """walks int32[n_seeds][M][m+1] on the GPU; ``set_sizes`` (int32[n_seeds], optional)
    receives the number of distinct nodes of every seed's walks."""
    n_nodes = row_ptr.numel() - 1
    n_seeds = seeds.numel()
    if out is None:
        out = torch.empty((n_seeds, M, m + 1), dtype=torch.int32, device=row_ptr.device)
    elif out.numel() != n_seeds * M * (m + 1):
        raise ValueError("out has the wrong size")
    rc = load().surel_sample_walks(
        ctx.handle, _ptr(row_ptr, torch.int32, "row_ptr"), _ptr(col_idx, torch.int32, "col_idx"),
        n_nodes, col_idx.numel(), _ptr(seeds, torch.int32, "seeds"), n_seeds, M, m,
        _u64(rng_seed), _ptr(out, torch.int32, "walks"),
        _ptr(set_sizes, torch.int32, "set_sizes"))
    if rc != OK:
        raise SurelError(rc, "surel_sample_walks")
    return out


def build_rpe_raw(ctx: Context, walks: torch.Tensor, n_nodes: int, cap_rows: int,
                  rpe_off: torch.Tensor, rpe_ids: torch.Tensor | None,
                  rpe_cnt: torch.Tensor | None, want_rows: bool = True,
                  set_sizes: torch.Tensor | None = None):
    """One call of surel_build_rpe into caller buffers.  Returns (status, rows or None)."""
    n_seeds, M, L = walks.shape
    rows = _i64(-1)
    rc = load().surel_build_rpe(
        ctx.handle, _ptr(walks, torch.int32, "walks"), n_seeds, M, L - 1, n_nodes,
        _ptr(set_sizes, torch.int32, "set_sizes"), cap_rows,
        _ptr(rpe_off, torch.int64, "rpe_off"), _ptr(rpe_ids, torch.int32, "rpe_ids"),
        _ptr(rpe_cnt, torch.uint16, "rpe_cnt"), ctypes.byref(rows) if want_rows else None)
    return rc, (rows.value if want_rows else None)


def build_rpe(ctx: Context, walks: torch.Tensor, n_nodes: int, cap_rows: int | None = None,
              set_sizes: torch.Tensor | None = None):
    """(rpe_off int64[n_seeds+1], rpe_ids int32[R], rpe_cnt uint16[R][m+1]) on the GPU.

    ``cap_rows=None`` sizes the outputs with a counting call first; a number allocates that
    many rows up front (``rpe_rows_bound`` always suffices for sampled walks) and returns
    views of the first R rows.
    """
    n_seeds, M, L = walks.shape
    dev = walks.device
    off = torch.empty(n_seeds + 1, dtype=torch.int64, device=dev)
    if cap_rows is None:
        rc, rows = build_rpe_raw(ctx, walks, n_nodes, 0, off, None, None, set_sizes=set_sizes)
        if rc != OK:
            raise SurelError(rc, "surel_build_rpe (count)")
        cap_rows = rows
    ids = torch.empty(cap_rows, dtype=torch.int32, device=dev)
    cnt = torch.empty((cap_rows, L), dtype=torch.uint16, device=dev)
    rc, rows = build_rpe_raw(ctx, walks, n_nodes, cap_rows, off, ids, cnt, set_sizes=set_sizes)
    if rc != OK:
        raise SurelError(rc, "surel_build_rpe")
    return off, ids[:rows], cnt[:rows]


def build_rpe_count(ctx: Context, walks: torch.Tensor, n_nodes: int, rpe_off: torch.Tensor,
                    set_sizes: torch.Tensor | None = None, want_rows: bool = True):
    """surel_build_rpe_count: the table's layout only.  Returns (status, rows or None)."""
    n_seeds, M, L = walks.shape
    rows = _i64(-1)
    rc = load().surel_build_rpe_count(
        ctx.handle, _ptr(walks, torch.int32, "walks"), n_seeds, M, L - 1, n_nodes,
        _ptr(set_sizes, torch.int32, "set_sizes"), _ptr(rpe_off, torch.int64, "rpe_off"),
        ctypes.byref(rows) if want_rows else None)
    return rc, (rows.value if want_rows else None)


def build_rpe_fill(ctx: Context, walks: torch.Tensor, n_nodes: int, rpe_off: torch.Tensor,
                   cap_rows: int, rpe_ids: torch.Tensor, rpe_cnt: torch.Tensor) -> int:
    """surel_build_rpe_fill: the rows only, at the offsets given.  Returns the status."""
    n_seeds, M, L = walks.shape
    return load().surel_build_rpe_fill(
        ctx.handle, _ptr(walks, torch.int32, "walks"), n_seeds, M, L - 1, n_nodes,
        _ptr(rpe_off, torch.int64, "rpe_off"), cap_rows, _ptr(rpe_ids, torch.int32, "rpe_ids"),
        _ptr(rpe_cnt, torch.uint16, "rpe_cnt"))


def sample_walks_rpe_raw(ctx: Context, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                         seeds: torch.Tensor, M: int, m: int, rng_seed: int, walks: torch.Tensor,
                         cap_rows: int, rpe_off: torch.Tensor, rpe_ids: torch.Tensor | None,
                         rpe_cnt: torch.Tensor | None, want_rows: bool = True):
    """One call of surel_sample_walks_rpe into caller buffers.  Returns (status, rows or None)."""
    n_seeds = seeds.numel()
    if walks.numel() != n_seeds * M * (m + 1):
        raise ValueError("walks has the wrong size")
    rows = _i64(-1)
    rc = load().surel_sample_walks_rpe(
        ctx.handle, _ptr(row_ptr, torch.int32, "row_ptr"), _ptr(col_idx, torch.int32, "col_idx"),
        row_ptr.numel() - 1, col_idx.numel(), _ptr(seeds, torch.int32, "seeds"), n_seeds, M, m,
        _u64(rng_seed), _ptr(walks, torch.int32, "walks"), cap_rows,
        _ptr(rpe_off, torch.int64, "rpe_off"), _ptr(rpe_ids, torch.int32, "rpe_ids"),
        _ptr(rpe_cnt, torch.uint16, "rpe_cnt"), ctypes.byref(rows) if want_rows else None)
    return rc, (rows.value if want_rows else None)


def sample_walks_rpe(ctx: Context, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                     seeds: torch.Tensor, M: int, m: int, rng_seed: int = 0):
    """(walks, rpe_off, rpe_ids, rpe_cnt) from the fused kernel; the table is allocated at the
    ``rpe_rows_bound`` size and returned as views of its first R rows."""
    n_seeds = seeds.numel()
    dev = row_ptr.device
    walks = torch.empty((n_seeds, M, m + 1), dtype=torch.int32, device=dev)
    cap_rows = rpe_rows_bound(n_seeds, M, m)
    off = torch.empty(n_seeds + 1, dtype=torch.int64, device=dev)
    ids = torch.empty(cap_rows, dtype=torch.int32, device=dev)
    cnt = torch.empty((cap_rows, m + 1), dtype=torch.uint16, device=dev)
    rc, rows = sample_walks_rpe_raw(ctx, row_ptr, col_idx, seeds, M, m, rng_seed, walks, cap_rows,
                                    off, ids, cnt)
    if rc != OK:
        raise SurelError(rc, "surel_sample_walks_rpe")
    return walks, off, ids[:rows], cnt[:rows]


def sample_walks_rpe_ids_raw(ctx: Context, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                             seeds: torch.Tensor, M: int, m: int, rng_seed: int,
                             walks: torch.Tensor, cap_rows: int, rpe_off: torch.Tensor,
                             rpe_ids: torch.Tensor, rpe_cnt: torch.Tensor | None,
                             code: torch.Tensor, cap_T: int, T: torch.Tensor):
    """One call of surel_sample_walks_rpe_ids into caller buffers.  Returns (status, rows, n_T)."""
    n_seeds = seeds.numel()
    if walks.numel() != n_seeds * M * (m + 1):
        raise ValueError("walks has the wrong size")
    rows, n_T = _i64(-1), _i64(-1)
    rc = load().surel_sample_walks_rpe_ids(
        ctx.handle, _ptr(row_ptr, torch.int32, "row_ptr"), _ptr(col_idx, torch.int32, "col_idx"),
        row_ptr.numel() - 1, col_idx.numel(), _ptr(seeds, torch.int32, "seeds"), n_seeds, M, m,
        _u64(rng_seed), _ptr(walks, torch.int32, "walks"), cap_rows,
        _ptr(rpe_off, torch.int64, "rpe_off"), _ptr(rpe_ids, torch.int32, "rpe_ids"),
        _ptr(rpe_cnt, torch.uint16, "rpe_cnt"), _ptr(code, torch.int32, "code"), cap_T,
        _ptr(T, torch.uint16, "T"), ctypes.byref(rows), ctypes.byref(n_T))
    return rc, rows.value, n_T.value


def sample_walks_rpe_ids(ctx: Context, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                         seeds: torch.Tensor, M: int, m: int, rng_seed: int = 0,
                         cap_T: int = 1 << 20, with_counts: bool = True):
    """(walks, rpe_off, rpe_ids, rpe_cnt or None, code, T): walks, RPE table and pruned array from
    one call (Algorithm 1 from end to end); rows carry T's index of their count vector."""
    n_seeds = seeds.numel()
    dev = row_ptr.device
    walks = torch.empty((n_seeds, M, m + 1), dtype=torch.int32, device=dev)
    cap_rows = rpe_rows_bound(n_seeds, M, m)
    off = torch.empty(n_seeds + 1, dtype=torch.int64, device=dev)
    ids = torch.empty(cap_rows, dtype=torch.int32, device=dev)
    cnt = torch.empty((cap_rows, m + 1), dtype=torch.uint16, device=dev) if with_counts else None
    code = torch.empty(cap_rows, dtype=torch.int32, device=dev)
    T = torch.empty((cap_T, m + 1), dtype=torch.uint16, device=dev)
    rc, rows, n_T = sample_walks_rpe_ids_raw(ctx, row_ptr, col_idx, seeds, M, m, rng_seed, walks,
                                             cap_rows, off, ids, cnt, code, cap_T, T)
    if rc != OK:
        raise SurelError(rc, "surel_sample_walks_rpe_ids")
    return walks, off, ids[:rows], (cnt[:rows] if with_counts else None), code[:rows], T[:n_T]


def join_queries_raw(ctx: Context, rpe_off: torch.Tensor, rpe_ids: torch.Tensor,
                     rpe_cnt: torch.Tensor, queries: torch.Tensor, max_set: int, cap_rows: int,
                     join_off: torch.Tensor, join_ids: torch.Tensor | None,
                     join_cnt: torch.Tensor | None, want_rows: bool = True, noalloc: bool = False):
    """One call of surel_join_queries (noalloc: of surel_join_queries_noalloc, which takes its
    device scratch from a static array inside the library) into caller buffers.  Returns
    (status, rows or None)."""
    n_q, k = queries.shape
    L = rpe_cnt.shape[1]
    rows = _i64(-1)
    fn = load().surel_join_queries_noalloc if noalloc else load().surel_join_queries
    rc = fn(
        ctx.handle, _ptr(rpe_off, torch.int64, "rpe_off"), _ptr(rpe_ids, torch.int32, "rpe_ids"),
        _ptr(rpe_cnt, torch.uint16, "rpe_cnt"), rpe_off.numel() - 1, L - 1, max_set,
        _ptr(queries, torch.int32, "queries"), n_q, k, cap_rows,
        _ptr(join_off, torch.int64, "join_off"), _ptr(join_ids, torch.int32, "join_ids"),
        _ptr(join_cnt, torch.uint16, "join_cnt"), ctypes.byref(rows) if want_rows else None)
    return rc, (rows.value if want_rows else None)


def join_queries(ctx: Context, rpe_off: torch.Tensor, rpe_ids: torch.Tensor,
                 rpe_cnt: torch.Tensor, queries: torch.Tensor, max_set: int,
                 cap_rows: int | None = None):
    """(join_off int64[n_q+1], join_ids int32[J], join_cnt uint16[J][k][m+1]) on the GPU."""
    n_q, k = queries.shape
    L = rpe_cnt.shape[1]
    dev = queries.device
    off = torch.empty(n_q + 1, dtype=torch.int64, device=dev)
    if cap_rows is None:
        rc, rows = join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, queries, max_set, 0, off,
                                    None, None)
        if rc != OK:
            raise SurelError(rc, "surel_join_queries (count)")
        cap_rows = rows
    ids = torch.empty(cap_rows, dtype=torch.int32, device=dev)
    cnt = torch.empty((cap_rows, k, L), dtype=torch.uint16, device=dev)
    rc, rows = join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, queries, max_set, cap_rows, off,
                                ids, cnt)
    if rc != OK:
        raise SurelError(rc, "surel_join_queries")
    return off, ids[:rows], cnt[:rows]


def join_count(ctx: Context, rpe_off: torch.Tensor, rpe_ids: torch.Tensor, queries: torch.Tensor,
               max_set: int, join_off: torch.Tensor, want_rows: bool = True):
    """surel_join_count: the join's layout only.  Returns (status, rows or None)."""
    n_q, k = queries.shape
    rows = _i64(-1)
    rc = load().surel_join_count(
        ctx.handle, _ptr(rpe_off, torch.int64, "rpe_off"), _ptr(rpe_ids, torch.int32, "rpe_ids"),
        rpe_off.numel() - 1, max_set, _ptr(queries, torch.int32, "queries"), n_q, k,
        _ptr(join_off, torch.int64, "join_off"), ctypes.byref(rows) if want_rows else None)
    return rc, (rows.value if want_rows else None)


def join_fill(ctx: Context, rpe_off: torch.Tensor, rpe_ids: torch.Tensor, rpe_cnt: torch.Tensor,
              queries: torch.Tensor, max_set: int, join_off: torch.Tensor, cap_rows: int,
              join_ids: torch.Tensor, join_cnt: torch.Tensor) -> int:
    """surel_join_fill: the joined rows only, at the offsets given.  Returns the status."""
    n_q, k = queries.shape
    L = rpe_cnt.shape[1]
    return load().surel_join_fill(
        ctx.handle, _ptr(rpe_off, torch.int64, "rpe_off"), _ptr(rpe_ids, torch.int32, "rpe_ids"),
        _ptr(rpe_cnt, torch.uint16, "rpe_cnt"), rpe_off.numel() - 1, L - 1, max_set,
        _ptr(queries, torch.int32, "queries"), n_q, k, _ptr(join_off, torch.int64, "join_off"),
        cap_rows, _ptr(join_ids, torch.int32, "join_ids"), _ptr(join_cnt, torch.uint16, "join_cnt"))


def join_query_ids_raw(ctx: Context, rpe_off: torch.Tensor, rpe_ids: torch.Tensor,
                       code: torch.Tensor, queries: torch.Tensor, max_set: int, cap_rows: int,
                       join_off: torch.Tensor, join_ids: torch.Tensor | None,
                       join_codes: torch.Tensor | None, want_rows: bool = True):
    """One call of surel_join_query_ids into caller buffers.  Returns (status, rows or None)."""
    n_q, k = queries.shape
    rows = _i64(-1)
    rc = load().surel_join_query_ids(
        ctx.handle, _ptr(rpe_off, torch.int64, "rpe_off"), _ptr(rpe_ids, torch.int32, "rpe_ids"),
        _ptr(code, torch.int32, "code"), rpe_off.numel() - 1, max_set,
        _ptr(queries, torch.int32, "queries"), n_q, k, cap_rows,
        _ptr(join_off, torch.int64, "join_off"), _ptr(join_ids, torch.int32, "join_ids"),
        _ptr(join_codes, torch.int32, "join_codes"), ctypes.byref(rows) if want_rows else None)
    return rc, (rows.value if want_rows else None)


def join_query_ids(ctx: Context, rpe_off: torch.Tensor, rpe_ids: torch.Tensor, code: torch.Tensor,
                   queries: torch.Tensor, max_set: int):
    """(join_off int64[n_q+1], join_ids int32[J], join_codes int32[J][k]) on the GPU: the union
    join with the rows' codes (indices into the pruned array T, -1 = absent) instead of counts."""
    n_q, k = queries.shape
    dev = queries.device
    off = torch.empty(n_q + 1, dtype=torch.int64, device=dev)
    rc, rows = join_query_ids_raw(ctx, rpe_off, rpe_ids, code, queries, max_set, 0, off, None, None)
    if rc != OK:
        raise SurelError(rc, "surel_join_query_ids")
    ids = torch.empty(rows, dtype=torch.int32, device=dev)
    codes = torch.empty((rows, k), dtype=torch.int32, device=dev)
    rc, rows2 = join_query_ids_raw(ctx, rpe_off, rpe_ids, code, queries, max_set, rows, off, ids,
                                   codes)
    if rc != OK:
        raise SurelError(rc, "surel_join_query_ids")
    return off, ids, codes


def query_rpe_ids(ctx: Context, walks: torch.Tensor, rpe_off: torch.Tensor, rpe_ids: torch.Tensor,
                  queries: torch.Tensor, max_set: int, out: torch.Tensor | None = None,
                  code: torch.Tensor | None = None):
    """int32[n_q][k][M][m+1][k] on the GPU: the query-level RPE-IDs of every walk position (table
    rows; with `code` from prune_rpe, the rows' codes, i.e. indices into the pruned array T)."""
    if code is not None and code.numel() != rpe_ids.numel():
        raise ValueError("code must have one entry per table row")
    n_blocks, M, L = walks.shape
    n_q, k = queries.shape
    if out is None:
        out = torch.empty((n_q, k, M, L, k), dtype=torch.int32, device=walks.device)
    elif out.numel() != n_q * k * M * L * k:
        raise ValueError("out has the wrong size")
    rc = load().surel_query_rpe_ids(
        ctx.handle, _ptr(walks, torch.int32, "walks"), _ptr(rpe_off, torch.int64, "rpe_off"),
        _ptr(rpe_ids, torch.int32, "rpe_ids"), _ptr(code, torch.int32, "code"), n_blocks,
        rpe_ids.numel(), M, L - 1, max_set, _ptr(queries, torch.int32, "queries"), n_q, k,
        _ptr(out, torch.int32, "out"))
    if rc != OK:
        raise SurelError(rc, "surel_query_rpe_ids")
    return out


def prune_rpe_raw(ctx: Context, rpe_cnt: torch.Tensor, cap_T: int, T: torch.Tensor,
                  code: torch.Tensor):
    """One call of surel_prune_rpe into caller buffers.  Returns (status, n_T)."""
    n_rows, L = rpe_cnt.shape
    n_T = _i64(-1)
    rc = load().surel_prune_rpe(ctx.handle, _ptr(rpe_cnt, torch.uint16, "rpe_cnt"), n_rows, L - 1,
                                cap_T, _ptr(T, torch.uint16, "T"), _ptr(code, torch.int32, "code"),
                                ctypes.byref(n_T))
    return rc, n_T.value


def prune_rpe(ctx: Context, rpe_cnt: torch.Tensor, cap_T: int = 1 << 20):
    """(T uint16[n_T][m+1], code int32[R]) on the GPU: the distinct count vectors, sorted, and
    every row's index among them."""
    n_rows, L = rpe_cnt.shape
    T = torch.empty((cap_T, L), dtype=torch.uint16, device=rpe_cnt.device)
    code = torch.empty(n_rows, dtype=torch.int32, device=rpe_cnt.device)
    rc, n_T = prune_rpe_raw(ctx, rpe_cnt, cap_T, T, code)
    if rc != OK:
        raise SurelError(rc, "surel_prune_rpe")
    return T[:n_T], code


def query_incidence(ctx: Context, queries: torch.Tensor, n_nodes: int):
    """(inc_off int64[n_nodes+1], inc_q int32[n_queries*k]) on the GPU: for every node the
    indices of the queries that name it, ascending (surel_query_incidence)."""
    n_queries, k = queries.shape
    inc_off = torch.empty(n_nodes + 1, dtype=torch.int64, device=queries.device)
    inc_q = torch.empty(n_queries * k, dtype=torch.int32, device=queries.device)
    rc = load().surel_query_incidence(ctx.handle, _ptr(queries, torch.int32, "queries"), n_queries,
                                      k, n_nodes, _ptr(inc_off, torch.int64, "inc_off"),
                                      _ptr(inc_q, torch.int32, "inc_q"))
    if rc != OK:
        raise SurelError(rc, "surel_query_incidence")
    return inc_off, inc_q


def bfs_batches_raw(ctx: Context, queries, n_nodes: int, inc_off, inc_q, start, B1: int, B2: int,
                    vbar, batch, tuples, counts) -> int:
    """One call of surel_bfs_batches into caller buffers.  Returns the status."""
    n_queries, k = queries.shape
    n_batches, n_start = start.shape
    return load().surel_bfs_batches(
        ctx.handle, _ptr(queries, torch.int32, "queries"), n_queries, k, n_nodes,
        _ptr(inc_off, torch.int64, "inc_off"), _ptr(inc_q, torch.int32, "inc_q"),
        _ptr(start, torch.int32, "start"), n_batches, n_start, B1, B2,
        _ptr(vbar, torch.int32, "vbar"), _ptr(batch, torch.int32, "batch"),
        None if tuples is None else _ptr(tuples, torch.int32, "tuples"),
        _ptr(counts, torch.int32, "counts"))


def bfs_batches(ctx: Context, queries: torch.Tensor, n_nodes: int, inc_off: torch.Tensor,
                inc_q: torch.Tensor, start: torch.Tensor, B1: int, B2: int, want_tuples=True):
    """(vbar int32[n_batches][B1], batch int32[n_batches][B2], tuples int32[n_batches][B2][k] or
    None, counts int32[n_batches][2]) on the GPU: one mini-batch per row of `start`
    (surel_bfs_batches).  Only the first counts[b] entries of a row are written."""
    n_batches = start.shape[0]
    k = queries.shape[1]
    dev = queries.device
    vbar = torch.empty((n_batches, B1), dtype=torch.int32, device=dev)
    batch = torch.empty((n_batches, B2), dtype=torch.int32, device=dev)
    tuples = torch.empty((n_batches, B2, k), dtype=torch.int32, device=dev) if want_tuples else None
    counts = torch.empty((n_batches, 2), dtype=torch.int32, device=dev)
    rc = bfs_batches_raw(ctx, queries, n_nodes, inc_off, inc_q, start, B1, B2, vbar, batch, tuples,
                         counts)
    if rc != OK:
        raise SurelError(rc, "surel_bfs_batches")
    return vbar, batch, tuples, counts
