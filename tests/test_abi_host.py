"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the public header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2202_13538_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "surel.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2202_13538_amd import build
        build.build()
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(surel_[a-z_]+)\s*\(", text)))


def test_header_and_binding_name_the_same_entry_points():
    assert declared_functions() == sorted(binding.SIGNATURES)


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_header_constants_match_binding():
    text = open(HEADER).read()
    defs = dict(re.findall(r"#define\s+(SUREL_[A-Z_]+)\s+\(?(-?[0-9a-fx]+)u?\)?", text))
    for kid, name in binding.KERNEL_NAMES.items():
        assert int(defs["SUREL_K_" + name.upper()]) == kid
    assert int(defs["SUREL_K_COUNT"]) == binding.K_COUNT == len(binding.KERNEL_NAMES)
    val = {k: int(v, 0) for k, v in defs.items()}
    assert val["SUREL_OK"] == binding.OK
    assert val["SUREL_E_NULL"] == binding.E_NULL
    assert val["SUREL_E_RANGE"] == binding.E_RANGE
    assert val["SUREL_E_HIP"] == binding.E_HIP
    assert val["SUREL_E_CAPACITY"] == binding.E_CAPACITY
    assert val["SUREL_E_CTX"] == binding.E_CTX
    assert val["SUREL_E_DEVICE"] == binding.E_DEVICE
    assert val["SUREL_DEV_BAD_SEED"] == binding.DEV_BAD_SEED
    assert val["SUREL_DEV_BAD_GRAPH"] == binding.DEV_BAD_GRAPH
    assert val["SUREL_DEV_BAD_WALK"] == binding.DEV_BAD_WALK
    assert val["SUREL_DEV_BAD_QUERY"] == binding.DEV_BAD_QUERY
    assert val["SUREL_DEV_SET_TOO_LARGE"] == binding.DEV_SET_TOO_LARGE
    assert val["SUREL_DEV_CAPACITY"] == binding.DEV_CAPACITY
    assert val["SUREL_DEV_BAD_TABLE"] == binding.DEV_BAD_TABLE
    assert val["SUREL_DEV_BAD_SIZES"] == binding.DEV_BAD_SIZES
    assert val["SUREL_MAX_NODES"] == binding.MAX_NODES
    assert val["SUREL_MAX_STEPS"] == binding.MAX_STEPS
    assert val["SUREL_MAX_WALKS"] == binding.MAX_WALKS
    assert val["SUREL_MAX_WALK_ENTRIES"] == binding.MAX_WALK_ENTRIES
    assert val["SUREL_MAX_SET"] == binding.MAX_SET
    assert val["SUREL_MAX_TUPLE"] == binding.MAX_TUPLE
    assert val["SUREL_MAX_DISTINCT"] == binding.MAX_DISTINCT
    assert val["SUREL_MAX_BATCH"] == binding.MAX_BATCH
    assert val["SUREL_DEV_STALL"] == binding.DEV_STALL
    assert val["SUREL_NOALLOC_MAX_QUERIES"] == binding.NOALLOC_MAX_QUERIES


def test_strerror_and_bound(lib):
    for status in range(-6, 1):
        assert lib.surel_strerror(status)
    assert lib.surel_strerror(-99) == b"unknown status"
    assert lib.surel_rpe_rows_bound(10, 50, 4) == 10 * 201
    assert lib.surel_rpe_rows_bound(2_900_000, 100, 4) == 2_900_000 * 401
    assert lib.surel_rpe_rows_bound(0, 50, 4) == 0
    assert lib.surel_rpe_rows_bound(-1, 50, 4) == 0


# A fake non-NULL pointer: argument checks must finish before anything is dereferenced.
P = ctypes.c_void_p(0x1000)
NULL = None


def walks_args(**kw):
    a = dict(ctx=NULL, row_ptr=P, col_idx=P, n_nodes=100, n_edges=500, seeds=P, n_seeds=10,
             M=50, m=4, rng_seed=0, walks=P, sizes=NULL)
    a.update(kw)
    return [a[k] for k in ("ctx", "row_ptr", "col_idx", "n_nodes", "n_edges", "seeds", "n_seeds",
                           "M", "m", "rng_seed", "walks", "sizes")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),                      # everything valid except the context
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(n_nodes=binding.MAX_NODES + 1), binding.E_RANGE),
    (dict(n_edges=-1), binding.E_RANGE),
    (dict(n_edges=1 << 31), binding.E_RANGE),
    (dict(n_seeds=-1), binding.E_RANGE),
    (dict(M=0), binding.E_RANGE),
    (dict(M=binding.MAX_WALKS + 1), binding.E_RANGE),
    (dict(m=0), binding.E_RANGE),
    (dict(m=binding.MAX_STEPS + 1), binding.E_RANGE),
    (dict(row_ptr=NULL), binding.E_NULL),
    (dict(col_idx=NULL), binding.E_NULL),
    (dict(col_idx=NULL, n_edges=0), binding.E_CTX),   # an edgeless graph needs no col_idx
    (dict(seeds=NULL), binding.E_NULL),
    (dict(walks=NULL), binding.E_NULL),
    (dict(seeds=NULL, walks=NULL, n_seeds=0), binding.E_CTX),
    (dict(sizes=P), binding.E_CTX),                   # set sizes requested, shape fits
    (dict(sizes=P, M=410, m=4), binding.E_RANGE),     # set sizes need M*(m+1) <= 2048
    (dict(M=410, m=4), binding.E_CTX),                # without them any M works
])
def test_sample_walks_argument_checks(lib, kw, want):
    assert lib.surel_sample_walks(*walks_args(**kw)) == want


def rpe_args(**kw):
    a = dict(ctx=NULL, walks=P, n_seeds=10, M=50, m=4, n_nodes=100, sizes=NULL, cap_rows=1000,
             off=P, ids=P, cnt=P, h_rows=NULL)
    a.update(kw)
    return [a[k] for k in ("ctx", "walks", "n_seeds", "M", "m", "n_nodes", "sizes", "cap_rows",
                           "off", "ids", "cnt", "h_rows")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(M=400, m=4), binding.E_CTX),            # 2000 walk entries: the paper's largest M
    (dict(M=410, m=4), binding.E_RANGE),          # 2050 > SUREL_MAX_WALK_ENTRIES
    (dict(M=128, m=15), binding.E_CTX),           # exactly 2048
    (dict(M=129, m=15), binding.E_RANGE),
    (dict(m=16), binding.E_RANGE),
    (dict(M=0), binding.E_RANGE),
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(cap_rows=-1), binding.E_RANGE),
    (dict(n_seeds=-5), binding.E_RANGE),
    (dict(off=NULL), binding.E_NULL),
    (dict(walks=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),             # ids and cnt go together
    (dict(cnt=NULL), binding.E_NULL),
    (dict(ids=NULL, cnt=NULL, cap_rows=0), binding.E_CTX),   # counting call
    (dict(sizes=P), binding.E_CTX),                          # caller-provided set sizes
    (dict(cnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),    # counts must be 4-byte aligned
])
def test_build_rpe_argument_checks(lib, kw, want):
    assert lib.surel_build_rpe(*rpe_args(**kw)) == want


def fused_args(**kw):
    a = dict(ctx=NULL, row_ptr=P, col_idx=P, n_nodes=100, n_edges=500, seeds=P, n_seeds=10,
             M=50, m=4, rng_seed=0, walks=P, cap_rows=1000, off=P, ids=P, cnt=P, h_rows=NULL)
    a.update(kw)
    return [a[k] for k in ("ctx", "row_ptr", "col_idx", "n_nodes", "n_edges", "seeds", "n_seeds",
                           "M", "m", "rng_seed", "walks", "cap_rows", "off", "ids", "cnt",
                           "h_rows")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(n_edges=-1), binding.E_RANGE),
    (dict(n_seeds=-1), binding.E_RANGE),
    (dict(M=0), binding.E_RANGE),
    (dict(m=16), binding.E_RANGE),
    (dict(M=400, m=4), binding.E_CTX),
    (dict(M=410, m=4), binding.E_RANGE),          # the fused kernel sorts M*(m+1) keys per seed
    (dict(cap_rows=-1), binding.E_RANGE),
    (dict(row_ptr=NULL), binding.E_NULL),
    (dict(col_idx=NULL), binding.E_NULL),
    (dict(col_idx=NULL, n_edges=0), binding.E_CTX),
    (dict(seeds=NULL), binding.E_NULL),
    (dict(walks=NULL), binding.E_NULL),
    (dict(off=NULL), binding.E_NULL),
    (dict(off=NULL, seeds=NULL, walks=NULL, n_seeds=0), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(cnt=NULL), binding.E_NULL),
    (dict(ids=NULL, cnt=NULL, cap_rows=0), binding.E_CTX),
    (dict(cnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),
])
def test_sample_walks_rpe_argument_checks(lib, kw, want):
    assert lib.surel_sample_walks_rpe(*fused_args(**kw)) == want


def fused_ids_args(**kw):
    a = dict(ctx=NULL, row_ptr=P, col_idx=P, n_nodes=100, n_edges=500, seeds=P, n_seeds=10,
             M=50, m=4, rng_seed=0, walks=P, cap_rows=1000, off=P, ids=P, cnt=P, code=P, cap_T=64,
             T=P, h_rows=ctypes.pointer(ctypes.c_int64(0)), h_n_T=ctypes.pointer(ctypes.c_int64(0)))
    a.update(kw)
    return [a[k] for k in ("ctx", "row_ptr", "col_idx", "n_nodes", "n_edges", "seeds", "n_seeds",
                           "M", "m", "rng_seed", "walks", "cap_rows", "off", "ids", "cnt", "code",
                           "cap_T", "T", "h_rows", "h_n_T")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(cnt=NULL), binding.E_CTX),              # a table of RPE-IDs only
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(n_edges=-1), binding.E_RANGE),
    (dict(M=410, m=4), binding.E_RANGE),
    (dict(cap_rows=-1), binding.E_RANGE),
    (dict(cap_T=0), binding.E_RANGE),
    (dict(cap_T=binding.MAX_DISTINCT + 1), binding.E_RANGE),
    (dict(row_ptr=NULL), binding.E_NULL),
    (dict(seeds=NULL), binding.E_NULL),
    (dict(walks=NULL), binding.E_NULL),
    (dict(off=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(code=NULL), binding.E_NULL),
    (dict(T=NULL), binding.E_NULL),
    (dict(h_rows=NULL), binding.E_NULL),
    (dict(h_n_T=NULL), binding.E_NULL),
    (dict(cnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),
])
def test_sample_walks_rpe_ids_argument_checks(lib, kw, want):
    assert lib.surel_sample_walks_rpe_ids(*fused_ids_args(**kw)) == want


def join_ids_args(**kw):
    a = dict(ctx=NULL, off=P, ids=P, code=P, n_blocks=100, max_set=201, queries=P, n_q=10, k=2,
             cap_rows=1000, joff=P, jids=P, jcodes=P, h_rows=NULL)
    a.update(kw)
    return [a[k] for k in ("ctx", "off", "ids", "code", "n_blocks", "max_set", "queries", "n_q", "k",
                           "cap_rows", "joff", "jids", "jcodes", "h_rows")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(k=3), binding.E_CTX),
    (dict(k=1), binding.E_RANGE),
    (dict(max_set=0), binding.E_RANGE),
    (dict(max_set=binding.MAX_SET + 1), binding.E_RANGE),
    (dict(n_q=-1), binding.E_RANGE),
    (dict(cap_rows=-1), binding.E_RANGE),
    (dict(joff=NULL), binding.E_NULL),
    (dict(queries=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(code=NULL), binding.E_NULL),
    (dict(jids=NULL), binding.E_NULL),
    (dict(jcodes=NULL), binding.E_NULL),
    (dict(jids=NULL, jcodes=NULL, code=NULL), binding.E_CTX),
])
def test_join_query_ids_argument_checks(lib, kw, want):
    assert lib.surel_join_query_ids(*join_ids_args(**kw)) == want


def ids_args(**kw):
    a = dict(ctx=NULL, walks=P, off=P, ids=P, code=NULL, n_blocks=100, table_rows=5000, M=50, m=4,
             max_set=201, queries=P, n_q=10, k=2, out=P)
    a.update(kw)
    return [a[k] for k in ("ctx", "walks", "off", "ids", "code", "n_blocks", "table_rows", "M", "m",
                           "max_set", "queries", "n_q", "k", "out")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(code=P), binding.E_CTX),
    (dict(M=0), binding.E_RANGE),
    (dict(m=16), binding.E_RANGE),
    (dict(k=1), binding.E_RANGE),
    (dict(k=4), binding.E_RANGE),
    (dict(max_set=0), binding.E_RANGE),
    (dict(max_set=binding.MAX_SET + 1), binding.E_RANGE),
    (dict(n_blocks=-1), binding.E_RANGE),
    (dict(n_q=-1), binding.E_RANGE),
    (dict(table_rows=-1), binding.E_RANGE),
    (dict(table_rows=1 << 31), binding.E_RANGE),      # a row index must fit int32
    (dict(walks=NULL), binding.E_NULL),
    (dict(off=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(queries=NULL), binding.E_NULL),
    (dict(out=NULL), binding.E_NULL),
    (dict(queries=NULL, out=NULL, walks=NULL, off=NULL, ids=NULL, n_q=0), binding.E_CTX),
])
def test_query_rpe_ids_argument_checks(lib, kw, want):
    assert lib.surel_query_rpe_ids(*ids_args(**kw)) == want


def prune_args(**kw):
    a = dict(ctx=NULL, cnt=P, n_rows=100, m=4, cap_T=1000, T=P, code=P,
             n_T=ctypes.pointer(ctypes.c_int64(0)))
    a.update(kw)
    return [a[k] for k in ("ctx", "cnt", "n_rows", "m", "cap_T", "T", "code", "n_T")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(m=0), binding.E_RANGE),
    (dict(m=16), binding.E_RANGE),
    (dict(n_rows=-1), binding.E_RANGE),
    (dict(cap_T=0), binding.E_RANGE),
    (dict(cap_T=binding.MAX_DISTINCT + 1), binding.E_RANGE),
    (dict(cnt=NULL), binding.E_NULL),
    (dict(T=NULL), binding.E_NULL),
    (dict(code=NULL), binding.E_NULL),
    (dict(n_T=NULL), binding.E_NULL),
    (dict(cnt=NULL, code=NULL, n_rows=0), binding.E_CTX),
])
def test_prune_rpe_argument_checks(lib, kw, want):
    assert lib.surel_prune_rpe(*prune_args(**kw)) == want


def incidence_args(**kw):
    a = dict(ctx=NULL, queries=P, n_q=10, k=2, n_nodes=100, inc_off=P, inc_q=P)
    a.update(kw)
    return [a[k] for k in ("ctx", "queries", "n_q", "k", "n_nodes", "inc_off", "inc_q")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(k=1), binding.E_CTX),
    (dict(k=0), binding.E_RANGE),
    (dict(k=4), binding.E_RANGE),
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(n_nodes=binding.MAX_NODES + 1), binding.E_RANGE),
    (dict(n_q=-1), binding.E_RANGE),
    (dict(n_q=(1 << 30), k=3), binding.E_RANGE),
    (dict(queries=NULL), binding.E_NULL),
    (dict(inc_off=NULL), binding.E_NULL),
    (dict(inc_q=NULL), binding.E_NULL),
    (dict(queries=NULL, inc_q=NULL, n_q=0), binding.E_CTX),
])
def test_query_incidence_argument_checks(lib, kw, want):
    assert lib.surel_query_incidence(*incidence_args(**kw)) == want


def batches_args(**kw):
    a = dict(ctx=NULL, queries=P, n_q=10, k=2, n_nodes=100, inc_off=P, inc_q=P, start=P,
             n_batches=4, n_start=2, B1=64, B2=32, vbar=P, batch=P, tuples=P, counts=P)
    a.update(kw)
    return [a[k] for k in ("ctx", "queries", "n_q", "k", "n_nodes", "inc_off", "inc_q", "start",
                           "n_batches", "n_start", "B1", "B2", "vbar", "batch", "tuples", "counts")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(tuples=NULL), binding.E_CTX),
    (dict(k=0), binding.E_RANGE),
    (dict(k=4), binding.E_RANGE),
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(n_q=-1), binding.E_RANGE),
    (dict(n_batches=-1), binding.E_RANGE),
    (dict(n_start=0), binding.E_RANGE),
    (dict(B1=0), binding.E_RANGE),
    (dict(B2=0), binding.E_RANGE),
    (dict(B1=binding.MAX_BATCH + 1), binding.E_RANGE),
    (dict(B2=binding.MAX_BATCH + 1), binding.E_RANGE),
    (dict(n_start=binding.MAX_BATCH + 1), binding.E_RANGE),
    (dict(B1=binding.MAX_BATCH, B2=binding.MAX_BATCH), binding.E_CTX),
    (dict(queries=NULL), binding.E_NULL),
    (dict(inc_off=NULL), binding.E_NULL),
    (dict(inc_q=NULL), binding.E_NULL),
    (dict(start=NULL), binding.E_NULL),
    (dict(vbar=NULL), binding.E_NULL),
    (dict(batch=NULL), binding.E_NULL),
    (dict(counts=NULL), binding.E_NULL),
    (dict(queries=NULL, inc_q=NULL, n_q=0), binding.E_CTX),
    (dict(start=NULL, vbar=NULL, batch=NULL, counts=NULL, n_batches=0), binding.E_CTX),
])
def test_bfs_batches_argument_checks(lib, kw, want):
    assert lib.surel_bfs_batches(*batches_args(**kw)) == want


def join_args(**kw):
    a = dict(ctx=NULL, off=P, ids=P, cnt=P, n_blocks=100, m=4, max_set=201, queries=P, n_q=10,
             k=2, cap_rows=1000, joff=P, jids=P, jcnt=P, h_rows=NULL)
    a.update(kw)
    return [a[k] for k in ("ctx", "off", "ids", "cnt", "n_blocks", "m", "max_set", "queries",
                           "n_q", "k", "cap_rows", "joff", "jids", "jcnt", "h_rows")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(k=3), binding.E_CTX),
    (dict(k=1), binding.E_RANGE),
    (dict(k=4), binding.E_RANGE),
    (dict(m=0), binding.E_RANGE),
    (dict(m=16), binding.E_RANGE),
    (dict(max_set=0), binding.E_RANGE),
    (dict(max_set=binding.MAX_SET), binding.E_CTX),
    (dict(max_set=binding.MAX_SET + 1), binding.E_RANGE),
    (dict(n_blocks=-1), binding.E_RANGE),
    (dict(n_q=-1), binding.E_RANGE),
    (dict(cap_rows=-1), binding.E_RANGE),
    (dict(joff=NULL), binding.E_NULL),
    (dict(queries=NULL), binding.E_NULL),
    (dict(off=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(cnt=NULL), binding.E_NULL),
    (dict(jids=NULL), binding.E_NULL),
    (dict(jids=NULL, jcnt=NULL, cap_rows=0), binding.E_CTX),
    (dict(jids=NULL, jcnt=NULL, cnt=NULL, cap_rows=0), binding.E_CTX),  # counting needs no counts
    (dict(cnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),
    (dict(jcnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),
])
def test_join_queries_argument_checks(lib, kw, want):
    assert lib.surel_join_queries(*join_args(**kw)) == want
    # the variant that allocates nothing checks the same arguments the same way
    assert lib.surel_join_queries_noalloc(*join_args(**kw)) == want


def test_join_queries_noalloc_rejects_more_queries_than_its_static_scratch_holds(lib):
    ctx = ctypes.c_void_p(0x2000)      # never dereferenced: the size check comes first
    too_many = binding.NOALLOC_MAX_QUERIES + 1
    assert lib.surel_join_queries_noalloc(*join_args(ctx=ctx, n_q=too_many)) == binding.E_RANGE
    assert lib.surel_join_queries_noalloc(*join_args(n_q=binding.NOALLOC_MAX_QUERIES)) == binding.E_CTX


def rpe_count_args(**kw):
    a = dict(ctx=NULL, walks=P, n_seeds=10, M=50, m=4, n_nodes=100, sizes=NULL, off=P, h_rows=NULL)
    a.update(kw)
    return [a[k] for k in ("ctx", "walks", "n_seeds", "M", "m", "n_nodes", "sizes", "off", "h_rows")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(sizes=P), binding.E_CTX),
    (dict(M=410, m=4), binding.E_RANGE),
    (dict(m=16), binding.E_RANGE),
    (dict(M=0), binding.E_RANGE),
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(n_seeds=-5), binding.E_RANGE),
    (dict(off=NULL), binding.E_NULL),
    (dict(walks=NULL), binding.E_NULL),
    (dict(walks=NULL, n_seeds=0), binding.E_CTX),
])
def test_build_rpe_count_argument_checks(lib, kw, want):
    assert lib.surel_build_rpe_count(*rpe_count_args(**kw)) == want


def rpe_fill_args(**kw):
    a = dict(ctx=NULL, walks=P, n_seeds=10, M=50, m=4, n_nodes=100, off=P, cap_rows=1000, ids=P,
             cnt=P)
    a.update(kw)
    return [a[k] for k in ("ctx", "walks", "n_seeds", "M", "m", "n_nodes", "off", "cap_rows", "ids",
                           "cnt")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(M=410, m=4), binding.E_RANGE),
    (dict(m=0), binding.E_RANGE),
    (dict(n_nodes=0), binding.E_RANGE),
    (dict(cap_rows=-1), binding.E_RANGE),
    (dict(off=NULL), binding.E_NULL),             # the offsets are an input here
    (dict(walks=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(cnt=NULL), binding.E_NULL),
    (dict(ids=NULL, cnt=NULL, cap_rows=0), binding.E_CTX),   # room for nothing: nothing to write to
    (dict(cnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),
])
def test_build_rpe_fill_argument_checks(lib, kw, want):
    assert lib.surel_build_rpe_fill(*rpe_fill_args(**kw)) == want


def join_count_args(**kw):
    a = dict(ctx=NULL, off=P, ids=P, n_blocks=100, max_set=201, queries=P, n_q=10, k=2, joff=P,
             h_rows=NULL)
    a.update(kw)
    return [a[k] for k in ("ctx", "off", "ids", "n_blocks", "max_set", "queries", "n_q", "k", "joff",
                           "h_rows")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(k=3), binding.E_CTX),
    (dict(k=1), binding.E_RANGE),
    (dict(k=4), binding.E_RANGE),
    (dict(max_set=0), binding.E_RANGE),
    (dict(max_set=binding.MAX_SET + 1), binding.E_RANGE),
    (dict(n_blocks=-1), binding.E_RANGE),
    (dict(n_q=-1), binding.E_RANGE),
    (dict(joff=NULL), binding.E_NULL),
    (dict(queries=NULL), binding.E_NULL),
    (dict(off=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(queries=NULL, off=NULL, ids=NULL, n_q=0), binding.E_CTX),
])
def test_join_count_argument_checks(lib, kw, want):
    assert lib.surel_join_count(*join_count_args(**kw)) == want


def join_fill_args(**kw):
    a = dict(ctx=NULL, off=P, ids=P, cnt=P, n_blocks=100, m=4, max_set=201, queries=P, n_q=10, k=2,
             joff=P, cap_rows=1000, jids=P, jcnt=P)
    a.update(kw)
    return [a[k] for k in ("ctx", "off", "ids", "cnt", "n_blocks", "m", "max_set", "queries", "n_q",
                           "k", "joff", "cap_rows", "jids", "jcnt")]


@pytest.mark.parametrize("kw,want", [
    (dict(), binding.E_CTX),
    (dict(k=3), binding.E_CTX),
    (dict(k=1), binding.E_RANGE),
    (dict(m=0), binding.E_RANGE),
    (dict(m=16), binding.E_RANGE),
    (dict(max_set=0), binding.E_RANGE),
    (dict(n_blocks=-1), binding.E_RANGE),
    (dict(n_q=-1), binding.E_RANGE),
    (dict(cap_rows=-1), binding.E_RANGE),
    (dict(joff=NULL), binding.E_NULL),            # the offsets are an input here
    (dict(queries=NULL), binding.E_NULL),
    (dict(off=NULL), binding.E_NULL),
    (dict(ids=NULL), binding.E_NULL),
    (dict(cnt=NULL), binding.E_NULL),
    (dict(jids=NULL), binding.E_NULL),
    (dict(jcnt=NULL), binding.E_NULL),
    (dict(cnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),
    (dict(jcnt=ctypes.c_void_p(0x1002)), binding.E_RANGE),
])
def test_join_fill_argument_checks(lib, kw, want):
    assert lib.surel_join_fill(*join_fill_args(**kw)) == want


def test_check_and_destroy_tolerate_null(lib):
    assert lib.surel_check(NULL, NULL) == binding.E_CTX
    assert lib.surel_profile_enable(NULL, 1) == binding.E_CTX
    assert lib.surel_profile_read(NULL, 0, None, None) == binding.E_CTX
    lib.surel_destroy(NULL)


def test_create_reports_missing_device_or_bad_arguments(lib):
    assert lib.surel_create(None, 0, None) == binding.E_NULL
    handle = ctypes.c_void_p()
    rc = lib.surel_create(ctypes.byref(handle), 1 << 20, None)   # no such device anywhere
    assert rc == binding.E_HIP and not handle.value


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/surel.h compiles as C99 with every warning on, and a C program that names every
    declared entry point links against libsurel.so (nothing is called: no GPU here)."""
    import subprocess
    names = declared_functions()
    src = tmp_path / "use_surel.c"
    src.write_text('#include "surel.h"\n#include <stdio.h>\n'
                   "int main(void) {\n    const void* fns[] = {\n"
                   + "".join(f"        (const void*)&{n},\n" for n in names)
                   + "    };\n    printf(\"%d entry points\\n\", (int)(sizeof fns / sizeof fns[0]));\n"
                   "    return 0;\n}\n")
    exe = tmp_path / "use_surel"
    lib_dir = os.path.dirname(binding.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                    "-Wno-pedantic",  # function-to-object pointer casts are the point here
                    "-I", os.path.dirname(HEADER), str(src), "-o", str(exe),
                    "-L", lib_dir, "-lsurel", f"-Wl,-rpath,{lib_dir}", "-Wl,--allow-shlib-undefined"],
                   check=True)


def test_the_product_never_reaches_for_the_oracle():
    """Only tests, smoke() and the benchmark's cpu_baseline leg may use oracle/: no file of the
    package names it, the benchmark imports it inside cpu_baseline only, and the oracle imports
    nothing of the package."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2202_13538_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath or "__pycache__" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f"{f} imports the oracle"
                assert "surel_oracle" not in text and "oracle_" not in text, f"{f} names oracle code"
    bench = open(os.path.join(root, "bench.py")).read()
    assert bench.count("import oracle") == 1
    start = bench.index("def cpu_baseline")
    assert start < bench.index("import oracle") < bench.index("def main")
    for f in os.listdir(os.path.join(root, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2202_13538_amd" not in open(os.path.join(root, "oracle", f)).read()
