"""surel_join_queries_noalloc, the entry point for callers that cannot allocate: through the C
ABI, its output against surel_join_queries' on the same inputs, byte for byte, on two calls in
a row, the second with a smaller input (the static scratch keeps the first call's contents)."""
import os

import numpy as np
import pytest
import torch

from paper_2202_13538_amd import binding, synth

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def join_into_fresh_buffers(ctx, table, d_q, max_set, rows, noalloc, fill=-7):
    off, ids, cnt = table
    n_q, k = d_q.shape
    L = cnt.shape[1]
    joff = torch.full((n_q + 1,), fill, dtype=torch.int64, device="cuda")
    jids = torch.full((rows,), fill, dtype=torch.int32, device="cuda")
    jcnt = torch.full((rows, k, L), 0x7777, dtype=torch.int16, device="cuda").view(torch.uint16)
    rc, got = binding.join_queries_raw(ctx, off, ids, cnt, d_q, max_set, rows, joff, jids, jcnt,
                                       noalloc=noalloc)
    assert rc == binding.OK and got == rows
    assert ctx.check() == 0
    return joff, jids, jcnt.view(torch.int16)


@pytest.mark.parametrize("k", [2, 3])
def test_noalloc_join_equals_the_allocating_one_on_two_calls_in_a_row(k):
    assert torch.cuda.is_available() and os.path.exists(binding.LIB_PATH)
    ctx = binding.Context()
    wl = synth.Workload("t", "rmat", 4096, 30000, 0.0, 50, 4, 0, k, "uniform", graph_seed=9)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(wl.n_nodes, dtype=np.int32)
    _, off, ids, cnt = binding.sample_walks_rpe(ctx, dev(rp), dev(ci), dev(seeds), wl.M, wl.m, 3)
    assert ctx.check() == 0
    table = (off, ids, cnt)
    max_set = 1 + wl.M * wl.m
    rng = np.random.default_rng(5 + k)
    big = dev(rng.integers(0, wl.n_nodes, size=(20011, k)).astype(np.int32))
    small = dev(rng.integers(0, wl.n_nodes, size=(777, k)).astype(np.int32))
    for d_q in (big, small):                       # the second call is the smaller one
        n_q = d_q.shape[0]
        joff = torch.empty(n_q + 1, dtype=torch.int64, device="cuda")
        rc, rows = binding.join_queries_raw(ctx, off, ids, cnt, d_q, max_set, 0, joff, None, None)
        assert rc == binding.OK
        # the counting form of the new entry point gives the same layout
        joff_n = torch.full_like(joff, -7)
        rc, rows_n = binding.join_queries_raw(ctx, off, ids, cnt, d_q, max_set, 0, joff_n, None,
                                              None, noalloc=True)
        assert rc == binding.OK and rows_n == rows and torch.equal(joff_n, joff)
        want = join_into_fresh_buffers(ctx, table, d_q, max_set, rows, noalloc=False)
        got = join_into_fresh_buffers(ctx, table, d_q, max_set, rows, noalloc=True)
        for g, w, what in zip(got, want, ("join_off", "join_ids", "join_cnt")):
            assert torch.equal(g, w), f"{what} differs at {n_q} queries"
    # an empty query list, and one query more than the static scratch holds
    joff = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    rc, rows = binding.join_queries_raw(ctx, off, ids, cnt, big[:0], max_set, 0, joff, None, None,
                                        noalloc=True)
    assert rc == binding.OK and rows == 0 and int(joff[0]) == 0
    too_many = torch.zeros((binding.NOALLOC_MAX_QUERIES + 1, k), dtype=torch.int32, device="cuda")
    joff = torch.empty(too_many.shape[0] + 1, dtype=torch.int64, device="cuda")
    rc, _ = binding.join_queries_raw(ctx, off, ids, cnt, too_many, max_set, 0, joff, None, None,
                                     noalloc=True)
    assert rc == binding.E_RANGE
    assert ctx.check() == 0
    ctx.close()


def test_noalloc_join_at_its_largest_size_and_device_memory_stays_as_it_was():
    # 2^20 queries, the most the static scratch holds; the library's own device memory does not
    # grow over the call (a fresh context has no workspace yet, so the allocating call would)
    ctx = binding.Context()
    wl = synth.Workload("t", "rmat", 4096, 30000, 0.0, 20, 2, 0, 2, "uniform", graph_seed=9)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(wl.n_nodes, dtype=np.int32)
    _, off, ids, cnt = binding.sample_walks_rpe(ctx, dev(rp), dev(ci), dev(seeds), wl.M, wl.m, 3)
    max_set = 1 + wl.M * wl.m
    n_q = binding.NOALLOC_MAX_QUERIES
    g = torch.Generator(device="cpu").manual_seed(3)
    d_q = torch.randint(0, wl.n_nodes, (n_q, 2), generator=g, dtype=torch.int32).cuda()
    joff = torch.empty(n_q + 1, dtype=torch.int64, device="cuda")
    fresh = binding.Context()                      # no workspace grown yet
    # a first small call, so that the runtime's own first-launch work (code loading) is done
    rc, _ = binding.join_queries_raw(fresh, off, ids, cnt, d_q[:64].contiguous(), max_set, 0,
                                     joff[:65], None, None, noalloc=True)
    assert rc == binding.OK
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    rc, rows = binding.join_queries_raw(fresh, off, ids, cnt, d_q, max_set, 0, joff, None, None,
                                        noalloc=True)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert rc == binding.OK and fresh.check() == 0
    assert free_after == free_before, "the call that must not allocate changed the free device memory"
    joff2 = torch.empty_like(joff)
    rc, rows2 = binding.join_queries_raw(ctx, off, ids, cnt, d_q, max_set, 0, joff2, None, None)
    assert rc == binding.OK and rows2 == rows and torch.equal(joff, joff2)
    jids = torch.empty(rows, dtype=torch.int32, device="cuda")
    jcnt = torch.empty((rows, 2, wl.m + 1), dtype=torch.uint16, device="cuda")
    jids2, jcnt2 = torch.empty_like(jids), torch.empty_like(jcnt)
    rc, _ = binding.join_queries_raw(fresh, off, ids, cnt, d_q, max_set, rows, joff, jids, jcnt,
                                     noalloc=True)
    assert rc == binding.OK and fresh.check() == 0
    rc, _ = binding.join_queries_raw(ctx, off, ids, cnt, d_q, max_set, rows, joff2, jids2, jcnt2)
    assert rc == binding.OK and ctx.check() == 0
    assert torch.equal(joff, joff2) and torch.equal(jids, jids2)
    assert torch.equal(jcnt.view(torch.int16), jcnt2.view(torch.int16))
    fresh.close()
    ctx.close()


def test_noalloc_join_under_graph_capture():
    # what the entry point is for: captured once (no allocation, no memset, no wait inside),
    # replayed with other work on the stream in between, every replay against the eager bytes
    wl = synth.Workload("t", "rmat", 4096, 30000, 0.0, 50, 4, 0, 2, "uniform", graph_seed=9)
    rp, ci = synth.make_graph(wl)
    rng = np.random.default_rng(4)
    queries = rng.integers(0, wl.n_nodes, size=(3001, 2)).astype(np.int32)
    max_set = 1 + wl.M * wl.m
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        c = binding.Context(stream=stream)
        seeds = torch.arange(wl.n_nodes, dtype=torch.int32, device="cuda")
        _, off, ids, cnt = binding.sample_walks_rpe(c, dev(rp), dev(ci), seeds, wl.M, wl.m, 3)
        d_q = dev(queries)
        want = join_into_fresh_buffers(c, (off, ids, cnt), d_q, max_set,
                                       rows=int(binding.join_queries(c, off, ids, cnt, d_q, max_set)[1].numel()),
                                       noalloc=False)
        rows = want[1].numel()
        joff = torch.empty(queries.shape[0] + 1, dtype=torch.int64, device="cuda")
        jids = torch.empty(rows, dtype=torch.int32, device="cuda")
        jcnt = torch.empty((rows, 2, wl.m + 1), dtype=torch.uint16, device="cuda")
        # a fresh context: nothing has grown its workspace, and nothing will
        g_ctx = binding.Context(stream=stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream, capture_error_mode="thread_local"):
            rc, _ = binding.join_queries_raw(g_ctx, off, ids, cnt, d_q, max_set, rows, joff, jids,
                                             jcnt, want_rows=False, noalloc=True)
        assert rc == binding.OK
        for replay in range(3):
            for t in (joff, jids, jcnt.view(torch.int16)):
                t.fill_(-7 - replay)                 # eager work between the replays
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            assert g_ctx.check() == 0, f"replay {replay}"
            for got, ref in zip((joff, jids, jcnt.view(torch.int16)), want):
                assert torch.equal(got, ref), f"replay {replay} differs from the eager call"
        g_ctx.close()
        c.close()
