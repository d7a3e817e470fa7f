"""Mini-batching on the GPU (Sec. 3.6; Algorithm 2, the BFS step) against the CPU oracle, through
the C ABI: the queries of every node against NumPy's stable sort, and every batch's node set and
query list, element by element and in order, against the oracle's first-in first-out search.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2202_13538_amd import binding, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(binding.LIB_PATH), "libsurel.so is not built"
    c = binding.Context()
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def random_queries(rng, n_nodes, n_queries, k, hubs=0, hub_share=0.3):
    q = rng.integers(0, n_nodes, size=(n_queries, k))
    if hubs:
        pick = rng.random(n_queries) < hub_share
        q[pick, int(rng.integers(0, k))] = rng.integers(0, hubs, size=int(pick.sum()))
    return q.astype(np.int32)


def numpy_incidence(queries, n_nodes):
    flat = queries.reshape(-1).astype(np.int64)
    order = np.argsort(flat, kind="stable")
    inc_q = (order // queries.shape[1]).astype(np.int32)
    inc_off = np.searchsorted(flat[order], np.arange(n_nodes + 1), side="left").astype(np.int64)
    return inc_off, inc_q


@pytest.mark.parametrize("n_nodes,n_queries,k", [(200, 37, 2), (200, 1, 3), (70000, 5000, 2),
                                                 (70000, 300001, 3), ((1 << 24) + 5, 40000, 2),
                                                 (5, 3000, 1)])
def test_query_incidence_equals_a_stable_sort(ctx, n_nodes, n_queries, k):
    rng = np.random.default_rng(n_nodes + n_queries)
    queries = random_queries(rng, n_nodes, n_queries, k, hubs=min(3, n_nodes))
    inc_off, inc_q = binding.query_incidence(ctx, dev(queries), n_nodes)
    assert ctx.check() == 0
    want_off, want_q = numpy_incidence(queries, n_nodes)
    assert np.array_equal(inc_off.cpu().numpy(), want_off)
    assert np.array_equal(inc_q.cpu().numpy(), want_q)


def test_query_incidence_of_an_empty_list_and_bad_ids(ctx):
    empty = torch.empty((0, 2), dtype=torch.int32, device="cuda")
    inc_off, inc_q = binding.query_incidence(ctx, empty, 17)
    assert ctx.check() == 0
    assert inc_off.cpu().tolist() == [0] * 18 and inc_q.numel() == 0
    # ids outside the graph are flagged and belong to no node's part
    queries = np.array([[3, 99], [-1, 3], [2, 3]], dtype=np.int32)
    inc_off, inc_q = binding.query_incidence(ctx, dev(queries), 10)
    assert ctx.check() == binding.DEV_BAD_QUERY
    off = inc_off.cpu().numpy()
    assert off.tolist() == [0, 0, 0, 1, 4, 4, 4, 4, 4, 4, 4]
    assert inc_q.cpu().numpy()[:4].tolist() == [2, 0, 1, 2]


def compare_batches(ctx, queries, n_nodes, start, B1, B2, which=None):
    """Runs every row of `start` on the GPU and the rows `which` (all by default) through the oracle."""
    d_q = dev(queries)
    inc_off, inc_q = binding.query_incidence(ctx, d_q, n_nodes)
    vbar, batch, tuples, counts = binding.bfs_batches(ctx, d_q, n_nodes, inc_off, inc_q, dev(start),
                                                      B1, B2)
    assert ctx.check() == 0
    vbar, batch, tuples, counts = (t.cpu().numpy() for t in (vbar, batch, tuples, counts))
    assert counts[:, 0].max(initial=0) <= B1 and counts[:, 1].max(initial=0) <= B2
    for b in (range(start.shape[0]) if which is None else which):
        want_v, want_b = oracle.bfs_batch(queries, n_nodes, start[b], B1, B2)
        n_v, n_b = counts[b]
        assert (n_v, n_b) == (len(want_v), len(want_b)), f"batch {b}: sizes {n_v, n_b}"
        assert np.array_equal(vbar[b, :n_v], want_v), f"batch {b}: node sets differ"
        assert np.array_equal(batch[b, :n_b], want_b), f"batch {b}: query lists differ"
        assert np.array_equal(tuples[b, :n_b], queries[want_b]), f"batch {b}: tuples differ"
    return counts


@pytest.mark.parametrize("k", [2, 3])
@pytest.mark.parametrize("B1,B2", [(10 ** 6, 10 ** 6), (40, 10 ** 6), (10 ** 6, 25), (300, 200),
                                   (1, 5), (5000, 3000)])
def test_bfs_batches_equal_the_queue_search(ctx, k, B1, B2):
    rng = np.random.default_rng(1000 * k + B1 % 977 + B2 % 31)
    n_nodes, n_queries = 3000, 4000
    queries = random_queries(rng, n_nodes, n_queries, k, hubs=4, hub_share=0.1)
    start = rng.integers(0, n_nodes, size=(24, 3)).astype(np.int32)
    start[0, :] = start[0, 0]                 # one seed three times
    counts = compare_batches(ctx, queries, n_nodes, start, B1, B2)
    print(f"k={k} B1={B1} B2={B2}: nodes {counts[:, 0].tolist()[:6]} queries {counts[:, 1].tolist()[:6]}")


def test_bfs_batches_with_long_lists_wide_levels_and_many_seeds(ctx):
    rng = np.random.default_rng(5)
    # a node held by 5000 queries (its list is taken in pieces), levels of thousands of nodes
    n_nodes, n_queries = 20000, 30000
    queries = random_queries(rng, n_nodes, n_queries, 2, hubs=2, hub_share=0.35)
    start = rng.integers(0, n_nodes, size=(12, 1)).astype(np.int32)
    start[0, 0] = 0
    start[1, 0] = 1
    compare_batches(ctx, queries, n_nodes, start, 10 ** 6, 10 ** 6)
    compare_batches(ctx, queries, n_nodes, start, 7000, 6000)
    compare_batches(ctx, queries, n_nodes, start, 4097, 10 ** 6)
    # seed-sets longer than one piece of the seed loop, with repeats; some fill B1 by themselves
    start = rng.integers(0, 3000, size=(6, 2500)).astype(np.int32)
    compare_batches(ctx, queries, n_nodes, start, 10 ** 6, 500)
    compare_batches(ctx, queries, n_nodes, start, 1500, 10 ** 6)
    # triples with a repeated node inside a query
    queries3 = random_queries(rng, 500, 2000, 3)
    queries3[::7, 2] = queries3[::7, 0]
    start = rng.integers(0, 500, size=(30, 2)).astype(np.int32)
    compare_batches(ctx, queries3, 500, start, 10 ** 6, 10 ** 6)
    compare_batches(ctx, queries3, 500, start, 57, 10 ** 6)
    compare_batches(ctx, queries3, 500, start, 10 ** 6, 33)


def test_bfs_batches_of_single_node_queries(ctx):
    # k = 1: a query shares its node with the queries that name the same node, nothing spreads
    rng = np.random.default_rng(12)
    queries = rng.integers(0, 50, size=(400, 1)).astype(np.int32)
    start = rng.integers(0, 50, size=(20, 3)).astype(np.int32)
    compare_batches(ctx, queries, 50, start, 100, 100)
    compare_batches(ctx, queries, 50, start, 100, 7)


def test_bfs_batches_degenerate_inputs(ctx):
    # no queries at all: every batch is its seed-set
    empty = torch.empty((0, 2), dtype=torch.int32, device="cuda")
    inc_off, inc_q = binding.query_incidence(ctx, empty, 9)
    start = dev(np.array([[4, 4], [8, 0]], dtype=np.int32))
    vbar, batch, tuples, counts = binding.bfs_batches(ctx, empty, 9, inc_off, inc_q, start, 5, 5)
    assert ctx.check() == 0
    assert counts.cpu().tolist() == [[1, 0], [2, 0]]
    assert vbar.cpu()[0, 0].item() == 4 and vbar.cpu()[1, :2].tolist() == [8, 0]
    # no batches
    none = torch.empty((0, 2), dtype=torch.int32, device="cuda")
    vbar, batch, tuples, counts = binding.bfs_batches(ctx, empty, 9, inc_off, inc_q, none, 5, 5)
    assert ctx.check() == 0 and counts.shape == (0, 2)
    # a start node outside the graph is flagged and skipped
    queries = np.array([[0, 1], [1, 2]], dtype=np.int32)
    d_q = dev(queries)
    inc_off, inc_q = binding.query_incidence(ctx, d_q, 3)
    start = dev(np.array([[7, 2]], dtype=np.int32))
    vbar, batch, tuples, counts = binding.bfs_batches(ctx, d_q, 3, inc_off, inc_q, start, 9, 9)
    assert ctx.check() == binding.DEV_BAD_QUERY
    assert counts.cpu().tolist() == [[3, 2]]
    assert vbar.cpu()[0, :3].tolist() == [2, 1, 0] and batch.cpu()[0, :2].tolist() == [1, 0]
    # lists that do not belong to the query list are flagged, nothing is read out of bounds
    bad_off = torch.tensor([0, 50, 60, 70], dtype=torch.int64, device="cuda")
    vbar, batch, tuples, counts = binding.bfs_batches(ctx, d_q, 3, bad_off, inc_q,
                                                      dev(np.array([[0]], dtype=np.int32)), 9, 9)
    assert ctx.check() & binding.DEV_BAD_TABLE


@pytest.mark.parametrize("name", ["cl235k", "cl2900k", "cl1m_triples"])
def test_bfs_batches_on_the_workloads_queries(ctx, name):
    wl = synth.WORKLOADS[name]
    rp, ci = synth.make_graph(wl)
    queries = synth.make_queries(wl, rp, ci)
    rng = np.random.default_rng(3)
    n_batches, n_start, B1, B2 = 256, 16, 4096, 2048
    in_queries = np.unique(queries)                       # the seed-set is drawn from the queried nodes
    start = rng.choice(in_queries, size=(n_batches, n_start)).astype(np.int32)
    counts = compare_batches(ctx, queries, wl.n_nodes, start, B1, B2,
                             which=rng.choice(n_batches, size=12, replace=False))
    print(f"[{name}] batches: mean nodes {counts[:, 0].mean():.0f}, mean queries {counts[:, 1].mean():.0f}",
          flush=True)
    # the paper's default limits (Sec. 4.1: batch capacity 1500, batch size 32), many batches
    start = rng.choice(in_queries, size=(4096, 4)).astype(np.int32)
    counts = compare_batches(ctx, queries, wl.n_nodes, start, 1500, 32,
                             which=rng.choice(4096, size=16, replace=False))
    assert counts[:, 1].max() <= 32 and counts[:, 0].max() <= 1500
