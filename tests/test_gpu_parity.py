"""Parity of the HIP path with the CPU oracle, through the C ABI, on a real MI355X.

Bit-exact comparison of walks, RPE tables and joins, element by element, on small and
medium inputs (several tiles, ragged tails, the degenerate cases) and of the device-detected
problems.  The workloads at their full sizes are in test_gpu_full_size.py.
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


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def host_u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def gpu_pipeline(ctx, rp, ci, seeds, M, m, rng_seed, queries=None, with_sizes=False):
    """walks -> RPE -> join on the GPU.  ``with_sizes``: the walk kernel reports |V_u| and
    build_rpe lays the table out from that; otherwise build_rpe counts by itself."""
    d_rp, d_ci, d_seeds = dev(rp), dev(ci), dev(np.asarray(seeds, dtype=np.int32))
    n_nodes = rp.size - 1
    sizes = None
    if with_sizes:
        sizes = torch.full((d_seeds.numel(),), -1, dtype=torch.int32, device="cuda")
    walks = binding.sample_walks(ctx, d_rp, d_ci, d_seeds, M, m, rng_seed, set_sizes=sizes)
    off, ids, cnt = binding.build_rpe(ctx, walks, n_nodes, set_sizes=sizes)
    out = {"walks": walks, "rpe": (off, ids, cnt), "sizes": sizes}
    if queries is not None:
        d_q = dev(np.asarray(queries, dtype=np.int32))
        out["join"] = binding.join_queries(ctx, off, ids, cnt, d_q, max_set=1 + M * m)
    assert ctx.check() == 0
    return out


def assert_table_equal(got, want, what):
    g_off, g_ids, g_cnt = got
    w_off, w_ids, w_cnt = want
    assert np.array_equal(g_off.cpu().numpy(), w_off), f"{what}: offsets differ"
    assert np.array_equal(g_ids.cpu().numpy(), w_ids), f"{what}: ids differ"
    assert np.array_equal(host_u16(g_cnt), w_cnt), f"{what}: counts differ"


def full_compare(ctx, rp, ci, seeds, M, m, rng_seed, queries):
    w = oracle.sample_walks(rp, ci, seeds, M, m, rng_seed)
    table = oracle.build_rpe(w)
    joined = oracle.join_queries(*table, queries) if queries is not None else None
    for with_sizes in (False, True):
        out = gpu_pipeline(ctx, rp, ci, seeds, M, m, rng_seed, queries, with_sizes)
        assert np.array_equal(out["walks"].cpu().numpy(), w), "walks differ"
        if with_sizes:
            assert np.array_equal(out["sizes"].cpu().numpy(), np.diff(table[0])), "set sizes"
        assert_table_equal(out["rpe"], table, f"rpe (sizes from walks: {with_sizes})")
        if queries is not None:
            assert_table_equal(out["join"], joined, "join")
    # the fused walk + RPE kernel gives the same walks and the same table
    d_seeds = dev(np.asarray(seeds, dtype=np.int32))
    f_walks, f_off, f_ids, f_cnt = binding.sample_walks_rpe(ctx, dev(rp), dev(ci), d_seeds, M, m,
                                                            rng_seed)
    assert ctx.check() == 0
    assert np.array_equal(f_walks.cpu().numpy(), w), "fused: walks differ"
    assert_table_equal((f_off, f_ids, f_cnt), table, "fused rpe")
    # the pruned central array and the re-indexed rows
    T, code = binding.prune_rpe(ctx, f_cnt, cap_T=max(1, table[2].shape[0]))
    assert ctx.check() == 0
    want_T, want_code = oracle.prune_rpe(table[2])
    assert np.array_equal(host_u16(T), want_T), "pruned array differs"
    assert np.array_equal(code.cpu().numpy(), want_code), "re-indexed rows differ"
    # walks, table and pruned array from one call, with and without the count vectors
    for with_counts in (True, False):
        i_walks, i_off, i_ids, i_cnt, i_code, i_T = binding.sample_walks_rpe_ids(
            ctx, dev(rp), dev(ci), d_seeds, M, m, rng_seed, cap_T=max(1, table[2].shape[0]),
            with_counts=with_counts)
        assert ctx.check() == 0
        assert np.array_equal(i_walks.cpu().numpy(), w), "one call: walks differ"
        assert np.array_equal(i_off.cpu().numpy(), table[0]), "one call: offsets differ"
        assert np.array_equal(i_ids.cpu().numpy(), table[1]), "one call: ids differ"
        if with_counts:
            assert np.array_equal(host_u16(i_cnt), table[2]), "one call: counts differ"
        assert np.array_equal(host_u16(i_T).reshape(want_T.shape), want_T), "one call: T differs"
        assert np.array_equal(i_code.cpu().numpy(), want_code), "one call: codes differ"
    if queries is not None and np.asarray(queries).shape[0] > 0:
        # query-level RPE-IDs of every walk position
        got = binding.query_rpe_ids(ctx, f_walks, f_off, f_ids, dev(np.asarray(queries, np.int32)),
                                    max_set=1 + M * m)
        assert ctx.check() == 0
        want = oracle.query_rpe_ids(w, table[0], table[1], queries)
        assert np.array_equal(got.cpu().numpy().astype(np.int64), want), "query RPE-IDs differ"
        # the same as indices into the pruned array: the code of the row, -1 where there is none
        got = binding.query_rpe_ids(ctx, f_walks, f_off, f_ids, dev(np.asarray(queries, np.int32)),
                                    max_set=1 + M * m, code=code)
        assert ctx.check() == 0
        want_ids = np.where(want < 0, -1, want_code.astype(np.int64)[np.maximum(want, 0)])
        assert np.array_equal(got.cpu().numpy().astype(np.int64), want_ids), "pruned RPE-IDs differ"
        # the union join over the codes: the same rows, every count vector replaced by its index
        # in the oracle's pruned array (-1 for the all-zero vector of an absent node)
        j_off, j_ids, j_codes = binding.join_query_ids(ctx, f_off, f_ids, code,
                                                       dev(np.asarray(queries, np.int32)),
                                                       max_set=1 + M * m)
        assert ctx.check() == 0
        index_of = {tuple(v): i for i, v in enumerate(want_T.tolist())}
        want_codes = np.array([[index_of.get(tuple(vec), -1) if any(vec) else -1 for vec in row]
                               for row in joined[2].tolist()], dtype=np.int32).reshape(-1, len(queries[0]))
        assert np.array_equal(j_off.cpu().numpy(), joined[0]), "join offsets differ (ids form)"
        assert np.array_equal(j_ids.cpu().numpy(), joined[1]), "join ids differ (ids form)"
        assert np.array_equal(j_codes.cpu().numpy(), want_codes), "joined RPE-IDs differ"
    return out


# --------------------------------------------------------------------------- #
# small and medium inputs, element by element
# --------------------------------------------------------------------------- #
def test_rmat4k_whole_pipeline_bit_exact(ctx):
    wl = synth.WORKLOADS["rmat4k"]
    rp, ci = synth.make_graph(wl)
    queries = synth.make_queries(wl, rp, ci)
    seeds = np.arange(wl.n_nodes, dtype=np.int32)
    full_compare(ctx, rp, ci, seeds, wl.M, wl.m, wl.rng_seed, queries)


@pytest.mark.parametrize("M,m", [(1, 1), (3, 2), (50, 4), (64, 3), (65, 3), (100, 4), (130, 3),
                                 (200, 4), (200, 3), (128, 15), (400, 4), (341, 5), (7, 15)])
@pytest.mark.parametrize("k", [2, 3])
def test_shapes_bit_exact(ctx, M, m, k):
    wl = synth.Workload("t", "rmat", 1024, 5000, 0.0, M, m, 300, k, "uniform",
                        graph_seed=100 + M + m)
    rp, ci = synth.make_graph(wl)
    rng = np.random.default_rng(M * 31 + m)
    # a ragged, unordered seed list with repeats: 4 waves per workgroup leave a tail
    seeds = rng.integers(0, wl.n_nodes, size=203).astype(np.int32)
    queries = rng.integers(0, seeds.size, size=(301, k)).astype(np.int32)
    queries[0] = 5                                    # every entry the same block
    full_compare(ctx, rp, ci, seeds, M, m, 0xABCDEF0123456789 & ((1 << 64) - 1), queries)


def test_tiny_graphs_and_isolated_nodes(ctx):
    # path 0-1-2-3, isolated node 4, star centred on 5 with leaves 6..9
    rp, ci = synth.csr_from_edge_list(10, [(0, 1), (1, 2), (2, 3), (5, 6), (5, 7), (5, 8), (5, 9)])
    seeds = np.arange(10, dtype=np.int32)
    queries = np.array([[4, 4], [4, 0], [0, 3], [5, 6], [9, 4]], dtype=np.int32)
    out = full_compare(ctx, rp, ci, seeds, 33, 4, 7, queries)
    walks = out["walks"].cpu().numpy()
    assert (walks[4] == 4).all()
    assert (walks[0, :, 1] == 1).all()


def test_edgeless_graph(ctx):
    rp = np.zeros(6, dtype=np.int32)
    ci = np.zeros(0, dtype=np.int32)
    seeds = np.array([3, 0, 4], dtype=np.int32)
    queries = np.array([[0, 1], [2, 2]], dtype=np.int32)
    full_compare(ctx, rp, ci, seeds, 10, 3, 1, queries)


def test_empty_seed_and_query_lists(ctx):
    wl = synth.WORKLOADS["rmat4k"]
    rp, ci = synth.make_graph(wl)
    out = gpu_pipeline(ctx, rp, ci, np.zeros(0, dtype=np.int32), 50, 4, 0,
                       np.zeros((0, 2), dtype=np.int32))
    assert out["walks"].shape == (0, 50, 5)
    off, ids, cnt = out["rpe"]
    assert off.cpu().tolist() == [0] and ids.numel() == 0 and cnt.numel() == 0
    joff, jids, jcnt = out["join"]
    assert joff.cpu().tolist() == [0] and jids.numel() == 0
    # an empty query list against a non-empty table
    out = gpu_pipeline(ctx, rp, ci, np.arange(8, dtype=np.int32), 50, 4, 0,
                       np.zeros((0, 3), dtype=np.int32))
    assert out["join"][0].cpu().tolist() == [0]


def test_paper_worked_example_on_the_gpu(ctx, golden_dir):
    from test_oracle_pins import _read_example
    ex = _read_example(golden_dir)
    m, M = ex["m"][0], ex["M"][0]
    walks = np.array([ex["walks_u"], ex["walks_v"]], dtype=np.int32).reshape(2, M, m + 1)
    off, ids, cnt = binding.build_rpe(ctx, dev(walks), n_nodes=7)
    joff, jids, jcnt = binding.join_queries(ctx, off, ids, cnt, dev(np.array([[0, 1]], np.int32)),
                                            max_set=1 + M * m)
    assert ctx.check() == 0
    ids_h, cnt_h = ids.cpu().numpy(), host_u16(cnt)
    blk = slice(int(off[0]), int(off[1]))
    assert cnt_h[blk][ids_h[blk] == 0][0].tolist() == ex["X_u,u"]
    assert cnt_h[blk][ids_h[blk] == 2][0].tolist() == ex["X_u,a"]
    assert cnt_h[blk][ids_h[blk] == 1][0].tolist() == ex["X_u,v"]
    row = host_u16(jcnt)[jids.cpu().numpy() == 0][0]
    assert row.reshape(-1).tolist() == ex["X_Q,u"]
    assert_table_equal((off, ids, cnt), oracle.build_rpe(walks), "rpe")


def test_hand_made_walks_with_mixed_start_nodes(ctx):
    # build_rpe counts whatever the walk block holds, also when position 0 varies
    rng = np.random.default_rng(4)
    walks = rng.integers(0, 40, size=(37, 20, 4)).astype(np.int32)
    off, ids, cnt = binding.build_rpe(ctx, dev(walks), n_nodes=40)
    assert ctx.check() == 0
    assert_table_equal((off, ids, cnt), oracle.build_rpe(walks), "rpe")


def test_two_runs_are_identical(ctx):
    wl = synth.WORKLOADS["rmat4k"]
    rp, ci = synth.make_graph(wl)
    queries = synth.make_queries(wl, rp, ci)
    seeds = np.arange(wl.n_nodes, dtype=np.int32)
    a = gpu_pipeline(ctx, rp, ci, seeds, wl.M, wl.m, 5, queries)
    b = gpu_pipeline(ctx, rp, ci, seeds, wl.M, wl.m, 5, queries)
    assert torch.equal(a["walks"], b["walks"])
    for x, y in zip(a["rpe"] + a["join"], b["rpe"] + b["join"]):
        assert torch.equal(x.view(torch.int16) if x.dtype == torch.uint16 else x,
                           y.view(torch.int16) if y.dtype == torch.uint16 else y)


# --------------------------------------------------------------------------- #
# device-detected problems never fault and are reported
# --------------------------------------------------------------------------- #
def test_bad_seed_is_flagged_and_skipped(ctx):
    rp, ci = synth.csr_from_edge_list(5, [(0, 1), (1, 2), (2, 3), (3, 4)])
    seeds = np.array([1, 99, -3, 2], dtype=np.int32)
    walks = binding.sample_walks(ctx, dev(rp), dev(ci), dev(seeds), 9, 3, 0)
    assert ctx.check() == binding.DEV_BAD_SEED
    assert ctx.check() == 0                                # the word is cleared by the read
    w = walks.cpu().numpy()
    assert (w[1] == -1).all() and (w[2] == -1).all()
    good = oracle.sample_walks(rp, ci, seeds[[0, 3]], 9, 3, 0)
    assert np.array_equal(w[[0, 3]], good)


def test_malformed_csr_is_flagged(ctx):
    rp = np.array([0, 2, 4, 6], dtype=np.int32)
    ci = np.array([1, 2, 0, 77, 0, 1], dtype=np.int32)     # node 77 does not exist
    walks = binding.sample_walks(ctx, dev(rp), dev(ci), dev(np.arange(3, dtype=np.int32)), 64, 4, 0)
    assert ctx.check() == binding.DEV_BAD_GRAPH
    w = walks.cpu().numpy()
    assert ((w >= 0) & (w < 3)).all()


def test_bad_walk_entry_is_flagged(ctx):
    walks = np.zeros((3, 4, 3), dtype=np.int32)
    walks[1, 2, 1] = 1000
    off = torch.empty(4, dtype=torch.int64, device="cuda")
    rc, rows = binding.build_rpe_raw(ctx, dev(walks), 10, 0, off, None, None)
    assert rc == binding.OK and rows == 3
    assert ctx.check() == binding.DEV_BAD_WALK


def test_wrong_set_sizes_are_flagged_and_do_not_overlap(ctx):
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(16, dtype=np.int32)
    sizes = torch.empty(16, dtype=torch.int32, device="cuda")
    walks = binding.sample_walks(ctx, dev(rp), dev(ci), dev(seeds), wl.M, wl.m, 0, set_sizes=sizes)
    want_off, want_ids, want_cnt = oracle.build_rpe(walks.cpu().numpy())
    sizes[5] += 3                                         # a size that is not this seed's
    total = int(want_off[-1]) + 3
    off = torch.empty(17, dtype=torch.int64, device="cuda")
    ids = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.zeros((total, wl.m + 1), dtype=torch.int16, device="cuda").view(torch.uint16)
    rc, rows = binding.build_rpe_raw(ctx, walks, wl.n_nodes, total, off, ids, cnt,
                                     set_sizes=sizes)
    assert rc == binding.OK and rows == total
    assert ctx.check() == binding.DEV_BAD_SIZES
    ids_h = ids.cpu().numpy()
    lo, hi = int(want_off[5]), int(want_off[6]) + 3
    assert (ids_h[lo:hi] == -7).all()                      # the mismatched seed wrote nothing
    assert np.array_equal(ids_h[:lo], want_ids[:lo])       # the others are where sizes put them
    assert np.array_equal(ids_h[hi:], want_ids[int(want_off[6]):])


def test_rpe_capacity_overflow_is_reported_and_nothing_is_written_past_it(ctx):
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(64, dtype=np.int32)
    walks = binding.sample_walks(ctx, dev(rp), dev(ci), dev(seeds), wl.M, wl.m, 0)
    want_off, want_ids, want_cnt = oracle.build_rpe(walks.cpu().numpy())
    total = int(want_off[-1])
    cap = total // 2
    L = wl.m + 1
    off = torch.empty(65, dtype=torch.int64, device="cuda")
    ids = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((total, L), 0x7777, dtype=torch.int16, device="cuda").view(torch.uint16)
    rc, rows = binding.build_rpe_raw(ctx, walks, wl.n_nodes, cap, off, ids, cnt)
    assert rc == binding.E_CAPACITY and rows == total
    assert ctx.check() == binding.DEV_CAPACITY
    assert np.array_equal(off.cpu().numpy(), want_off)      # offsets are complete anyway
    ids_h, cnt_h = ids.cpu().numpy(), host_u16(cnt)
    assert (ids_h[cap:] == -7).all() and (cnt_h[cap:] == 0x7777).all()
    fits = want_off[1:] <= cap                               # blocks that fit are written
    last = int(want_off[1:][fits].max())
    assert np.array_equal(ids_h[:last], want_ids[:last])
    assert np.array_equal(cnt_h[:last], want_cnt[:last])


def test_fused_bad_seed_capacity_and_count_only(ctx):
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    M, m, L = wl.M, wl.m, wl.m + 1
    seeds = np.arange(64, dtype=np.int32)
    seeds[7] = 1000                                          # not a node
    seeds[20] = -1
    good = np.ones(64, dtype=bool)
    good[[7, 20]] = False
    w = oracle.sample_walks(rp, ci, seeds[good], M, m, 3)
    want_off, want_ids, want_cnt = oracle.build_rpe(w)
    sizes = np.zeros(64, dtype=np.int64)
    sizes[good] = np.diff(want_off)
    full_off = np.concatenate([[0], np.cumsum(sizes)])
    total = int(full_off[-1])
    d_rp, d_ci, d_seeds = dev(rp), dev(ci), dev(seeds)
    walks = torch.empty((64, M, L), dtype=torch.int32, device="cuda")
    off = torch.empty(65, dtype=torch.int64, device="cuda")
    # offsets and total only
    rc, rows = binding.sample_walks_rpe_raw(ctx, d_rp, d_ci, d_seeds, M, m, 3, walks, 0, off,
                                            None, None)
    assert rc == binding.OK and rows == total
    assert ctx.check() == binding.DEV_BAD_SEED
    assert np.array_equal(off.cpu().numpy(), full_off)
    wh = walks.cpu().numpy()
    assert (wh[7] == -1).all() and (wh[20] == -1).all() and np.array_equal(wh[good], w)
    # a table that is too small: complete offsets, nothing written at or past cap_rows
    cap = total // 2
    ids = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((total, L), 0x7777, dtype=torch.int16, device="cuda").view(torch.uint16)
    rc, rows = binding.sample_walks_rpe_raw(ctx, d_rp, d_ci, d_seeds, M, m, 3, walks, cap, off,
                                            ids, cnt)
    assert rc == binding.E_CAPACITY and rows == total
    assert ctx.check() == binding.DEV_BAD_SEED | binding.DEV_CAPACITY
    assert np.array_equal(off.cpu().numpy(), full_off)
    ids_h, cnt_h = ids.cpu().numpy(), host_u16(cnt)
    assert (ids_h[cap:] == -7).all() and (cnt_h[cap:] == 0x7777).all()
    last = int(full_off[1:][full_off[1:] <= cap].max())
    assert np.array_equal(ids_h[:last], want_ids[:last])
    assert np.array_equal(cnt_h[:last], want_cnt[:last])
    # no seeds at all
    rc, rows = binding.sample_walks_rpe_raw(ctx, d_rp, d_ci, d_seeds[:0], M, m, 3, walks[:0], 0,
                                            off[:1], None, None)
    assert rc == binding.OK and rows == 0 and int(off[0]) == 0


@pytest.mark.parametrize("M,m", [(50, 4), (200, 3)])
def test_fused_kernel_seed_counts_around_its_group_and_window_sizes(ctx, M, m):
    # seeds are handed out in groups of 8 and the offset scan reads 2048 counts a round: seed
    # counts on, just below and just above those sizes, against the two-call path
    wl = synth.Workload("t", "rmat", 2048, 12000, 0.0, M, m, 0, 2, "uniform", graph_seed=5)
    rp, ci = synth.make_graph(wl)
    d_rp, d_ci = dev(rp), dev(ci)
    rng = np.random.default_rng(8)
    all_seeds = dev(rng.integers(0, wl.n_nodes, size=20000).astype(np.int32))
    for n in (1, 2, 7, 8, 9, 15, 16, 17, 63, 64, 65, 511, 2047, 2048, 2049, 4104, 16384, 16391,
              20000):
        d_seeds = all_seeds[:n].contiguous()
        walks = binding.sample_walks(ctx, d_rp, d_ci, d_seeds, M, m, 11)
        off, ids, cnt = binding.build_rpe(ctx, walks, wl.n_nodes)
        f_walks, f_off, f_ids, f_cnt = binding.sample_walks_rpe(ctx, d_rp, d_ci, d_seeds, M, m, 11)
        assert ctx.check() == 0
        assert torch.equal(f_walks, walks), f"walks differ at {n} seeds"
        assert torch.equal(f_off, off), f"offsets differ at {n} seeds"
        assert torch.equal(f_ids, ids), f"ids differ at {n} seeds"
        assert torch.equal(f_cnt.view(torch.int16), cnt.view(torch.int16)), f"counts differ at {n}"


def test_one_pass_captured_in_a_graph_replays_to_the_same_bytes():
    # with no row totals asked for, the calls only enqueue kernels: a pass can be captured once
    # and replayed; every replay (with other work on the stream in between) gives the eager bytes
    wl = synth.Workload("t", "rmat", 4096, 30000, 0.0, 50, 4, 0, 2, "uniform", graph_seed=9)
    rp, ci = synth.make_graph(wl)
    rng = np.random.default_rng(4)
    seeds = rng.integers(0, wl.n_nodes, size=1500).astype(np.int32)
    queries = rng.integers(0, seeds.size, size=(700, 2)).astype(np.int32)
    M, m, L, S = wl.M, wl.m, wl.m + 1, seeds.size
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        c = binding.Context(stream=stream)
        d_rp, d_ci, d_seeds, d_q = dev(rp), dev(ci), dev(seeds), dev(queries)
        cap_r = binding.rpe_rows_bound(S, M, m)
        walks = torch.empty((S, M, L), dtype=torch.int32, device="cuda")
        off = torch.empty(S + 1, dtype=torch.int64, device="cuda")
        ids = torch.empty(cap_r, dtype=torch.int32, device="cuda")
        cnt = torch.empty((cap_r, L), dtype=torch.uint16, device="cuda")
        joff = torch.empty(queries.shape[0] + 1, dtype=torch.int64, device="cuda")
        max_set = 1 + M * m
        # eager pass: sizes the join's output, warms the context's workspaces, is the reference
        rc, R = binding.sample_walks_rpe_raw(c, d_rp, d_ci, d_seeds, M, m, 5, walks, cap_r, off, ids, cnt)
        assert rc == binding.OK
        rc, J = binding.join_queries_raw(c, off, ids, cnt, d_q, max_set, 0, joff, None, None)
        assert rc == binding.OK
        jids = torch.empty(J, dtype=torch.int32, device="cuda")
        jcnt = torch.empty((J, 2, L), dtype=torch.uint16, device="cuda")
        rc, _ = binding.join_queries_raw(c, off, ids, cnt, d_q, max_set, J, joff, jids, jcnt)
        assert rc == binding.OK and c.check() == 0
        outs = [walks, off, ids[:R], cnt[:R].view(torch.int16), joff, jids, jcnt.view(torch.int16)]
        want = [t.clone() for t in outs]

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream, capture_error_mode="thread_local"):
            rc1, _ = binding.sample_walks_rpe_raw(c, d_rp, d_ci, d_seeds, M, m, 5, walks, cap_r, off,
                                                  ids, cnt, want_rows=False)
            rc2, _ = binding.join_queries_raw(c, off, ids, cnt, d_q, max_set, J, joff, jids, jcnt,
                                              want_rows=False)
        assert rc1 == binding.OK and rc2 == binding.OK
        for replay in range(3):
            for t in outs:
                t.fill_(-7 - replay)                 # eager work between the replays
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            assert c.check() == 0, f"replay {replay}"
            for got, ref in zip(outs, want):
                assert torch.equal(got, ref), f"replay {replay} differs from the eager pass"
        c.close()


def test_fused_kernel_waits_are_bounded(ctx):
    # with a spin limit of zero every wait inside the fused kernel gives up at once: the kernel
    # must still end, say so, and write nothing out of place; the default limit then gives the
    # right table again
    wl = synth.Workload("t", "rmat", 4096, 30000, 0.0, 50, 4, 0, 2, "uniform", graph_seed=9)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(wl.n_nodes, dtype=np.int32)
    d_rp, d_ci, d_seeds = dev(rp), dev(ci), dev(seeds)
    M, m, L = wl.M, wl.m, wl.m + 1
    cap = binding.rpe_rows_bound(seeds.size, M, m)
    walks = torch.empty((seeds.size, M, L), dtype=torch.int32, device="cuda")
    off = torch.empty(seeds.size + 1, dtype=torch.int64, device="cuda")
    ids = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.zeros((cap, L), dtype=torch.int16, device="cuda").view(torch.uint16)
    ctx.set_spin_limit(0)
    try:
        rc, _ = binding.sample_walks_rpe_raw(ctx, d_rp, d_ci, d_seeds, M, m, 0, walks, cap, off,
                                             ids, cnt, want_rows=False)
        assert rc == binding.OK
        flags = ctx.check()
    finally:
        ctx.set_spin_limit(1 << 22)
    assert flags & ~binding.DEV_STALL == 0
    w = oracle.sample_walks(rp, ci, seeds, M, m, 0)
    want = oracle.build_rpe(w)
    if flags == 0:
        assert_table_equal((off, ids[:int(off[-1])], cnt[:int(off[-1])]), want, "rpe")
    else:
        # whatever was written is a correct prefix of the table or untouched memory
        ids_h = ids.cpu().numpy()[:want[1].size]
        assert ((ids_h == want[1]) | (ids_h == -7)).all()
    f_walks, f_off, f_ids, f_cnt = binding.sample_walks_rpe(ctx, d_rp, d_ci, d_seeds, M, m, 0)
    assert ctx.check() == 0
    assert np.array_equal(f_walks.cpu().numpy(), w)
    assert_table_equal((f_off, f_ids, f_cnt), want, "rpe after the limit was restored")


def test_prune_capacity_and_degenerate_tables(ctx):
    rng = np.random.default_rng(3)
    cnt = rng.integers(0, 3, size=(5000, 4)).astype(np.uint16)          # at most 81 vectors
    want_T, want_code = oracle.prune_rpe(cnt)
    d_cnt = dev(cnt.view(np.int16)).view(torch.uint16)
    n_T = want_T.shape[0]
    T = torch.zeros((n_T, 4), dtype=torch.int16, device="cuda").view(torch.uint16)
    code = torch.empty(5000, dtype=torch.int32, device="cuda")
    rc, got = binding.prune_rpe_raw(ctx, d_cnt, n_T, T, code)           # exactly enough room
    assert rc == binding.OK and got == n_T and ctx.check() == 0
    assert np.array_equal(host_u16(T), want_T) and np.array_equal(code.cpu().numpy(), want_code)
    rc, got = binding.prune_rpe_raw(ctx, d_cnt, n_T - 1, T, code)       # one too few
    assert rc == binding.E_CAPACITY and got == n_T
    assert ctx.check() == binding.DEV_CAPACITY
    # one row, all rows equal, widest vectors (m = 15), no rows
    for arr in (np.array([[7, 0, 9]], np.uint16), np.full((300, 5), 65535, np.uint16),
                rng.integers(0, 2, size=(700, 16)).astype(np.uint16),
                np.zeros((0, 4), np.uint16)):
        T, code = binding.prune_rpe(ctx, dev(arr.view(np.int16)).view(torch.uint16), cap_T=1024)
        assert ctx.check() == 0
        w_T, w_code = oracle.prune_rpe(arr)
        assert np.array_equal(host_u16(T).reshape(w_T.shape), w_T)
        assert np.array_equal(code.cpu().numpy(), w_code)


def test_query_rpe_ids_problems_are_flagged(ctx):
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(32, dtype=np.int32)
    walks, off, ids, cnt = binding.sample_walks_rpe(ctx, dev(rp), dev(ci), dev(seeds), wl.M, wl.m, 0)
    q = np.array([[1, 2], [5, 32], [3, 4]], dtype=np.int32)          # 32 is not a block
    got = binding.query_rpe_ids(ctx, walks, off, ids, dev(q), max_set=61).cpu().numpy()
    assert ctx.check() == binding.DEV_BAD_QUERY
    assert (got[1] == -1).all()
    want = oracle.query_rpe_ids(walks.cpu().numpy(), off.cpu().numpy(), ids.cpu().numpy(),
                                q[[0, 2]])
    assert np.array_equal(got[[0, 2]].astype(np.int64), want)
    sizes = np.diff(off.cpu().numpy())
    big = int(np.argmax(sizes))
    got = binding.query_rpe_ids(ctx, walks, off, ids, dev(np.array([[big, 0]], np.int32)),
                                max_set=int(sizes[big]) - 1)
    assert ctx.check() == binding.DEV_SET_TOO_LARGE and bool((got == -1).all())


def test_join_problems_are_flagged(ctx):
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(32, dtype=np.int32)
    out = gpu_pipeline(ctx, rp, ci, seeds, wl.M, wl.m, 0)
    off, ids, cnt = out["rpe"]
    table = oracle.build_rpe(out["walks"].cpu().numpy())
    good = np.array([[1, 2], [3, 4]], dtype=np.int32)
    want = oracle.join_queries(*table, good)
    # a query entry outside the table: that query yields no rows, the others are intact
    q = np.array([[1, 2], [5, 32], [-1, 0], [3, 4]], dtype=np.int32)
    joff, jids, jcnt = binding.join_queries(ctx, off, ids, cnt, dev(q), max_set=61)
    assert ctx.check() == binding.DEV_BAD_QUERY
    joff_h = joff.cpu().numpy()
    assert joff_h[2] == joff_h[1] and joff_h[3] == joff_h[2]
    assert np.array_equal(jids.cpu().numpy(), want[1])
    assert np.array_equal(host_u16(jcnt), want[2])
    # max_set smaller than a queried block
    sizes = np.diff(table[0])
    big = int(np.argmax(sizes))
    assert sizes[big] >= 2
    joff, jids, jcnt = binding.join_queries(ctx, off, ids, cnt,
                                            dev(np.array([[big, big]], np.int32)),
                                            max_set=int(sizes[big]) - 1)
    assert ctx.check() == binding.DEV_SET_TOO_LARGE
    assert jids.numel() == 0
    # capacity
    joff = torch.empty(3, dtype=torch.int64, device="cuda")
    total = int(want[0][-1])
    jids = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    jcnt = torch.zeros((total, 2, 4), dtype=torch.int16, device="cuda").view(torch.uint16)
    cap = int(want[0][1])                                    # room for the first query only
    rc, rows = binding.join_queries_raw(ctx, off, ids, cnt, dev(good), 61, cap, joff, jids, jcnt)
    assert rc == binding.E_CAPACITY and rows == total
    assert ctx.check() == binding.DEV_CAPACITY
    assert np.array_equal(jids.cpu().numpy()[:cap], want[1][:cap])
    assert (jids.cpu().numpy()[cap:] == -7).all()


# --------------------------------------------------------------------------- #
# the two phases as calls of their own: size, allocate, fill
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("M,m,k", [(50, 4, 2), (200, 3, 3), (33, 2, 2), (20, 7, 3)])
def test_count_then_fill_calls_against_the_oracle(ctx, M, m, k):
    wl = synth.Workload("t", "rmat", 2048, 12000, 0.0, M, m, 0, k, "uniform", graph_seed=21)
    rp, ci = synth.make_graph(wl)
    rng = np.random.default_rng(M + m)
    seeds = rng.integers(0, wl.n_nodes, size=777).astype(np.int32)
    queries = rng.integers(0, seeds.size, size=(1501, k)).astype(np.int32)
    L = m + 1
    w = oracle.sample_walks(rp, ci, seeds, M, m, 9)
    table = oracle.build_rpe(w)
    joined = oracle.join_queries(*table, queries)

    walks = binding.sample_walks(ctx, dev(rp), dev(ci), dev(seeds), M, m, 9)
    off = torch.empty(seeds.size + 1, dtype=torch.int64, device="cuda")
    rc, R = binding.build_rpe_count(ctx, walks, wl.n_nodes, off)
    assert rc == binding.OK and R == table[1].size
    assert np.array_equal(off.cpu().numpy(), table[0])
    ids = torch.empty(R, dtype=torch.int32, device="cuda")
    cnt = torch.empty((R, L), dtype=torch.uint16, device="cuda")
    kept = off.clone()
    assert binding.build_rpe_fill(ctx, walks, wl.n_nodes, off, R, ids, cnt) == binding.OK
    assert ctx.check() == 0
    assert torch.equal(off, kept), "the filling call changed the offsets it was given"
    assert_table_equal((off, ids, cnt), table, "rpe by count + fill")

    d_q = dev(queries)
    joff = torch.empty(queries.shape[0] + 1, dtype=torch.int64, device="cuda")
    rc, J = binding.join_count(ctx, off, ids, d_q, 1 + M * m, joff)
    assert rc == binding.OK and J == joined[1].size
    jids = torch.empty(J, dtype=torch.int32, device="cuda")
    jcnt = torch.empty((J, k, L), dtype=torch.uint16, device="cuda")
    kept = joff.clone()
    assert binding.join_fill(ctx, off, ids, cnt, d_q, 1 + M * m, joff, J, jids, jcnt) == binding.OK
    assert ctx.check() == 0
    assert torch.equal(joff, kept)
    assert_table_equal((joff, jids, jcnt), joined, "join by count + fill")
    # offsets kept from an earlier call fill again without any counting
    jids.fill_(-7)
    assert binding.join_fill(ctx, off, ids, cnt, d_q, 1 + M * m, joff, J, jids, jcnt) == binding.OK
    assert ctx.check() == 0
    assert np.array_equal(jids.cpu().numpy(), joined[1])


def test_fill_calls_with_offsets_of_something_else_are_flagged(ctx):
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(40, dtype=np.int32)
    walks, off, ids, cnt = binding.sample_walks_rpe(ctx, dev(rp), dev(ci), dev(seeds), wl.M, wl.m, 0)
    table = oracle.build_rpe(walks.cpu().numpy())
    q = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.int32)
    want = oracle.join_queries(*table, q)
    joff = torch.from_numpy(want[0].copy()).cuda()
    joff[2:] += 2                                      # query 1 is given two rows too many
    total = int(joff[-1])
    jids = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    jcnt = torch.zeros((total, 2, 4), dtype=torch.int16, device="cuda").view(torch.uint16)
    assert binding.join_fill(ctx, off, ids, cnt, dev(q), 61, joff, total, jids, jcnt) == binding.OK
    assert ctx.check() == binding.DEV_BAD_SIZES
    got = jids.cpu().numpy()
    lo, hi = int(want[0][1]), int(want[0][2]) + 2
    assert (got[lo:hi] == -7).all()                    # the mismatched query wrote nothing
    assert np.array_equal(got[:lo], want[1][:lo])      # the others are where the offsets put them
    assert np.array_equal(got[hi:], want[1][int(want[0][2]):])
    # the same for the table's rows
    roff = torch.from_numpy(table[0].copy()).cuda()
    roff[6:] += 1
    total = int(roff[-1])
    rids = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    rcnt = torch.zeros((total, 4), dtype=torch.int16, device="cuda").view(torch.uint16)
    assert binding.build_rpe_fill(ctx, walks, wl.n_nodes, roff, total, rids, rcnt) == binding.OK
    assert ctx.check() == binding.DEV_BAD_SIZES
    got = rids.cpu().numpy()
    lo, hi = int(table[0][5]), int(table[0][6]) + 1
    assert (got[lo:hi] == -7).all()
    assert np.array_equal(got[:lo], table[1][:lo]) and np.array_equal(got[hi:], table[1][int(table[0][6]):])


def test_bad_seeds_give_the_same_table_on_both_paths(ctx):
    # a seed that is not a node gets walks of -1 and no rows, whether the table is built by the
    # fused kernel or by surel_build_rpe over those walks
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(50, dtype=np.int32)
    seeds[[0, 17, 49]] = [-1, 256, 1 << 30]
    good = np.ones(50, dtype=bool)
    good[[0, 17, 49]] = False
    d_rp, d_ci, d_seeds = dev(rp), dev(ci), dev(seeds)
    f_walks, f_off, f_ids, f_cnt = binding.sample_walks_rpe(ctx, d_rp, d_ci, d_seeds, wl.M, wl.m, 2)
    assert ctx.check() == binding.DEV_BAD_SEED
    for sizes in (None, torch.empty(50, dtype=torch.int32, device="cuda")):
        walks = binding.sample_walks(ctx, d_rp, d_ci, d_seeds, wl.M, wl.m, 2, set_sizes=sizes)
        assert ctx.check() == binding.DEV_BAD_SEED
        off, ids, cnt = binding.build_rpe(ctx, walks, wl.n_nodes, set_sizes=sizes)
        assert ctx.check() == binding.DEV_BAD_WALK          # the -1 entries are left out, and said so
        assert torch.equal(walks, f_walks) and torch.equal(off, f_off) and torch.equal(ids, f_ids)
        assert torch.equal(cnt.view(torch.int16), f_cnt.view(torch.int16))
    w = oracle.sample_walks(rp, ci, seeds[good], wl.M, wl.m, 2)
    t_off, t_ids, t_cnt = oracle.build_rpe(w)
    sizes_h = np.zeros(50, dtype=np.int64)
    sizes_h[good] = np.diff(t_off)
    assert np.array_equal(f_off.cpu().numpy(), np.concatenate([[0], np.cumsum(sizes_h)]))
    assert np.array_equal(f_ids.cpu().numpy(), t_ids) and np.array_equal(host_u16(f_cnt), t_cnt)


@pytest.mark.parametrize("k", [2, 3])
def test_join_query_counts_around_workgroup_and_scan_tile_sizes(ctx, k):
    # 4 waves a workgroup, 2048 counts per tile of the offset scan: query counts on and around
    # those sizes against the oracle
    wl = synth.Workload("t", "rmat", 2048, 12000, 0.0, 50, 4, 0, k, "uniform", graph_seed=5)
    rp, ci = synth.make_graph(wl)
    seeds = np.arange(wl.n_nodes, dtype=np.int32)
    walks, off, ids, cnt = binding.sample_walks_rpe(ctx, dev(rp), dev(ci), dev(seeds), wl.M, wl.m, 4)
    table = oracle.build_rpe(walks.cpu().numpy())
    rng = np.random.default_rng(k)
    all_q = rng.integers(0, wl.n_nodes, size=(20000, k)).astype(np.int32)
    for n in (1, 2, 7, 8, 9, 15, 16, 17, 31, 33, 64, 2047, 2048, 2049, 4104, 16391, 20000):
        want = oracle.join_queries(*table, all_q[:n])
        got = binding.join_queries(ctx, off, ids, cnt, dev(all_q[:n]), max_set=201,
                                   cap_rows=int(want[0][-1]) + 5)
        assert ctx.check() == 0
        assert_table_equal(got, want, f"join of {n} queries")


def hand_made_table(blocks, L, rng):
    """An RPE table whose blocks hold the given ascending id lists and random counts."""
    off = np.zeros(len(blocks) + 1, dtype=np.int64)
    off[1:] = np.cumsum([len(b) for b in blocks])
    ids = np.concatenate([np.asarray(b, dtype=np.int32) for b in blocks]) if off[-1] else \
        np.zeros(0, dtype=np.int32)
    cnt = rng.integers(0, 65536, size=(int(off[-1]), L)).astype(np.uint16)
    return off, ids, cnt


@pytest.mark.parametrize("max_set", [1, 31, 32, 33, 64, 96, 2048])
@pytest.mark.parametrize("L", [2, 4, 5, 7])
def test_join_of_hand_made_tables_around_64_row_boundaries(ctx, max_set, L):
    # pairs whose unions end exactly at, one before and one after a multiple of 64 rows (the
    # union's bit masks are 64-bit words; a round of the filling loop is 64 rows), from lists
    # that are disjoint, equal, interleaved, nested, empty, and full sets of max_set nodes
    rng = np.random.default_rng(1000 * max_set + L)
    n = max_set
    even, odd = np.arange(0, 2 * n, 2), np.arange(1, 2 * n, 2)
    low, high = np.arange(n), np.arange(n, 2 * n)
    blocks = [even, odd, low, high, low[: n // 2], low[n // 2:], np.zeros(0, dtype=np.int64),
              low[:1], high[-1:], even[: max(n - 1, 0)], np.sort(rng.choice(4 * n, n, replace=False)),
              np.sort(rng.choice(4 * n, n, replace=False))]
    table = hand_made_table(blocks, L, rng)
    nb = len(blocks)
    queries = np.array([(a, b) for a in range(nb) for b in range(nb)], dtype=np.int32)
    want = oracle.join_queries(*table, queries)
    sizes = np.diff(want[0])
    assert sizes.max() == 2 * n and (sizes == 0).any()
    d_table = (dev(table[0]), dev(table[1]), dev(table[2].view(np.int16)).view(torch.uint16))
    got = binding.join_queries(ctx, *d_table, dev(queries), max_set=max_set)
    assert ctx.check() == 0
    assert_table_equal(got, want, f"hand-made join, max_set {max_set}, L {L}")
    if max_set > 96:
        return
    # and as triples: (a, b, b) and (a, a, b) have the union of (a, b) with a list repeated
    tri = np.concatenate([queries[:, [0, 1, 1]], queries[:, [0, 0, 1]]])[:: 3]
    want3 = oracle.join_queries(*table, tri)
    got3 = binding.join_queries(ctx, *d_table, dev(tri), max_set=max_set)
    assert ctx.check() == 0
    assert_table_equal(got3, want3, f"hand-made join of triples, max_set {max_set}, L {L}")


def test_largest_node_ids(ctx):
    # a graph with the most nodes the library takes (2^28 - 1): the largest ids make sort keys
    # (id << 4 | position) that use all 32 bits and must still sort in front of the padding
    n = binding.MAX_NODES
    top = [n - 1, n - 2, n - 3, n - 4]
    edges = [(a, b) for i, a in enumerate(top) for b in top[i + 1:]]
    edges += [(0, n - 1), (12345, n - 2), (n - 5, 7), (7, 12345)]
    rp, ci = synth.csr_from_edge_list(n, edges)
    seeds = np.array([n - 1, 0, n - 2, 12345, n - 5, 7, n - 3, 5, n - 1], dtype=np.int32)  # 5: isolated
    queries = np.array([[0, 2], [1, 6], [8, 0], [7, 7], [3, 4], [5, 2]], dtype=np.int32)
    out = full_compare(ctx, rp, ci, seeds, 60, 4, 3, queries)
    assert int(out["walks"].max()) == n - 1


def hub_and_ring(n_leaves):
    """Node 0 joined to every one of n_leaves leaves, the leaves joined in a chain."""
    leaf = np.arange(1, n_leaves + 1, dtype=np.int64)
    deg = np.full(n_leaves + 1, 3, dtype=np.int64)
    deg[0], deg[1], deg[n_leaves] = n_leaves, 2, 2
    rp = np.zeros(n_leaves + 2, dtype=np.int64)
    np.cumsum(deg, out=rp[1:])
    ci = np.empty(int(rp[-1]), dtype=np.int32)
    ci[:n_leaves] = leaf
    ci[rp[1:-1]] = 0                                       # every leaf's row: hub, left, right
    ci[rp[2:-1] + 1] = leaf[1:] - 1
    ci[rp[1:-2] + 2 - (leaf[:-1] == 1)] = leaf[:-1] + 1
    return rp.astype(np.int32), ci


def test_packed_edge_records_and_a_degree_beyond_their_field(ctx):
    # from 2^22 edge entries on, the walks read 8-byte neighbour records; the hub's degree
    # (1.2 M) does not fit the 20 bits the record leaves for it and is taken from the CSR
    n_leaves = 1_200_000
    rp, ci = hub_and_ring(n_leaves)
    assert ci.size >= 1 << 22 and np.all(np.diff(rp) > 0)
    rng = np.random.default_rng(5)
    seeds = rng.integers(0, n_leaves + 1, size=50_000, dtype=np.int32)
    seeds[:3] = [0, 1, n_leaves]
    M, m = 200, 3
    assert seeds.size * M * (m - 1) >= 4 * ci.size         # enough steps to make the records
    w = oracle.sample_walks(rp, ci, seeds, M, m, 11)
    assert (w[:, :, 1:] == 0).mean() > 0.2                 # walks do pass through the hub
    table = oracle.build_rpe(w)
    d_rp, d_ci, d_seeds = dev(rp), dev(ci), dev(seeds)
    walks = binding.sample_walks(ctx, d_rp, d_ci, d_seeds, M, m, 11)
    assert ctx.check() == 0
    assert np.array_equal(walks.cpu().numpy(), w), "walks differ"
    del walks
    f_walks, f_off, f_ids, f_cnt = binding.sample_walks_rpe(ctx, d_rp, d_ci, d_seeds, M, m, 11)
    assert ctx.check() == 0
    assert np.array_equal(f_walks.cpu().numpy(), w), "fused: walks differ"
    assert_table_equal((f_off, f_ids, f_cnt), table, "fused rpe")
    # an entry that names no node: flagged, the walker stays where it is
    bad = ci.copy()
    bad[rp[7]] = n_leaves + 1 + 40
    walks = binding.sample_walks(ctx, d_rp, dev(bad), dev(np.full(seeds.size, 7, dtype=np.int32)),
                                 M, m, 11)
    assert ctx.check() == binding.DEV_BAD_GRAPH
    got = walks.cpu().numpy()
    assert ((got >= 0) & (got <= n_leaves)).all()
    stay = (got[:, :, 1] == 7)
    assert 0.2 < stay.mean() < 0.5                         # one of node 7's three entries


def test_one_call_rpe_ids_capacity(ctx):
    # surel_sample_walks_rpe_ids with too little room: for the table, for the distinct vectors
    wl = synth.Workload("t", "rmat", 256, 900, 0.0, 20, 3, 0, 2, "uniform", graph_seed=3)
    rp, ci = synth.make_graph(wl)
    M, m, L = wl.M, wl.m, wl.m + 1
    seeds = np.arange(64, dtype=np.int32)
    w = oracle.sample_walks(rp, ci, seeds, M, m, 3)
    t_off, t_ids, t_cnt = oracle.build_rpe(w)
    want_T, want_code = oracle.prune_rpe(t_cnt)
    total, n_T = int(t_off[-1]), want_T.shape[0]
    d_rp, d_ci, d_seeds = dev(rp), dev(ci), dev(seeds)
    walks = torch.empty((64, M, L), dtype=torch.int32, device="cuda")
    off = torch.empty(65, dtype=torch.int64, device="cuda")
    ids = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    code = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    T = torch.zeros((n_T, L), dtype=torch.int16, device="cuda").view(torch.uint16)
    # exactly enough room for both
    rc, rows, got_T = binding.sample_walks_rpe_ids_raw(ctx, d_rp, d_ci, d_seeds, M, m, 3, walks,
                                                       total, off, ids, None, code, n_T, T)
    assert rc == binding.OK and rows == total and got_T == n_T and ctx.check() == 0
    assert np.array_equal(host_u16(T), want_T) and np.array_equal(code.cpu().numpy(), want_code)
    assert np.array_equal(ids.cpu().numpy(), t_ids) and np.array_equal(off.cpu().numpy(), t_off)
    # one distinct vector too many
    rc, rows, got_T = binding.sample_walks_rpe_ids_raw(ctx, d_rp, d_ci, d_seeds, M, m, 3, walks,
                                                       total, off, ids, None, code, n_T - 1, T)
    assert rc == binding.E_CAPACITY and rows == total and got_T == n_T
    assert ctx.check() == binding.DEV_CAPACITY
    # a table that is too small: complete offsets and walks, the totals reported, nothing
    # written at or past cap_rows
    cap = total // 2
    ids.fill_(-7)
    code.fill_(-7)
    rc, rows, got_T = binding.sample_walks_rpe_ids_raw(ctx, d_rp, d_ci, d_seeds, M, m, 3, walks,
                                                       cap, off, ids, None, code, n_T, T)
    assert rc == binding.E_CAPACITY and rows == total
    assert ctx.check() == binding.DEV_CAPACITY
    assert np.array_equal(off.cpu().numpy(), t_off) and np.array_equal(walks.cpu().numpy(), w)
    assert (ids.cpu().numpy()[cap:] == -7).all() and (code.cpu().numpy()[cap:] == -7).all()
    last = int(t_off[1:][t_off[1:] <= cap].max())
    assert np.array_equal(ids.cpu().numpy()[:last], t_ids[:last])
    # no seeds at all
    rc, rows, got_T = binding.sample_walks_rpe_ids_raw(ctx, d_rp, d_ci, d_seeds[:0], M, m, 3,
                                                       walks[:0], 0, off[:1], ids, None, code, n_T, T)
    assert rc == binding.OK and rows == 0 and got_T == 0 and int(off[0]) == 0
