"""The workloads at their full sizes: every output of the HIP path against the CPU oracle.

Nothing is sampled.  The oracle runs over ALL seeds and ALL queries of a workload, in
contiguous blocks on a pool of host threads (its outputs are per seed and per query, its
random stream is counter-based, and ctypes drops the GIL), and every block is compared byte
for byte with the same slice of what the GPU wrote: walks, RPE offsets / ids / counts, join
offsets / ids / counts, the per-walk-position RPE-IDs, and the pruned array with the rows'
codes.  The oracle only ever sees inputs (the graph, the seeds, the queries) and its own
outputs; the invariants that hold at any size stay as a second net.
"""
import os
from collections import deque
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_2202_13538_amd import binding, synth
from test_gpu_parity import dev, host_u16

pytestmark = pytest.mark.gpu

HOST_THREADS = max(1, min(16, os.cpu_count() or 1))


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(binding.LIB_PATH), "libsurel.so is not built"
    c = binding.Context()
    yield c
    c.close()


@pytest.fixture
def say(capsys):
    """Progress lines that reach the terminal although pytest captures output."""
    def emit(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return emit


def in_order(pool, fn, items, window):
    """fn(item) for every item on the pool; results in item order, at most `window` in flight
    or waiting (so that the blocks' arrays never pile up)."""
    pending = deque()
    for item in items:
        pending.append(pool.submit(fn, item))
        if len(pending) >= window:
            yield pending.popleft().result()
    while pending:
        yield pending.popleft().result()


def segment_sums(flat_u16, off, chunk=1 << 24):
    """Per-segment column sums of a uint16 [rows][cols] tensor, segments given by ``off``."""
    n_seg = off.numel() - 1
    rows, cols = flat_u16.shape
    sizes = off[1:] - off[:-1]
    seg_of_row = torch.repeat_interleave(torch.arange(n_seg, device=off.device), sizes)
    sums = torch.zeros((n_seg, cols), dtype=torch.int64, device=off.device)
    as_i16 = flat_u16.view(torch.int16)
    for s in range(0, rows, chunk):
        e = min(rows, s + chunk)
        sums.index_add_(0, seg_of_row[s:e], as_i16[s:e].to(torch.int64) & 0xFFFF)
    return sums


def same_u16(a, b, chunk=1 << 28):
    """torch.equal for uint16 tensors of any size (compared as int16, piece by piece)."""
    if a.shape != b.shape:
        return False
    a, b = a.view(torch.int16).reshape(-1), b.view(torch.int16).reshape(-1)
    return all(torch.equal(a[s:s + chunk], b[s:s + chunk]) for s in range(0, a.numel(), chunk))


def sweep_seeds(pool, rp, ci, N, M, m, rng_seed, walks, off, ids, cnt, say, tag, keep_walks=True):
    """All seeds 0..N-1, block by block: the oracle's walks and RPE rows against the GPU's.
    Returns the oracle's own walks (None unless keep_walks) and table (host arrays) for the
    query sweeps."""
    L = m + 1
    block = max(1024, (1 << 24) // (M * L))
    bound = N * (1 + M * m)                       # App. D.4; pages are only touched when written
    o_walks = np.empty((N, M, L), dtype=np.int32) if keep_walks else None
    o_off = np.zeros(N + 1, dtype=np.int64)
    o_ids = np.empty(bound, dtype=np.int32)
    o_cnt = np.empty((bound, L), dtype=np.uint16)
    off_h = off.cpu().numpy()

    def job(s0):
        s1 = min(N, s0 + block)
        w = oracle.sample_walks(rp, ci, np.arange(s0, s1, dtype=np.int32), M, m, rng_seed)
        return s0, s1, w, oracle.build_rpe(w)

    done = 0
    for s0, s1, w, (b_off, b_ids, b_cnt) in in_order(pool, job, range(0, N, block),
                                                    2 * HOST_THREADS):
        assert np.array_equal(walks[s0:s1].cpu().numpy(), w), f"{tag}: walks differ in seeds {s0}..{s1}"
        r0 = int(o_off[s0])
        r1 = r0 + b_ids.size
        o_off[s0 + 1:s1 + 1] = r0 + b_off[1:]
        assert np.array_equal(off_h[s0:s1 + 1], o_off[s0:s1 + 1]), f"{tag}: rpe_off differs in seeds {s0}..{s1}"
        assert np.array_equal(ids[r0:r1].cpu().numpy(), b_ids), f"{tag}: rpe_ids differ in seeds {s0}..{s1}"
        assert np.array_equal(host_u16(cnt[r0:r1]), b_cnt), f"{tag}: rpe_cnt differs in seeds {s0}..{s1}"
        if keep_walks:
            o_walks[s0:s1] = w
        o_ids[r0:r1] = b_ids
        o_cnt[r0:r1] = b_cnt
        done += 1
        if done % 16 == 0:
            say(f"[{tag}] walks + table: seeds ..{s1} of {N} equal the oracle's")
    R = int(o_off[N])
    assert ids.shape[0] == R and cnt.shape[0] == R, f"{tag}: row total differs"
    return o_walks, (o_off, o_ids[:R], o_cnt[:R])


def sweep_join(pool, table, queries, joff, jids, jcnt, say, tag):
    """All queries, block by block: the oracle's join of its own table against the GPU's."""
    Q = queries.shape[0]
    block = 1 << 13
    joff_h = joff.cpu().numpy()

    def job(q0):
        q1 = min(Q, q0 + block)
        return q0, q1, oracle.join_queries(*table, queries[q0:q1])

    j0 = 0
    for q0, q1, (b_off, b_ids, b_cnt) in in_order(pool, job, range(0, Q, block), 2 * HOST_THREADS):
        j1 = j0 + b_ids.size
        assert np.array_equal(joff_h[q0:q1 + 1], j0 + b_off), f"{tag}: join_off differs in queries {q0}..{q1}"
        assert np.array_equal(jids[j0:j1].cpu().numpy(), b_ids), f"{tag}: join_ids differ in queries {q0}..{q1}"
        assert np.array_equal(host_u16(jcnt[j0:j1]), b_cnt), f"{tag}: join_cnt differs in queries {q0}..{q1}"
        j0 = j1
    assert jids.shape[0] == j0 and int(joff_h[Q]) == j0, f"{tag}: joined row total differs"
    say(f"[{tag}] join: all {Q} queries ({j0} rows) equal the oracle's")
    return j0


def sweep_query_ids(pool, o_walks, table, queries, qids, say, tag):
    """All queries, block by block: the oracle's per-walk-position RPE-IDs against the GPU's."""
    Q, k = queries.shape
    per_query = k * o_walks.shape[1] * o_walks.shape[2] * k
    block = max(64, (1 << 24) // per_query)

    def job(q0):
        q1 = min(Q, q0 + block)
        return q0, q1, oracle.query_rpe_ids(o_walks, table[0], table[1], queries[q0:q1])

    for q0, q1, want in in_order(pool, job, range(0, Q, block), 2 * HOST_THREADS):
        assert np.array_equal(qids[q0:q1].cpu().numpy(), want), f"{tag}: RPE-IDs differ in queries {q0}..{q1}"
    say(f"[{tag}] query-level RPE-IDs: all {Q} queries equal the oracle's")


def oracle_prune_blockwise(pool, o_cnt):
    """oracle.prune_rpe over a table too long for one single-threaded call, through calls on row
    blocks: the table's distinct vectors are the distinct vectors among the blocks' distinct
    vectors (one more call, on their concatenation), and a row's index in the whole follows
    through its index in its block."""
    R = o_cnt.shape[0]
    block = 1 << 23
    starts = list(range(0, R, block))
    parts = list(in_order(pool, lambda r0: oracle.prune_rpe(o_cnt[r0:r0 + block]), starts,
                          2 * HOST_THREADS))
    T, where = oracle.prune_rpe(np.concatenate([T_b for T_b, _ in parts]))
    code = np.empty(R, dtype=np.int32)
    base = 0
    for r0, (T_b, code_b) in zip(starts, parts):
        code[r0:r0 + code_b.size] = where[base + code_b]
        base += T_b.shape[0]
    return T, code


def check_workload(ctx, name, say):
    wl = synth.WORKLOADS[name]
    rp, ci = synth.make_graph(wl)
    queries = synth.make_queries(wl, rp, ci)
    N, M, m, k = wl.n_nodes, wl.M, wl.m, wl.k
    L = m + 1
    max_set = 1 + M * m
    d_rp, d_ci, d_q = dev(rp), dev(ci), dev(queries)
    d_seeds = torch.arange(N, dtype=torch.int32, device="cuda")
    say(f"[{name}] graph ready: N={N} E2={ci.size} M={M} m={m} queries={queries.shape}, "
        f"{HOST_THREADS} oracle threads")

    # the fused kernel (what the benchmark times): whole output against the oracle
    walks, off, ids, cnt = binding.sample_walks_rpe(ctx, d_rp, d_ci, d_seeds, M, m, wl.rng_seed)
    assert ctx.check() == 0
    R = int(off[-1])
    with ThreadPoolExecutor(HOST_THREADS) as pool:
        o_walks, table = sweep_seeds(pool, rp, ci, N, M, m, wl.rng_seed, walks, off, ids, cnt, say,
                                     name)
        say(f"[{name}] fused walk + RPE: all {N} seeds, {R} rows equal the oracle's")

        # the two-call path gives the same bytes (with the walk kernel's set sizes, and with the
        # RPE builder's own counting pass for the layout)
        sizes = torch.empty(N, dtype=torch.int32, device="cuda")
        walks2 = binding.sample_walks(ctx, d_rp, d_ci, d_seeds, M, m, wl.rng_seed, set_sizes=sizes)
        off2, ids2, cnt2 = binding.build_rpe(ctx, walks2, N, cap_rows=R, set_sizes=sizes)
        assert ctx.check() == 0
        assert torch.equal(walks2, walks) and torch.equal(off2, off) and torch.equal(ids2, ids)
        assert same_u16(cnt2, cnt), "two calls: counts differ"
        off3 = torch.empty_like(off)
        rc, rows3 = binding.build_rpe_raw(ctx, walks2, N, 0, off3, None, None)
        assert rc == binding.OK and rows3 == R and torch.equal(off3, off)
        del walks2, off2, ids2, cnt2, off3, sizes
        say(f"[{name}] sample_walks + build_rpe equal the fused kernel")

        # invariants over the whole table
        assert int(off[0]) == 0 and bool((off[1:] > off[:-1]).all())
        assert bool((segment_sums(cnt, off) == M).all()), "a step's counts do not sum to M"
        inner = torch.ones(R, dtype=torch.bool, device="cuda")
        inner[off[:-1]] = False                                  # first row of every block
        assert bool((ids[1:] > ids[:-1])[inner[1:]].all()), "ids not ascending inside a block"
        slot0 = cnt.view(torch.int16)[:, 0].to(torch.int32) & 0xFFFF
        assert int((slot0 > 0).sum()) == N and bool((slot0[slot0 > 0] == M).all())
        del inner, slot0

        # the join, all queries
        joff, jids, jcnt = binding.join_queries(ctx, off, ids, cnt, d_q, max_set=max_set)
        assert ctx.check() == 0
        J = sweep_join(pool, table, queries, joff, jids, jcnt, say, name)
        sizes_q = (off[1:] - off[:-1])[d_q.long()]
        jn = joff[1:] - joff[:-1]
        assert bool((jn >= sizes_q.max(dim=1).values).all()) and bool((jn <= sizes_q.sum(dim=1)).all())
        assert bool((segment_sums(jcnt.reshape(J, k * L), joff) == M).all()), \
            "a joined half does not sum to M per step"

        # pruning: the whole array T and every row's code
        T, code = binding.prune_rpe(ctx, cnt)
        assert ctx.check() == 0
        want_T, want_code = oracle_prune_blockwise(pool, table[2])
        assert np.array_equal(host_u16(T), want_T), "pruned array differs"
        assert np.array_equal(code.cpu().numpy(), want_code), "re-indexed rows differ"
        say(f"[{name}] pruning: {T.shape[0]} distinct vectors, all {R} codes equal the oracle's")
        # the same from the call that walks, builds and prunes at once (table of RPE-IDs only)
        i_walks, i_off, i_ids, _, i_code, i_T = binding.sample_walks_rpe_ids(
            ctx, d_rp, d_ci, d_seeds, M, m, wl.rng_seed, with_counts=False)
        assert ctx.check() == 0
        assert torch.equal(i_walks, walks) and torch.equal(i_off, off) and torch.equal(i_ids, ids)
        assert torch.equal(i_code, code) and same_u16(i_T, T), "one call: codes or T differ"
        del i_walks, i_off, i_ids, i_code, i_T
        say(f"[{name}] walks + RPE-IDs + T from one call equal the separate calls")

        # the union join over the codes: same offsets and ids as the join over counts (checked
        # above), and every code names, in T (checked above), the count vector that the join over
        # counts holds there (-1 <-> all zeros; the vectors of T are distinct, so that fixes it)
        i_off, i_ids, i_codes = binding.join_query_ids(ctx, off, ids, code, d_q, max_set=max_set)
        assert ctx.check() == 0
        assert torch.equal(i_off, joff) and torch.equal(i_ids, jids), "ids form: rows differ"
        T_ext = torch.cat([T.view(torch.int16), torch.zeros((1, L), dtype=torch.int16, device="cuda")])
        for s in range(0, J, 1 << 25):
            e = min(J, s + (1 << 25))
            c = i_codes[s:e].long()
            c = torch.where(c < 0, torch.full_like(c, T.shape[0]), c)        # -1 -> the zero row
            assert torch.equal(T_ext[c], jcnt.view(torch.int16)[s:e]), "ids form: a code names another vector"
        del i_off, i_ids, i_codes, T_ext, joff, jids, jcnt
        say(f"[{name}] join over RPE-IDs ok")

        # query-level RPE-IDs of every walk position, all queries; then the same call with the
        # rows' codes: everywhere the code of the row it names without them
        qids = binding.query_rpe_ids(ctx, walks, off, ids, d_q, max_set=max_set)
        assert ctx.check() == 0
        sweep_query_ids(pool, o_walks, table, queries, qids, say, name)
        qcodes = binding.query_rpe_ids(ctx, walks, off, ids, d_q, max_set=max_set, code=code)
        assert ctx.check() == 0
        for s in range(0, qids.shape[0], 1 << 16):
            rows_part = qids[s:s + (1 << 16)].long()
            want_part = torch.where(rows_part < 0, torch.full_like(rows_part, -1),
                                    code[rows_part.clamp(min=0)].long())
            assert torch.equal(qcodes[s:s + (1 << 16)].long(), want_part), "pruned RPE-IDs differ"
        say(f"[{name}] RPE-IDs into the pruned array ok")


def test_cl235k_full_size(ctx, say):
    check_workload(ctx, "cl235k", say)


def test_rmat512k_full_size(ctx, say):
    check_workload(ctx, "rmat512k", say)


def test_cl2900k_full_size(ctx, say):
    check_workload(ctx, "cl2900k", say)


def test_cl1m_triples_full_size(ctx, say):
    check_workload(ctx, "cl1m_triples", say)


def test_table_with_more_than_2_31_rows(ctx, say):
    # the 2.9M-node graph with M = 330: 2.35 G table rows, so row numbers and byte offsets pass
    # 2^31 and 2^32.  All seeds and all queries against the oracle, and the two-call path
    # against the fused kernel.
    wl = synth.WORKLOADS["cl2900k"]
    M, m = 330, 4
    L = m + 1
    rp, ci = synth.make_graph(wl)
    queries = synth.make_queries(wl, rp, ci)[:200000]
    N = wl.n_nodes
    d_rp, d_ci, d_q = dev(rp), dev(ci), dev(queries)
    seeds = torch.arange(N, dtype=torch.int32, device="cuda")
    walks, off, ids, cnt = binding.sample_walks_rpe(ctx, d_rp, d_ci, seeds, M, m, 0)
    assert ctx.check() == 0
    R = int(off[-1])
    assert R > 2 ** 31 and bool((off[1:] > off[:-1]).all())
    say(f"[2^31] fused done: R={R}")
    with ThreadPoolExecutor(HOST_THREADS) as pool:
        _, table = sweep_seeds(pool, rp, ci, N, M, m, 0, walks, off, ids, cnt, say, "2^31",
                               keep_walks=False)
        say(f"[2^31] all {N} seeds, {R} rows equal the oracle's")
        sizes = torch.empty(N, dtype=torch.int32, device="cuda")
        walks2 = binding.sample_walks(ctx, d_rp, d_ci, seeds, M, m, 0, set_sizes=sizes)
        assert torch.equal(walks2, walks)
        del walks2
        off2 = torch.empty(N + 1, dtype=torch.int64, device="cuda")
        ids2 = torch.empty(R, dtype=torch.int32, device="cuda")
        cnt2 = torch.empty((R, L), dtype=torch.uint16, device="cuda")
        rc, R2 = binding.build_rpe_raw(ctx, walks, N, R, off2, ids2, cnt2, set_sizes=sizes)
        assert rc == binding.OK and R2 == R and ctx.check() == 0
        assert torch.equal(off2, off) and torch.equal(ids2, ids) and same_u16(cnt2, cnt)
        del ids2, cnt2, off2
        say("[2^31] the two-call path equals the fused kernel")
        joff, jids, jcnt = binding.join_queries(ctx, off, ids, cnt, d_q, max_set=1 + M * m)
        assert ctx.check() == 0
        sweep_join(pool, table, queries, joff, jids, jcnt, say, "2^31")
