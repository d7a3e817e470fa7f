#!/usr/bin/env python3
"""Benchmark of the walk -> RPE -> join hot path on one MI355X.

A step is one pass of the whole path over the workload: walks for every node and the RPE
table of all walks (one fused kernel by default; --unfused runs sample_walks and build_rpe
as two calls), then join_queries over all query tuples, inputs already resident in HBM and
output buffers allocated beforehand.  The line printed at the end follows the
driver's contract; `value` is walk-steps/s through the whole pipeline (the stage rates and
the HBM-roofline fractions are extra keys of the same line).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cl2900k]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
METRIC = "walk-steps/s + joined query-RPE rows/s at 1 GPU; % of HBM roofline"


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def algorithmic_bytes(N, M, m, k, R, J, in_rows, Q, fused):
    """Bytes the method itself must move, per stage (one pass).  The fused kernel never reads
    the walks back, so that read is not part of its figure."""
    L = m + 1
    walk = N * M * m * 12 + N * M * L * 4 + N * 4
    rpe_out = R * (4 + 2 * L) + (N + 1) * 8
    join = in_rows * (4 + 2 * L) + Q * k * (4 + 16) + J * (4 + 2 * k * L) + (Q + 1) * 8
    if fused:
        return {"walk_rpe": walk + rpe_out, "join": join}
    return {"walk": walk, "rpe": N * M * L * 4 + rpe_out, "join": join}


# The paper's own timings for this path (Table 2 and Table 4, "Prep." column; App. D.3 for the
# (M, m) settings), all on one server with 4x Intel Xeon Gold 6248R, 16 threads.  Context only:
# another machine, real datasets, and what the times include is not itemised.
PAPER_CONTEXT = {
    "hardware": "4x Intel Xeon Gold 6248R, 1 TB DRAM; walks, RPE and joins on 16 CPU threads",
    "subgraph_sampling_citation2_s": 26,
    "prep_citation2_s": 31, "prep_collab_s": "<1", "prep_dblp_coauthor_s": 10,
    "derived_walk_steps_per_s_citation2": 2_927_963 * 50 * 4 / 31,
    "derived_walk_steps_per_s_dblp_coauthor": 1_924_991 * 100 * 3 / 10,
    "note": "context, not a target: citation2 (2,927,963 nodes, M=50, m=4) is what workload "
            "cl2900k stands in for in shape; the paper does not say what the times include",
}


def read_requests(workload: str):
    """Fabric requests per launch measured with rocprofv3 --pmc, from profiles/ (or {}):
    kernel -> {counter: value}."""
    path = os.path.join(ROOT, "profiles", f"requests_{workload}.txt")
    table = {}
    if not os.path.exists(path):
        return table
    header = None
    with open(path) as fh:
        for line in fh:
            if line.startswith("# columns:"):
                header = line.split(":", 1)[1].split()
            tok = line.split()
            if header and tok and not line.startswith("#") and len(tok) == len(header):
                table[tok[0]] = {h: float(v) for h, v in zip(header[1:], tok[1:])}
    return table


def read_membench():
    """The measured ceilings of profiles/membench_mi355x.txt (or {}): name -> value."""
    path = os.path.join(ROOT, "profiles", "membench_mi355x.txt")
    out = {}
    if os.path.exists(path):
        with open(path) as fh:
            for line in fh:
                tok = line.split()
                if len(tok) >= 2 and not line.startswith("#"):
                    try:
                        out[tok[0]] = float(tok[1])
                    except ValueError:
                        pass
    return out


def membench(torch) -> dict:
    """Streaming, gather and scatter rates of this GPU (libsurel_membench.so)."""
    import ctypes

    from paper_2202_13538_amd import build
    if not os.path.exists(build.MEMBENCH_LIB_PATH):
        raise SystemExit("libsurel_membench.so is not built; run python __graft_entry__.py")
    lib = ctypes.CDLL(build.MEMBENCH_LIB_PATH)
    vp, dbl = ctypes.c_void_p, ctypes.c_double
    lib.surel_membench_init.argtypes = [vp, ctypes.c_size_t, vp]
    lib.surel_membench_stream.argtypes = [ctypes.c_int, vp, ctypes.c_size_t, vp, vp, ctypes.POINTER(dbl)]
    lib.surel_membench_gather.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp,
                                          ctypes.POINTER(dbl), ctypes.POINTER(dbl)]
    lib.surel_membench_scatter.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp,
                                           ctypes.POINTER(dbl), ctypes.POINTER(dbl)]
    lib.surel_membench_bin.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp, vp,
                                       ctypes.POINTER(dbl), ctypes.POINTER(dbl)]
    size = 8 << 30
    buf = torch.empty(size, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    stream = vp(torch.cuda.current_stream().cuda_stream)
    p, sk = vp(buf.data_ptr()), vp(sink.data_ptr())
    assert lib.surel_membench_init(p, size, stream) == 0
    out = {}
    ms, units = dbl(0), dbl(0)
    for kind, name, moved in ((0, "stream_read_TBs", 4 << 30), (1, "stream_write_TBs", 4 << 30),
                              (2, "stream_copy_TBs", 8 << 30),
                              (3, "stream_read1_write2_TBs", 6 << 30)):
        nbytes = (4 << 30) if kind < 2 else (8 << 30)
        assert lib.surel_membench_stream(kind, p, nbytes, sk, stream, ctypes.byref(ms)) == 0
        out[name] = round(moved / (ms.value * 1e-3) / 1e12, 3)
    for width in (4, 8, 16):
        assert lib.surel_membench_gather(p, 1 << 30, width, 8, sk, stream, ctypes.byref(ms),
                                         ctypes.byref(units)) == 0
        out[f"gather_{width}B_1GiB_Gs"] = round(units.value / (ms.value * 1e-3) / 1e9, 2)
    for mib in (2, 4, 8, 16, 32, 64, 128, 256, 4096):
        assert lib.surel_membench_gather(p, mib << 20, 16, 8, sk, stream, ctypes.byref(ms),
                                         ctypes.byref(units)) == 0
        out[f"gather_16B_{mib}MiB_Gs"] = round(units.value / (ms.value * 1e-3) / 1e9, 2)
    for width in (4, 20, 64):
        assert lib.surel_membench_scatter(p, 4 << 30, width, 8, stream, ctypes.byref(ms),
                                          ctypes.byref(units)) == 0
        out[f"scatter_{width}B_rows_Gs"] = round(units.value / (ms.value * 1e-3) / 1e9, 2)
    # one pass of binning 290 M 12-byte items (as many as the 2.9M-node workload has walkers)
    # into 256 bins through LDS: what regrouping walkers by graph region would cost per exchange
    assert lib.surel_membench_init(p, size, stream) == 0
    n_items = 290_000_000
    out_off = 7 << 29                                     # 3.5 GiB in: behind the items
    cursor = torch.zeros(512, dtype=torch.int32, device="cuda")
    assert lib.surel_membench_bin(p, n_items, vp(buf.data_ptr() + out_off), size - out_off,
                                  vp(cursor.data_ptr()), stream, ctypes.byref(ms),
                                  ctypes.byref(units)) == 0
    out["bin_12B_256bins_ms_per_290M"] = round(ms.value, 3)
    out["bin_12B_256bins_TBs"] = round(2 * n_items * 12 / (ms.value * 1e-3) / 1e12, 3)
    out["bin_dropped_items"] = units.value
    placed = int(cursor[:256].long().sum())               # every item has a place in its bin
    assert placed + int(units.value) == n_items, (placed, units.value)
    del buf
    return out


def read_traffic(workload: str):
    """HBM traffic per launch measured with rocprofv3 --pmc, from profiles/ (or None)."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    table = {}
    if not os.path.exists(path):
        return table
    with open(path) as fh:
        for line in fh:
            tok = line.split()
            if len(tok) == 3 and not line.startswith("#"):
                table[tok[0]] = float(tok[1]) + float(tok[2])
    return table


def cpu_baseline(wl, rp, ci, queries, n_seeds_sample, n_query_sample):
    """The oracle, as it stands, on one host core over a bounded sample of the workload."""
    import numpy as np

    import oracle

    N, M, m = wl.n_nodes, wl.M, wl.m
    seeds = np.arange(min(n_seeds_sample, N), dtype=np.int32)
    t0 = time.perf_counter()
    w = oracle.sample_walks(rp, ci, seeds, M, m, wl.rng_seed)
    t1 = time.perf_counter()
    sample_off, _, _ = oracle.build_rpe(w)
    t2 = time.perf_counter()
    # the join leg needs the RPE blocks of its queries' nodes; building them is not timed
    sub_q = queries[:n_query_sample]
    nodes, local = np.unique(sub_q, return_inverse=True)
    table = oracle.build_rpe(oracle.sample_walks(rp, ci, nodes.astype(np.int32), M, m,
                                                 wl.rng_seed))
    local = local.reshape(sub_q.shape).astype(np.int32)
    t3 = time.perf_counter()
    _, jids, _ = oracle.join_queries(*table, local)
    t4 = time.perf_counter()
    per_seed = (t2 - t0) / seeds.size
    per_query = (t4 - t3) / sub_q.shape[0]
    full = per_seed * N + per_query * wl.n_queries      # scaled to the whole workload
    # the same oracle calls on disjoint seed / query ranges from P threads (its outputs are
    # per seed and per query, the random stream is counter-based, and ctypes drops the GIL)
    from concurrent.futures import ThreadPoolExecutor
    P = max(1, os.cpu_count() or 1)                     # every host core the box shows
    seed_parts = np.array_split(seeds, P)
    query_parts = np.array_split(local, P)
    with ThreadPoolExecutor(P) as pool:
        p0 = time.perf_counter()
        list(pool.map(lambda part: oracle.build_rpe(
            oracle.sample_walks(rp, ci, part, M, m, wl.rng_seed)), seed_parts))
        p1 = time.perf_counter()
        list(pool.map(lambda part: oracle.join_queries(*table, part), query_parts))
        p2 = time.perf_counter()
    full_p = (p1 - p0) / seeds.size * N + (p2 - p1) / sub_q.shape[0] * wl.n_queries
    return {
        "value": N * M * m / full, "unit": "walk-steps/s", "cores": 1, "kind": "oracle",
        "all_cores": {"value": N * M * m / full_p, "unit": "walk-steps/s", "cores": P,
                      "sample": f"the same sample split into {P} ranges, one thread each "
                                f"(walks+RPE {p1 - p0:.1f} s, join {p2 - p1:.2f} s)"},
        "sample": (f"seeds 0..{seeds.size - 1} for walks+RPE ({t2 - t0:.1f} s: walks "
                   f"{t1 - t0:.1f} s, RPE {t2 - t1:.1f} s), first {sub_q.shape[0]} queries for "
                   f"the join ({t4 - t3:.1f} s); per-seed and per-query times scaled to the "
                   "whole workload"),
        "walk_steps_per_s": seeds.size * M * m / (t1 - t0),
        "rpe_rows_per_s": float(sample_off[-1]) / (t2 - t1),
        "joined_rows_per_s": jids.size / (t4 - t3),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cl2900k")
    ap.add_argument("--cpu-seeds", type=int, default=1 << 17)
    ap.add_argument("--cpu-queries", type=int, default=1 << 14)
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--unfused", action="store_true",
                    help="sample_walks and build_rpe as two calls instead of the fused kernel")
    ap.add_argument("--query-ids", action="store_true",
                    help="also time surel_query_rpe_ids (Sec. 3.4's per-walk-position form of the "
                         "join) after the timed region; reported under 'query_rpe_ids', not part "
                         "of 'value'")
    ap.add_argument("--prune", action="store_true",
                    help="also time surel_prune_rpe (Sec. 3.3: distinct count vectors stored once) "
                         "after the timed region; reported under 'prune_rpe', not part of 'value'")
    ap.add_argument("--join-ids", action="store_true",
                    help="also time surel_join_query_ids (the union join over RPE-IDs into the "
                         "pruned array instead of count vectors) after the timed region; reported "
                         "under 'join_query_ids', not part of 'value'")
    ap.add_argument("--batches", action="store_true",
                    help="also time surel_query_incidence + surel_bfs_batches (Sec. 3.6: mini-batches "
                         "of queries that share nodes) after the timed region, and the join over "
                         "the batches' queries next to the join over as many queries in the given "
                         "order; reported under 'bfs_batches', not part of 'value'")
    ap.add_argument("--batch-size", type=int, default=4096, help="B2 of --batches")
    ap.add_argument("--batch-nodes", type=int, default=0,
                    help="B1 of --batches (default k * B2, so that B2 is the limit that binds)")
    ap.add_argument("--relabel-by-degree", action="store_true",
                    help="renumber the nodes by descending degree before the run (hubs get the "
                         "smallest ids and lie together in memory): a different input labelling, "
                         "not a different method; the line says so in config.labelling")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one pass (no row totals read back) into a HIP graph and time "
                         "its replays; reported under 'graph_replay', not part of 'value'")
    ap.add_argument("--membench", action="store_true",
                    help="instead of the pipeline, run the memory-system micro-benchmarks "
                         "(streaming, dependent random gathers by table size, scatters) and print "
                         "them as one JSON line: the measured ceilings of this GPU that the "
                         "roofline.as_moved figures are compared with")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run three plain 1 GiB read + 1 GiB write "
                         "elementwise kernels (the known-size reference for rocprofv3 FETCH_SIZE "
                         "/ WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build is the one-GPU hot path; --gpus must be 1 "
            "(seeds and queries shard with no change to the kernels, but no multi-GPU run "
            "is part of this benchmark)")
        return 2

    import numpy as np
    import torch

    from paper_2202_13538_amd import binding, synth

    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2

    if args.membench:
        torch.cuda.set_device(0)
        print(json.dumps({"membench": membench(torch), "unit": "TB/s for stream_*, G gathers or "
                          "rows per second for *_Gs", "data": "synthetic"}))
        return 0

    wl = synth.WORKLOADS[args.workload]
    N, M, m, k, Q = wl.n_nodes, wl.M, wl.m, wl.k, wl.n_queries
    L = m + 1
    t0 = time.time()
    rp, ci = synth.make_graph(wl)
    queries = synth.make_queries(wl, rp, ci)
    if args.relabel_by_degree:
        deg0 = np.diff(rp)
        order = np.argsort(-deg0, kind="stable")            # old id of the node that becomes id i
        new_id = np.empty(N, dtype=np.int64)
        new_id[order] = np.arange(N)
        src = np.repeat(new_id, deg0)                        # new id of every entry's row
        dst = new_id[ci]
        keys = np.argsort(src * N + dst, kind="stable")     # rows in new order, ascending inside
        ci = dst[keys].astype(np.int32)
        rp = np.concatenate([[0], np.cumsum(deg0[order])]).astype(np.int32)
        queries = new_id[queries].astype(np.int32)
    log(f"[bench] {wl.name}: N={N} E2={ci.size} M={M} m={m} queries={Q}x{k} "
        f"(generated in {time.time() - t0:.1f} s)")

    torch.cuda.set_device(0)
    if args.graph:
        torch.cuda.set_stream(torch.cuda.Stream())   # graphs are not captured on the default stream
    ctx = binding.Context(0)
    d_rp, d_ci = torch.from_numpy(rp).cuda(), torch.from_numpy(ci).cuda()
    d_q = torch.from_numpy(queries).cuda()
    d_seeds = torch.arange(N, dtype=torch.int32, device="cuda")
    walks = torch.empty((N, M, L), dtype=torch.int32, device="cuda")
    cap_r = binding.rpe_rows_bound(N, M, m)
    rpe_off = torch.empty(N + 1, dtype=torch.int64, device="cuda")
    rpe_ids = torch.empty(cap_r, dtype=torch.int32, device="cuda")
    rpe_cnt = torch.empty((cap_r, L), dtype=torch.uint16, device="cuda")
    join_off = torch.empty(Q + 1, dtype=torch.int64, device="cuda")
    set_sizes = torch.empty(N, dtype=torch.int32, device="cuda")
    max_set = 1 + M * m

    fused = not args.unfused

    def walks_and_rpe():
        if fused:
            return binding.sample_walks_rpe_raw(ctx, d_rp, d_ci, d_seeds, M, m, wl.rng_seed, walks,
                                                cap_r, rpe_off, rpe_ids, rpe_cnt)
        binding.sample_walks(ctx, d_rp, d_ci, d_seeds, M, m, wl.rng_seed, out=walks,
                             set_sizes=set_sizes)
        return binding.build_rpe_raw(ctx, walks, N, cap_r, rpe_off, rpe_ids, rpe_cnt,
                                     set_sizes=set_sizes)

    # sizing pass (untimed): the join's row total fixes its output allocation
    rc, R = walks_and_rpe()
    assert rc == binding.OK, rc
    rc, J = binding.join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, d_q, max_set, 0, join_off,
                                     None, None)
    assert rc == binding.OK, rc
    join_ids = torch.empty(J, dtype=torch.int32, device="cuda")
    join_cnt = torch.empty((J, k, L), dtype=torch.uint16, device="cuda")
    in_rows = int((rpe_off[1:] - rpe_off[:-1])[d_q.long()].sum())
    # what the synthetic input looks like (the byte formulas depend on it)
    deg = np.diff(rp)
    set_len = (rpe_off[1:] - rpe_off[:-1]).float()
    input_stats = {
        "csr_entries": int(ci.size), "max_degree": int(deg.max()), "isolated_nodes": int((deg == 0).sum()),
        "set_size_mean": round(float(set_len.mean()), 2),
        "set_size_p95": int(torch.quantile(set_len[:: max(1, N // 1_000_000)], 0.95)),
        "joined_rows_per_query": round(J / Q, 2),
        "shared_nodes_per_query": round((in_rows - J) / Q, 2),
    }
    log(f"[bench] R={R} RPE rows, J={J} joined rows, {in_rows} table rows read by the join")

    def one_step():
        rc1, r = walks_and_rpe()
        rc2, j = binding.join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, d_q, max_set, J,
                                          join_off, join_ids, join_cnt)
        assert rc1 == binding.OK and rc2 == binding.OK and r == R and j == J

    for _ in range(args.warmup):
        one_step()
    assert ctx.check() == 0

    ctx.profile(True)            # HIP events around every kernel launch, on the ctx's stream
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    prof = ctx.profile_read()
    ctx.profile(False)
    assert ctx.check() == 0

    ms_per_step = elapsed * 1e3 / args.steps
    kern = {name: (tot / n if n else 0.0) for name, (tot, n) in prof.items()}   # avg ms / launch
    per_step = {name: tot / args.steps for name, (tot, n) in prof.items()}       # ms / step
    join_ms = per_step.get("join_count", 0.0) + per_step.get("join_fill", 0.0)
    expand_ms = per_step.get("edge_records", 0.0)   # CSR -> per-edge records, part of the walk
    if fused:
        stage_ms = {"walk_rpe": per_step.get("walk_rpe", 0.0) + expand_ms, "join": join_ms}
        walk_ms = rpe_ms = stage_ms["walk_rpe"]     # one kernel makes both outputs
    else:
        stage_ms = {"walk": per_step.get("walk", 0.0) + expand_ms,
                    "rpe": per_step.get("rpe_count", 0.0) + per_step.get("rpe_fill", 0.0),
                    "join": join_ms}
        walk_ms, rpe_ms = stage_ms["walk"], stage_ms["rpe"]
    alg = algorithmic_bytes(N, M, m, k, R, J, in_rows, Q, fused)
    pipeline_bytes = sum(alg.values())
    traffic = read_traffic(wl.name)

    # roofline of the dominant kernel (largest average launch duration)
    dom = max(kern, key=lambda n: kern[n])
    dom_stage = dom if dom in alg else dom.split("_")[0]
    dom_gbs = alg[dom_stage] / (kern[dom] * 1e-3) / 1e9 if kern[dom] > 0 else 0.0
    roofline = {
        "bound": "hbm", "kernel": dom, "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
        "traffic": traffic.get(dom),
        "avg_launch_ms": round(kern[dom], 4),
        "algorithmic_bytes_per_launch": alg[dom_stage],
    }
    # Beside the graded figure, never instead of it: (1) the same kernel with the graph counted
    # ONCE (compulsory traffic: a perfect cache would read the CSR once, not 12 bytes a step);
    # (2) what the kernel really moves, from the request counters of profiles/ (per launch;
    # 128-byte reads and 64-byte writes between the L2s and the memory fabric) over the launch
    # time measured here, against the HBM peak and against the time the bus needs for them at
    # the measured rates of line fetches and streaming writes (profiles/membench_mi355x.txt).
    if dom_stage in ("walk_rpe", "walk"):
        walk_steps_read = N * M * m * 12
        csr_once = (N + 1) * 4 + ci.size * 4
        comp = alg[dom_stage] - walk_steps_read + csr_once
        roofline["compulsory"] = {
            "bytes_per_launch": comp,
            "frac": round(comp / (kern[dom] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "note": "the graph counted once instead of 12 bytes per walk step"}
    req = read_requests(wl.name).get(dom)
    if req and kern[dom] > 0:
        rd = req.get("RDREQ_128B", 0.0) * 128 + req.get("RDREQ_64B", 0.0) * 64 + req.get("RDREQ_32B", 0.0) * 32
        wr = req.get("WRREQ_64B", 0.0) * 64 + (req.get("WRREQ", 0.0) - req.get("WRREQ_64B", 0.0)) * 32
        n_req = req.get("RDREQ", 0.0) + req.get("WRREQ", 0.0)
        ceil = read_membench()
        as_moved = {
            "kernel": dom, "read_requests": req.get("RDREQ"), "write_requests": req.get("WRREQ"),
            "read_requests_128B": req.get("RDREQ_128B"), "bytes_per_launch": rd + wr,
            "achieved_GBs": round((rd + wr) / (kern[dom] * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round((rd + wr) / (kern[dom] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "requests_per_s": round(n_req / (kern[dom] * 1e-3), 1),
            "source": f"profiles/requests_{wl.name}.txt (counts per launch) / launch time measured here",
        }
        if "gather_16B_1GiB_Gs" in ceil and "stream_write_TBs" in ceil:
            # the time the memory bus needs for these requests at the rates it was measured to
            # give: line fetches at the rate of dependent random gathers, writes at the rate
            # of streaming writes, one after the other
            fetch_rate = ceil["gather_16B_1GiB_Gs"] * 1e9 * 128        # bytes/s as moved
            write_rate = ceil["stream_write_TBs"] * 1e12
            bus_ms = (rd / fetch_rate + wr / write_rate) * 1e3
            as_moved["measured_line_fetch_GBs"] = round(fetch_rate / 1e9, 1)
            as_moved["measured_stream_write_GBs"] = round(write_rate / 1e9, 1)
            as_moved["bus_time_ms_at_measured_rates"] = round(bus_ms, 3)
            as_moved["bus_time_over_launch_time"] = round(bus_ms / kern[dom], 4)
        roofline["as_moved"] = as_moved

    out = {
        "metric": METRIC,
        "value": N * M * m / (ms_per_step * 1e-3),
        "unit": "walk-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": wl.name, "graph": wl.graph, "n_nodes": N, "n_edges": wl.n_edges,
                   "M": M, "m": m, "n_queries": Q, "k": k, "rpe_rows": R, "joined_rows": J,
                   "walk_and_rpe": "one fused kernel" if fused else "two calls",
                   "labelling": "by descending degree" if args.relabel_by_degree else "random permutation",
                   "input_stats": input_stats},
        "walk_steps_per_s": N * M * m / (walk_ms * 1e-3) if walk_ms else None,
        "rpe_rows_per_s": R / (rpe_ms * 1e-3) if rpe_ms else None,
        "joined_rows_per_s": J / (join_ms * 1e-3) if join_ms else None,
        "stage_ms": {s: round(v, 4) for s, v in stage_ms.items()},
        "kernel_avg_ms": {n: round(v, 4) for n, v in kern.items()},
        "stage_hbm_frac": {s: round(alg[s] / (stage_ms[s] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                           for s in stage_ms if stage_ms[s] > 0},
        "pipeline_algorithmic_bytes": pipeline_bytes,
        "pipeline_hbm_frac": round(pipeline_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": roofline,
        "paper_context": PAPER_CONTEXT,
    }
    if args.query_ids:
        qid = torch.empty((Q, k, M, L, k), dtype=torch.int32, device="cuda")
        binding.query_rpe_ids(ctx, walks, rpe_off, rpe_ids[:R], d_q, max_set, out=qid)
        ctx.profile(True)
        for _ in range(args.steps):
            binding.query_rpe_ids(ctx, walks, rpe_off, rpe_ids[:R], d_q, max_set, out=qid)
        ms = ctx.profile_read()["query_ids"][0] / args.steps
        ctx.profile(False)
        assert ctx.check() == 0
        # read: the k walk blocks and id lists of every query; written: k row indices per entry
        q_bytes = Q * k * M * L * 4 + in_rows * 4 + Q * k * M * L * k * 4
        out["query_rpe_ids"] = {
            "ms": round(ms, 4), "walk_positions_per_s": Q * k * M * L / (ms * 1e-3),
            "algorithmic_bytes": q_bytes,
            "hbm_frac": round(q_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if args.prune:
            # the same with the rows' codes from surel_prune_rpe: RPE-IDs into the pruned array
            cap_T = 1 << 20
            T = torch.empty((cap_T, L), dtype=torch.uint16, device="cuda")
            code = torch.empty(R, dtype=torch.int32, device="cuda")
            rc, n_T = binding.prune_rpe_raw(ctx, rpe_cnt[:R], cap_T, T, code)
            assert rc == binding.OK, rc
            binding.query_rpe_ids(ctx, walks, rpe_off, rpe_ids[:R], d_q, max_set, out=qid, code=code)
            ctx.profile(True)
            for _ in range(args.steps):
                binding.query_rpe_ids(ctx, walks, rpe_off, rpe_ids[:R], d_q, max_set, out=qid,
                                      code=code)
            ms_c = ctx.profile_read()["query_ids"][0] / args.steps
            ctx.profile(False)
            assert ctx.check() == 0
            out["query_rpe_ids"]["with_codes_ms"] = round(ms_c, 4)
            del T, code
        del qid
    if args.prune:
        cap_T = 1 << 20
        T = torch.empty((cap_T, L), dtype=torch.uint16, device="cuda")
        code = torch.empty(R, dtype=torch.int32, device="cuda")
        rc, n_T = binding.prune_rpe_raw(ctx, rpe_cnt[:R], cap_T, T, code)
        assert rc == binding.OK, rc
        ctx.profile(True)
        for _ in range(args.steps):
            rc, n_T = binding.prune_rpe_raw(ctx, rpe_cnt[:R], cap_T, T, code)
        ms = ctx.profile_read()["prune"][0] / args.steps
        ctx.profile(False)
        assert ctx.check() == 0
        p_bytes = R * 2 * L + R * 4 + n_T * 2 * L          # vectors read, codes and T written
        out["prune_rpe"] = {
            "ms": round(ms, 4), "rows_per_s": R / (ms * 1e-3), "distinct_vectors": n_T,
            "algorithmic_bytes": p_bytes,
            "hbm_frac": round(p_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        # Algorithm 1 from end to end in one call: the fused kernel feeds the set of distinct
        # vectors itself; with the count vectors, and with a table that carries RPE-IDs only
        for key, cnt_arg in (("with_counts", rpe_cnt), ("ids_only", None)):
            def one_call():
                rc, rows, nt = binding.sample_walks_rpe_ids_raw(
                    ctx, d_rp, d_ci, d_seeds, M, m, wl.rng_seed, walks, cap_r, rpe_off, rpe_ids,
                    cnt_arg, code, cap_T, T)
                assert rc == binding.OK and rows == R and nt == n_T, (rc, rows, nt)
            one_call()
            ctx.profile(True)
            torch.cuda.synchronize()
            t_p = time.perf_counter()
            for _ in range(args.steps):
                one_call()
            torch.cuda.synchronize()
            wall = (time.perf_counter() - t_p) * 1e3 / args.steps
            pr = ctx.profile_read()
            ctx.profile(False)
            assert ctx.check() == 0
            out["prune_rpe"]["one_call_" + key] = {
                "ms": round(wall, 4),
                "walk_rpe_kernel_ms": round(pr["walk_rpe"][0] / args.steps, 4),
                "edge_records_ms": round(pr["edge_records"][0] / args.steps, 4),
                "finish_ms": round(pr["prune"][0] / args.steps, 4)}
        out["prune_rpe"]["separate_calls_ms"] = round(stage_ms.get("walk_rpe", 0.0) + ms, 4)
        del T, code
    if args.join_ids:
        cap_T = 1 << 20
        T = torch.empty((cap_T, L), dtype=torch.uint16, device="cuda")
        code = torch.empty(R, dtype=torch.int32, device="cuda")
        rc, n_T = binding.prune_rpe_raw(ctx, rpe_cnt[:R], cap_T, T, code)
        assert rc == binding.OK, rc
        j_codes = torch.empty((J, k), dtype=torch.int32, device="cuda")
        rc, rows = binding.join_query_ids_raw(ctx, rpe_off, rpe_ids, code, d_q, max_set, J, join_off,
                                              join_ids, j_codes)
        assert rc == binding.OK and rows == J
        ctx.profile(True)
        for _ in range(args.steps):
            binding.join_query_ids_raw(ctx, rpe_off, rpe_ids, code, d_q, max_set, J, join_off,
                                       join_ids, j_codes)
        pr = ctx.profile_read()
        ctx.profile(False)
        assert ctx.check() == 0
        ms = (pr["join_count"][0] + pr["join_fill"][0] + pr["scan"][0]) / args.steps
        i_bytes = in_rows * 8 + J * (4 + 4 * k)            # ids + codes read, ids + k codes written
        out["join_query_ids"] = {
            "ms": round(ms, 4), "joined_rows_per_s": J / (ms * 1e-3), "algorithmic_bytes": i_bytes,
            "hbm_frac": round(i_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "join_over_counts_ms": round(stage_ms["join"], 4)}
        del T, code, j_codes
    if args.batches:
        B2 = args.batch_size
        B1 = args.batch_nodes or B2 * k   # default: the batch size is the limit that binds
        n_batches, n_start = max(1, Q // B2), 16
        g = torch.Generator(device="cpu").manual_seed(7)
        # Algorithm 2 draws the seed-set from the nodes that queries name
        start = d_q.reshape(-1)[torch.randint(0, Q * k, (n_batches * n_start,), generator=g).cuda()]
        start = start.reshape(n_batches, n_start).contiguous()
        inc_off, inc_q = binding.query_incidence(ctx, d_q, N)
        vbar, batch, tuples, counts = binding.bfs_batches(ctx, d_q, N, inc_off, inc_q, start, B1, B2)
        assert ctx.check() == 0
        ctx.profile(True)
        for _ in range(args.steps):
            binding.query_incidence(ctx, d_q, N)
        inc_ms = ctx.profile_read()["batch"][0] / args.steps
        ctx.profile(True)
        for _ in range(args.steps):
            binding.bfs_batches_raw(ctx, d_q, N, inc_off, inc_q, start, B1, B2, vbar, batch, tuples,
                                    counts)
        bfs_ms = ctx.profile_read()["batch"][0] / args.steps
        ctx.profile(False)
        assert ctx.check() == 0
        n_b = counts[:, 1].long()
        keep = torch.arange(B2, device="cuda")[None, :] < n_b[:, None]
        bq = tuples[keep].contiguous()                      # the batches' queries, batch after batch
        Qb = bq.shape[0]
        given = d_q[:Qb].contiguous()                       # as many queries in the given order
        nodes_bfs = float(counts[:, 0].float().sum()) / max(Qb, 1)
        nodes_given = sum(int(torch.unique(d_q[i * B2:(i + 1) * B2]).numel())
                          for i in range(min(n_batches, 32))) / (min(n_batches, 32) * B2)

        def time_join(qs):
            off = torch.empty(qs.shape[0] + 1, dtype=torch.int64, device="cuda")
            rc, rows = binding.join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, qs, max_set, 0, off,
                                                None, None)
            assert rc == binding.OK, rc
            ids = torch.empty(rows, dtype=torch.int32, device="cuda")
            cnt = torch.empty((rows, k, L), dtype=torch.uint16, device="cuda")
            binding.join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, qs, max_set, rows, off, ids, cnt)
            ctx.profile(True)
            for _ in range(args.steps):
                binding.join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, qs, max_set, rows, off, ids,
                                         cnt)
            pr = ctx.profile_read()
            ctx.profile(False)
            return (pr["join_count"][0] + pr["join_fill"][0] + pr["scan"][0]) / args.steps, rows

        join_bfs_ms, rows_bfs = time_join(bq)
        join_given_ms, rows_given = time_join(given)
        assert ctx.check() == 0
        out["bfs_batches"] = {
            "n_batches": n_batches, "B1": B1, "B2": B2, "seed_set": n_start,
            "incidence_ms": round(inc_ms, 4), "bfs_ms": round(bfs_ms, 4),
            "queries_in_batches": Qb, "batched_queries_per_s": Qb / (bfs_ms * 1e-3),
            "distinct_nodes_per_query": {"bfs_batches": round(nodes_bfs, 4),
                                         "given_order": round(nodes_given, 4)},
            "join_ms": {"bfs_batches": round(join_bfs_ms, 4), "given_order": round(join_given_ms, 4)},
            "joined_rows": {"bfs_batches": rows_bfs, "given_order": rows_given},
            "joined_rows_per_s": {"bfs_batches": rows_bfs / (join_bfs_ms * 1e-3),
                                  "given_order": rows_given / (join_given_ms * 1e-3)}}
        del vbar, batch, tuples, counts, inc_off, inc_q
    if args.graph:
        if not fused:
            raise SystemExit("--graph replays the fused pass; drop --unfused")

        def one_step_enqueued():
            rc1, _ = binding.sample_walks_rpe_raw(ctx, d_rp, d_ci, d_seeds, M, m, wl.rng_seed, walks,
                                                  cap_r, rpe_off, rpe_ids, rpe_cnt, want_rows=False)
            rc2, _ = binding.join_queries_raw(ctx, rpe_off, rpe_ids, rpe_cnt, d_q, max_set, J,
                                              join_off, join_ids, join_cnt, want_rows=False)
            assert rc1 == binding.OK and rc2 == binding.OK

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.current_stream(),
                              capture_error_mode="thread_local"):
            one_step_enqueued()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t_g) * 1e3 / args.steps
        assert ctx.check() == 0 and int(rpe_off[-1]) == R and int(join_off[-1]) == J
        out["graph_replay"] = {"ms_per_step": round(graph_ms, 4),
                               "eager_ms_per_step": round(ms_per_step, 4)}
    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            torch.add(a, 1, out=b)        # an elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
    if not args.no_cpu:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(wl, rp, ci, queries, args.cpu_seeds, args.cpu_queries)
        log(f"[bench] cpu_baseline took {time.time() - t0:.1f} s")
    ctx.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
