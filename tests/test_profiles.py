"""The committed profiler summaries are usable as evidence: each names the command that made
it, that command runs a committed file, and the two that the benchmark reads parse into the
figures it quotes."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")


def test_every_summary_names_a_command_that_runs_committed_files():
    names = sorted(f for f in os.listdir(PROFILES) if f.endswith((".txt", ".md")))
    assert names, "no profiler summaries"
    for name in names:
        text = open(os.path.join(PROFILES, name)).read()
        commands = re.findall(r"^#\s+(rocprofv3 --.*|python3 bench\.py.*)$", text, flags=re.M)
        assert commands, f"{name} does not say how it was made"
        for cmd in commands:
            program = cmd.split(" -- ", 1)[1] if " -- " in cmd else cmd
            assert program.startswith("python3 bench.py"), f"{name}: {program}"
        assert os.path.getsize(os.path.join(PROFILES, name)) < 32 * 1024, f"{name} is not a summary"
    assert os.path.exists(os.path.join(ROOT, "bench.py"))


def test_the_benchmark_reads_its_request_counters_and_ceilings():
    req = bench.read_requests("cl2900k")
    for kernel in ("walk_rpe", "edge_records", "join_count", "join_fill"):
        row = req[kernel]
        assert row["RDREQ"] >= row["RDREQ_128B"] + row["RDREQ_64B"] + row["RDREQ_32B"] - 1
        assert row["WRREQ"] >= row["WRREQ_64B"]
    assert req["walk_rpe"]["RDREQ_128B"] > 0.99 * req["walk_rpe"]["RDREQ"]
    ceilings = bench.read_membench()
    assert 10 < ceilings["gather_16B_1GiB_Gs"] < 1000
    assert 1 < ceilings["stream_copy_TBs"] < 8
    traffic = bench.read_traffic("cl2900k")
    assert traffic["walk_rpe"] > 0
