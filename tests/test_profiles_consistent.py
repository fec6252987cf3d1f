"""bench.py carries the measured HBM traffic per kernel launch as constants (counters cannot be read inside the
benchmark process); they must be the figures of the committed counter summary, so that a refreshed profile cannot leave
a stale number behind."""

import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_traffic_constants_match_the_committed_counter_summary():
    text = open(os.path.join(ROOT, "profiles", "keyswitch_cfg2_hbm_traffic.txt")).read()
    measured = {}
    for name, value in re.findall(r"^\s*ks::([a-z_0-9]+)<[^\n]*?measured\s+(\d+)", text, flags=re.M):
        measured[name] = int(value)
    assert measured, "no 'measured' lines found in the counter summary"
    table = {kernel: v for (workload, kernel), v in bench.MEASURED_TRAFFIC_BYTES.items() if workload == "keyswitch"}
    assert set(table) == set(measured), (sorted(table), sorted(measured))
    for kernel, v in table.items():
        assert v == measured[kernel], (kernel, v, measured[kernel])
