"""The counter-derived HBM traffic that bench.py prints as `roofline.traffic` is a constant copied from a tracked
rocprofv3 summary: this test keeps the two from drifting apart (CPU only, reads text files of the repository)."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_traffic_constants_are_the_profiles_figures():
    bench = load_bench()
    seen = {}
    for name in ("ctx32k_hbm_traffic_pmc.md", "ragged16_hbm_traffic_pmc.md"):
        text = open(os.path.join(ROOT, "profiles", name)).read()
        for workload, value in re.findall(r"^traffic_bytes_per_launch\[(\w+)\] = (\d+)$", text, flags=re.M):
            seen[workload] = int(value)
    assert seen == bench.VERIFY_TRAFFIC_BYTES


def test_traffic_is_close_to_the_algorithmic_bytes():
    """The figures themselves: a verification launch moves its K + V bytes once, plus a few percent of queries, page
    table, collected log-sum-exps and partial results (re-reads would show up here first)."""
    bench = load_bench()
    assert 1.0 <= bench.VERIFY_TRAFFIC_BYTES["ctx32k"] / (32768 * 4096) <= 1.05
    text = open(os.path.join(ROOT, "profiles", "ragged16_hbm_traffic_pmc.md")).read()
    kv = int(re.search(r"K \+ V = ([\d,]+) bytes", text).group(1).replace(",", ""))
    assert 1.0 <= bench.VERIFY_TRAFFIC_BYTES["ragged16"] / kv <= 1.05
