"""The counter summaries under profiles/ belong to the kernels as they stand: bench.py reports their traffic figure only
if the hash they record equals the hash of the kernel sources, and this test says so before a benchmark run does."""
import glob
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_summaries_were_taken_with_the_present_kernels():
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "pagerank_iteration_*_hbm_traffic_counters.txt")))
    assert {os.path.basename(f).split("_")[2] for f in files} >= {"cfg2", "cfg3", "cfg5"}
    now = bench.kernel_sources_sha256()
    for f in files:
        text = open(f).read()
        sha = re.search(r"kernel_sources_sha256:\s*([0-9a-f]{64})", text)
        assert sha and sha.group(1) == now, "%s was taken with other kernels: run its commands again" % os.path.basename(f)
        cfg = os.path.basename(f).split("_")[2]
        value, source = bench.traffic_from_profiles(cfg)
        assert value and value > 0 and source.endswith(os.path.basename(f))


def test_a_summary_of_other_kernels_is_not_used(tmp_path, monkeypatch):
    text = "kernel_sources_sha256: %s\ntraffic_bytes_per_iteration: 123.0\n" % ("0" * 64)
    os.makedirs(tmp_path / "profiles")
    (tmp_path / "profiles" / "pagerank_iteration_cfgX_hbm_traffic_counters.txt").write_text(text)
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "kernel_sources_sha256", lambda: "1" * 64)
    value, why = bench.traffic_from_profiles("cfgX")
    assert value is None and "changed" in why
    assert bench.traffic_from_profiles("cfgY")[0] is None
