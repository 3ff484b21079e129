"""The evidence folder stays consistent: every kernel-statistics summary has its counter summary, both
name the full command that made them (rocprofv3 in front of the committed bench.py), the rate printed
in a summary follows from its own duration and byte count, and the index lists every pair."""
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")


def tags():
    return sorted(os.path.basename(f)[:-len("_kernel_stats.txt")] for f in glob.glob(os.path.join(PROFILES, "*_kernel_stats.txt")))


def test_every_summary_pair_is_complete_and_self_consistent():
    assert len(tags()) >= 18
    for tag in tags():
        stats = open(os.path.join(PROFILES, tag + "_kernel_stats.txt")).read()
        pmc_path = os.path.join(PROFILES, tag + "_pmc.txt")
        assert os.path.exists(pmc_path), tag
        pmc = open(pmc_path).read()
        for text in (stats, pmc):
            assert re.search(r"rocprofv3 .* -- python3 bench\.py ", text), tag
            assert re.search(r"^kernel_source_id: [0-9a-f]{16}$", text, re.M), tag
        m = re.search(r"algorithmic bytes per launch (\d+) / average duration (\d+) ns = ([0-9.]+) GB/s = ([0-9.]+) %", stats)
        assert m, tag
        nbytes, ns, gbps, pct = int(m.group(1)), int(m.group(2)), float(m.group(3)), float(m.group(4))
        assert abs(nbytes / ns - gbps) <= 0.06 and abs(gbps / 80.0 - pct) <= 0.006, tag
        t = re.search(r"^traffic_bytes_per_launch: ([0-9.]+)$", pmc, re.M)
        r = re.search(r"traffic / algorithmic[^0-9]*([0-9.]+)", pmc)
        assert t and r and abs(float(t.group(1)) / nbytes - float(r.group(1))) <= 2e-4, tag
        assert 0.99 <= float(r.group(1)) <= 1.2, tag         # never below the algorithmic bytes, never far above


def test_index_lists_every_pair_with_its_figures():
    index = open(os.path.join(PROFILES, "INDEX.md")).read()
    listed = re.findall(r"^\| `([A-Za-z0-9_]+)` \| `\w+` \| [0-9.]+ \| ([0-9.]+) \| ([0-9.]+) \|", index, re.M)
    assert sorted(t for t, _, _ in listed) == tags()
    for tag, pct, ratio in listed:
        stats = open(os.path.join(PROFILES, tag + "_kernel_stats.txt")).read()
        pmc = open(os.path.join(PROFILES, tag + "_pmc.txt")).read()
        assert f"= {pct} % of the 8 TB/s" in stats, tag
        assert re.search(r"traffic / algorithmic[^0-9]*" + re.escape(ratio), pmc), tag


def test_nothing_in_the_folder_runs_or_is_raw_profiler_output():
    for f in os.listdir(PROFILES):
        assert f.endswith((".txt", ".md")), f
        assert os.path.getsize(os.path.join(PROFILES, f)) < 64 * 1024, f
