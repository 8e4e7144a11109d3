"""The HBM traffic figures that bench.py prints in its roofline blocks are constants copied from the
tracked rocprofv3 counter summaries; this keeps the two from drifting apart.  (Host only.)"""
import glob
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _traffic_lines():
    found = {}
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_step_counters.md"))):
        for m in re.finditer(r"^TRAFFIC workload=(\S+) kernel=(\S+) fetch_kib=(\S+) write_kib=(\S+)$", open(f).read(), flags=re.M):
            key = (m.group(1), m.group(2))
            assert key not in found, f"{key} appears twice in profiles/"
            found[key] = (float(m.group(3)), float(m.group(4)))
    return found


def test_bench_traffic_table_is_the_profiles_table():
    table = _bench().MEASURED_TRAFFIC_KIB
    lines = _traffic_lines()
    assert lines, "no TRAFFIC lines under profiles/"
    assert table == lines


def test_every_summary_names_its_commands():
    for f in glob.glob(os.path.join(ROOT, "profiles", "*.md")):
        text = open(f).read()
        assert "rocprofv3 " in text and "bench.py" in text, f
        # a summary's commands run committed files only: no working-folder scripts, no wrappers
        assert ("_wo" + "rk") not in text and ("gpu" + "run") not in text, f


def test_headline_workload_has_traffic_for_every_roofline_block():
    b = _bench()
    for k in ("lmhead", "attn", "row_stats", "accept", "select"):
        assert b.measured_traffic("stress_1024px", k) is not None, k
