"""The per-launch counters that bench.py uses for `roofline.traffic` and the issue fractions are copies of the
committed rocprofv3 summary: this keeps the two from drifting apart."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)          # defines constants and main(); runs nothing
    return mod


def test_measured_table_matches_the_committed_counter_summary():
    bench = _bench_module()
    rows = {}
    with open(os.path.join(ROOT, "profiles", "keyswitch_step_n16_l24_d4_hbm_traffic.txt")) as f:
        for line in f:
            m = re.match(r"^(\S.*?>)\s+([\d.]+)\s+([\d.]+)\s+(\d+)\s+(\d+)\s+(\d+)\s*$", line)
            if m:
                rows[m.group(1)] = (float(m.group(2)), float(m.group(3)), int(m.group(5)))
    assert set(rows) == set(bench.MEASURED), "kernel lists differ"
    for name, (rd, wr, insts) in bench.MEASURED.items():
        prd, pwr, pinsts = rows[name]
        assert abs(rd - prd) < 0.05 and abs(wr - pwr) < 0.05 and insts == pinsts, name


def test_kernel_stats_summary_lists_the_same_kernels():
    bench = _bench_module()
    names = set()
    with open(os.path.join(ROOT, "profiles", "keyswitch_step_n16_l24_d4_kernel_stats.txt")) as f:
        for line in f:
            m = re.match(r"^(\S.*?>)\s+\d+\s+[\d.]+\s+[\d.]+\s+[\d.]+\s*$", line)
            if m:
                names.add(m.group(1))
    assert names == set(bench.MEASURED)
