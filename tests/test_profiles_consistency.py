"""bench.py takes the per-launch counters behind `roofline.traffic`, the issue fractions and `step_roofline` from the
committed rocprofv3 summary; these checks keep the parser, the two summaries and the kernel names in step."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)          # defines constants and main(); runs nothing
    return mod


def test_counter_table_is_read_from_the_committed_summary():
    bench = _bench_module()
    rows = bench.load_counter_table()
    assert rows and rows == bench.MEASURED
    assert os.path.exists(os.path.join(ROOT, bench.TRAFFIC_SOURCE))
    for name, (rd, wr, insts) in rows.items():
        assert re.match(r"^[a-z_]+<.*>$", name), name
        assert 0 < rd < 4096 and 0 < wr < 4096 and insts > 100000, name
    # the kernels of the default step: both conversions, the inner product on the special limbs and, for HMult
    # and HRot, the q-limb inner product that also ends the ModDown (no separate final kernel)
    for frag in ("conv_fwd_strided_kernel<FpAr, 8, 1", "conv_mfma_kernel<8,", "ks_inner_kernel<FpAr, 8, 1, false, true", "ks_inner_kernel<FpAr, 8, 2, false, true",
                 "ks_inner_kernel<IntAr, 8, 0, false, false", "inv_contig_kernel<FpAr, 8, 1", "inv_strided_kernel<IntAr, 8"):
        assert any(k.startswith(frag) for k in rows), frag
    assert not any(k.startswith("ks_final_kernel") for k in rows)
    assert bench.load_counter_table(os.path.join(ROOT, "no_such_file")) == {}


def test_kernel_stats_summary_lists_the_same_kernels():
    bench = _bench_module()
    names = set()
    with open(os.path.join(ROOT, "profiles", "keyswitch_step_n16_l24_d4_kernel_stats.txt")) as f:
        for line in f:
            m = re.match(r"^(\S.*?>)\s+\d+\s+[\d.]+\s+[\d.]+\s+[\d.]+\s*$", line)
            if m:
                names.add(m.group(1))
    assert names == set(bench.MEASURED)
