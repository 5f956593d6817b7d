"""The tracked table of measured HBM bytes per launch (profiles/hbm_traffic_per_launch.txt) is what bench.py's
`traffic` figures are computed from: it has to parse, cover every timed workload and every kernel of the step, and
agree with the per-kernel tables of the profile summaries beside it (same counter means, same factors)."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
STEP_KERNELS = ["class_pass_kernel(priority_pass)", "class_pass_kernel(deferred_pass)", "gather_rows_kernel",
                "radix_hist_kernel(first_pass)", "radix_hist_kernel(later_passes)", "radix_scatter_kernel(first_pass)",
                "radix_scatter_kernel(later_passes)", "unique_count_kernel", "unique_compact_kernel", "split_flag_kernel",
                "split_compact_kernel", "class_scatter_kernel"]


def test_every_timed_workload_has_every_kernel_of_the_step():
    tab = bench.read_traffic()
    assert tab, "profiles/hbm_traffic_per_launch.txt is missing or empty"
    for c in (1, 2, 3, 4):
        names = {k.split("/")[0] for (w, k) in tab if w == f"configs[{c}]"}
        assert set(STEP_KERNELS) <= names, (c, sorted(set(STEP_KERNELS) - names))
        for (w, k), v in tab.items():
            assert v["bytes"] > 0 and v["launches_per_step"] in (0.5, 1.0, 2.0), (w, k, v)


def test_the_table_is_the_source_of_the_summaries():
    tab = bench.read_traffic()
    for c in (1, 2, 3, 4):
        text = open(os.path.join(ROOT, "profiles", f"step_config{c}_trace_and_traffic.md")).read()
        rows = re.findall(r"^\| (\S+) \| (\d+) \| ([\d.]+) \| ([\d.]+) \| ([\d.]+) \| ([\d.]+) \| ([\d.]+) \|$", text, re.M)
        assert len(rows) >= len(STEP_KERNELS)
        total = 0.0
        for name, _disp, lps, fetch, write, mb, mb_step in rows:
            v = tab[(f"configs[{c}]", name)]
            assert abs(v["bytes"] - (2.0 * float(fetch) + float(write)) * 1024.0) < 1.0, (c, name)
            assert abs(v["bytes"] / 1e6 - float(mb)) < 0.06 and v["launches_per_step"] == float(lps), (c, name)
            total += v["bytes"] * v["launches_per_step"]
        said = float(re.search(r"One step moves ([\d.]+) MB", text).group(1))
        assert abs(total / 1e6 - said) < 0.6, (c, total / 1e6, said)
