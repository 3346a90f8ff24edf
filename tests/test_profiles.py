"""The measured HBM traffic that bench.py reports (`roofline.traffic`) is the figure the
committed rocprofv3 summaries under profiles/ hold: the two must not drift apart."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_traffic_equals_the_profiles():
    assert bench.MEASURED_TRAFFIC_BYTES, "bench.py reports no measured traffic"
    for cfg, value in bench.MEASURED_TRAFFIC_BYTES.items():
        text = open(os.path.join(ROOT, "profiles", f"sweep_kernel_config{cfg}.md")).read()
        m = re.search(r"^traffic_bytes_per_launch: (\d+)$", text, re.M)
        assert m, f"profiles/sweep_kernel_config{cfg}.md has no traffic_bytes_per_launch line"
        assert int(m.group(1)) == value
        # the summary derives that figure from its own counter table: FETCH x scale + WRITE x scale
        rows = dict(re.findall(r"^\| (FETCH_SIZE|WRITE_SIZE) \| (\d+) KiB \| \d+ KiB \| [\d.]+ \| [\d.]+ MB \|$", text, re.M))
        scale = dict(re.findall(r"^\| (FETCH_SIZE|WRITE_SIZE) \| \d+ KiB \| \d+ KiB \| ([\d.]+) \|", text, re.M))
        total = sum(int(rows[k]) * 1024 * float(scale[k]) for k in ("FETCH_SIZE", "WRITE_SIZE"))
        assert abs(total - value) <= 0.002 * value
        # and the command that produced it runs committed files only
        assert "bench.py" in text and "_work" not in text
