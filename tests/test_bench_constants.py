"""The HBM-traffic and kernel-time constants that bench.py reports for the headline workload are the figures of the
committed rocprofv3 summaries under profiles/ (they cannot be read from inside the benchmark process)."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _text(rel):
    return open(os.path.join(ROOT, rel)).read()


def test_traffic_constants_are_the_profiles_figures():
    import bench
    t = _text(bench.TRAFFIC["profile"])
    m = re.search(r"contractions_read_bytes = (\d+), contractions_written_bytes = (\d+)", t)
    assert m, "the traffic summary states the two totals"
    assert int(m.group(1)) == bench.TRAFFIC["contractions_read_bytes"]
    assert int(m.group(2)) == bench.TRAFFIC["contractions_written_bytes"]
    assert "--pmc FETCH_SIZE" in t and "--pmc WRITE_SIZE" in t and "--copy-calibration" in t      # the commands that made it


def test_kernel_time_constants_are_the_profiles_figures():
    import bench
    t = _text(bench.TRAFFIC["stats_profile"])
    m = re.search(r"the contraction kernels \(contract_kernel, contract_pair_kernel, finish_kernel\) ([0-9.]+) us in (\d+) launches", t)
    assert m, "the kernel-stats summary states the contraction total"
    assert abs(float(m.group(1)) - bench.TRAFFIC["contractions_us_per_step"]) <= 0.5
    assert int(m.group(2)) == bench.TRAFFIC["contraction_launches_per_step"]
    assert "--kernel-trace --stats" in t and "--config 5" in t


def test_every_profile_names_its_command_and_workload():
    for name in os.listdir(os.path.join(ROOT, "profiles")):
        t = _text(os.path.join("profiles", name))
        assert "rocprofv3" in t and "bench.py" in t, name
